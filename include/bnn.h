/*
 * bnn.h -- C ABI of libbnn: inference of a binarized neural network's own layers on one
 * AMD MI355X (gfx950).
 *
 * The library computes what the HEP-BNN paper (Sec. II-A, "Basics of Binarized Neural
 * Networks") defines for the layers of a BNN, and what its problem definition
 * (Sec. II-D) and mapping algorithm (Alg. 1, the "profile(layer(batch_size))" step) ask of
 * an execution backend: run a given model layer by layer on a batch, return the class
 * scores and each layer's device time next to its host-core time.
 *
 * Data conventions.  Every input, output and intermediate tensor is an integer or a bit.  The
 * dense binary layers multiply on the matrix cores with +-1 operands held as FP4 (E2M1) values
 * and FP32 accumulators; all their sums are integers (or odd multiples of 1/2) of magnitude
 * below 2^24, which FP32 holds exactly, so every result equals the integer definition bit for
 * bit.  The first layer uses int8 operands with int32 accumulators, batch <= 8 FC layers use
 * xor + popcount on the vector ALU.
 *   - +1/-1 values are stored one bit each: bit 1 = +1, bit 0 = -1.
 *   - packed vectors: element t lives in 32-bit word t/32 at bit t%32 (LSB first); a row of
 *     k elements takes ceil(k/32) words and the unused high bits of its last word are 0.
 *   - packed activations: uint32 [n][h][w][cw], cw = ceil(c/32), channel c -> word c/32.
 *   - binary conv weights: uint32 [c_out][3][3][cw_in]; FC weights: uint32 [n][ceil(k/32)]
 *     (each output's K bits contiguous).
 *   - int8 images and int32 pre-activations are NHWC.
 *   - flattening a packed activation for an FC layer is the identity on memory
 *     ((h, w, c) order, c fastest); it requires c % 32 == 0.
 *
 * Pointers and ownership
 *   Every pointer named *_dev or documented "device" is device memory owned by the caller,
 *   16-byte aligned, valid until the work queued on `stream` has finished.  The library
 *   never allocates, frees or keeps device memory.  bnn_epilogue, bnn_layer_desc and
 *   bnn_layer_timing are host structs.  `stream` is a hipStream_t passed as void*
 *   (NULL = the default stream).
 *
 * Execution and errors
 *   Layer calls validate all arguments on the host before any HIP call, then enqueue
 *   kernels on `stream` and return without synchronizing.  Every function returns a
 *   bnn_status; BNN_ERR_HIP means a HIP runtime call failed and bnn_last_hip_error()
 *   returns its hipError_t (per thread).  A call with n == 0 / m == 0 / rows == 0
 *   succeeds and does nothing.  Calls on distinct streams may be made from distinct
 *   threads.
 */
#ifndef BNN_H
#define BNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum bnn_status {
    BNN_OK = 0,
    BNN_ERR_NULL = 1,        /* a required pointer is NULL                               */
    BNN_ERR_SHAPE = 2,       /* a size is negative / zero where it may not be / odd pool */
    BNN_ERR_ALIGN = 3,       /* a device pointer is not 16-byte aligned                  */
    BNN_ERR_UNSUPPORTED = 4, /* valid request outside what the kernels implement         */
    BNN_ERR_WORKSPACE = 5,   /* workspace too small                                      */
    BNN_ERR_HIP = 6          /* HIP runtime error, see bnn_last_hip_error()              */
} bnn_status;

/* Static, NUL-terminated name of a status code ("BNN_OK", ...). */
const char *bnn_status_string(bnn_status s);

/* hipError_t (as int) of the calling thread's most recent BNN_ERR_HIP, else 0. */
int bnn_last_hip_error(void);

/* Library version, "major.minor". */
const char *bnn_version(void);

/*
 * Step layer (+ optional max-pool) fused behind a conv / FC layer.
 * Paper Sec. II-A: the step layer is batch-norm followed by the binary activation,
 * evaluated at inference as a comparison with a signed-integer threshold; the maxpool
 * layer takes the maximum over 2x2 windows.
 *   bit[c] = (x[c] > thr[c]) xor (flip[c] != 0)     strict '>', thr int32
 *   pool == 2, pool_first == 0: step, then OR of the four bits of each 2x2 / stride-2 window
 *                               (= max of the +-1 values; the benchmark configurations' order)
 *   pool == 2, pool_first == 1: max of the four int32 pre-activations of the window, then the
 *                               step (the order of the paper's model tables, C -> MP -> S)
 * The two orders agree on channels with flip == 0 and differ where flip != 0.
 * thr:  device, int32 [c_out].   flip: device, uint8 [c_out], or NULL for "no flips".
 * pool: 1 or 2.  pool_first: 0 or 1 (ignored when pool == 1).
 */
typedef struct bnn_epilogue {
    const int32_t *thr;
    const uint8_t *flip;
    int pool;
    int pool_first;
} bnn_epilogue;

/*
 * Bit-pack +-1 values (paper Sec. II-A: weights and activations are 1-bit).
 *   src_dev: device, int8 [rows][k]; an element is +1 iff it is > 0.
 *   dst_dev: device, uint32 [rows][ceil(k/32)], tail bits written as 0.
 * Errors: NULL pointers, rows < 0 or k <= 0 (SHAPE), misaligned pointers.
 */
bnn_status bnn_pack_bits(const int8_t *src_dev, int64_t rows, int64_t k, uint32_t *dst_dev,
                         void *stream);

/*
 * First layer: int8 activations times +-1 weights (paper Sec. II-A convolutional layer,
 * applied to the 8-bit input image; with kh = kw = 1, h = w = 1 it is a fully-connected
 * layer on a flattened image).
 *   x[n,y,x,o] = sum_{i<kh, j<kw, c<c_in} a(n, y+i-pad, x+j-pad, c) * W[o,i,j,c]
 *   a() = in_dev inside the image, pad_value outside; stride 1; int32 accumulation.
 *   in_dev:   device, int8 [n][h][w][c_in].
 *   w_dev:    device, int8 [c_out][kh][kw][c_in], values +1/-1 (any int8 is multiplied as is).
 *   Output size ho = h + 2*pad - kh + 1, wo likewise (must be >= 1).
 *   ep == NULL: preact_out_dev (int32 [n][ho][wo][c_out]) is required, packed_out_dev unused.
 *   ep != NULL: packed_out_dev (uint32 [n][ho/pool][wo/pool][ceil(c_out/32)]) is required
 *               and preact_out_dev is optional (written too when non-NULL).
 * Errors: NULL, SHAPE (also odd ho/wo with pool 2, pool not 1|2, pad_value outside int8),
 *         ALIGN, UNSUPPORTED (kh*kw*c_in > 65536).
 */
bnn_status bnn_conv_first_int8(const int8_t *in_dev, int n, int h, int w, int c_in,
                               const int8_t *w_dev, int c_out, int kh, int kw, int pad,
                               int pad_value, const bnn_epilogue *ep, int32_t *preact_out_dev,
                               uint32_t *packed_out_dev, void *stream);

/*
 * Binary 3x3 convolution, stride 1, one ring of padding whose value is -1 (bit 0), so
 * every output sums exactly K = 9*c_in products (paper Sec. II-A: neuron output
 * 2*popcount(xnor(W, I)) - #bits, i.e. the sum of the K products of +-1 values; evaluated here
 * as that sum on the matrix cores, bits expanded to FP4 +-1.0, FP32 accumulators, exact).
 *   in_dev: device, packed uint32 [n][h][w][ceil(c_in/32)].
 *   w_dev:  device, packed uint32 [c_out][3][3][ceil(c_in/32)].
 *   When c_in % 32 != 0 the unused high bits of every pixel's and every tap's last word must be
 *   0 in both operands (bnn_pack_bits and the fused epilogues write them as 0); they are
 *   counted as matching pairs and the constant is subtracted.
 *   Outputs as for bnn_conv_first_int8 (ho = h, wo = w).
 * Errors: NULL, SHAPE, ALIGN, UNSUPPORTED (c_in > 1024, or one image's packed input of
 *         2 GiB or more).
 * Layers of at most 1024 tiles of 32 pixels x 32 channels (a few images) with c_in in
 * {64, 128, 256, 512, 1024} run on a latency kernel, everything else on the persistent tile
 * kernels; the choice depends on the shape only and the results are identical.
 */
bnn_status bnn_conv_binary(const uint32_t *in_dev, int n, int h, int w, int c_in,
                           const uint32_t *w_dev, int c_out, const bnn_epilogue *ep,
                           int32_t *preact_out_dev, uint32_t *packed_out_dev, void *stream);

/*
 * Binary fully-connected layer / binary GEMM (paper Sec. II-A fully-connected layer):
 *   C[r][o] = sum_t a[r][t]*b[o][t]  ( = K - 2 * sum_words popcount(A[r][.] xor B[o][.]) )
 *   m > 8: matrix cores (FP4 +-1.0 operands, FP32 accumulators, exact for the K accepted);
 *   m <= 8: xor + popcount on the vector ALU (bandwidth bound).
 *   a_dev: device, packed uint32 [m][ceil(k/32)]  (row-major along K)
 *   b_dev: device, packed uint32 [n][ceil(k/32)]  (each output's K bits contiguous)
 *   ep == NULL: c_out_dev (int32 [m][n]) required.
 *   ep != NULL: ep->pool must be 1; packed_out_dev (uint32 [m][ceil(n/32)]) required,
 *               c_out_dev optional.
 * Tail bits of both operands' last words must be 0 (bnn_pack_bits guarantees it).
 * Errors: NULL, SHAPE (also k > 2^30), ALIGN, UNSUPPORTED (m > 8 and k > 2^24 - 2048: the
 *         FP32 accumulators of the matrix-core path would no longer be exact).
 */
bnn_status bnn_fc_binary(const uint32_t *a_dev, int64_t m, int64_t k, const uint32_t *b_dev,
                         int64_t n, const bnn_epilogue *ep, int32_t *c_out_dev,
                         uint32_t *packed_out_dev, void *stream);

/*
 * Stand-alone step (+ pool) layer on int32 pre-activations (paper Sec. II-A step and
 * maxpool layers), same arithmetic and same meaning of pool / pool_first as bnn_epilogue:
 *   preact_dev: device, int32 [n][h][w][c];  thr_dev int32 [c];  flip_dev uint8 [c] or NULL.
 *   packed_out_dev: device, uint32 [n][h/pool][w/pool][ceil(c/32)].
 * Errors: NULL, SHAPE (pool not 1|2, odd h/w with pool 2), ALIGN.
 */
bnn_status bnn_threshold_sign_maxpool(const int32_t *preact_dev, int n, int h, int w, int c,
                                      const int32_t *thr_dev, const uint8_t *flip_dev, int pool,
                                      int pool_first, uint32_t *packed_out_dev, void *stream);

/* ------------------------------------------------------------------ whole model ----- */

typedef enum bnn_layer_kind {
    BNN_LAYER_CONV_FIRST_INT8 = 0,
    BNN_LAYER_CONV_BINARY = 1,
    BNN_LAYER_FC_BINARY = 2
} bnn_layer_kind;

/*
 * One fused layer of a model: conv / FC, then (has_step) step, then (pool == 2) max-pool.
 * Paper Tab. I / Tab. II list these as separate C / S / MP / FLAT / FC entries; the last FC
 * has no step and emits int32 class scores.
 */
typedef struct bnn_layer_desc {
    int kind;               /* bnn_layer_kind                                              */
    int c_in;               /* input channels (conv) or input features (FC)                */
    int c_out;              /* output channels / features                                  */
    int kh, kw, pad;        /* CONV_FIRST_INT8 only (CONV_BINARY is always 3,3,1)          */
    int pad_value;          /* CONV_FIRST_INT8 only                                        */
    int has_step;           /* 1 for hidden layers, 0 for the last layer                   */
    int pool;               /* 1 or 2 (conv layers only; requires has_step)                */
    int pool_first;         /* 0: step then pool, 1: pool then step (see bnn_epilogue)     */
    const void *weights_dev;/* int8 [c_out][kh][kw][c_in] for CONV_FIRST_INT8, else packed */
    const int32_t *thr_dev; /* [c_out], required iff has_step                              */
    const uint8_t *flip_dev;/* [c_out] or NULL                                             */
    int32_t *preact_tap_dev;/* optional: receives this layer's int32 pre-activations       */
    uint32_t *packed_tap_dev;/* optional: receives a copy of this layer's packed output    */
} bnn_layer_desc;

/* One row of the latency table (the per-layer CPU-time / GPU-time pair of Alg. 1). */
typedef struct bnn_layer_timing {
    double gpu_us;            /* hipEvent time of the layer's kernels                      */
    double host_us;           /* wall time of host_fn(layer) on the host cores, 0 if none  */
    int64_t macs;             /* multiply-accumulates of the layer for the whole batch     */
    int64_t bytes_algorithmic;/* bytes the layer must read + write (inputs, weights, out)  */
} bnn_layer_timing;

typedef enum bnn_run_mode {
    BNN_RUN_TIMED = 0,  /* events around every layer, synchronizes, fills `timings`        */
    BNN_RUN_GRAPH = 1,  /* replays the layer chain as one captured hipGraph; asynchronous  */
    BNN_RUN_STREAM = 2  /* plain asynchronous launches on `stream`                         */
} bnn_run_mode;

/* Host callback that runs layer `layer` of the same model on the host cores. */
typedef void (*bnn_host_layer_fn)(int layer, void *ctx);

typedef struct bnn_model bnn_model; /* host object; owns no device memory */

/*
 * Validate a layer list for a fixed batch size and input shape and build the host-side
 * plan.  `layers` is copied.  The first layer must be CONV_FIRST_INT8, the last must be
 * FC_BINARY with has_step == 0, every other layer has has_step == 1.  The transition from
 * a conv layer to an FC layer flattens (h, w, c) and needs c % 32 == 0.
 * Errors: NULL, SHAPE, ALIGN, UNSUPPORTED.  On error *out is NULL.
 */
bnn_status bnn_model_create(const bnn_layer_desc *layers, int n_layers, int batch, int in_h,
                            int in_w, int in_c, bnn_model **out);

/* Bytes of device workspace bnn_run_model needs (two ping-pong activation buffers). */
size_t bnn_model_workspace_bytes(const bnn_model *m);

/* Number of layers / of class scores per image. */
int bnn_model_num_layers(const bnn_model *m);
int bnn_model_num_classes(const bnn_model *m);

/*
 * Run the model on one batch.
 *   input_dev:  device, int8 [batch][in_h][in_w][in_c].
 *   logits_dev: device, int32 [batch][classes].
 *   workspace_dev / workspace_bytes: device scratch >= bnn_model_workspace_bytes().
 *   timings:    host array of n_layers entries; required in TIMED mode, ignored otherwise.
 *   host_fn:    optional (TIMED mode): called once per layer after the device work has
 *               finished, timed with a steady clock into timings[l].host_us.
 * TIMED synchronizes `stream`; GRAPH and STREAM only enqueue.  In GRAPH mode the chain is
 * captured the first time it is run with a given (input, logits, workspace) triple and
 * replayed afterwards; taps are ignored in GRAPH mode.
 * Small batches (three or more layers, the last two FC_BINARY; batch <= 8 with batch x
 * classes <= 512 and a last hidden layer of at most 8192 outputs, or a larger batch whose last
 * hidden layer has at most 1024 outputs, is too small for the 64 x 64 GEMM tiles and feeds at
 * most 16 classes): in GRAPH and STREAM mode the last layer (no step, hence
 * linear in its input bits; Sec. II-A) has no launch of its own.  The first layer's launch zeroes `logits_dev` and the blocks of
 * the layer before the last add their output word's share of every logit with integer
 * atomics (exact in any order).  Results are those of TIMED mode, which keeps one launch per
 * layer; `logits_dev` is written by more than one launch, so it must not alias the input,
 * the workspace or a tap.
 * Errors: NULL, ALIGN, WORKSPACE, HIP.
 */
bnn_status bnn_run_model(bnn_model *m, const int8_t *input_dev, int32_t *logits_dev,
                         void *workspace_dev, size_t workspace_bytes, int mode,
                         bnn_layer_timing *timings, bnn_host_layer_fn host_fn, void *host_ctx,
                         void *stream);

/*
 * bnn_run_model for callers that cannot allocate device memory and have no workspace to hand
 * over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same model, same kernels and same results as bnn_run_model in BNN_RUN_STREAM mode (plain
 * asynchronous launches on `stream`, taps honoured), but the two ping-pong activation buffers
 * live in a fixed array of BNN_NOALLOC_SCRATCH_BYTES bytes of device memory inside the
 * library (each GPU the library runs on holds one from load time until the process ends).
 * The call allocates and frees nothing, on the host side of HIP or through any library.  Its
 * first call on a device looks the array's address up (one hipGetSymbolAddress, no stream
 * work); make that call outside any capture.
 *   - a model whose bnn_model_workspace_bytes() exceeds BNN_NOALLOC_SCRATCH_BYTES is refused
 *     with BNN_ERR_WORKSPACE before any HIP call (VGG-small fits up to batch 512);
 *   - all calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 *     (two streams, two threads) race and give undefined activations; order them;
 *   - the array keeps the previous call's contents; no call depends on them (every layer
 *     overwrites its whole output before it is read).
 * Errors: NULL, ALIGN, WORKSPACE, UNSUPPORTED (device ordinal >= 64), HIP.
 */
#define BNN_NOALLOC_SCRATCH_BYTES (16u << 20)
bnn_status bnn_run_model_noalloc(bnn_model *m, const int8_t *input_dev, int32_t *logits_dev,
                                 void *stream);

/* Free the host object (and its captured graph).  NULL is allowed. */
void bnn_model_destroy(bnn_model *m);

/* ------------------------------------------------------------- host-only helpers ----- */

/*
 * Layer-to-implementation mapping (paper Alg. 1).  Host arrays only, no GPU work.
 *   cpu_us, gpu_us: [n_batch][n_layers][n_impl], the (CPU time, GPU time) pair that profiling
 *                   layer l with implementation j at batch-size index b returned; the
 *                   inference time of the triple is their sum.
 * For every batch size the implementation with the smallest inference time is chosen per
 * layer (the first one wins a tie, as a strict '<' scan does) and the minima are summed; the
 * batch size with the smallest sum wins (first one on a tie).
 *   best_batch:  out, index of that batch size.
 *   mapping:     out, [n_layers] implementation indices at that batch size.
 *   total_us:    out (nullable), its summed inference time.
 * Errors: NULL, SHAPE (any count < 1, a negative or non-finite time).
 */
bnn_status bnn_map_layers(const double *cpu_us, const double *gpu_us, int n_batch, int n_layers,
                          int n_impl, int *best_batch, int *mapping, double *total_us);

/*
 * Batch-norm + sign folded into an integer threshold and a flip flag (paper Sec. II-A: the
 * step layer "can be computed with binary thresholding"; the formula is not given there).
 * For integer pre-activations x the step output is +1 iff
 *     gamma * (x - mean) / sqrt(var + eps) + beta > 0 .
 * With tau = mean - beta * sqrt(var + eps) / gamma this is x > floor(tau) for gamma > 0 and
 * NOT (x > ceil(tau) - 1) for gamma < 0; gamma == 0 gives a constant (beta > 0).
 * All arrays are host arrays of n entries; arithmetic is IEEE double; thresholds are clamped
 * to the int32 range.  Errors: NULL, SHAPE (n < 1, var + eps <= 0, non-finite input).
 */
bnn_status bnn_fold_batchnorm(const double *gamma, const double *beta, const double *mean,
                              const double *var, double eps, int n, int32_t *thr, uint8_t *flip);

#ifdef __cplusplus
}
#endif
#endif /* BNN_H */

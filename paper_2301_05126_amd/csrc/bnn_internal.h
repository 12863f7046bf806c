// Internal declarations shared by the translation units of libbnn (not installed).
#ifndef BNN_INTERNAL_H
#define BNN_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bnn.h"

namespace bnn {

// Where a fused step (+pool) epilogue reads its parameters and writes its results.
// preact == nullptr: int32 pre-activations are not stored.
// packed == nullptr: no step is applied (raw int32 output only).
struct EpiArgs {
    const int32_t *thr;
    const uint8_t *flip;   // may be nullptr (no flips)
    int32_t *preact;
    uint32_t *packed;
    int pool;              // 1 or 2
    int pool_first;        // 1: max of the int32 window first, then the step
};

// The model's last layer (fully connected, no step) folded into the layer that produces its
// input: `w` = that last layer's packed weights [n_out][ceil(n/32)], `logits` = [m][n_out] int32,
// zero when the producing launch starts; every block of the producer adds its share.
struct FcTailArgs {
    const uint32_t *w;
    int32_t *logits;
    int n_out;
};

// A few int32 words that a first-layer launch sets to zero on the side (its blocks with
// blockIdx.y == 0 share them): the accumulator that a later launch of the same chain adds into.
// count == 0: nothing.
struct ClearArgs {
    int32_t *ptr;
    int count;
};

// Records a HIP error for bnn_last_hip_error() and returns BNN_ERR_HIP, or BNN_OK.
bnn_status hip_result(hipError_t e);

// Kernel launchers.  Arguments are already validated; they only pick a launch shape,
// enqueue on `s` and report launch errors.
bnn_status launch_pack_bits(const int8_t *src, int64_t rows, int64_t k, uint32_t *dst,
                            hipStream_t s);
bnn_status launch_threshold_sign_maxpool(const int32_t *x, int n, int h, int w, int c,
                                         const int32_t *thr, const uint8_t *flip, int pool,
                                         int pool_first, uint32_t *out, hipStream_t s);
bnn_status launch_fc_binary(const uint32_t *a, int64_t m, int64_t k, const uint32_t *b, int64_t n,
                            const EpiArgs &ep, hipStream_t s);
// launch_fc_binary with the following (last, step-less) layer of n_out classes folded in, for the
// shapes that run on bgemv_rows or bgemm_small; fc_binary_tail_qualifies says which those are.
// The logits (m x n_out <= FC_TAIL_MAX_LOGITS words) are zeroed on the side by an earlier launch.
constexpr int64_t FC_TAIL_MAX_LOGITS = 1 << 16;
bool fc_binary_tail_qualifies(int64_t m, int64_t n, int64_t n_out);
bnn_status launch_fc_binary_tail(const uint32_t *a, int64_t m, int64_t k, const uint32_t *b, int64_t n,
                                 const EpiArgs &ep, const FcTailArgs &tail, hipStream_t s);
bnn_status launch_conv_binary(const uint32_t *in, int n, int h, int w, int c_in,
                              const uint32_t *wt, int c_out, const EpiArgs &ep, hipStream_t s);
bnn_status launch_conv_first_int8(const int8_t *in, int n, int h, int w, int c_in,
                                  const int8_t *wt, int c_out, int kh, int kw, int pad,
                                  int pad_value, const EpiArgs &ep, const ClearArgs &clear, hipStream_t s);

// The small-problem kernel of launch_conv_binary; BNN_ERR_UNSUPPORTED if the layer does not qualify.
bnn_status launch_conv_binary_small(const uint32_t *in, int n, int h, int w, int c_in,
                                    const uint32_t *wt, int c_out, const EpiArgs &ep, hipStream_t s);

// The persistent tile kernels of launch_conv_binary for any supported shape (launch_conv_binary
// itself sends small layers to the latency kernel first).
bnn_status launch_conv_binary_tiles(const uint32_t *in, int n, int h, int w, int c_in,
                                    const uint32_t *wt, int c_out, const EpiArgs &ep, hipStream_t s);

// Argument checks of bnn_conv_binary (everything before the first HIP call); fills *ea.
bnn_status check_conv_binary(const uint32_t *in_dev, int n, int h, int w, int c_in, const uint32_t *w_dev,
                             int c_out, const bnn_epilogue *ep, int32_t *preact_out_dev,
                             uint32_t *packed_out_dev, EpiArgs *ea);

// Whether launch_conv_binary_small takes this layer.
bool conv_binary_small_qualifies(int n, int h, int w, int c_in, int c_out);

// Which kernel a binary convolution of this shape runs on (host-side query, launches nothing):
// 10 = small-problem kernel, 3 = 256 x 128 block tile, 2 = 128 x 128 with streamed weights,
// 1 = 128 x 128, 0 = 64 x 64, -1 = unsupported shape.  tiles_only: as launch_conv_binary_tiles.
int conv_binary_kernel_choice(int n, int h, int w, int c_in, int c_out, bool tiles_only);

// Whether launch_conv_binary can run this shape (LDS budget of the input patch).
bool conv_binary_supported(int h, int w, int c_in);

// Largest K of bnn_fc_binary on the matrix-core path (m > 8): K plus the zero padding to a whole
// LDS chunk (at most 2047 bits) must not exceed 2^24, the range in which FP32 holds integers exactly.
constexpr int64_t FC_MFMA_MAX_K = ((int64_t)1 << 24) - 2048;

static inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace bnn

#endif

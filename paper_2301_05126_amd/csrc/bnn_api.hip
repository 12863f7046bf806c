// C ABI of libbnn: host-side validation, dispatch to the kernel launchers, and the
// whole-model runner with per-layer timing and hipGraph replay.
#include <chrono>
#include <mutex>
#include <new>
#include <vector>

#include "bnn_internal.h"

namespace bnn {

static thread_local int g_last_hip_error = 0;

bnn_status hip_result(hipError_t e)
{
    if (e == hipSuccess) return BNN_OK;
    g_last_hip_error = (int)e;
    return BNN_ERR_HIP;
}

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Validates an optional fused epilogue and its output pointers.
//   ep == NULL  -> raw output required.
//   ep != NULL  -> packed output required, raw output optional.
static bnn_status check_epilogue(const bnn_epilogue *ep, const void *raw_out, const void *packed_out,
                                 int ho, int wo, bool pool_allowed, EpiArgs *out)
{
    out->thr = nullptr; out->flip = nullptr; out->pool = 1; out->pool_first = 0;
    out->preact = (int32_t *)raw_out;
    out->packed = nullptr;
    if (!ep) {
        if (!raw_out) return BNN_ERR_NULL;
        if (!aligned16(raw_out)) return BNN_ERR_ALIGN;
        return BNN_OK;
    }
    if (!ep->thr || !packed_out) return BNN_ERR_NULL;
    if (ep->pool != 1 && ep->pool != 2) return BNN_ERR_SHAPE;
    if (ep->pool_first != 0 && ep->pool_first != 1) return BNN_ERR_SHAPE;
    if (ep->pool == 2 && (!pool_allowed || (ho & 1) || (wo & 1))) return BNN_ERR_SHAPE;
    if (!aligned16(ep->thr) || !aligned16(packed_out) || (raw_out && !aligned16(raw_out)))
        return BNN_ERR_ALIGN;
    out->thr = ep->thr;
    out->flip = ep->flip;
    out->pool = ep->pool;
    out->pool_first = (ep->pool == 2) ? ep->pool_first : 0;
    out->packed = (uint32_t *)packed_out;
    return BNN_OK;
}

bnn_status check_conv_binary(const uint32_t *in_dev, int n, int h, int w, int c_in, const uint32_t *w_dev,
                             int c_out, const bnn_epilogue *ep, int32_t *preact_out_dev,
                             uint32_t *packed_out_dev, EpiArgs *ea)
{
    if (!in_dev || !w_dev) return BNN_ERR_NULL;
    if (n < 0 || h <= 0 || w <= 0 || c_in <= 0 || c_out <= 0) return BNN_ERR_SHAPE;
    if (c_in > (1 << 24) || (int64_t)h * w > (1 << 30)) return BNN_ERR_SHAPE;
    const bnn_status st = check_epilogue(ep, preact_out_dev, packed_out_dev, h, w, true, ea);
    if (st != BNN_OK) return st;
    if (!aligned16(in_dev) || !aligned16(w_dev)) return BNN_ERR_ALIGN;
    if (!conv_binary_supported(h, w, c_in)) return BNN_ERR_UNSUPPORTED;
    return BNN_OK;
}

}  // namespace bnn

using namespace bnn;

extern "C" {

const char *bnn_status_string(bnn_status s)
{
    switch (s) {
    case BNN_OK: return "BNN_OK";
    case BNN_ERR_NULL: return "BNN_ERR_NULL";
    case BNN_ERR_SHAPE: return "BNN_ERR_SHAPE";
    case BNN_ERR_ALIGN: return "BNN_ERR_ALIGN";
    case BNN_ERR_UNSUPPORTED: return "BNN_ERR_UNSUPPORTED";
    case BNN_ERR_WORKSPACE: return "BNN_ERR_WORKSPACE";
    case BNN_ERR_HIP: return "BNN_ERR_HIP";
    }
    return "BNN_ERR_UNKNOWN";
}

int bnn_last_hip_error(void) { return g_last_hip_error; }

const char *bnn_version(void) { return "0.1"; }

bnn_status bnn_pack_bits(const int8_t *src_dev, int64_t rows, int64_t k, uint32_t *dst_dev, void *stream)
{
    if (!src_dev || !dst_dev) return BNN_ERR_NULL;
    if (rows < 0 || k <= 0) return BNN_ERR_SHAPE;
    if (!aligned16(src_dev) || !aligned16(dst_dev)) return BNN_ERR_ALIGN;
    if (rows > (INT64_MAX / 64) / k) return BNN_ERR_SHAPE;
    return launch_pack_bits(src_dev, rows, k, dst_dev, (hipStream_t)stream);
}

bnn_status bnn_threshold_sign_maxpool(const int32_t *preact_dev, int n, int h, int w, int c,
                                      const int32_t *thr_dev, const uint8_t *flip_dev, int pool,
                                      int pool_first, uint32_t *packed_out_dev, void *stream)
{
    if (!preact_dev || !thr_dev || !packed_out_dev) return BNN_ERR_NULL;
    if (n < 0 || h <= 0 || w <= 0 || c <= 0) return BNN_ERR_SHAPE;
    if (pool != 1 && pool != 2) return BNN_ERR_SHAPE;
    if (pool_first != 0 && pool_first != 1) return BNN_ERR_SHAPE;
    if (pool == 2 && ((h & 1) || (w & 1))) return BNN_ERR_SHAPE;
    if (!aligned16(preact_dev) || !aligned16(thr_dev) || !aligned16(packed_out_dev)) return BNN_ERR_ALIGN;
    return launch_threshold_sign_maxpool(preact_dev, n, h, w, c, thr_dev, flip_dev, pool,
                                         pool == 2 ? pool_first : 0, packed_out_dev,
                                         (hipStream_t)stream);
}

// bnn_fc_binary; with `tail` (small batches only) the model's last layer is folded into this launch.
static bnn_status fc_binary_checked(const uint32_t *a_dev, int64_t m, int64_t k, const uint32_t *b_dev, int64_t n,
                                    const bnn_epilogue *ep, int32_t *c_out_dev, uint32_t *packed_out_dev,
                                    const FcTailArgs *tail, void *stream)
{
    if (!a_dev || !b_dev) return BNN_ERR_NULL;
    if (m < 0 || k <= 0 || n <= 0) return BNN_ERR_SHAPE;
    if (k > (int64_t)1 << 30 || n > (int64_t)1 << 31 || m > (int64_t)1 << 31) return BNN_ERR_SHAPE;
    EpiArgs ea;
    bnn_status st = check_epilogue(ep, c_out_dev, packed_out_dev, 1, 1, false, &ea);
    if (st != BNN_OK) return st;
    if (!aligned16(a_dev) || !aligned16(b_dev)) return BNN_ERR_ALIGN;
    // More than 8 rows run on the matrix cores with FP32 accumulators, which hold the raw sums
    // (at most K rounded up to a whole chunk of 2048 bits in magnitude) exactly only up to 2^24.
    if (m > 8 && k > FC_MFMA_MAX_K) return BNN_ERR_UNSUPPORTED;
    const int64_t tiles = ceil_div64(m, 128) * ceil_div64(n, 128);
    if (tiles > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
    if (tail) return launch_fc_binary_tail(a_dev, m, k, b_dev, n, ea, *tail, (hipStream_t)stream);
    return launch_fc_binary(a_dev, m, k, b_dev, n, ea, (hipStream_t)stream);
}

bnn_status bnn_fc_binary(const uint32_t *a_dev, int64_t m, int64_t k, const uint32_t *b_dev, int64_t n,
                         const bnn_epilogue *ep, int32_t *c_out_dev, uint32_t *packed_out_dev, void *stream)
{
    return fc_binary_checked(a_dev, m, k, b_dev, n, ep, c_out_dev, packed_out_dev, nullptr, stream);
}

bnn_status bnn_conv_binary(const uint32_t *in_dev, int n, int h, int w, int c_in, const uint32_t *w_dev,
                           int c_out, const bnn_epilogue *ep, int32_t *preact_out_dev,
                           uint32_t *packed_out_dev, void *stream)
{
    EpiArgs ea;
    const bnn_status st = check_conv_binary(in_dev, n, h, w, c_in, w_dev, c_out, ep, preact_out_dev, packed_out_dev, &ea);
    if (st != BNN_OK) return st;
    return launch_conv_binary(in_dev, n, h, w, c_in, w_dev, c_out, ea, (hipStream_t)stream);
}

// bnn_conv_first_int8; `clr` names words that the launch also sets to zero (count 0: none).
static bnn_status conv_first_int8_checked(const int8_t *in_dev, int n, int h, int w, int c_in, const int8_t *w_dev,
                                          int c_out, int kh, int kw, int pad, int pad_value,
                                          const bnn_epilogue *ep, int32_t *preact_out_dev,
                                          uint32_t *packed_out_dev, const ClearArgs &clr, void *stream)
{
    if (!in_dev || !w_dev) return BNN_ERR_NULL;
    if (n < 0 || h <= 0 || w <= 0 || c_in <= 0 || c_out <= 0 || kh <= 0 || kw <= 0 || pad < 0)
        return BNN_ERR_SHAPE;
    if (pad_value < -128 || pad_value > 127) return BNN_ERR_SHAPE;
    if (h > (1 << 15) || w > (1 << 15) || pad > (1 << 10)) return BNN_ERR_SHAPE;
    const int64_t ho = (int64_t)h + 2 * pad - kh + 1, wo = (int64_t)w + 2 * pad - kw + 1;
    if (ho <= 0 || wo <= 0) return BNN_ERR_SHAPE;
    if ((int64_t)kh * kw * c_in > 65536) return BNN_ERR_UNSUPPORTED;
    EpiArgs ea;
    bnn_status st = check_epilogue(ep, preact_out_dev, packed_out_dev, (int)ho, (int)wo, true, &ea);
    if (st != BNN_OK) return st;
    if (!aligned16(in_dev) || !aligned16(w_dev)) return BNN_ERR_ALIGN;
    return launch_conv_first_int8(in_dev, n, h, w, c_in, w_dev, c_out, kh, kw, pad, pad_value, ea, clr,
                                  (hipStream_t)stream);
}

bnn_status bnn_conv_first_int8(const int8_t *in_dev, int n, int h, int w, int c_in, const int8_t *w_dev,
                               int c_out, int kh, int kw, int pad, int pad_value, const bnn_epilogue *ep,
                               int32_t *preact_out_dev, uint32_t *packed_out_dev, void *stream)
{
    const ClearArgs none = {nullptr, 0};
    return conv_first_int8_checked(in_dev, n, h, w, c_in, w_dev, c_out, kh, kw, pad, pad_value, ep,
                                   preact_out_dev, packed_out_dev, none, stream);
}

/* ------------------------------------------------------------------ whole model ----- */

struct bnn_model {
    std::vector<bnn_layer_desc> layers;
    int batch, in_h, in_w, in_c;
    // per layer: input spatial shape, output (post-pool) spatial shape, packed output bytes
    std::vector<int> h_in, w_in, h_out, w_out;
    std::vector<int64_t> macs, bytes_alg;
    size_t buf_bytes;          // one ping-pong buffer (256-byte multiple)
    int n_classes;
    // the last two layers fully connected and the one before the last on bgemv_rows or bgemm_small
    // (small batches): outside TIMED mode the last layer (no step, so linear in its input bits)
    // runs inside the launch of the layer before it, which adds each output word's share to the
    // logits; the first layer's launch zeroes them
    bool fold_last;
    // captured graph (GRAPH mode)
    hipGraph_t graph;
    hipGraphExec_t graph_exec;
    const void *g_input; void *g_logits; void *g_ws;
    std::vector<hipEvent_t> events;
};

static size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- device scratch of bnn_run_model_noalloc: the two ping-pong activation buffers that
// bnn_run_model takes from its caller's workspace, here in a fixed array that every GPU the
// library runs on holds from the moment the library is loaded until the process ends.
}  // extern "C"

static __device__ __align__(256) unsigned char scratch[BNN_NOALLOC_SCRATCH_BYTES];

namespace {

// In host code the array's name is only a handle for the symbol lookup below, never an address:
// each device holds its own copy at its own address, fetched once per device (with that device
// current) and used from then on for everything the host does with the array's memory.
constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void *scratch_ptr[MAX_DEVICES] = {};

bnn_status static_scratch_of_current_device(void **out)
{
    int dev = -1;
    bnn_status st = bnn::hip_result(hipGetDevice(&dev));
    if (st != BNN_OK) return st;
    if (dev < 0 || dev >= MAX_DEVICES) return BNN_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        st = bnn::hip_result(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (st != BNN_OK) return st;
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u) != 0) return BNN_ERR_ALIGN;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return BNN_OK;
}

}  // namespace

extern "C" {

bnn_status bnn_model_create(const bnn_layer_desc *layers, int n_layers, int batch, int in_h, int in_w,
                            int in_c, bnn_model **out)
{
    if (out) *out = nullptr;
    if (!layers || !out) return BNN_ERR_NULL;
    if (n_layers < 2 || n_layers > 1024 || batch <= 0 || in_h <= 0 || in_w <= 0 || in_c <= 0)
        return BNN_ERR_SHAPE;
    bnn_model *m = new (std::nothrow) bnn_model();
    if (!m) return BNN_ERR_UNSUPPORTED;
    m->layers.assign(layers, layers + n_layers);
    m->batch = batch; m->in_h = in_h; m->in_w = in_w; m->in_c = in_c;
    m->graph = nullptr; m->graph_exec = nullptr;
    m->g_input = nullptr; m->g_logits = nullptr; m->g_ws = nullptr;
    m->buf_bytes = 0;

    bnn_status st = BNN_OK;
    int h = in_h, w = in_w, c = in_c;
    bool flat = false;
    for (int l = 0; l < n_layers && st == BNN_OK; ++l) {
        const bnn_layer_desc &L = m->layers[l];
        const bool last = (l == n_layers - 1);
        if (!L.weights_dev) { st = BNN_ERR_NULL; break; }
        if (!aligned16(L.weights_dev)) { st = BNN_ERR_ALIGN; break; }
        if (L.c_in <= 0 || L.c_out <= 0) { st = BNN_ERR_SHAPE; break; }
        if ((l == 0) != (L.kind == BNN_LAYER_CONV_FIRST_INT8)) { st = BNN_ERR_UNSUPPORTED; break; }
        if (last && (L.kind != BNN_LAYER_FC_BINARY || L.has_step)) { st = BNN_ERR_UNSUPPORTED; break; }
        if (!last && !L.has_step) { st = BNN_ERR_UNSUPPORTED; break; }
        if (L.has_step) {
            if (!L.thr_dev) { st = BNN_ERR_NULL; break; }
            if (!aligned16(L.thr_dev)) { st = BNN_ERR_ALIGN; break; }
            if (L.pool != 1 && L.pool != 2) { st = BNN_ERR_SHAPE; break; }
            if (L.pool_first != 0 && L.pool_first != 1) { st = BNN_ERR_SHAPE; break; }
        }
        if ((L.preact_tap_dev && !aligned16(L.preact_tap_dev)) ||
            (L.packed_tap_dev && !aligned16(L.packed_tap_dev))) { st = BNN_ERR_ALIGN; break; }
        int ho, wo;
        int64_t fan_in;
        if (L.kind == BNN_LAYER_FC_BINARY) {
            if (!flat) {
                if (l > 0 && (c % 32) != 0 && (int64_t)h * w > 1) { st = BNN_ERR_UNSUPPORTED; break; }
                const int64_t feat = (int64_t)h * w * c;
                if (feat > (1 << 30)) { st = BNN_ERR_SHAPE; break; }
                h = 1; w = 1; c = (int)feat;
                flat = true;
            }
            if (L.c_in != c) { st = BNN_ERR_SHAPE; break; }
            if (L.has_step && L.pool != 1) { st = BNN_ERR_SHAPE; break; }
            ho = 1; wo = 1; fan_in = c;
        } else if (L.kind == BNN_LAYER_CONV_BINARY) {
            if (flat) { st = BNN_ERR_UNSUPPORTED; break; }
            if (L.c_in != c) { st = BNN_ERR_SHAPE; break; }
            if (!conv_binary_supported(h, w, c)) { st = BNN_ERR_UNSUPPORTED; break; }
            ho = h; wo = w; fan_in = 9LL * c;
        } else if (L.kind == BNN_LAYER_CONV_FIRST_INT8) {
            if (L.c_in != c) { st = BNN_ERR_SHAPE; break; }
            if (L.kh <= 0 || L.kw <= 0 || L.pad < 0 || L.pad_value < -128 || L.pad_value > 127) {
                st = BNN_ERR_SHAPE; break;
            }
            ho = h + 2 * L.pad - L.kh + 1; wo = w + 2 * L.pad - L.kw + 1;
            if (ho <= 0 || wo <= 0) { st = BNN_ERR_SHAPE; break; }
            fan_in = (int64_t)L.kh * L.kw * c;
            if (fan_in > 65536) { st = BNN_ERR_UNSUPPORTED; break; }
        } else { st = BNN_ERR_UNSUPPORTED; break; }
        m->h_in.push_back(h); m->w_in.push_back(w);
        const int64_t out_px = (int64_t)batch * ho * wo;
        m->macs.push_back(out_px * L.c_out * fan_in);
        int hp = ho, wp = wo;
        if (L.has_step && L.pool == 2) {
            if ((ho & 1) || (wo & 1)) { st = BNN_ERR_SHAPE; break; }
            hp = ho / 2; wp = wo / 2;
        }
        m->h_out.push_back(hp); m->w_out.push_back(wp);
        // algorithmic bytes: input activations + weights (+ thresholds) + output
        int64_t in_bytes = (L.kind == BNN_LAYER_CONV_FIRST_INT8)
                               ? (int64_t)batch * h * w * c
                               : (int64_t)batch * h * w * ((c + 31) / 32) * 4;
        int64_t w_bytes = (L.kind == BNN_LAYER_CONV_FIRST_INT8)
                              ? (int64_t)L.c_out * fan_in
                              : (int64_t)L.c_out * ((L.kind == BNN_LAYER_CONV_BINARY ? 9 : 1) *
                                                    (int64_t)((c + 31) / 32)) * 4;
        int64_t out_bytes;
        if (L.has_step) {
            out_bytes = (int64_t)batch * hp * wp * ((L.c_out + 31) / 32) * 4;
            w_bytes += (int64_t)L.c_out * 5;
            if ((size_t)out_bytes > m->buf_bytes) m->buf_bytes = (size_t)out_bytes;
        } else {
            out_bytes = (int64_t)batch * L.c_out * 4;
        }
        m->bytes_alg.push_back(in_bytes + w_bytes + out_bytes);
        h = hp; w = wp; c = L.c_out;
    }
    if (st != BNN_OK) { delete m; return st; }
    m->buf_bytes = round_up(m->buf_bytes ? m->buf_bytes : 16, 256);
    m->n_classes = m->layers.back().c_out;
    m->fold_last = n_layers >= 3 && m->layers[n_layers - 2].kind == BNN_LAYER_FC_BINARY &&
                   fc_binary_tail_qualifies(batch, m->layers[n_layers - 2].c_out, m->n_classes);
    *out = m;
    return BNN_OK;
}

size_t bnn_model_workspace_bytes(const bnn_model *m) { return m ? 2 * m->buf_bytes : 0; }
int bnn_model_num_layers(const bnn_model *m) { return m ? (int)m->layers.size() : 0; }
int bnn_model_num_classes(const bnn_model *m) { return m ? m->n_classes : 0; }

// Enqueue layer l: reads `src` (int8 image for l == 0, packed otherwise), writes `dst`
// (packed) or the logits.
// fold: the last layer rides on the launch of the one before it (see bnn_model::fold_last).
static bnn_status enqueue_layer(bnn_model *m, int l, const void *src, void *dst, int32_t *logits,
                                bool taps, bool fold, hipStream_t s)
{
    const bnn_layer_desc &L = m->layers[l];
    const int nl = (int)m->layers.size();
    bnn_epilogue ep;
    ep.thr = L.thr_dev; ep.flip = L.flip_dev; ep.pool = L.has_step ? L.pool : 1;
    ep.pool_first = L.pool_first;
    const bnn_epilogue *epp = L.has_step ? &ep : nullptr;
    int32_t *raw = L.has_step ? (taps ? L.preact_tap_dev : nullptr) : logits;
    uint32_t *packed = L.has_step ? (uint32_t *)dst : nullptr;
    bnn_status st = BNN_OK;
    switch (L.kind) {
    case BNN_LAYER_CONV_FIRST_INT8: {
        const ClearArgs clr = {fold ? logits : nullptr, fold ? m->batch * m->n_classes : 0};
        st = conv_first_int8_checked((const int8_t *)src, m->batch, m->h_in[l], m->w_in[l], L.c_in,
                                     (const int8_t *)L.weights_dev, L.c_out, L.kh, L.kw, L.pad, L.pad_value,
                                     epp, raw, packed, clr, s);
        break;
    }
    case BNN_LAYER_CONV_BINARY:
        st = bnn_conv_binary((const uint32_t *)src, m->batch, m->h_in[l], m->w_in[l], L.c_in,
                             (const uint32_t *)L.weights_dev, L.c_out, epp, raw, packed, s);
        break;
    default:
        if (fold && l == nl - 1) break;             // done by the launch of layer nl - 2
        if (fold && l == nl - 2) {
            const FcTailArgs tail = {(const uint32_t *)m->layers[nl - 1].weights_dev, logits, m->n_classes};
            st = fc_binary_checked((const uint32_t *)src, m->batch, L.c_in, (const uint32_t *)L.weights_dev,
                                   L.c_out, epp, raw, packed, &tail, s);
            break;
        }
        st = bnn_fc_binary((const uint32_t *)src, m->batch, L.c_in, (const uint32_t *)L.weights_dev, L.c_out,
                           epp, raw, packed, s);
        break;
    }
    if (st != BNN_OK) return st;
    if (!L.has_step && taps && L.preact_tap_dev && L.preact_tap_dev != logits) {
        st = hip_result(hipMemcpyAsync(L.preact_tap_dev, logits, (size_t)m->batch * L.c_out * 4,
                                       hipMemcpyDeviceToDevice, s));
        if (st != BNN_OK) return st;
    }
    if (L.has_step && taps && L.packed_tap_dev) {
        const size_t bytes = (size_t)m->batch * m->h_out[l] * m->w_out[l] * ((L.c_out + 31) / 32) * 4;
        st = hip_result(hipMemcpyAsync(L.packed_tap_dev, dst, bytes, hipMemcpyDeviceToDevice, s));
    }
    return st;
}

static bnn_status enqueue_chain(bnn_model *m, const int8_t *input, int32_t *logits, void *ws, bool taps,
                                hipStream_t s, bool timed)
{
    unsigned char *buf[2] = {(unsigned char *)ws, (unsigned char *)ws + m->buf_bytes};
    const void *src = input;
    const int nl = (int)m->layers.size();
    for (int l = 0; l < nl; ++l) {
        if (timed) {
            bnn_status e = hip_result(hipEventRecord(m->events[l], s));
            if (e != BNN_OK) return e;
        }
        void *dst = buf[l & 1];
        bnn_status st = enqueue_layer(m, l, src, dst, logits, taps, !timed && m->fold_last, s);
        if (st != BNN_OK) return st;
        src = dst;
    }
    if (timed) return hip_result(hipEventRecord(m->events[nl], s));
    return BNN_OK;
}

static void drop_graph(bnn_model *m)
{
    if (m->graph_exec) { (void)hipGraphExecDestroy(m->graph_exec); m->graph_exec = nullptr; }
    if (m->graph) { (void)hipGraphDestroy(m->graph); m->graph = nullptr; }
}

bnn_status bnn_run_model(bnn_model *m, const int8_t *input_dev, int32_t *logits_dev, void *workspace_dev,
                         size_t workspace_bytes, int mode, bnn_layer_timing *timings,
                         bnn_host_layer_fn host_fn, void *host_ctx, void *stream)
{
    if (!m || !input_dev || !logits_dev || !workspace_dev) return BNN_ERR_NULL;
    if (mode != BNN_RUN_TIMED && mode != BNN_RUN_GRAPH && mode != BNN_RUN_STREAM) return BNN_ERR_UNSUPPORTED;
    if (mode == BNN_RUN_TIMED && !timings) return BNN_ERR_NULL;
    if (!aligned16(input_dev) || !aligned16(logits_dev) || !aligned16(workspace_dev)) return BNN_ERR_ALIGN;
    if (workspace_bytes < 2 * m->buf_bytes) return BNN_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int nl = (int)m->layers.size();

    if (mode == BNN_RUN_STREAM) return enqueue_chain(m, input_dev, logits_dev, workspace_dev, true, s, false);

    if (mode == BNN_RUN_GRAPH) {
        if (!m->graph_exec || m->g_input != input_dev || m->g_logits != logits_dev || m->g_ws != workspace_dev) {
            drop_graph(m);
            // capture needs a real (non-NULL) stream; use a private one when given the default
            hipStream_t cap = s;
            bool own = false;
            if (!cap) {
                bnn_status e = hip_result(hipStreamCreateWithFlags(&cap, hipStreamNonBlocking));
                if (e != BNN_OK) return e;
                own = true;
            }
            bnn_status st = hip_result(hipStreamBeginCapture(cap, hipStreamCaptureModeThreadLocal));
            if (st == BNN_OK) {
                st = enqueue_chain(m, input_dev, logits_dev, workspace_dev, false, cap, false);
                hipGraph_t gr = nullptr;
                bnn_status st2 = hip_result(hipStreamEndCapture(cap, &gr));
                if (st == BNN_OK) st = st2;
                m->graph = gr;
            }
            if (st == BNN_OK) st = hip_result(hipGraphInstantiate(&m->graph_exec, m->graph, nullptr, nullptr, 0));
            if (own) (void)hipStreamDestroy(cap);
            if (st != BNN_OK) { drop_graph(m); return st; }
            m->g_input = input_dev; m->g_logits = logits_dev; m->g_ws = workspace_dev;
        }
        return hip_result(hipGraphLaunch(m->graph_exec, s));
    }

    // TIMED
    if ((int)m->events.size() != nl + 1) {
        for (hipEvent_t e : m->events) (void)hipEventDestroy(e);
        m->events.clear();
        for (int i = 0; i <= nl; ++i) {
            hipEvent_t e;
            bnn_status st = hip_result(hipEventCreate(&e));
            if (st != BNN_OK) return st;
            m->events.push_back(e);
        }
    }
    bnn_status st = enqueue_chain(m, input_dev, logits_dev, workspace_dev, true, s, true);
    if (st != BNN_OK) return st;
    st = hip_result(hipStreamSynchronize(s));
    if (st != BNN_OK) return st;
    for (int l = 0; l < nl; ++l) {
        float ms = 0.f;
        st = hip_result(hipEventElapsedTime(&ms, m->events[l], m->events[l + 1]));
        if (st != BNN_OK) return st;
        timings[l].gpu_us = (double)ms * 1000.0;
        timings[l].host_us = 0.0;
        timings[l].macs = m->macs[l];
        timings[l].bytes_algorithmic = m->bytes_alg[l];
        if (host_fn) {
            const auto t0 = std::chrono::steady_clock::now();
            host_fn(l, host_ctx);
            const auto t1 = std::chrono::steady_clock::now();
            timings[l].host_us = std::chrono::duration<double, std::micro>(t1 - t0).count();
        }
    }
    return BNN_OK;
}

bnn_status bnn_run_model_noalloc(bnn_model *m, const int8_t *input_dev, int32_t *logits_dev, void *stream)
{
    if (!m || !input_dev || !logits_dev) return BNN_ERR_NULL;
    if (!aligned16(input_dev) || !aligned16(logits_dev)) return BNN_ERR_ALIGN;
    if (2 * m->buf_bytes > (size_t)BNN_NOALLOC_SCRATCH_BYTES) return BNN_ERR_WORKSPACE;
    void *ws = nullptr;
    const bnn_status st = static_scratch_of_current_device(&ws);
    if (st != BNN_OK) return st;
    // every layer overwrites the whole of its output buffer before the next layer reads it, so
    // nothing in the array has to start at zero, whatever an earlier call left there
    return enqueue_chain(m, input_dev, logits_dev, ws, true, (hipStream_t)stream, false);
}

void bnn_model_destroy(bnn_model *m)
{
    if (!m) return;
    drop_graph(m);
    for (hipEvent_t e : m->events) (void)hipEventDestroy(e);
    delete m;
}

}  // extern "C"

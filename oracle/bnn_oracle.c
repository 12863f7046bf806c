/*
 * bnn_oracle.c -- plain CPU definition of the binarized-network layers.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what
 * the GPU library must compute.  It works on UNPACKED values (int8 activations that are
 * +1/-1, or raw int8 pixels for the first layer; int8 +1/-1 weights; int32 sums).  It
 * contains no bit packing, no xor/popcount, no tiling, no fusion, and shares no code,
 * header, table or helper with the HIP library.  Only tests, the smoke check and the
 * CPU-baseline leg of the benchmark may call it.
 *
 * What each function follows (HEP-BNN paper, Sec. II-A "Basics of Binarized Neural
 * Networks"):
 *   - neuron:  the output of a binarized neuron is the +-1 dot product of weights and
 *     inputs compared against a signed-integer threshold T; the paper writes the dot
 *     product as 2*popcount(xnor(W, I)) - #bits.  Here it is written as the plain sum of
 *     products, which is the quantity that expression equals.
 *   - convolutional layer: 2-D convolution, fixed 3x3 filters, output keeps the input's
 *     spatial size (so stride 1 and one ring of padding).
 *   - maxpool layer: maximum over 2x2 windows, halving height and width.
 *   - step layer: batch-norm + binary activation evaluated as a threshold comparison.
 *   - fully-connected layer, flatten layer (a pure re-indexing, (h, w, c) with c fastest).
 *   - model tables (Tab. I, Tab. II): the last fully-connected layer produces the class
 *     scores and is not followed by a step layer.
 *
 * Readings the paper leaves open (pad value, strictness of the comparison, the flip
 * flag, step/pool order) are parameters or separate functions here; the caller picks.
 *
 * All loops are in definition order.  OpenMP, when enabled, splits only the outermost
 * loop over images / rows; every output element is still one sequential sum.
 */
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int ref_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void ref_set_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/*
 * 2-D convolution, stride 1, `pad` rings of padding filled with `pad_value`.
 *   in  : int8  [n][h][w][c_in]          (raw pixels, or +1/-1 activations)
 *   wt  : int8  [c_out][kh][kw][c_in]    (+1/-1)
 *   out : int32 [n][ho][wo][c_out],  ho = h + 2*pad - kh + 1, wo likewise
 * x[n,y,x,o] = sum_{i<kh} sum_{j<kw} sum_{c<c_in} a(n, y+i-pad, x+j-pad, c) * W[o,i,j,c]
 * where a() is the stored value inside the image and pad_value outside it.
 * Returns 0, or -1 on a bad shape.
 */
int ref_conv2d(const int8_t *in, int n, int h, int w, int c_in,
               const int8_t *wt, int c_out, int kh, int kw, int pad, int pad_value,
               int32_t *out)
{
    const int ho = h + 2 * pad - kh + 1;
    const int wo = w + 2 * pad - kw + 1;
    if (n < 0 || h <= 0 || w <= 0 || c_in <= 0 || c_out <= 0 || kh <= 0 || kw <= 0 ||
        pad < 0 || ho <= 0 || wo <= 0)
        return -1;
#pragma omp parallel for schedule(static)
    for (int b = 0; b < n; ++b) {
        for (int y = 0; y < ho; ++y) {
            for (int x = 0; x < wo; ++x) {
                for (int o = 0; o < c_out; ++o) {
                    int32_t sum = 0;
                    for (int i = 0; i < kh; ++i) {
                        for (int j = 0; j < kw; ++j) {
                            const int yy = y + i - pad;
                            const int xx = x + j - pad;
                            const int inside = (yy >= 0 && yy < h && xx >= 0 && xx < w);
                            for (int c = 0; c < c_in; ++c) {
                                int32_t a;
                                if (inside)
                                    a = in[(((size_t)b * h + yy) * w + xx) * c_in + c];
                                else
                                    a = pad_value;
                                const int32_t wv =
                                    wt[(((size_t)o * kh + i) * kw + j) * c_in + c];
                                sum += a * wv;
                            }
                        }
                    }
                    out[(((size_t)b * ho + y) * wo + x) * c_out + o] = sum;
                }
            }
        }
    }
    return 0;
}

/*
 * Fully-connected layer.
 *   a   : int8  [m][k]   (+1/-1, or raw int8)
 *   wt  : int8  [n][k]   (+1/-1)
 *   out : int32 [m][n],  out[r][o] = sum_{t<k} a[r][t] * wt[o][t]
 */
int ref_fc(const int8_t *a, int64_t m, int64_t k, const int8_t *wt, int64_t n, int32_t *out)
{
    if (m < 0 || k <= 0 || n <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < m; ++r) {
        for (int64_t o = 0; o < n; ++o) {
            int32_t sum = 0;
            for (int64_t t = 0; t < k; ++t)
                sum += (int32_t)a[r * k + t] * (int32_t)wt[o * k + t];
            out[r * n + o] = sum;
        }
    }
    return 0;
}

/* One +-1 dot product (used for sampled entries of large products). */
int32_t ref_dot(const int8_t *a, const int8_t *b, int64_t k)
{
    int32_t sum = 0;
    for (int64_t t = 0; t < k; ++t) sum += (int32_t)a[t] * (int32_t)b[t];
    return sum;
}

/*
 * Step layer.  x: int32 [rows][c] (rows = n*h*w), thr: int32 [c], flip: uint8 [c] or NULL.
 * s = +1 if (x > T[c]) xor flip[c], else -1.  Strict comparison: x == T gives -1 when
 * flip = 0 and +1 when flip = 1.
 */
int ref_step(const int32_t *x, int64_t rows, int c, const int32_t *thr, const uint8_t *flip,
             int8_t *out)
{
    if (rows < 0 || c <= 0) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        for (int ch = 0; ch < c; ++ch) {
            int above = x[r * c + ch] > thr[ch];
            int f = flip ? (flip[ch] != 0) : 0;
            out[r * c + ch] = (above != f) ? 1 : -1;
        }
    }
    return 0;
}

/*
 * 2x2 / stride-2 max-pool without padding, on int32 [n][h][w][c] -> [n][h/2][w/2][c].
 * h and w must be even.
 */
int ref_maxpool2_i32(const int32_t *x, int n, int h, int w, int c, int32_t *out)
{
    if (n < 0 || h <= 0 || w <= 0 || c <= 0 || (h & 1) || (w & 1)) return -1;
    const int ho = h / 2, wo = w / 2;
    for (int b = 0; b < n; ++b)
        for (int y = 0; y < ho; ++y)
            for (int xx = 0; xx < wo; ++xx)
                for (int ch = 0; ch < c; ++ch) {
                    int32_t best = x[(((size_t)b * h + 2 * y) * w + 2 * xx) * c + ch];
                    for (int i = 0; i < 2; ++i)
                        for (int j = 0; j < 2; ++j) {
                            int32_t v =
                                x[(((size_t)b * h + 2 * y + i) * w + 2 * xx + j) * c + ch];
                            if (v > best) best = v;
                        }
                    out[(((size_t)b * ho + y) * wo + xx) * c + ch] = best;
                }
    return 0;
}

/* Same pool on int8 values (+1/-1 activations). */
int ref_maxpool2_i8(const int8_t *x, int n, int h, int w, int c, int8_t *out)
{
    if (n < 0 || h <= 0 || w <= 0 || c <= 0 || (h & 1) || (w & 1)) return -1;
    const int ho = h / 2, wo = w / 2;
    for (int b = 0; b < n; ++b)
        for (int y = 0; y < ho; ++y)
            for (int xx = 0; xx < wo; ++xx)
                for (int ch = 0; ch < c; ++ch) {
                    int8_t best = x[(((size_t)b * h + 2 * y) * w + 2 * xx) * c + ch];
                    for (int i = 0; i < 2; ++i)
                        for (int j = 0; j < 2; ++j) {
                            int8_t v =
                                x[(((size_t)b * h + 2 * y + i) * w + 2 * xx + j) * c + ch];
                            if (v > best) best = v;
                        }
                    out[(((size_t)b * ho + y) * wo + xx) * c + ch] = best;
                }
    return 0;
}

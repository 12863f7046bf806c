// First layer for gfx950: int8 activations x +-1 (int8) weights, int32 accumulation.
//
// x[n,y,x,o] = sum_{i<kh, j<kw, c<c_in} a(n, y+i-pad, x+j-pad, c) * W[o,i,j,c]
// (paper Sec. II-A convolutional layer applied to the 8-bit input image; with
// kh = kw = h = w = 1 it is the fully-connected first layer of an MLP).
//
// One lane = one output pixel x 32 output channels.  The flattened taps (i, j, c) are taken
// four at a time with v_dot4_i32_i8: the lane gathers its four activation bytes into a
// dword, the block keeps the weights of its 32 channels in LDS as [tap group][channel]
// dwords (zero beyond K), so every lane of a wave reads the same LDS address (broadcast).
// With pool == 2 lanes are ordered window-major: four neighbouring lanes hold the 2x2
// window and OR their bit words.
#include "bnn_internal.h"

namespace bnn {

namespace {

constexpr int K4C = 256;   // tap groups (of 4) per LDS chunk -> 32 KB of weights

struct FirstGeom {
    int n, h, w, c_in, c_out, kh, kw, pad, pad_value;
    int ho, wo, pool, k, k4;
};

__global__ __launch_bounds__(256) void conv_first_kernel(const int8_t *__restrict__ in,
                                                         const int8_t *__restrict__ wt, FirstGeom g,
                                                         EpiArgs ep)
{
    __shared__ int W4[K4C][32];

    const int t = threadIdx.x;
    const int cg = blockIdx.y;                 // group of 32 output channels
    const int hp = g.ho / g.pool, wp = g.wo / g.pool;
    const int sub_n = g.pool * g.pool;
    const int64_t total = (int64_t)g.n * hp * wp * sub_n;
    const int64_t idx = (int64_t)blockIdx.x * 256 + t;
    const bool live = idx < total;

    int img = 0, y = 0, x = 0, yo = 0, xo = 0;
    {
        int64_t p = live ? idx : 0;
        const int sub = (int)(p % sub_n); p /= sub_n;
        xo = (int)(p % wp); p /= wp;
        yo = (int)(p % hp);
        img = (int)(p / hp);
        y = yo * g.pool + (sub >> 1);
        x = xo * g.pool + (sub & 1);
    }
    const int8_t *img_base = in + (int64_t)img * g.h * g.w * g.c_in;

    int acc[32];
#pragma unroll
    for (int o = 0; o < 32; ++o) acc[o] = 0;

    // running (i, j, c) of flattened tap k; uniform over the block
    int ti = 0, tj = 0, tc = 0;
    for (int k4_base = 0; k4_base < g.k4; k4_base += K4C) {
        const int cnt = min(K4C, g.k4 - k4_base);
        __syncthreads();
        for (int e = t; e < cnt * 32; e += 256) {
            const int k4l = e >> 5, co = e & 31;
            const int o = cg * 32 + co;
            unsigned d = 0;
            if (o < g.c_out) {
                const int kb = (k4_base + k4l) * 4;
                const int8_t *wp8 = wt + (int64_t)o * g.k + kb;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (kb + q < g.k) d |= (unsigned)(uint8_t)wp8[q] << (8 * q);
            }
            W4[k4l][co] = (int)d;
        }
        __syncthreads();

        for (int k4l = 0; k4l < cnt; ++k4l) {
            unsigned a4 = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int k = (k4_base + k4l) * 4 + q;
                if (k < g.k) {
                    const int yy = y + ti - g.pad, xx = x + tj - g.pad;
                    int v = g.pad_value;
                    if (yy >= 0 && yy < g.h && xx >= 0 && xx < g.w)
                        v = img_base[((int64_t)yy * g.w + xx) * g.c_in + tc];
                    a4 |= (unsigned)(uint8_t)(int8_t)v << (8 * q);
                    if (++tc == g.c_in) { tc = 0; if (++tj == g.kw) { tj = 0; ++ti; } }
                }
            }
#pragma unroll
            for (int o = 0; o < 32; ++o)
                acc[o] = __builtin_amdgcn_sdot4((int)a4, W4[k4l][o], acc[o], false);
        }
    }

    const int o0 = cg * 32;
    if (ep.preact && live) {
        int32_t *dst = ep.preact + (((int64_t)img * g.ho + y) * g.wo + x) * g.c_out + o0;
#pragma unroll
        for (int o = 0; o < 32; ++o)
            if (o0 + o < g.c_out) dst[o] = acc[o];
    }
    if (ep.packed) {
        unsigned word = 0;
#pragma unroll
        for (int o = 0; o < 32; ++o) {
            if (o0 + o < g.c_out) {
                bool bit = acc[o] > ep.thr[o0 + o];
                if (ep.flip && ep.flip[o0 + o]) bit = !bit;
                word |= (bit ? 1u : 0u) << o;
            }
        }
        if (!live) word = 0;
        if (g.pool == 2) {
            word |= __shfl_xor(word, 1);
            word |= __shfl_xor(word, 2);
        }
        const int cwo = (g.c_out + 31) >> 5;
        if (live && (g.pool == 1 || (t & 3) == 0))
            ep.packed[(((int64_t)img * hp + yo) * wp + xo) * cwo + cg] = word;
    }
}

}  // namespace

bnn_status launch_conv_first_int8(const int8_t *in, int n, int h, int w, int c_in, const int8_t *wt,
                                  int c_out, int kh, int kw, int pad, int pad_value, const EpiArgs &ep,
                                  hipStream_t s)
{
    if (n == 0) return BNN_OK;
    FirstGeom g;
    g.n = n; g.h = h; g.w = w; g.c_in = c_in; g.c_out = c_out;
    g.kh = kh; g.kw = kw; g.pad = pad; g.pad_value = pad_value;
    g.ho = h + 2 * pad - kh + 1;
    g.wo = w + 2 * pad - kw + 1;
    g.pool = ep.packed ? ep.pool : 1;
    g.k = kh * kw * c_in;
    g.k4 = (g.k + 3) / 4;
    const int64_t total = (int64_t)n * g.ho * g.wo;     // pooled pixels x window size = all pixels
    const int64_t bx = (total + 255) / 256;
    const int by = (c_out + 31) / 32;
    if (bx > 0x7fffffffLL || by > 65535) return BNN_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(conv_first_kernel, dim3((unsigned)bx, (unsigned)by), dim3(256), 0, s, in, wt, g, ep);
    return hip_result(hipGetLastError());
}

}  // namespace bnn

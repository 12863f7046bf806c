// Bandwidth-bound helpers for gfx950: bit packing of +-1 values, and the stand-alone
// step (+ 2x2 max-pool) layer on int32 pre-activations (paper Sec. II-A step / maxpool).
#include "bnn_internal.h"

namespace bnn {

namespace {

// 4 int8 in a dword -> 4 bits, bit q = (byte q > 0).
__device__ __forceinline__ unsigned positive_bits4(uint32_t w)
{
    // bit 7 of each byte: low 7 bits non-zero and sign bit clear
    const uint32_t m = (((w & 0x7f7f7f7fu) + 0x7f7f7f7fu) & ~w) & 0x80808080u;
    // gather bits 7,15,23,31 into bits 24..27 (distinct partial products, no carries)
    return (((m >> 7) * 0x01020408u) >> 24) & 0xfu;
}

__device__ __forceinline__ unsigned positive_bits16(const uint4 &v)
{
    return positive_bits4(v.x) | (positive_bits4(v.y) << 4) | (positive_bits4(v.z) << 8) |
           (positive_bits4(v.w) << 12);
}

// k % 32 == 0 and 16-byte aligned rows: one 16-byte load per lane, two lanes per word.
__global__ __launch_bounds__(256) void pack_bits_fast(const uint4 *__restrict__ src, int64_t n_half,
                                                      uint32_t *__restrict__ dst)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    // n_half is even and the loop trip count is wave-uniform up to the last partial wave;
    // lanes past the end compute zeros so that the pair shuffle stays convergent.
    for (int64_t base = (int64_t)blockIdx.x * 256; base < n_half; base += stride) {
        const int64_t i = base + threadIdx.x;
        unsigned bits = 0;
        if (i < n_half) bits = positive_bits16(src[i]);
        const unsigned other = __shfl_xor(bits, 1);
        if (i < n_half && (threadIdx.x & 1) == 0) dst[i >> 1] = bits | (other << 16);
    }
}

// any k: one thread per output word, byte loads.
__global__ __launch_bounds__(256) void pack_bits_generic(const int8_t *__restrict__ src, int64_t rows,
                                                         int64_t k, int64_t kw, uint32_t *__restrict__ dst)
{
    const int64_t total = rows * kw;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
        const int64_t r = i / kw, wi = i - r * kw;
        const int64_t k0 = wi * 32;
        const int8_t *p = src + r * k + k0;
        const int cnt = (int)((k - k0) < 32 ? (k - k0) : 32);
        unsigned word = 0;
        for (int q = 0; q < cnt; ++q) word |= (p[q] > 0 ? 1u : 0u) << q;
        dst[i] = word;
    }
}

struct StepGeom {
    int n, h, w, c;
    int ho, wo, cwo, pool, pool_first;
};

// One thread per (output pixel, 8-channel group); four neighbouring lanes own one word.
template <bool VEC>
__global__ __launch_bounds__(256) void step_pool_kernel(const int32_t *__restrict__ x,
                                                        const int32_t *__restrict__ thr,
                                                        const uint8_t *__restrict__ flip, StepGeom g,
                                                        uint32_t *__restrict__ out)
{
    const int gpp = g.cwo * 4;                                   // 8-channel groups per pixel
    const int64_t total = (int64_t)g.n * g.ho * g.wo * gpp;      // multiple of 4
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t base = (int64_t)blockIdx.x * 256; base < total; base += stride) {
        const int64_t idx = base + threadIdx.x;
        unsigned byte = 0;
        if (idx < total) {
            const int grp = (int)(idx % gpp);
            int64_t p = idx / gpp;
            const int xo = (int)(p % g.wo); p /= g.wo;
            const int yo = (int)(p % g.ho);
            const int img = (int)(p / g.ho);
            const int c0 = grp * 8;
            if (c0 < g.c) {
                int t[8];
                unsigned fm = 0, valid = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool ok = c0 + j < g.c;
                    t[j] = ok ? thr[c0 + j] : 0;
                    if (ok) valid |= 1u << j;
                    if (ok && flip && flip[c0 + j]) fm |= 1u << j;
                }
                int vmax[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) vmax[j] = INT32_MIN;
                for (int sy = 0; sy < g.pool; ++sy)
                    for (int sx = 0; sx < g.pool; ++sx) {
                        const int y = yo * g.pool + sy, xx = xo * g.pool + sx;
                        const int32_t *src = x + (((int64_t)img * g.h + y) * g.w + xx) * g.c + c0;
                        int v[8];
                        if (VEC) {
                            const int4 v0 = *reinterpret_cast<const int4 *>(src);
                            const int4 v1 = *reinterpret_cast<const int4 *>(src + 4);
                            v[0] = v0.x; v[1] = v0.y; v[2] = v0.z; v[3] = v0.w;
                            v[4] = v1.x; v[5] = v1.y; v[6] = v1.z; v[7] = v1.w;
                        } else {
#pragma unroll
                            for (int j = 0; j < 8; ++j) v[j] = (c0 + j < g.c) ? src[j] : 0;
                        }
                        unsigned b = 0;
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            b |= (v[j] > t[j] ? 1u : 0u) << j;
                            vmax[j] = max(vmax[j], v[j]);
                        }
                        byte |= (b ^ fm) & valid;
                    }
                if (g.pool_first) {
                    // paper order: max of the window's pre-activations, then the step
                    unsigned b = 0;
#pragma unroll
                    for (int j = 0; j < 8; ++j) b |= (vmax[j] > t[j] ? 1u : 0u) << j;
                    byte = (b ^ fm) & valid;
                }
            }
        }
        unsigned word = byte << (8 * (threadIdx.x & 3));
        word |= __shfl_xor(word, 1);
        word |= __shfl_xor(word, 2);
        if (idx < total && (threadIdx.x & 3) == 0) out[idx >> 2] = word;
    }
}

unsigned grid_for(int64_t items)
{
    int64_t blocks = (items + 255) / 256;
    const int64_t cap = 256 * 32;     // 32 blocks per compute unit, grid-stride beyond
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (unsigned)blocks;
}

}  // namespace

bnn_status launch_pack_bits(const int8_t *src, int64_t rows, int64_t k, uint32_t *dst, hipStream_t s)
{
    if (rows == 0) return BNN_OK;
    const int64_t kw = (k + 31) / 32;
    if ((k & 31) == 0) {
        const int64_t n_half = rows * kw * 2;
        hipLaunchKernelGGL(pack_bits_fast, dim3(grid_for(n_half)), dim3(256), 0, s,
                           reinterpret_cast<const uint4 *>(src), n_half, dst);
    } else {
        hipLaunchKernelGGL(pack_bits_generic, dim3(grid_for(rows * kw)), dim3(256), 0, s, src, rows, k, kw,
                           dst);
    }
    return hip_result(hipGetLastError());
}

bnn_status launch_threshold_sign_maxpool(const int32_t *x, int n, int h, int w, int c, const int32_t *thr,
                                         const uint8_t *flip, int pool, int pool_first, uint32_t *out,
                                         hipStream_t s)
{
    if (n == 0) return BNN_OK;
    StepGeom g;
    g.n = n; g.h = h; g.w = w; g.c = c;
    g.pool = pool; g.pool_first = pool_first; g.ho = h / pool; g.wo = w / pool; g.cwo = (c + 31) / 32;
    const int64_t total = (int64_t)n * g.ho * g.wo * g.cwo * 4;
    if ((c & 7) == 0)
        hipLaunchKernelGGL(step_pool_kernel<true>, dim3(grid_for(total)), dim3(256), 0, s, x, thr, flip, g, out);
    else
        hipLaunchKernelGGL(step_pool_kernel<false>, dim3(grid_for(total)), dim3(256), 0, s, x, thr, flip, g, out);
    return hip_result(hipGetLastError());
}

}  // namespace bnn

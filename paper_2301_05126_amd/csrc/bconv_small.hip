// Binary 3x3 convolution for problems too small to fill the chip with the persistent tile
// kernels (a few images): latency, not throughput, is what counts there, and a block of the
// tile kernels runs its K loop on one wave per SIMD.  Here a block owns 32 output pixels x 32
// output channels and its four waves split K in units of up to four MFMA steps (a step = 64 bits
// of K = one channel word per lane half of one tap; a unit = consecutive words of one tap, one
// vector load per operand): wave v takes the units v, v + 4, ..., reads its operand words straight
// from global memory (all loads in flight together with the thresholds and flips, no staging),
// and the partial sums meet in LDS.  (Eight waves per block were measured and are not faster.)  Wave 0
// then runs the step, the pooling and the packing in its registers (a batch-1 launch is bound by its
// instruction count: the tile kernels' epilogue through LDS is three times as long).
// Same conventions: pixels in window-major order, weights as the MFMA's first matrix (rows =
// channels, lanes = pixels), out-of-image taps = -1 = zero bits, FP4 +-1 operands.
#include "bnn_internal.h"
#include "conv_epilogue.h"
#include "lds_dma.h"

namespace bnn {

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));

struct SmallGeom {
    int n, h, w, cw, c_out, k_bits;
    int lth, ltw, ni, tiles_x, tiles_y, n_co_tiles;
    unsigned mg_co, mg_tpg, mg_tx;       // magic_floor of n_co_tiles, tiles per image group, tiles_x
};

// WPH = channel words per lane half per tap; the layer has exactly 2 * WPH words per pixel.
template <int WPH>
__global__ __launch_bounds__(256) void bconv_small(const uint32_t *__restrict__ in, const uint32_t *__restrict__ wt,
                                                   SmallGeom g, EpiArgs ep)
{
    constexpr int NW = 4;                // waves of the block
    __shared__ float red[NW - 1][16][64];    // partial sums of waves 1..NW-1
    constexpr int UW = WPH < 4 ? WPH : 4;    // words (= steps) per unit
    constexpr int UPT = WPH / UW;            // units per tap
    constexpr int NU = 9 * UPT;              // units of the whole K
    constexpr int NUW = (NU + NW - 1) / NW;  // units per wave (the last one may be missing)
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, half = lane >> 5;

    const int ptile = div_by((int)blockIdx.x, g.n_co_tiles, g.mg_co);
    const int o0 = ((int)blockIdx.x - ptile * g.n_co_tiles) * 32;
    const int tpg = g.tiles_x * g.tiles_y;
    const int group = div_by(ptile, tpg, g.mg_tpg);
    const int ty = div_by(ptile - group * tpg, g.tiles_x, g.mg_tx);
    const int tx = ptile - group * tpg - ty * g.tiles_x;
    TilePos pos;
    pos.n = g.n; pos.h = g.h; pos.w = g.w; pos.c_out = g.c_out;
    pos.lth = g.lth; pos.ltw = g.ltw; pos.img0 = group * g.ni; pos.y0 = ty << g.lth; pos.x0 = tx << g.ltw;

    // this lane's pixel (MFMA column) and channel (MFMA row of the weight operand)
    int img, y, x;
    row_to_pixel(l32, pos, img, y, x);
    const bool pix_ok = img < g.n && y < g.h && x < g.w;
    const int o = o0 + l32;
    const bool ch_ok = o < g.c_out;

    // operand words of this wave's units: branch-free, so that all loads are in flight together
    // (a unit that does not exist reads the start of its tensor and is zeroed)
    uint32_t aw[NUW][UW], bw[NUW][UW];
    auto load_unit = [&](const uint32_t *p, uint32_t (&dst)[UW]) {
        if constexpr (UW == 4) {
            const uint4 v = *reinterpret_cast<const uint4 *>(p);
            dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
        } else if constexpr (UW == 2) {
            const uint2 v = *reinterpret_cast<const uint2 *>(p);
            dst[0] = v.x; dst[1] = v.y;
        } else {
            dst[0] = *p;
        }
    };
#pragma unroll
    for (int k = 0; k < NUW; ++k) {
        const int u = wave + NW * k;
        const int tap = u / UPT, cw0 = (u % UPT) * UW;
        const int ti = tap / 3, tj = tap - 3 * ti;
        const int yy = y + ti - 1, xx = x + tj - 1;
        const bool a_ok = u < NU && pix_ok && yy >= 0 && yy < g.h && xx >= 0 && xx < g.w;
        const bool b_ok = u < NU && ch_ok;
        load_unit(in + (unsigned)(a_ok ? ((img * g.h + yy) * g.w + xx) * g.cw + half * WPH + cw0 : 0), aw[k]);
        load_unit(wt + (unsigned)(b_ok ? (o * 9 + tap) * g.cw + half * WPH + cw0 : 0), bw[k]);
#pragma unroll
        for (int q = 0; q < UW; ++q) {
            aw[k][q] = a_ok ? aw[k][q] : 0u;
            bw[k][q] = b_ok ? bw[k][q] : 0u;
        }
    }

    // wave 0's epilogue parameters, requested now so that they arrive with the operands: the
    // thresholds of the lane's 16 channels, and the flip of channel o0 + l32 (one per lane)
    int th[16];
    unsigned flipv = 0;
    if (wave == 0 && ep.packed) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int c = o0 + (r >> 2) * 8 + half * 4 + (r & 3);
            th[r] = ep.thr[c < g.c_out ? c : 0];
        }
        if (ep.flip) flipv = ep.flip[ch_ok ? o : 0];
    }

    uint32_t sgn = 0x88888888u, one = 0x22222222u;
    asm volatile("" : "+s"(sgn));
    asm volatile("" : "+v"(one));
    v16f acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
    for (int k = 0; k < NUW; ++k) {
        if (wave + NW * k < NU) {        // uniform per wave
#pragma unroll
            for (int q = 0; q < UW; ++q) {
                const v8i a = expand_fp4(aw[k][q], sgn, one), b = expand_fp4(bw[k][q], sgn, one);
                acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b, a, acc, 4, 4, 0, 0, 0, 0);
            }
        }
    }

    // ---- the partial sums meet in wave 0 (all values are small integers: exact)
    if (wave > 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wave - 1][r][lane] = acc[r];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
#pragma unroll
            for (int v = 0; v < NW - 1; ++v) acc[r] += red[v][r][lane];

        if (ep.preact) {
            auto getx = [&](int, int, int r) { return (int)acc[r]; };
            conv_tile_store_preact<1, 1>(getx, 0, o0, l32, half, pos, ep.preact);
        }
        if (ep.packed) {
            // The step in registers: register r of lane (l32, half) is channel 8 (r / 4) + 4 half + r % 4
            // of pixel l32; the four lanes 4 j .. 4 j + 3 are one 2x2 window (window-major pixels).
            const bool pool2 = ep.pool == 2, pool_first = pool2 && ep.pool_first != 0;
            int xv[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) xv[r] = (int)acc[r];
            if (pool_first) {                       // max over the window, then the step
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int v = max(xv[r], __shfl_xor(xv[r], 1));
                    xv[r] = max(v, __shfl_xor(v, 2));
                }
            }
            unsigned dec = 0;                       // bit r: x > T, the sign of T - x shifted in from the right
#pragma unroll
            for (int r = 15; r >= 0; --r) {
                const int64_t diff = (int64_t)th[r] - (int64_t)xv[r];
                dec = (dec << 1) | (unsigned)((uint64_t)diff >> 63);
            }
            unsigned bits = (dec & 0x000fu) | ((dec & 0x00f0u) << 4) | ((dec & 0x0f00u) << 8) | ((dec & 0xf000u) << 12);
            bits <<= 4 * half;
            unsigned word = bits | (unsigned)__shfl_xor((int)bits, 32);
            word ^= (unsigned)__ballot(flipv != 0);             // both wave halves hold the tile's 32 flips
            const int left = g.c_out - o0;
            word &= left >= 32 ? 0xffffffffu : (1u << left) - 1u;
            if (pool2 && !pool_first) {             // max of +-1 values = OR of the bits
                word |= (unsigned)__shfl_xor((int)word, 1);
                word |= (unsigned)__shfl_xor((int)word, 2);
            }
            const int nw = (g.c_out + 31) >> 5;
            const int sh = pool2 ? 1 : 0;
            const int64_t at = ((int64_t)(img * (g.h >> sh) + (y >> sh)) * (g.w >> sh) + (x >> sh)) * nw + (o0 >> 5);
            if (half == 0 && pix_ok && (!pool2 || (l32 & 3) == 0)) ep.packed[at] = word;
        }
    }
}

template <int WPH>
bnn_status launch_small(const uint32_t *in, const uint32_t *wt, const SmallGeom &g, unsigned blocks,
                        const EpiArgs &ep, hipStream_t s)
{
    hipLaunchKernelGGL((bconv_small<WPH>), dim3(blocks), dim3(256), 0, s, in, wt, g, ep);
    return hip_result(hipGetLastError());
}

}  // namespace

// Runs the layer on the small-problem kernel if it qualifies: exactly 2 * WPH channel words per
// pixel (C_in a multiple of 64 with a power-of-two word count) and at most 1024 blocks (four per
// compute unit; measured on the VGG-type model: faster than the tile kernels up to there, slower
// beyond).  Returns BNN_ERR_UNSUPPORTED otherwise (the caller then takes the tile kernels).
bool conv_binary_small_qualifies(int n, int h, int w, int c_in, int c_out)
{
    const int cw = (c_in + 31) / 32;
    if ((c_in & 63) != 0 || (cw & (cw - 1)) != 0 || cw > 32) return false;
    const TileShape ts = make_tile_shape(h, w, 32);
    const int64_t ptiles = (int64_t)ts.tiles_x * ts.tiles_y * ((n + ts.ni - 1) / ts.ni);
    return ptiles * ((c_out + 31) / 32) <= 1024;
}

bnn_status launch_conv_binary_small(const uint32_t *in, int n, int h, int w, int c_in, const uint32_t *wt,
                                    int c_out, const EpiArgs &ep, hipStream_t s)
{
    if (!conv_binary_small_qualifies(n, h, w, c_in, c_out)) return BNN_ERR_UNSUPPORTED;
    const int cw = (c_in + 31) / 32;
    const TileShape ts = make_tile_shape(h, w, 32);
    const int64_t ptiles = (int64_t)ts.tiles_x * ts.tiles_y * ((n + ts.ni - 1) / ts.ni);
    const int n_co = (c_out + 31) / 32;
    SmallGeom g;
    g.n = n; g.h = h; g.w = w; g.cw = cw; g.c_out = c_out; g.k_bits = 9 * c_in;
    g.lth = ts.lth; g.ltw = ts.ltw; g.ni = ts.ni; g.tiles_x = ts.tiles_x; g.tiles_y = ts.tiles_y;
    g.n_co_tiles = n_co;
    g.mg_co = magic_floor(n_co);
    g.mg_tpg = magic_floor(ts.tiles_x * ts.tiles_y);
    g.mg_tx = magic_floor(ts.tiles_x);
    const unsigned blocks = (unsigned)(ptiles * n_co);
    switch (cw) {
    case 2: return launch_small<1>(in, wt, g, blocks, ep, s);
    case 4: return launch_small<2>(in, wt, g, blocks, ep, s);
    case 8: return launch_small<4>(in, wt, g, blocks, ep, s);
    case 16: return launch_small<8>(in, wt, g, blocks, ep, s);
    case 32: return launch_small<16>(in, wt, g, blocks, ep, s);
    }
    return BNN_ERR_UNSUPPORTED;
}

}  // namespace bnn

// Epilogue shared by the convolution kernels that run on the matrix cores.
//
// A wave holds TM x TN accumulator tiles of 32 x 32.  GEMM rows are pixels numbered
// window-major inside the block (row = 4 * window + 2*dy + dx, windows enumerated x-fastest
// over the spatial tile, then over the block's images); columns are output channels.
// Accumulator register r of lane (l32, half) is row 8*(r/4) + 4*half + r%4 of its tile and
// column l32, so the four registers r = 4a..4a+3 of a lane are one 2x2 window: max-pool
// after the step layer (paper Sec. II-A) is an OR of four predicates, and a wave-wide ballot
// of a predicate is the packed word of 32 consecutive channels (lower / upper 32 lanes).
#ifndef BNN_CONV_EPILOGUE_H
#define BNN_CONV_EPILOGUE_H

#include <utility>

#include "bnn_internal.h"

namespace bnn {

struct TilePos {
    int n, h, w, c_out;      // output tensor: images, height, width, channels
    int lth, ltw;            // log2 of the spatial tile height / width
    int img0, y0, x0;        // first image and tile origin of this block
};

// Raw int32 output of one wave's tiles (debug / "no step" path).
// getx(i, j, r) returns the integer pre-activation held in accumulator (i, j, r).
// row0 = first GEMM row of this wave inside the block, ch0 = first channel of this wave.
template <int TM, int TN, typename GetX>
__device__ __forceinline__ void conv_tile_store_preact(GetX getx, int row0, int ch0, int l32, int half,
                                                       const TilePos &p, int32_t *preact)
{
    const int lhw = p.ltw - 1, lhh = p.lth - 1;
    const int col0 = ch0 + l32;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int a4 = 0; a4 < 4; ++a4) {
            const int wq = (row0 + i * 32) / 4 + 2 * a4 + half;
            const int wx = wq & ((1 << lhw) - 1);
            const int wy = (wq >> lhw) & ((1 << lhh) - 1);
            const int img = p.img0 + (wq >> (lhw + lhh));
#pragma unroll
            for (int sub = 0; sub < 4; ++sub) {
                const int y = p.y0 + 2 * wy + (sub >> 1), x = p.x0 + 2 * wx + (sub & 1);
                if (img < p.n && y < p.h && x < p.w) {
                    int32_t *dst = preact + (((int64_t)img * p.h + y) * p.w + x) * p.c_out;
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const int col = col0 + j * 32;
                        if (col < p.c_out) dst[col] = getx(i, j, a4 * 4 + sub);
                    }
                }
            }
        }
}

// v_writelane_b32: put a wave-uniform value into lane `LANE` of a register.
template <int LANE>
__device__ __forceinline__ int write_lane(int old, unsigned value)
{
    const unsigned uniform = __builtin_amdgcn_readfirstlane(value);   // pins the value to a scalar register
    asm("v_writelane_b32 %0, %1, %2" : "+v"(old) : "s"(uniform), "n"(LANE));
    return old;
}

// Per-column step parameters of one lane: the threshold of its channel in each of the wave's
// TN tiles and two flags (bit 0: comparison flipped, bit 1: channel exists).  Loaded once
// per block; kept in vector registers, the wave-wide masks are rebuilt where they are used.
template <int TN>
struct StepCols {
    int thr[TN];
    int flags[TN];
};

template <int TN>
__device__ __forceinline__ StepCols<TN> load_step_cols(const EpiArgs &ep, int ch0, int l32, int c_out)
{
    StepCols<TN> sc;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = ch0 + j * 32 + l32;
        const bool cok = col < c_out;
        sc.thr[j] = cok ? ep.thr[col] : 0;
        sc.flags[j] = (cok ? 2 : 0) | ((cok && ep.flip && ep.flip[col]) ? 1 : 0);
    }
    return sc;
}

// One parked word pair: mask halves -> lanes K and 32 + K of `parked`.
template <int K>
__device__ __forceinline__ int park_pair(int parked, unsigned long long m)
{
    parked = write_lane<K>(parked, (unsigned)m);
    parked = write_lane<32 + K>(parked, (unsigned)(m >> 32));
    return parked;
}

template <int TM, int TN, typename GetX, int... R>
__device__ __forceinline__ int park_rows(GetX getx, int i, int j, int thr, unsigned long long fm,
                                         unsigned long long om, std::integer_sequence<int, R...>)
{
    int parked = 0;
    ((parked = park_pair<R>(parked, (__ballot(getx(i, j, R) > thr) ^ fm) & om)), ...);
    return parked;
}

template <int TM, int TN, typename GetX, int... W>
__device__ __forceinline__ int park_windows(GetX getx, int j, int thr, unsigned long long fm,
                                            unsigned long long om, bool pool_first,
                                            std::integer_sequence<int, W...>)
{
    int parked = 0;
    auto window = [&](int i, int a4) {
        unsigned long long m = 0;
        if (pool_first) {
            // max of the four pre-activations, then one comparison
            int x = getx(i, j, a4 * 4);
#pragma unroll
            for (int sub = 1; sub < 4; ++sub) x = max(x, getx(i, j, a4 * 4 + sub));
            m = __ballot(x > thr) ^ fm;
        } else {
#pragma unroll
            for (int sub = 0; sub < 4; ++sub) m |= __ballot(getx(i, j, a4 * 4 + sub) > thr) ^ fm;
        }
        return m & om;
    };
    ((parked = park_pair<W>(parked, window(W / 4, W % 4))), ...);
    return parked;
}

template <int TM, int TN, typename GetX>
__device__ __forceinline__ void conv_tile_step_to_lds(GetX getx, int row0, int word0, int bw, int lane,
                                                      const StepCols<TN> &sc, int pool, bool pool_first,
                                                      uint32_t *out_lds)
{
    const int k = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const unsigned long long fm = __ballot((sc.flags[j] & 1) != 0), om = __ballot((sc.flags[j] & 2) != 0);
        const int thr = sc.thr[j];
        if (pool == 2) {
            // window W = 4i + a4 of this wave -> lanes W (lower rows) and 32 + W
            const int parked = park_windows<TM, TN>(getx, j, thr, fm, om, pool_first, std::make_integer_sequence<int, TM * 4>{});
            // lane (k, hf) holds window (row0/4) + 8*(k/4) + 2*(k%4) + hf
            if (k < TM * 4) out_lds[((row0 >> 2) + (k >> 2) * 8 + (k & 3) * 2 + hf) * bw + word0 + j] = (uint32_t)parked;
        } else {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int parked = park_rows<TM, TN>(getx, i, j, thr, fm, om, std::make_integer_sequence<int, 16>{});
                // lane (k, hf), k < 16, holds row row0 + 32i + 8*(k/4) + 4*hf + k%4
                if (k < 16) out_lds[(row0 + i * 32 + (k >> 2) * 8 + hf * 4 + (k & 3)) * bw + word0 + j] = (uint32_t)parked;
            }
        }
    }
}

// Copy the block's LDS output tile to the packed activation tensor: one thread per output
// pixel in raster order of the tile, bw consecutive words each (vector stores when the
// tensor's words-per-pixel is a multiple of bw).  All threads of the block call it, after a
// barrier that follows conv_tile_step_to_lds.  blk_word0 = first word index of the block.
template <int BW>
__device__ __forceinline__ void conv_tile_copy_out(const uint32_t *out_lds, int block_rows, int blk_word0,
                                                   const TilePos &p, const EpiArgs &ep, int t)
{
    const int pool = ep.pool;
    const int cwo = (p.c_out + 31) >> 5;
    const int lw = pool == 2 ? p.ltw - 1 : p.ltw, lh = pool == 2 ? p.lth - 1 : p.lth;
    const int oh = pool == 2 ? p.h >> 1 : p.h, ow = pool == 2 ? p.w >> 1 : p.w;
    const int oy0 = pool == 2 ? p.y0 >> 1 : p.y0, ox0 = pool == 2 ? p.x0 >> 1 : p.x0;
    const int n_out = pool == 2 ? block_rows >> 2 : block_rows;
    const bool vec_ok = (cwo % BW) == 0;
    for (int q = t; q < n_out; q += 256) {
        const int tx = q & ((1 << lw) - 1);
        const int ty = (q >> lw) & ((1 << lh) - 1);
        const int il = q >> (lw + lh);
        // LDS index: windows are stored x-fastest; un-pooled pixels are window-major
        int src;
        if (pool == 2) {
            src = q;
        } else {
            const int wq = (il << (lw + lh - 2)) | ((ty >> 1) << (lw - 1)) | (tx >> 1);
            src = wq * 4 + (ty & 1) * 2 + (tx & 1);
        }
        const int img = p.img0 + il, y = oy0 + ty, x = ox0 + tx;
        if (img < p.n && y < oh && x < ow) {
            uint32_t *dst = ep.packed + (((int64_t)img * oh + y) * ow + x) * cwo + blk_word0;
            const uint32_t *sp = out_lds + src * BW;
            if (vec_ok) {
                if (BW == 8) {
                    reinterpret_cast<uint4 *>(dst)[0] = reinterpret_cast<const uint4 *>(sp)[0];
                    reinterpret_cast<uint4 *>(dst)[1] = reinterpret_cast<const uint4 *>(sp)[1];
                } else if (BW == 4) *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(sp);
                else if (BW == 2) *reinterpret_cast<uint2 *>(dst) = *reinterpret_cast<const uint2 *>(sp);
                else {
#pragma unroll
                    for (int k = 0; k < BW; ++k) dst[k] = sp[k];
                }
            } else {
#pragma unroll
                for (int k = 0; k < BW; ++k)
                    if (blk_word0 + k < cwo) dst[k] = sp[k];
            }
        }
    }
}

// Spatial tile for `pixels` (a power of two) output pixels per block: as wide as the image
// allows (at most 16), then as tall as allowed; the rest is filled with further images.
struct TileShape {
    int lth, ltw, ni, tiles_x, tiles_y;
};

inline TileShape make_tile_shape(int h, int w, int pixels)
{
    auto log2_ceil = [](int v) { int l = 0; while ((1 << l) < v) ++l; return l; };
    TileShape s;
    const int lp = log2_ceil(pixels);
    int ltw = log2_ceil(w);
    ltw = ltw < 1 ? 1 : (ltw > 4 ? 4 : ltw);
    int lth = log2_ceil(h);
    lth = lth < 1 ? 1 : lth;
    if (lth > lp - ltw) lth = lp - ltw;
    s.ltw = ltw; s.lth = lth;
    s.ni = pixels >> (ltw + lth);
    s.tiles_x = (w + (1 << ltw) - 1) >> ltw;
    s.tiles_y = (h + (1 << lth) - 1) >> lth;
    return s;
}

}  // namespace bnn
#endif

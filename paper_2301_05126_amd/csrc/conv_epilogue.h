// Epilogue shared by the convolution kernels that run on the matrix cores.
//
// A wave holds TM x TN accumulator tiles of 32 x 32 computed as (weights) x (pixels)^T: the
// weight operand is the MFMA's first matrix, so accumulator register r of lane (l32, half)
// is output channel 8*(r/4) + 4*half + r%4 of the tile and pixel l32.  A lane therefore
// owns 16 channels of one pixel:
//   - the step layer (paper Sec. II-A) is, per register, a subtract and a funnel shift that
//     appends the sign bit of (thr - x) to a 16-bit code (x > thr  <=>  thr - x < 0);
//   - the four nibbles of the code are spread to their channel positions, the two lane
//     halves are merged, the per-channel flip word is xor-ed in: one packed word per pixel;
//   - pixels are numbered window-major inside the block (GEMM row = 4 * window + 2*dy + dx,
//     windows x-fastest over the spatial tile, then over the block's images), so a 2x2 pool
//     window is four neighbouring lanes: max-pool after the step is an OR over a lane quad,
//     max-pool before the step a max over the quad (DPP quad permutes).
// Thresholds sit in LDS (clamped to +-2^30, which no sum can reach, so thr - x never
// overflows); words go to an LDS output tile and leave as one vector store per pixel.
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

// Position of GEMM row `row` (window-major) inside the block's tile.
__device__ __forceinline__ void row_to_pixel(int row, const TilePos &p, int &img, int &y, int &x)
{
    const int lhw = p.ltw - 1, lhh = p.lth - 1;
    const int wq = row >> 2, sub = row & 3;
    const int wx = wq & ((1 << lhw) - 1);
    const int wy = (wq >> lhw) & ((1 << lhh) - 1);
    img = p.img0 + (wq >> (lhw + lhh));
    y = p.y0 + 2 * wy + (sub >> 1);
    x = p.x0 + 2 * wx + (sub & 1);
}

// Raw int32 output of one wave's tiles (debug / "no step" path).
// getx(i, j, r): pre-activation of pixel tile i, channel tile j, register r.
// row0 = first GEMM row of this wave inside the block, ch0 = first channel of this wave.
template <int TM, int TN, typename GetX>
__device__ __forceinline__ void conv_tile_store_preact(GetX getx, int row0, int ch0, int l32, int half,
                                                       const TilePos &p, int32_t *preact)
{
    const bool vec_ok = (p.c_out & 3) == 0;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int img, y, x;
        row_to_pixel(row0 + i * 32 + l32, p, img, y, x);
        if (img >= p.n || y >= p.h || x >= p.w) continue;
        int32_t *dst = preact + (((int64_t)img * p.h + y) * p.w + x) * p.c_out;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = ch0 + j * 32 + q * 8 + half * 4;
                if (vec_ok && c + 4 <= p.c_out) {
                    *reinterpret_cast<int4 *>(dst + c) =
                        make_int4(getx(i, j, q * 4), getx(i, j, q * 4 + 1), getx(i, j, q * 4 + 2), getx(i, j, q * 4 + 3));
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (c + k < p.c_out) dst[c + k] = getx(i, j, q * 4 + k);
                }
            }
    }
}

// Block-cooperative: thresholds of the block's `nch` channels (first one ch_blk0) into LDS,
// clamped to +-2^30; channels beyond c_out get 0.  Followed by a barrier before use.
__device__ __forceinline__ void stage_thresholds(const EpiArgs &ep, int ch_blk0, int nch, int c_out,
                                                 int *thr_lds, int t)
{
    for (int c = t; c < nch; c += 256) {
        int v = 0;
        if (ch_blk0 + c < c_out) v = ep.thr[ch_blk0 + c];
        v = v > (1 << 30) ? (1 << 30) : (v < -(1 << 30) ? -(1 << 30) : v);
        thr_lds[c] = v;
    }
}

// Per 32-channel tile of a wave: packed words of the flipped / existing channels.
template <int TN>
struct StepWords {
    unsigned flipw[TN], okw[TN];
};

template <int TN>
__device__ __forceinline__ StepWords<TN> load_step_words(const EpiArgs &ep, int ch0, int l32, int c_out)
{
    StepWords<TN> sw;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = ch0 + j * 32 + l32;
        const bool cok = col < c_out;
        sw.flipw[j] = (unsigned)__ballot(cok && ep.flip && ep.flip[col]);      // lanes 0..31 = channels
        sw.okw[j] = (unsigned)__ballot(cok);
    }
    return sw;
}

// quad-lane exchanges (DPP quad_perm [1,0,3,2] and [2,3,0,1])
__device__ __forceinline__ int quad_xor1(int v) { return __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false); }
__device__ __forceinline__ int quad_xor2(int v) { return __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false); }

// Step (+ pool) of one wave's tiles into the block's LDS output tile.
// out_lds is [output pixel of the block][bw words]; an output pixel is a GEMM row (pool 1) or
// a window (pool 2).  word0 = index, inside the block's bw words, of this wave's first 32
// channels; thr_wave = LDS thresholds of this wave's first channel.
template <int TM, int TN, typename GetX>
__device__ __forceinline__ void conv_tile_step_to_lds(GetX getx, int row0, int word0, int bw, int l32, int half,
                                                      const int *thr_wave, const StepWords<TN> &sw, int pool,
                                                      bool pool_first, uint32_t *out_lds)
{
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        // this lane's 16 thresholds: channels 8q + 4*half + (0..3), q = 0..3
        int thr[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int4 t4 = *reinterpret_cast<const int4 *>(thr_wave + j * 32 + q * 8 + half * 4);
            thr[q * 4] = t4.x; thr[q * 4 + 1] = t4.y; thr[q * 4 + 2] = t4.z; thr[q * 4 + 3] = t4.w;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            unsigned code = 0;                       // bit r = (x_r > thr_r)
#pragma unroll
            for (int r = 15; r >= 0; --r) {
                int x = getx(i, j, r);
                if (pool == 2 && pool_first) {       // max over the window's four pixels first
                    x = max(x, quad_xor1(x));
                    x = max(x, quad_xor2(x));
                }
                code = __builtin_amdgcn_alignbit(code, (unsigned)(thr[r] - x), 31);
            }
            // nibble q of the code -> channels 8q + 4*half .. +3
            unsigned w = (code & 0xFu) | ((code & 0xF0u) << 4) | ((code & 0xF00u) << 8) | ((code & 0xF000u) << 12);
            w <<= 4 * half;
            w |= (unsigned)__shfl_xor((int)w, 32);
            w = (w ^ sw.flipw[j]) & sw.okw[j];
            const int row = row0 + i * 32 + l32;
            if (pool == 2) {
                if (!pool_first) {                   // OR over the window
                    w |= (unsigned)quad_xor1((int)w);
                    w |= (unsigned)quad_xor2((int)w);
                }
                if (half == 0 && (l32 & 3) == 0) out_lds[(row >> 2) * bw + word0 + j] = w;
            } else {
                if (half == 0) out_lds[row * bw + word0 + j] = w;
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

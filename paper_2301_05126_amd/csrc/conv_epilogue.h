// Epilogue shared by the convolution kernels that run on the matrix cores.
//
// A wave holds TM x TN accumulator tiles of 32 x 32 computed as (weights) x (pixels)^T: the
// weight operand is the MFMA's first matrix, so accumulator register r of lane (l32, half)
// is output channel 8*(r/4) + 4*half + r%4 of the tile and pixel l32.  A lane therefore
// owns 16 channels of one pixel:
//   - the step layer (paper Sec. II-A) costs one instruction per value: the accumulators do
//     not start at zero but at a per-channel bias chosen so that the finished sum
//     s = x - thr - 1 (integer sums) or x - thr - 1/2 (FP32 sums) is negative exactly when
//     x <= thr, and a funnel shift appends the sign bit of s to a 16-bit code;
//   - the four nibbles are put at their channel positions, the two lane halves are merged
//     (v_permlane32_swap), and the word is xor-ed with the complement of the per-channel flip
//     word (sign bit set means step = 0): one packed word per pixel;
//   - pixels are numbered window-major inside the block (GEMM row = 4 * window + 2*dy + dx,
//     windows x-fastest over the spatial tile, then over the block's images), so a 2x2 pool
//     window is four neighbouring lanes: max-pool after the step is an OR over a lane quad,
//     max-pool before the step a max over the quad (DPP quad permutes).
// The biases sit in LDS (thresholds clamped to a range no sum can leave, so that nothing
// overflows or rounds); words go to an LDS output tile and leave as one vector store per pixel.
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

// floor(n / d) for 0 <= n < 2^31 and d >= 1 with mg = magic_floor(d) = floor(2^32 / d) (2^32 - 1 for
// d == 1): one multiply-high, which is at most one too small, and a correction.  Stands in for the
// integer divisions of block and tile indices (a run-time division costs some thirty instructions).
__host__ __device__ __forceinline__ unsigned magic_floor(int d) { return d == 1 ? 0xffffffffu : (unsigned)(0x100000000ULL / (unsigned)d); }
__device__ __forceinline__ int div_by(int n, int d, unsigned mg)
{
    unsigned q = __umulhi((unsigned)n, mg);
    if ((unsigned)n - q * (unsigned)d >= (unsigned)d) ++q;
    return (int)q;
}

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
    // (the address arithmetic below hangs on a value the compiler cannot see through, so that it
    // stays inside the caller's "raw output requested" branch instead of running for every tile)
    asm volatile("" : "+v"(l32));
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

// Block-cooperative: accumulator start values of the block's `nch` channels (first one
// ch_blk0) into LDS; followed by a barrier before use.  With a step layer the start value of
// channel c is -(thr_c clamped to +-bound) - 1, otherwise 0: a sum x then ends as
// x - thr - 1, negative iff x <= thr.  |x| <= bound - 1 must hold for every reachable sum.
__device__ __forceinline__ void stage_bias_i32(const EpiArgs &ep, int ch_blk0, int nch, int c_out, int bound,
                                               int *bias_lds, int t)
{
    for (int c = t; c < nch; c += 256) {
        int v = 0;
        if (ep.packed && ch_blk0 + c < c_out) {
            v = ep.thr[ch_blk0 + c];
            v = v > bound ? bound : (v < -bound ? -bound : v);
            v = -v - 1;
        }
        bias_lds[c] = v;
    }
}

// FP32 accumulators whose raw sum is x + corr (corr >= 0: padded positions all count +1):
// start value -(thr_c clamped) - corr - 1/2 with a step layer, otherwise -corr, so the sum
// ends as x - thr - 1/2 (never zero, negative iff x <= thr) or as x.  All values are
// multiples of 1/2 far below 2^23: exact.
__device__ __forceinline__ void stage_bias_f32(const EpiArgs &ep, int ch_blk0, int nch, int c_out, int bound,
                                               int corr, float *bias_lds, int t)
{
    for (int c = t; c < nch; c += 256) {
        float v = -(float)corr;
        if (ep.packed) {
            int th = 0;
            if (ch_blk0 + c < c_out) th = ep.thr[ch_blk0 + c];
            th = th > bound ? bound : (th < -bound ? -bound : th);
            v = -(float)(th + corr) - 0.5f;
        }
        bias_lds[c] = v;
    }
}

// This lane's 16 start values of a 32-channel tile (channels 8q + 4*half + (0..3), q = 0..3),
// in accumulator register order.  bias_tile = LDS start values of the tile's first channel.
template <typename VecT, typename T>
__device__ __forceinline__ VecT load_bias16(const T *bias_tile, int half)
{
    VecT v;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        struct alignas(16) Quad { T a, b, c, d; };
        const Quad f = *reinterpret_cast<const Quad *>(bias_tile + q * 8 + half * 4);
        v[q * 4] = f.a; v[q * 4 + 1] = f.b; v[q * 4 + 2] = f.c; v[q * 4 + 3] = f.d;
    }
    return v;
}

// Per 32-channel tile of a wave: packed words of the not-flipped / existing channels.
template <int TN>
struct StepWords {
    unsigned nflipw[TN], okw[TN];
};

template <int TN>
__device__ __forceinline__ StepWords<TN> load_step_words(const EpiArgs &ep, int ch0, int l32, int c_out)
{
    StepWords<TN> sw;
    uint8_t fl[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = ch0 + j * 32 + l32;
        const bool cok = col < c_out;
        fl[j] = ep.flip ? ep.flip[cok ? col : 0] : (uint8_t)0;      // loads of all tiles in flight together
        sw.okw[j] = (unsigned)__ballot(cok);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) sw.nflipw[j] = ~((unsigned)__ballot(fl[j] != 0) & sw.okw[j]);   // lanes 0..31 = channels
    return sw;
}

// Reductions over the four lanes of a quad, one DPP instruction per exchange (the operation
// reads its first operand through the quad permute).  Written as inline assembly: the compiler
// keeps a separate v_mov_dpp per exchange (and, for fmaxf, a canonicalising v_max).  The
// s_nop covers the two wait states a DPP read needs after a VALU write of the same register.
#define BNN_QUAD_OP(name, type, cons, insn)                                                                   \
    __device__ __forceinline__ type name(type v)                                                              \
    {                                                                                                         \
        type r;                                                                                               \
        asm volatile("s_nop 1\n\t" insn " %0, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf"          \
                     : "=" cons(r) : cons(v));                                                                \
        asm volatile("s_nop 1\n\t" insn " %0, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf"          \
                     : "=" cons(v) : cons(r));                                                                \
        return v;                                                                                             \
    }
BNN_QUAD_OP(quad_max, int, "v", "v_max_i32_dpp")
BNN_QUAD_OP(quad_max, float, "v", "v_max_f32_dpp")
BNN_QUAD_OP(quad_or, unsigned, "v", "v_or_b32_dpp")
#undef BNN_QUAD_OP
__device__ __forceinline__ unsigned value_bits(int v) { return (unsigned)v; }
__device__ __forceinline__ unsigned value_bits(float v) { return __float_as_uint(v); }

// This lane's 16 result bits of one 32 x 32 accumulator tile (register r = 4q + m holds channel
// 8q + 4*half + m; bit set iff x <= thr): one funnel shift per value appends the sign bits to a
// 16-bit chain, ordered so that chain | chain << 12 has nibble q of the result in the low
// nibble of byte q; the other nibbles hold leftovers that merge_half_words drops.
// QMAX: the values are first replaced by the maximum over the window's four pixels.
template <bool QMAX, typename GetR>
__device__ __forceinline__ unsigned tile_half_word(GetR getr)
{
    unsigned chain = 0u;
#pragma unroll
    for (int q : {3, 1, 2, 0}) {                  // chain nibbles 3, 2, 1, 0 = result nibbles 3, 1, 2, 0
#pragma unroll
        for (int m = 3; m >= 0; --m) {
            auto v = getr(4 * q + m);
            if (QMAX) v = quad_max(v);
            chain = __builtin_amdgcn_alignbit(chain, value_bits(v), 31);
        }
    }
    return (chain << 12) | chain;
}

// lo / hi: tile_half_word of the lanes with half == 0 / half == 1 for the same 32 channels and
// pixel -> the 32 result bits (low nibble of every byte from lo, high nibble from hi).
__device__ __forceinline__ unsigned merge_half_words(unsigned lo, unsigned hi)
{
    return (lo & 0x0f0f0f0fu) | ((hi << 4) & 0xf0f0f0f0u);
}

// MODE 0: step; 1: step, then OR over each 2 x 2 window; 2: maximum over the window, then step.
template <int TM, int TN, int MODE, typename GetS>
__device__ __forceinline__ void conv_tile_step_mode(GetS gets, int row0, int word0, int bw, int l32, int half,
                                                    const StepWords<TN> &sw, uint32_t *out_lds)
{
    // LDS word index of pixel tile 0, channel tile 0 (row0 is a multiple of 32); kept in a
    // register as it is (the compiler would rebuild it from its parts before every store)
    unsigned idx0 = (MODE != 0 ? (unsigned)(row0 + l32) >> 2 : (unsigned)(row0 + l32)) * bw + word0;
    if (TN % 2 == 0) idx0 += half;
    asm volatile("" : "+v"(idx0));
    constexpr int ISTRIDE = MODE != 0 ? 8 : 32;              // output pixels per pixel tile
    if constexpr (TN % 2 == 0) {
        // Two channel tiles at a time: lane l and lane l ^ 32 hold complementary nibbles of
        // both tiles' words; one swap leaves the first tile's word complete in lanes 0..31
        // and the second tile's in lanes 32..63, and each lane half finishes and stores its own.
#pragma unroll
        for (int jp = 0; jp < TN / 2; ++jp) {
            const unsigned nflip = half ? sw.nflipw[2 * jp + 1] : sw.nflipw[2 * jp];
            const unsigned ok = half ? sw.okw[2 * jp + 1] : sw.okw[2 * jp];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const unsigned wa = tile_half_word<MODE == 2>([&](int r) { return gets(i, 2 * jp, r); });
                const unsigned wb = tile_half_word<MODE == 2>([&](int r) { return gets(i, 2 * jp + 1, r); });
                // after the swap: [0] = what the half-0 lanes computed, [1] = the half-1 lanes
                const auto sw2 = __builtin_amdgcn_permlane32_swap(wa, wb, false, false);
                unsigned w = (merge_half_words(sw2[0], sw2[1]) ^ nflip) & ok;
                if (MODE == 1) w = quad_or(w);
                if (MODE == 0 || (l32 & 3) == 0) out_lds[idx0 + i * ISTRIDE * bw + 2 * jp] = w;
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                unsigned w = tile_half_word<MODE == 2>([&](int r) { return gets(i, j, r); });
                // merge the two lane halves (lane l and lane l ^ 32 hold complementary nibbles)
                const auto sw2 = __builtin_amdgcn_permlane32_swap(w, w, false, false);
                w = (merge_half_words(sw2[0], sw2[1]) ^ sw.nflipw[j]) & sw.okw[j];
                if (MODE == 1) w = quad_or(w);
                if (half == 0 && (MODE == 0 || (l32 & 3) == 0)) out_lds[idx0 + i * ISTRIDE * bw + j] = w;
            }
        }
    }
}

// Step (+ pool) of one wave's tiles into the block's LDS output tile.
// gets(i, j, r): finished biased sum (int or float) of pixel tile i, channel tile j, register
// r; its sign bit is set iff x <= thr.  out_lds is [output pixel of the block][bw words]; an
// output pixel is a GEMM row (pool 1) or a window (pool 2).  word0 = index, inside the
// block's bw words, of this wave's first 32 channels.  (One straight-line variant per mode.)
template <int TM, int TN, typename GetS>
__device__ __forceinline__ void conv_tile_step_to_lds(GetS gets, int row0, int word0, int bw, int l32, int half,
                                                      const StepWords<TN> &sw, int pool, bool pool_first,
                                                      uint32_t *out_lds)
{
    if (pool == 2 && pool_first) conv_tile_step_mode<TM, TN, 2>(gets, row0, word0, bw, l32, half, sw, out_lds);
    else if (pool == 2) conv_tile_step_mode<TM, TN, 1>(gets, row0, word0, bw, l32, half, sw, out_lds);
    else conv_tile_step_mode<TM, TN, 0>(gets, row0, word0, bw, l32, half, sw, out_lds);
}

// Copy of the block's LDS output tile to the packed activation tensor: thread t moves output
// pixel t of the tile (raster order; block_rows <= 256 pixels, bw consecutive words each, as
// vector stores when the tensor's words-per-pixel is a multiple of bw).  What does not depend
// on the tile's position is worked out once per kernel (make_copy_lane); all threads of the
// block call conv_tile_copy_out after a barrier that follows conv_tile_step_to_lds.
struct CopyLane {
    int tx, ty, il;     // output pixel relative to the tile origin: column, row, image
    int src;            // its index in the LDS tile
    int rel;            // its word offset from the tile origin's pixel in the output tensor
    bool active;        // the tile has such a pixel
};

// p: any tile position of this kernel (only the geometry is used).
__device__ __forceinline__ CopyLane make_copy_lane(int block_rows, const TilePos &p, int pool, int t)
{
    const int cwo = (p.c_out + 31) >> 5;
    const int lw = pool == 2 ? p.ltw - 1 : p.ltw, lh = pool == 2 ? p.lth - 1 : p.lth;
    const int oh = pool == 2 ? p.h >> 1 : p.h, ow = pool == 2 ? p.w >> 1 : p.w;
    const int n_out = pool == 2 ? block_rows >> 2 : block_rows;
    CopyLane c;
    c.active = t < n_out;
    c.tx = t & ((1 << lw) - 1);
    c.ty = (t >> lw) & ((1 << lh) - 1);
    c.il = t >> (lw + lh);
    // LDS index: windows are stored x-fastest; un-pooled pixels are window-major
    if (pool == 2) {
        c.src = t;
    } else {
        const int wq = (c.il << (lw + lh - 2)) | ((c.ty >> 1) << (lw - 1)) | (c.tx >> 1);
        c.src = wq * 4 + (c.ty & 1) * 2 + (c.tx & 1);
    }
    // several images per tile only when an image is smaller than the tile: the offset is small
    c.rel = ((c.il * oh + c.ty) * ow + c.tx) * cwo;
    return c;
}

// blk_word0 = first word index of the block inside a pixel's words.
template <int BW>
__device__ __forceinline__ void conv_tile_copy_out(const uint32_t *out_lds, const CopyLane &c, int blk_word0,
                                                   const TilePos &p, const EpiArgs &ep)
{
    const int pool = ep.pool;
    const int cwo = (p.c_out + 31) >> 5;
    const int oh = pool == 2 ? p.h >> 1 : p.h, ow = pool == 2 ? p.w >> 1 : p.w;
    const int oy0 = pool == 2 ? p.y0 >> 1 : p.y0, ox0 = pool == 2 ? p.x0 >> 1 : p.x0;
    const bool vec_ok = (cwo % BW) == 0;
    if (c.active && p.img0 + c.il < p.n && oy0 + c.ty < oh && ox0 + c.tx < ow) {
        // the origin's part of the address is the same for every thread
        uint32_t *dst = ep.packed + ((((int64_t)p.img0 * oh + oy0) * ow + ox0) * cwo + blk_word0) + c.rel;
        const uint32_t *sp = out_lds + c.src * BW;
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

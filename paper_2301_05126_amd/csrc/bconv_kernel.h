// Binary 3x3 convolution (stride 1, pad 1 with -1) for gfx950: im2col-free, on the matrix
// cores.
//
// x[n,y,x,o] = sum_{tap, c} a(n, y+i-1, x+j-1, c) * W[o, tap, c] over +-1 values (paper
// Sec. II-A: convolutional layer of binarized neurons, 2*popcount(xnor) - #bits).  Taps that
// fall outside the image read zero words, i.e. -1 activations, so every output sums exactly
// K = 9*c_in products.
//
// A block of 4 waves (2 x 2) computes (64*TM pixels) x (64*TN output channels) per pixel
// tile and is persistent: it keeps one channel tile and walks over pixel tiles.  The pixels
// of a tile are `ni` images x (th x tw) spatial tile whose input patch, halo included, sits
// in LDS as packed words; the nine taps are read from it with shifted addresses.  Weights
// are resident in LDS when they fit, else they stream through it in chunks of a few taps.
// Every 32-bit word of either operand is expanded in registers into 32 FP4 values +-1.0 and
// multiplied by v_mfma_f32_32x32x64_f8f6f4 (no block scales); all sums are multiples of 1/2
// far below 2^23, so the FP32 accumulators are exact.  Within one MFMA the lower 32 lanes
// supply the first half of a pixel's channel words and the upper 32 lanes the second half
// (same split on the weight side).
//
// The weights are the MFMA's first operand, so a lane owns 16 channels of one pixel, and
// pixels are numbered window-major (four consecutive rows of the implicit GEMM are one 2x2
// window = one lane quad); the step and pool layers fused behind the sums are described in
// conv_epilogue.h.
#ifndef BNN_BCONV_KERNEL_H
#define BNN_BCONV_KERNEL_H
#include <mutex>

#include "bnn_internal.h"
#include "conv_epilogue.h"
#include "lds_dma.h"

namespace bnn {

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));

// LDS per block: gfx950 has 160 KB per compute unit and lets one block take all of it; two
// resident blocks per compute unit leave 80 KB each.
constexpr int MAX_SMEM = 80 * 1024;

template <int V> struct WordVec;
template <> struct WordVec<4> { using type = uint4; };
template <> struct WordVec<2> { using type = uint2; };
template <> struct WordVec<1> { using type = uint32_t; };

__device__ __forceinline__ uint32_t vec_word(const uint4 &v, int q) { return q == 0 ? v.x : (q == 1 ? v.y : (q == 2 ? v.z : v.w)); }
__device__ __forceinline__ uint32_t vec_word(const uint2 &v, int q) { return q == 0 ? v.x : v.y; }
__device__ __forceinline__ uint32_t vec_word(const uint32_t &v, int) { return v; }
// operand of a word group's first step (see expand_pair_half for the two-word groups)
template <int V, typename VecT>
__device__ __forceinline__ v8i expand_first(const VecT &v, uint32_t sgn, uint32_t one)
{
    if constexpr (V == 2) {
        const uint2 lo = expand_pair_half(v, 0, 0, sgn, one), hi = expand_pair_half(v, 0, 1, sgn, one);
        v8i r;
        r[0] = (int)lo.x; r[1] = (int)lo.y; r[2] = (int)hi.x; r[3] = (int)hi.y;
        r[4] = 0; r[5] = 0; r[6] = 0; r[7] = 0;
        return r;
    } else {
        return expand_fp4(vec_word(v, 0), sgn, one);
    }
}

__device__ __forceinline__ void vec_set(uint4 &v, int q, uint32_t x) { if (q == 0) v.x = x; else if (q == 1) v.y = x; else if (q == 2) v.z = x; else v.w = x; }
__device__ __forceinline__ void vec_set(uint2 &v, int q, uint32_t x) { if (q == 0) v.x = x; else v.y = x; }
__device__ __forceinline__ void vec_set(uint32_t &v, int, uint32_t x) { v = x; }

// Steps (one MFMA K-slice = one word per lane half) per weight chunk, by words per half.
constexpr int steps_per_chunk(int wph) { return wph == 1 ? 9 : (wph == 2 ? 18 : (wph == 4 ? 12 : 8)); }

// Whether a block keeps all of its weight chunks in LDS at once: up to 40 KB for any tile
// (C_in <= 256 with 128 output channels), up to 48 KB for the 64-channel tile.
constexpr bool weights_resident(int tm, int tn, int wph)
{
    const int v = wph >= 2 ? 2 : wph;
    const int lsb = 2 * steps_per_chunk(wph) + v;
    const int nchunk = 9 * wph / steps_per_chunk(wph);
    const int bytes = nchunk * 64 * tn * lsb * 4;
    return bytes <= 40 * 1024 || (tm * tn == 1 && bytes <= 48 * 1024);
}

struct TileCoord {
    int group, ty, tx;           // image group, tile row, tile column
};

struct ConvGeom {
    int n, h, w, cw;             // input: images, height, width, words per pixel
    int c_out, k_bits;           // outputs, K = 9*c_in
    int lth, ltw;                // log2 of the spatial tile height / width (both >= 1)
    int ni;                      // images per pixel tile; ni * th * tw == pixels per block
    int tiles_x, tiles_y, n_co_tiles;
    int n_ptiles;                // pixel tiles in the layer
    int slots;                   // blocks per channel tile = pixel tiles in flight
    int patch_words;             // LDS words of one patch buffer (rounded up)
    int dbuf;                    // 1: two patch buffers, the next tile's patch is fetched during the MFMAs
    unsigned mg_pw, mg_ph;       // ceil(2^32 / d) for d = patch width, patch height (staging index math)
    int step_group, step_ty, step_tx;    // `slots` pixel tiles as an (image group, tile row, tile column) increment
    unsigned mg_co, mg_tpg, mg_tx;       // magic_floor of n_co_tiles, tiles per image group, tiles_x
};

// WPH = words per lane half per tap; the layer's cw words per pixel are zero-padded to 2*WPH.
//
// Blocks are persistent: block b owns channel tile b % n_co_tiles for its whole life (so
// thresholds, and the weights when they are resident, are fetched once) and walks the pixel
// tiles slot, slot + slots, ...  The input patch of a tile goes global -> LDS without passing
// through registers (buffer_load ... lds; lanes outside the image or beyond the last image
// address past the buffer's end and deliver zeros, i.e. -1 padding); with two patch buffers
// the next tile's patch is in flight while the current tile is multiplied.
//
// WDMA (wide layers whose weights are not resident; needs cw == 2*WPH words per pixel and
// c_out a multiple of the block's channels): weight chunks also travel global -> LDS without
// passing through registers, into two buffers that alternate; the chunk sequence is cyclic
// over the tiles (weights do not depend on the tile), so the next chunk is always in flight
// behind the current one and a chunk costs one barrier.  Rows are unpadded (16 words) and
// their 8-byte units are stored at position unit ^ ((row >> 1) & 7), which keeps the 32 rows
// read by one instruction on distinct banks.
template <int TM, int TN, int WPH, bool WDMA = false>
__global__ __launch_bounds__(256, 2)
void bconv_mfma(const uint32_t *__restrict__ in, const uint32_t *__restrict__ wt, ConvGeom g, EpiArgs ep)
{
    constexpr int BN = 64 * TN;
    constexpr int BW = 2 * TN;                         // packed output words per pixel of a block
    constexpr int CWP = 2 * WPH;                       // padded words per pixel
    constexpr int V = WPH >= 2 ? 2 : WPH;              // words per LDS access
    constexpr int SPC = steps_per_chunk(WPH);
    constexpr int NCHUNK = 9 * WPH / SPC;
    constexpr int LSB = WDMA ? 2 * SPC : 2 * SPC + V;  // weight row stride (words); padded: LSB/V is odd
    constexpr int UPRW = 2 * SPC / V;                  // weight units per row per chunk
    constexpr int STG = (BN * UPRW + 255) / 256;       // weight units per thread per chunk
    constexpr int NVG = SPC / V;                       // V-step groups per chunk
    constexpr bool RES = !WDMA && weights_resident(TM, TN, WPH);
    constexpr int NBUF = RES ? NCHUNK : (WDMA ? 2 : 1);
    static_assert(!WDMA || (SPC == 8 && V == 2 && BN == 128), "weight DMA layout: 16-word rows, 128 rows");
    static_assert(NCHUNK == 1 || (SPC % 2 == 0 && NVG % 2 == 0), "operand pipeline across chunks: buffer parity");
    using vec_t = typename WordVec<V>::type;

    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *Bs = reinterpret_cast<uint32_t *>(smem);                 // [NBUF][BN][LSB] weights
    float *Ts = reinterpret_cast<float *>(Bs + NBUF * BN * LSB);       // [BN] accumulator start values
    uint32_t *Os = reinterpret_cast<uint32_t *>(Ts + BN);              // [2][64*TM][BW] output tiles
    uint32_t *Ps = Os + 2 * 64 * TM * BW;                              // [1 or 2][patch_words]

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, half = lane >> 5;

    // XCD-aware order: hardware deals consecutive block ids round-robin to the 8 XCDs (one L2
    // each); renumber so that blocks working on the same pixel tile (its channel tiles) share
    // an XCD and the patch is fetched from HBM once.
    int bid = blockIdx.x;
    if ((gridDim.x & 7) == 0) bid = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int slot = div_by(bid, g.n_co_tiles, g.mg_co);
    const int co_tile = bid - slot * g.n_co_tiles;
    const int th = 1 << g.lth, tw = 1 << g.ltw;
    const int o_blk = co_tile * BN;
    const int pw = tw + 2, ph = th + 2;
    const int tiles_per_group = g.tiles_x * g.tiles_y;

    // ---- per-channel step parameters and (if resident) all weight chunks: once per block,
    // requested further down, behind the first patch, so that all of it is in flight together
    const int corr = 9 * CWP * 32 - g.k_bits;          // padded positions all counted as +1
    StepWords<TN> sw;
    const float *Tw = Ts + wn * TN * 32;               // this wave's channels

    // weight staging: LDS row = [half 0: SPC words][half 1: SPC words]; the word of
    // (half, step) is W[o][tap][half*WPH + cwi] with tap = step / WPH, cwi = step % WPH.
    vec_t pb[STG];
    const bool wvec_ok = (g.cw % V) == 0;
    // A thread's units keep their row and position inside the chunk; per chunk only a uniform
    // (tap, word) offset is added.  (step = chunk * SPC + vg * V splits into a chunk part and a
    // unit part without carry because SPC is a multiple of WPH or the other way round.)
    static_assert(SPC % WPH == 0 || WPH % SPC == 0, "chunk and unit parts of a step index add without carry");
    int wu_off[STG], wu_cw[STG];                       // word offset / word inside the pixel, chunk 0
    bool wu_row[STG];
    if (!WDMA) {
#pragma unroll
        for (int r = 0; r < STG; ++r) {
            const int idx = t + 256 * r;
            const int row = idx / UPRW, u = idx % UPRW;
            const int hh = u / NVG, s0 = (u % NVG) * V;
            const int tapr = WPH <= SPC ? s0 / WPH : 0, cwir = WPH <= SPC ? s0 % WPH : s0;
            const int o = o_blk + row;
            wu_row[r] = row < BN && o < g.c_out;
            wu_cw[r] = hh * WPH + cwir;
            wu_off[r] = (o * 9 + tapr) * g.cw + wu_cw[r];
        }
    }
    auto load_w_to = [&](int chunk, vec_t (&dst)[STG]) {
        // Branch-free inside each loop, so that all loads of a chunk are in flight together:
        // rows or words that do not exist read the first weight word and are zeroed afterwards.
        const int sc = chunk * SPC;
        const int cwic = sc % WPH;
        const int coff = (sc / WPH) * g.cw + cwic;
        auto unit = [&](int r, bool &row_ok, int &cwpos) {
            cwpos = wu_cw[r] + cwic;
            row_ok = wu_row[r];
            return wu_off[r] + coff;
        };
        if (wvec_ok) {
#pragma unroll
            for (int r = 0; r < STG; ++r) {
                bool row_ok;
                int cwpos;
                const int off = unit(r, row_ok, cwpos);
                const bool ok = row_ok && cwpos < g.cw;
                vec_t v = *reinterpret_cast<const vec_t *>(wt + (unsigned)(ok ? off : 0));
#pragma unroll
                for (int q = 0; q < V; ++q) vec_set(v, q, ok ? vec_word(v, q) : 0u);
                dst[r] = v;
            }
        } else {
#pragma unroll
            for (int r = 0; r < STG; ++r) {
                bool row_ok;
                int cwpos;
                const int off = unit(r, row_ok, cwpos);
                vec_t v;
#pragma unroll
                for (int q = 0; q < V; ++q) {
                    const bool ok = row_ok && cwpos + q < g.cw;
                    const uint32_t x = wt[(unsigned)(ok ? off + q : 0)];
                    vec_set(v, q, ok ? x : 0u);
                }
                dst[r] = v;
            }
        }
    };
    auto store_w_from = [&](int buf, const vec_t (&src)[STG]) {
#pragma unroll
        for (int r = 0; r < STG; ++r) {
            const int idx = t + 256 * r;
            const int row = idx / UPRW, u = idx % UPRW;
            if (row < BN) *reinterpret_cast<vec_t *>(Bs + (buf * BN + row) * LSB + u * V) = src[r];
        }
    };
    auto load_w = [&](int chunk) { load_w_to(chunk, pb); };
    auto store_w = [&](int buf) { store_w_from(buf, pb); };

    // WDMA: instruction k (0..7) of this wave fills LDS words [(wave + 4k) * 64, +64) of a
    // chunk buffer = rows 4*(wave + 4k) .. +3.  The word a lane delivers depends on k and on
    // the chunk only through a scalar offset.
    unsigned wd_voff = 0;
    v4i wd_rsrc = make_raw_rsrc(wt, (unsigned)g.c_out * 9u * (unsigned)g.cw * 4u);
    if (WDMA) {
        const int phys = (lane & 15) >> 1, sub = lane & 1;
        const int lw = ((phys ^ ((2 * wave + (lane >> 5)) & 7)) << 1) | sub;    // logical word of the chunk row
        const int hh = lw >> 3, st = lw & 7;
        wd_voff = (unsigned)(((o_blk + 4 * wave + (lane >> 4)) * 9 * g.cw + hh * WPH + st) * 4);
    }
    auto dma_w = [&](int chunk, int buf) {
        const int s0 = chunk * SPC;
        // (wave-uniform; read through readfirstlane so that it reaches the transfer's scalar
        // operand in a scalar register whatever the compiler makes of the chunk index)
        const unsigned soff0 = (unsigned)__builtin_amdgcn_readfirstlane(((s0 / WPH) * g.cw + (s0 % WPH)) * 4);
        const unsigned dst = (unsigned)(size_t)(__attribute__((address_space(3))) uint32_t *)(Bs + buf * BN * LSB) +
                             (unsigned)__builtin_amdgcn_readfirstlane(wave) * 256u;
#pragma unroll
        for (int k = 0; k < 8; ++k)
            lds_dma4_soff(wd_rsrc, dst + k * 1024u, wd_voff, soff0 + (unsigned)(k * 16 * 9 * 4) * (unsigned)g.cw);
    };
    // this lane's read offsets (words) inside a weight row, per V-step group
    int wd_boff[NVG];
#pragma unroll
    for (int vg = 0; vg < NVG; ++vg) wd_boff[vg] = (((half * NVG + vg) ^ ((l32 >> 1) & 7)) << 1);

    // ---- patch fetch, global -> LDS directly.  Unit = 16 bytes (a whole-pixel multiple) when
    // the layer has exactly CWP words per pixel and CWP >= 4, else one word.
    const bool wide = (g.cw == CWP) && (CWP >= 4);
    auto fetch_patch = [&](const TileCoord &tc, int buf) {
        const int img0 = tc.group * g.ni;
        const int y0 = tc.ty * th, x0 = tc.tx * tw;
        const int imgs = min(g.ni, g.n - img0);
        const uint32_t *base = in + (int64_t)img0 * g.h * g.w * g.cw;
        const unsigned bytes = (unsigned)imgs * g.h * g.w * g.cw * 4;
        const v4i rsrc = make_raw_rsrc(base, bytes);
        // LDS byte address of the destination buffer
        const unsigned dst = (unsigned)(size_t)(__attribute__((address_space(3))) uint32_t *)(Ps + buf * g.patch_words);
        const int upp = wide ? CWP / 4 : CWP;               // units per pixel
        const int total = g.ni * ph * pw * upp;
        for (int b0 = 0; b0 < total; b0 += 256) {
            const int idx = b0 + t;
            // idx -> (image, row, column, unit) of the patch; divisions by multiply-high
            const int p0 = idx / upp, u = idx - p0 * upp;
            const int p1 = (int)__umulhi((unsigned)p0, g.mg_pw), px = p0 - p1 * pw;
            const int il = (int)__umulhi((unsigned)p1, g.mg_ph), py = p1 - il * ph;
            const int y = y0 + py - 1, x = x0 + px - 1;
            const bool inside = y >= 0 && y < g.h && x >= 0 && x < g.w && (wide || u < g.cw);
            unsigned voff = 0x80000000u;                    // past the end of the buffer: zeros
            if (inside) voff = (unsigned)(((il * g.h + y) * g.w + x) * g.cw) * 4u + (unsigned)u * (wide ? 16u : 4u);
            const unsigned wave_base = (unsigned)__builtin_amdgcn_readfirstlane(b0 + wave * 64);
            if (idx < total) {
                if (wide) lds_dma16(rsrc, dst + wave_base * 16u, voff);
                else lds_dma4(rsrc, dst + wave_base * 4u, voff);
            }
        }
    };

    // ---- this lane's pixels: implicit-GEMM row p = 4 * window + (2*dy + dx)
    int pixoff[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int p = wm * TM * 32 + i * 32 + l32;
        const int wq = p >> 2, sub = p & 3;
        const int wx = wq & ((tw >> 1) - 1);
        const int wy = (wq >> (g.ltw - 1)) & ((th >> 1) - 1);
        const int il = wq >> (g.ltw - 1 + g.lth - 1);
        const int py = 2 * wy + (sub >> 1), px = 2 * wx + (sub & 1);
        pixoff[i] = ((il * ph + py) * pw + px) * CWP + half * WPH;
    }
    const int browoff = (wn * TN * 32 + l32) * LSB + half * SPC;

    uint32_t sgn = 0x88888888u, one = 0x22222222u;
    asm volatile("" : "+s"(sgn));
    asm volatile("" : "+v"(one));
    constexpr int DPM = (4 * (TM + TN) + TM * TN - 1) / (TM * TN);   // operand dwords made per MFMA

    // tile coordinates of the previous, current and next pixel tile of this block; a step of
    // `slots` tiles is a fixed (group, y, x) increment with carries
    TileCoord step, prev, cur, next;
    step.group = g.step_group; step.ty = g.step_ty; step.tx = g.step_tx;
    next.group = div_by(slot, tiles_per_group, g.mg_tpg);
    next.ty = div_by(slot - next.group * tiles_per_group, g.tiles_x, g.mg_tx);
    next.tx = slot - next.group * tiles_per_group - next.ty * g.tiles_x;
    prev = cur = next;
    auto advance = [&](TileCoord &c) {
        c.tx += step.tx;
        if (c.tx >= g.tiles_x) { c.tx -= g.tiles_x; ++c.ty; }
        c.ty += step.ty;
        if (c.ty >= g.tiles_y) { c.ty -= g.tiles_y; ++c.group; }
        c.group += step.group;
    };
    auto tile_pos = [&](const TileCoord &c) {
        TilePos pos;
        pos.n = g.n; pos.h = g.h; pos.w = g.w; pos.c_out = g.c_out;
        pos.lth = g.lth; pos.ltw = g.ltw; pos.img0 = c.group * g.ni; pos.y0 = c.ty * th; pos.x0 = c.tx * tw;
        return pos;
    };

    const CopyLane copy_lane = make_copy_lane(64 * TM, tile_pos(next), ep.pool, t);
    if (slot < g.n_ptiles) fetch_patch(next, 0);
    if (WDMA && slot < g.n_ptiles) dma_w(0, 0);
    // resident weights (at most 48 registers per thread), flips and thresholds: every load is
    // issued before the first one is waited for, one memory latency for all of them
    if (RES) {
        vec_t pall[NCHUNK][STG];
#pragma unroll
        for (int c = 0; c < NCHUNK; ++c) load_w_to(c, pall[c]);
        if (ep.packed) sw = load_step_words<TN>(ep, o_blk + wn * TN * 32, l32, g.c_out);
        stage_bias_f32(ep, o_blk, BN, g.c_out, g.k_bits + 1, corr, Ts, t);
#pragma unroll
        for (int c = 0; c < NCHUNK; ++c) store_w_from(c, pall[c]);
    } else {
        if (ep.packed) sw = load_step_words<TN>(ep, o_blk + wn * TN * 32, l32, g.c_out);
        stage_bias_f32(ep, o_blk, BN, g.c_out, g.k_bits + 1, corr, Ts, t);
    }
    int cc = 0;                                            // chunks done so far (WDMA buffer parity)

    // The packed words of a tile go to one of two LDS output tiles and are copied to global
    // memory after the next tile's barrier, so the stores drain while the next tile is
    // multiplied and the block needs one barrier per tile.
    int it = 0;
    for (int ptile = slot; ptile < g.n_ptiles; ptile += g.slots, ++it) {
        const int buf = g.dbuf ? (it & 1) : 0;
        const uint32_t *Pc = Ps + buf * g.patch_words;
        uint32_t *Oc = Os + (it & 1) * (64 * TM * BW);
        prev = cur;
        cur = next;
        advance(next);
        if (!RES && !WDMA) load_w(0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this tile's patch (and first weight chunk) has landed
        __syncthreads();                                      // ... for every wave; previous tile fully consumed
        if (g.dbuf && ptile + g.slots < g.n_ptiles) fetch_patch(next, buf ^ 1);
        if (ep.packed && it > 0)
            conv_tile_copy_out<BW>(Os + ((it - 1) & 1) * (64 * TM * BW), copy_lane, o_blk >> 5, tile_pos(prev), ep);

        __builtin_amdgcn_s_setprio(1);                        // the multiply phase outranks another wave's epilogue
        // accumulators start at the channels' biases (see stage_bias_f32)
        v16f acc[TM][TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const v16f b16 = load_bias16<v16f>(Tw + j * 32, half);
#pragma unroll
            for (int i = 0; i < TM; ++i) acc[i][j] = b16;
        }

        // Raw words of a V-step group (TM pixels' words, TN channels' words) and the expanded
        // operands of the current and the next MFMA step.  The pipeline "read words, expand
        // them, multiply" runs across chunk borders where the data allows it (XA: pixel words
        // always, the patch is resident; XB: channel words only when the weights are resident).
        constexpr bool XA = RES || WDMA, XB = RES;
        vec_t ra[2][TM], rb[2][TN];
        v8i a[2][TM], b[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int q = 4; q < 8; ++q) a[0][i][q] = a[1][i][q] = 0;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 4; q < 8; ++q) b[0][j][q] = b[1][j][q] = 0;
        auto load_a = [&](int c, int vg, int slot2) {
            const int s = c * SPC + vg * V;
            const int tap = s / WPH, cwi = s % WPH;
            const int ti = tap / 3, tj = tap - ti * 3;
            const int aoff = (ti * pw + tj) * CWP + cwi;
#pragma unroll
            for (int i = 0; i < TM; ++i) ra[slot2][i] = *reinterpret_cast<const vec_t *>(Pc + pixoff[i] + aoff);
        };
        auto load_b = [&](const uint32_t *Bc, int vg, int slot2) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
                rb[slot2][j] = *reinterpret_cast<const vec_t *>(
                    WDMA ? Bc + (wn * TN * 32 + j * 32 + l32) * LSB + wd_boff[vg] : Bc + browoff + j * 32 * LSB + vg * V);
        };
        if (XA) {                                           // pixel operands of the tile's first step
            load_a(0, 0, 0);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const v8i e = expand_first<V>(ra[0][i], sgn, one);
#pragma unroll
                for (int q = 0; q < 4; ++q) a[0][i][q] = e[q];
            }
        }

        // resident weights: the chunk loop is unrolled too (straight-line code keeps the operand
        // pipeline in registers without copies)
        constexpr int CUNROLL = RES ? NCHUNK : 1;
#pragma unroll CUNROLL
        for (int c = 0; c < NCHUNK; ++c) {
            if (WDMA) {
                if (c > 0) {
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // this chunk has landed
                    __syncthreads();              // ... for every wave; previous chunk consumed
                }
                // next chunk of the cyclic sequence into the other buffer
                if (c + 1 < NCHUNK || ptile + g.slots < g.n_ptiles) dma_w(c + 1 < NCHUNK ? c + 1 : 0, (cc + 1) & 1);
            } else if (!RES) {
                if (c > 0) __syncthreads();       // previous chunk consumed
                store_w(0);
                __syncthreads();
                if (c + 1 < NCHUNK) load_w(c + 1);
            }
            const uint32_t *Bc = RES ? Bs + c * BN * LSB : (WDMA ? Bs + (cc & 1) * BN * LSB : Bs);
            const uint32_t *Bn = Bc + BN * LSB;            // next chunk's weights (resident weights only)
            if (WDMA) ++cc;
            const bool more = c + 1 < NCHUNK;

            // operands of the chunk's first step that did not come from the previous chunk
            if (!XA) {
                load_a(c, 0, 0);
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const v8i e = expand_first<V>(ra[0][i], sgn, one);
#pragma unroll
                    for (int q = 0; q < 4; ++q) a[0][i][q] = e[q];
                }
            }
            if (!XB || c == 0) {
                load_b(Bc, 0, 0);
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const v8i e = expand_first<V>(rb[0][j], sgn, one);
#pragma unroll
                    for (int q = 0; q < 4; ++q) b[0][j][q] = e[q];
                }
            }
            // The instruction order below is the issue order (scheduling barriers pin it): the
            // LDS reads of the next word group, then each MFMA followed by its share of the
            // next step's operand dwords, so that VALU work runs in the shadow of the MFMAs.
#pragma unroll
            for (int st = 0; st < SPC; ++st) {
                const int cur_s = st & 1, nxt = cur_s ^ 1;
                const int vg = st / V, q = st % V;
                const bool last_group = vg + 1 == NVG;
                if (q == 0) {
                    if (!last_group) {
                        load_a(c, vg + 1, (vg + 1) & 1);
                        load_b(Bc, vg + 1, (vg + 1) & 1);
                    } else if (more) {                    // first group of the next chunk
                        if (XA) load_a(c + 1, 0, 0);
                        if (XB) load_b(Bn, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                const bool in_chunk = st + 1 < SPC;
                const int vg1 = in_chunk ? (st + 1) / V : 0, q1 = in_chunk ? (st + 1) % V : 0;
                // (streamed weights: the chunk index is a run-time value, and the last chunk expands
                // stale words into operands that the next tile overwrites, rather than branching)
                const bool next_a = in_chunk || (XA && (WDMA || more)), next_b = in_chunk || (XB && more);
                uint2 pend[2 * (TM + TN)];                // shifted pairs awaiting their masks
#pragma unroll
                for (int k = 0; k < TM * TN; ++k) {
                    const int i = k / TN, j = k % TN;
                    // weights first: accumulator rows = channels, columns (lanes) = pixels
                    // (zero scale operands select the instruction form without block scales)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        b[cur_s][j], a[cur_s][i], acc[i][j], 4, 4, 0, 0, 0, 0);
                    if constexpr (V == 2) {
                        // Word pairs: TM + TN pairs, two (shift, mask, mask) items each.  An item's
                        // masks come one MFMA after its shift (no VALU instruction waits for the one
                        // before it); with a single MFMA per step both fall behind that one.
                        constexpr int NIT = 2 * (TM + TN), NM = TM * TN, LAG = NM > 1 ? 1 : 0;
#pragma unroll
                        for (int t2 = 0; t2 < NIT; ++t2) {
                            const int ks = t2 * (NM - LAG) / NIT;            // MFMA the shift follows
                            const int wi = t2 >> 1, dp = t2 & 1;
                            if (!(wi < TM ? next_a : next_b)) continue;
                            if (ks == k) pend[t2] = shift_pair_half(wi < TM ? ra[vg1 & 1][wi] : rb[vg1 & 1][wi - TM], q1, dp);
                            if (ks + LAG == k) {
                                const uint2 e = mask_pair(pend[t2], sgn, one);
                                if (wi < TM) {
                                    a[nxt][wi][2 * dp] = (int)e.x;
                                    a[nxt][wi][2 * dp + 1] = (int)e.y;
                                } else {
                                    b[nxt][wi - TM][2 * dp] = (int)e.x;
                                    b[nxt][wi - TM][2 * dp + 1] = (int)e.y;
                                }
                            }
                        }
                    } else {
#pragma unroll
                        for (int d = k * DPM; d < (k + 1) * DPM && d < 4 * (TM + TN); ++d) {
                            const int wi = d >> 2, part = d & 3;
                            if (wi < TM) {
                                if (next_a) a[nxt][wi][part] = (int)expand_part(vec_word(ra[vg1 & 1][wi], q1), part, sgn, one);
                            } else {
                                if (next_b)
                                    b[nxt][wi - TM][part] = (int)expand_part(vec_word(rb[vg1 & 1][wi - TM], q1), part, sgn, one);
                            }
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }

        // ---- epilogue (shared with the first layer)
        __builtin_amdgcn_s_setprio(0);
        const TilePos pos = tile_pos(cur);
        if (ep.preact) {
            auto getx = [&](int i, int j, int r) {
                return (int)(acc[i][j][r] - Tw[j * 32 + (r >> 2) * 8 + half * 4 + (r & 3)]) - corr;
            };
            conv_tile_store_preact<TM, TN>(getx, wm * TM * 32, o_blk + wn * TN * 32, l32, half, pos, ep.preact);
        }
        if (ep.packed) {
            // bits -> LDS tile [output pixel][2*TN words]; one vector store per pixel later
            auto gets = [&](int i, int j, int r) { return acc[i][j][r]; };
            conv_tile_step_to_lds<TM, TN>(gets, wm * TM * 32, wn * TN, BW, l32, half, sw,
                                          ep.pool, ep.pool_first != 0, Oc);
        }
        if (!g.dbuf && ptile + g.slots < g.n_ptiles) {
            __syncthreads();                                  // every wave is done with the only patch buffer
            fetch_patch(next, 0);
        }
    }
    if (ep.packed && it > 0) {
        __syncthreads();
        conv_tile_copy_out<BW>(Os + ((it - 1) & 1) * (64 * TM * BW), copy_lane, o_blk >> 5, tile_pos(cur), ep);
    }
}

template <int TM, int TN, int WPH, bool WDMA>
bool make_geom(int n, int h, int w, int c_in, int c_out, ConvGeom &g, size_t &smem)
{
    constexpr int V = WPH >= 2 ? 2 : WPH;
    constexpr int LSB = WDMA ? 2 * steps_per_chunk(WPH) : 2 * steps_per_chunk(WPH) + V;
    constexpr int NBUF = WDMA ? 2 : (weights_resident(TM, TN, WPH) ? 9 * WPH / steps_per_chunk(WPH) : 1);
    // weights by DMA: exact channel words, whole channel tiles, byte offsets below 2^31
    if (WDMA && ((c_in + 31) / 32 != 2 * WPH || c_out % (64 * TN) != 0 ||
                 (int64_t)c_out * 9 * ((c_in + 31) / 32) * 4 >= 0x7fffffffLL))
        return false;
    g.n = n; g.h = h; g.w = w;
    g.cw = (c_in + 31) / 32;
    g.c_out = c_out;
    g.k_bits = 9 * c_in;
    const TileShape ts = make_tile_shape(h, w, 64 * TM);
    g.ltw = ts.ltw; g.lth = ts.lth; g.ni = ts.ni;
    g.tiles_x = ts.tiles_x; g.tiles_y = ts.tiles_y;
    g.n_co_tiles = (c_out + 64 * TN - 1) / (64 * TN);
    const int64_t ptiles = (int64_t)ts.tiles_x * ts.tiles_y * ((n + ts.ni - 1) / ts.ni);
    if (ptiles > 0x3fffffffLL || (int64_t)ts.ni * h * w * g.cw * 4 >= 0x7fffffffLL) return false;
    if (((int64_t)c_out + 64 * TN) * 9 * g.cw >= 0x7fffffffLL) return false;     // 32-bit weight word offsets
    g.n_ptiles = (int)ptiles;
    // exact for dividends below 2^16 (a patch has at most a few thousand units)
    g.mg_pw = (unsigned)((0x100000000ULL + (1 << ts.ltw) + 1) / ((1 << ts.ltw) + 2));
    g.mg_ph = (unsigned)((0x100000000ULL + (1 << ts.lth) + 1) / ((1 << ts.lth) + 2));
    // one patch buffer: pixels x padded words, rounded up to a wave's worth of 16-byte units
    const int pwords = ts.ni * ((1 << ts.lth) + 2) * ((1 << ts.ltw) + 2) * (2 * WPH);
    g.patch_words = (pwords + 255) & ~255;
    const size_t fixed = (size_t)NBUF * 64 * TN * LSB * 4 + 64 * TN * 4 + (size_t)2 * 64 * TM * 2 * TN * 4;
    g.dbuf = (fixed + 2 * (size_t)g.patch_words * 4 <= (size_t)MAX_SMEM) ? 1 : 0;
    smem = fixed + (size_t)(g.dbuf ? 2 : 1) * g.patch_words * 4;
    // persistent grid: two resident blocks per compute unit, a whole number of channel-tile sets
    int slots = 512 / g.n_co_tiles;
    if (slots < 1) slots = 1;
    if (slots > g.n_ptiles) slots = g.n_ptiles;
    g.slots = slots;
    const int tpg = ts.tiles_x * ts.tiles_y;
    g.step_group = slots / tpg;
    g.step_ty = (slots - g.step_group * tpg) / ts.tiles_x;
    g.step_tx = slots - g.step_group * tpg - g.step_ty * ts.tiles_x;
    g.mg_co = magic_floor(g.n_co_tiles);
    g.mg_tpg = magic_floor(tpg);
    g.mg_tx = magic_floor(ts.tiles_x);
    return smem <= (size_t)MAX_SMEM;
}

template <int TM, int TN, int WPH, bool WDMA = false>
bnn_status launch_one(const uint32_t *in, const uint32_t *wt, int n, int h, int w, int c_in, int c_out,
                      const EpiArgs &ep, hipStream_t s)
{
    ConvGeom g;
    size_t smem;
    if (!make_geom<TM, TN, WPH, WDMA>(n, h, w, c_in, c_out, g, smem)) return BNN_ERR_UNSUPPORTED;
    const unsigned blocks = (unsigned)(g.slots * g.n_co_tiles);
    if (smem > 64 * 1024) {          // above the default limit of dynamic LDS: opt in, once per kernel
        // (callers on distinct threads may arrive here together; a failed attempt is reported to
        // every caller of this kernel, a successful one is never repeated)
        static std::once_flag once;
        static hipError_t raise_err = hipSuccess;
        std::call_once(once, [] {
            raise_err = hipFuncSetAttribute((const void *)bconv_mfma<TM, TN, WPH, WDMA>,
                                            hipFuncAttributeMaxDynamicSharedMemorySize, MAX_SMEM);
        });
        if (raise_err != hipSuccess) return hip_result(raise_err);
    }
    hipLaunchKernelGGL((bconv_mfma<TM, TN, WPH, WDMA>), dim3(blocks), dim3(256), smem, s, in, wt, g, ep);
    return hip_result(hipGetLastError());
}

// Work items (pixel tiles x channel tiles) a (64*TM pixels) x (64*TN channels) block tile
// would give, or -1 if its LDS footprint does not fit.
template <int TM, int TN, int WPH, bool WDMA = false>
int64_t blocks_one(int n, int h, int w, int c_in, int c_out)
{
    ConvGeom g;
    size_t smem;
    if (!make_geom<TM, TN, WPH, WDMA>(n, h, w, c_in, c_out, g, smem)) return -1;
    return (int64_t)g.n_co_tiles * g.n_ptiles;
}

// Largest block tile that fits LDS and still fills most of the 256 compute units.
}  // namespace

// The 256 x 128 tile of a channel width is compiled in a translation unit of its own (it is the
// slowest to build); the dispatcher below reaches it through this function.
template <int WPH>
bnn_status launch_conv_big_tile(const uint32_t *in, const uint32_t *wt, int n, int h, int w, int c_in,
                                int c_out, const EpiArgs &ep, hipStream_t s);

namespace {

// Which block tile launch_wph takes: the largest that fits LDS and still gives two resident
// blocks per compute unit.  3: 256 x 128, 2: 128 x 128 with streamed weights, 1: 128 x 128,
// 0: 64 x 64.
template <int WPH>
int tile_choice_wph(int n, int h, int w, int c_in, int c_out)
{
    const int64_t want = 512;     // two resident blocks per compute unit
    // the largest tile keeps its weights resident (WPH <= 4) or streams them by DMA
    constexpr bool WD = WPH >= 8;
    if (blocks_one<4, 2, WPH, WD>(n, h, w, c_in, c_out) >= want) return 3;
    if (WD && blocks_one<2, 2, WPH, WD>(n, h, w, c_in, c_out) >= want) return 2;
    if (blocks_one<2, 2, WPH>(n, h, w, c_in, c_out) >= want) return 1;
    return 0;
}

template <int WPH>
bnn_status launch_wph(const uint32_t *in, const uint32_t *wt, int n, int h, int w, int c_in, int c_out,
                      const EpiArgs &ep, hipStream_t s)
{
    constexpr bool WD = WPH >= 8;
    switch (tile_choice_wph<WPH>(n, h, w, c_in, c_out)) {
    case 3: return launch_conv_big_tile<WPH>(in, wt, n, h, w, c_in, c_out, ep, s);
    case 2: return launch_one<2, 2, WPH, WD>(in, wt, n, h, w, c_in, c_out, ep, s);
    case 1: return launch_one<2, 2, WPH>(in, wt, n, h, w, c_in, c_out, ep, s);
    }
    return launch_one<1, 1, WPH>(in, wt, n, h, w, c_in, c_out, ep, s);
}

}  // namespace

}  // namespace bnn
#endif

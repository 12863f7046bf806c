// Binary 3x3 convolution (stride 1, pad 1 with -1) for gfx950: im2col-free, on the matrix
// cores.
//
// x[n,y,x,o] = sum_{tap, c} a(n, y+i-1, x+j-1, c) * W[o, tap, c] over +-1 values (paper
// Sec. II-A: convolutional layer of binarized neurons, 2*popcount(xnor) - #bits).  Taps that
// fall outside the image read zero words, i.e. -1 activations, so every output sums exactly
// K = 9*c_in products.
//
// A block of 4 waves (2 x 2) computes (64*TM pixels) x (64*TN output channels).  The pixels
// are `ni` images x (th x tw) spatial tile whose input patch, halo included, is staged once
// in LDS as packed words; the nine taps are read from it with shifted addresses.  Weights
// stream through LDS in chunks of a few taps.  Every 32-bit word of either operand is
// expanded in registers into 32 FP4 values +-1.0 and multiplied by
// v_mfma_scale_f32_32x32x64_f8f6f4; sums stay below 2^24 so the FP32 accumulators are exact.
// Within one MFMA the lower 32 lanes supply the first half of a pixel's channel words and
// the upper 32 lanes the second half (same split on the weight side).
//
// Pixels are numbered window-major (four consecutive rows of the implicit GEMM are one 2x2
// window), which puts a pool window into four accumulator registers of one lane: max-pool
// after the sign is an OR of four predicate bits.  A wave-wide ballot of the predicate is the
// packed output word (32 lanes = 32 consecutive channels).
#ifndef BNN_BCONV_KERNEL_H
#define BNN_BCONV_KERNEL_H
#include "bnn_internal.h"
#include "conv_epilogue.h"

namespace bnn {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int MAX_SMEM = 64 * 1024;

struct ConvGeom {
    int n, h, w, cw;             // input: images, height, width, words per pixel
    int c_out, k_bits;           // outputs, K = 9*c_in
    int lth, ltw;                // log2 of the spatial tile height / width (both >= 1)
    int ni;                      // images per block; ni * th * tw == pixels per block
    int tiles_x, tiles_y, n_co_tiles;
};

template <int V> struct WordVec;
template <> struct WordVec<4> { using type = uint4; };
template <> struct WordVec<2> { using type = uint2; };
template <> struct WordVec<1> { using type = uint32_t; };

__device__ __forceinline__ uint32_t vec_word(const uint4 &v, int q) { return q == 0 ? v.x : (q == 1 ? v.y : (q == 2 ? v.z : v.w)); }
__device__ __forceinline__ uint32_t vec_word(const uint2 &v, int q) { return q == 0 ? v.x : v.y; }
__device__ __forceinline__ uint32_t vec_word(const uint32_t &v, int) { return v; }

__device__ __forceinline__ void vec_set(uint4 &v, int q, uint32_t x) { if (q == 0) v.x = x; else if (q == 1) v.y = x; else if (q == 2) v.z = x; else v.w = x; }
__device__ __forceinline__ void vec_set(uint2 &v, int q, uint32_t x) { if (q == 0) v.x = x; else v.y = x; }
__device__ __forceinline__ void vec_set(uint32_t &v, int, uint32_t x) { v = x; }

// 32 packed bits -> 32 FP4 values (0b0010 = +1.0, 0b1010 = -1.0) in the low four dwords of an
// MFMA operand; sgn / one hold 0x88888888 / 0x22222222 in registers (one v_and_or_b32 each).
__device__ __forceinline__ v8i expand_fp4(uint32_t w, uint32_t sgn, uint32_t one)
{
    v8i r;
    r[0] = (int)(((w << 3) & sgn) | one);
    r[1] = (int)(((w << 2) & sgn) | one);
    r[2] = (int)(((w << 1) & sgn) | one);
    r[3] = (int)((w & sgn) | one);
    r[4] = 0; r[5] = 0; r[6] = 0; r[7] = 0;
    return r;
}

// Steps (one MFMA K-slice = one word per lane half) per weight chunk, by words per half.
constexpr int steps_per_chunk(int wph) { return wph == 1 ? 9 : (wph == 2 ? 6 : (wph == 4 ? 12 : 8)); }

// Whether a block keeps all of its weight chunks in LDS at once (64-channel tiles, <= 48 KB).
constexpr bool weights_resident(int tm, int tn, int wph)
{
    const int v = wph >= 4 ? 4 : wph;
    const int lsb = 2 * steps_per_chunk(wph) + v;
    const int nchunk = 9 * wph / steps_per_chunk(wph);
    return tm * tn == 1 && nchunk * 64 * tn * lsb * 4 <= 48 * 1024;
}

// WPH = words per lane half per tap; the layer's cw words per pixel are zero-padded to 2*WPH.
template <int TM, int TN, int WPH>
__global__ __launch_bounds__(256, 2)
void bconv_mfma(const uint32_t *__restrict__ in, const uint32_t *__restrict__ wt, ConvGeom g, EpiArgs ep)
{
    constexpr int BN = 64 * TN;
    constexpr int CWP = 2 * WPH;                       // padded words per pixel
    constexpr int V = WPH >= 4 ? 4 : WPH;              // words per LDS access
    constexpr int SPC = steps_per_chunk(WPH);
    constexpr int NCHUNK = 9 * WPH / SPC;
    constexpr int LSB = 2 * SPC + V;                   // weight row stride (words); LSB/V is odd
    constexpr int UPRW = 2 * SPC / V;                  // weight units per row per chunk
    constexpr int STG = (BN * UPRW + 255) / 256;       // weight units per thread per chunk
    constexpr int NVG = SPC / V;                       // V-step groups per chunk
    // Smallest tile (latency-bound launches, e.g. batch 1): all weight chunks of the block are
    // loaded up front into their own LDS buffers, so the K loop has no barrier and no global
    // load latency in it.
    constexpr bool RES = weights_resident(TM, TN, WPH);
    constexpr int NBUF = RES ? NCHUNK : 1;
    using vec_t = typename WordVec<V>::type;

    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *Bs = reinterpret_cast<uint32_t *>(smem);                 // [NBUF][BN][LSB]
    int *Ts = reinterpret_cast<int *>(Bs + NBUF * BN * LSB);           // [BN] thresholds
    uint32_t *Ps = reinterpret_cast<uint32_t *>(Ts + BN);              // [ni][ph][pw][CWP]

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, half = lane >> 5;

    // XCD-aware order: hardware deals consecutive block ids round-robin to the 8 XCDs (one L2
    // each); renumber so that blocks sharing an input patch (the channel tiles of one pixel
    // tile) run on the same XCD and the patch is fetched from HBM once.
    int bid = blockIdx.x;
    if ((gridDim.x & 7) == 0) bid = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int co_tile = bid % g.n_co_tiles; bid /= g.n_co_tiles;
    const int tile_x = bid % g.tiles_x;     bid /= g.tiles_x;
    const int tile_y = bid % g.tiles_y;     bid /= g.tiles_y;
    const int img0 = bid * g.ni;
    const int th = 1 << g.lth, tw = 1 << g.ltw;
    const int y0 = tile_y * th, x0 = tile_x * tw;
    const int o_blk = co_tile * BN;
    const int pw = tw + 2, ph = th + 2;

    // per-channel step parameters: fetched first so their latency hides behind the main loop
    StepWords<TN> sw;
    if (ep.packed) {
        sw = load_step_words<TN>(ep, o_blk + wn * TN * 32, l32, g.c_out);
        stage_thresholds(ep, o_blk, BN, g.c_out, Ts, t);
    }

    // ---- stage the input patch (halo included; outside the image / beyond cw = zero words).
    // Four units per thread are loaded before any is stored, so the loads overlap.
    {
        constexpr int UPP = CWP / V;                  // units per pixel
        const int total = g.ni * ph * pw * UPP;
        const bool vec_ok = (g.cw % V) == 0;
        for (int base = 0; base < total; base += 256 * 4) {
            vec_t v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int idx = base + k * 256 + t;
#pragma unroll
                for (int q = 0; q < V; ++q) vec_set(v[k], q, 0u);
                if (idx < total) {
                    const int u = idx % UPP;
                    int p = idx / UPP;
                    const int px = p % pw; p /= pw;
                    const int py = p % ph;
                    const int il = p / ph;
                    const int y = y0 + py - 1, x = x0 + px - 1, img = img0 + il;
                    if (img < g.n && y >= 0 && y < g.h && x >= 0 && x < g.w) {
                        const uint32_t *src = in + (((int64_t)img * g.h + y) * g.w + x) * g.cw + u * V;
                        if (vec_ok) {
                            if (u * V < g.cw) v[k] = *reinterpret_cast<const vec_t *>(src);
                        } else {
#pragma unroll
                            for (int q = 0; q < V; ++q)
                                if (u * V + q < g.cw) vec_set(v[k], q, src[q]);
                        }
                    }
                }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int idx = base + k * 256 + t;
                if (idx < total) *reinterpret_cast<vec_t *>(Ps + idx * V) = v[k];
            }
        }
    }

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

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // ---- weight staging: LDS row = [half 0: SPC words][half 1: SPC words]; the word of
    // (half, step) is W[o][tap][half*WPH + cwi] with tap = step / WPH, cwi = step % WPH.
    vec_t pb[STG];
    const bool wvec_ok = (g.cw % V) == 0;
    auto load_w = [&](int chunk) {
#pragma unroll
        for (int r = 0; r < STG; ++r) {
            const int idx = t + 256 * r;
            const int row = idx / UPRW, u = idx % UPRW;
            const int hh = u / NVG, vg = u % NVG;
            const int s = chunk * SPC + vg * V;
            const int tap = s / WPH, cwi = s % WPH;
            const int cwpos = hh * WPH + cwi;
            const int o = o_blk + row;
            vec_t v;
#pragma unroll
            for (int q = 0; q < V; ++q) vec_set(v, q, 0u);
            if (row < BN && o < g.c_out) {
                const uint32_t *src = wt + ((int64_t)o * 9 + tap) * g.cw + cwpos;
                if (wvec_ok) {
                    if (cwpos < g.cw) v = *reinterpret_cast<const vec_t *>(src);
                } else {
#pragma unroll
                    for (int q = 0; q < V; ++q)
                        if (cwpos + q < g.cw) vec_set(v, q, src[q]);
                }
            }
            pb[r] = v;
        }
    };
    if (RES) {
        // every chunk: loads of all chunks are in flight together, then one barrier
        vec_t all[NCHUNK][STG];
#pragma unroll
        for (int c = 0; c < NCHUNK; ++c) {
            load_w(c);
#pragma unroll
            for (int r = 0; r < STG; ++r) all[c][r] = pb[r];
        }
#pragma unroll
        for (int c = 0; c < NCHUNK; ++c)
#pragma unroll
            for (int r = 0; r < STG; ++r) {
                const int idx = t + 256 * r;
                const int row = idx / UPRW, u = idx % UPRW;
                if (row < BN) *reinterpret_cast<vec_t *>(Bs + (c * BN + row) * LSB + u * V) = all[c][r];
            }
        __syncthreads();
    } else {
        load_w(0);
    }

    uint32_t sgn = 0x88888888u, one = 0x22222222u;
    asm volatile("" : "+s"(sgn));
    asm volatile("" : "+v"(one));
    constexpr int VPM = (7 * (TM + TN) + TM * TN - 1) / (TM * TN);

    for (int c = 0; c < NCHUNK; ++c) {
        if (!RES) {
            __syncthreads();      // patch staged (first pass) / previous chunk consumed
#pragma unroll
            for (int r = 0; r < STG; ++r) {
                const int idx = t + 256 * r;
                const int row = idx / UPRW, u = idx % UPRW;
                if (row < BN) *reinterpret_cast<vec_t *>(Bs + row * LSB + u * V) = pb[r];
            }
            __syncthreads();
            if (c + 1 < NCHUNK) load_w(c + 1);
        }
        const uint32_t *Bc = RES ? Bs + c * BN * LSB : Bs;

        // raw words of V-step group vg: TM pixels' words and TN channels' words
        vec_t ra[2][TM], rb[2][TN];
        auto load_group = [&](int vg, int slot) {
            const int s = c * SPC + vg * V;
            const int tap = s / WPH, cwi = s % WPH;
            const int ti = tap / 3, tj = tap - ti * 3;
            const int aoff = (ti * pw + tj) * CWP + cwi;
#pragma unroll
            for (int i = 0; i < TM; ++i) ra[slot][i] = *reinterpret_cast<const vec_t *>(Ps + pixoff[i] + aoff);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                rb[slot][j] = *reinterpret_cast<const vec_t *>(Bc + browoff + j * 32 * LSB + vg * V);
        };
        load_group(0, 0);
        v8i a[2][TM], b[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[0][i] = expand_fp4(vec_word(ra[0][i], 0), sgn, one);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[0][j] = expand_fp4(vec_word(rb[0][j], 0), sgn, one);
#pragma unroll
        for (int st = 0; st < SPC; ++st) {
            const int cur = st & 1, nxt = cur ^ 1;
            const int vg = st / V, q = st % V;
            if (q == 0 && vg + 1 < NVG) load_group(vg + 1, (vg + 1) & 1);
            if (st + 1 < SPC) {
                const int vg1 = (st + 1) / V, q1 = (st + 1) % V;
#pragma unroll
                for (int i = 0; i < TM; ++i) a[nxt][i] = expand_fp4(vec_word(ra[vg1 & 1][i], q1), sgn, one);
#pragma unroll
                for (int j = 0; j < TN; ++j) b[nxt][j] = expand_fp4(vec_word(rb[vg1 & 1][j], q1), sgn, one);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    // weights first: accumulator rows = channels, columns (lanes) = pixels
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        b[cur][j], a[cur][i], acc[i][j], 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
#pragma unroll
            for (int k = 0; k < TM * TN; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, VPM, 0);
            }
        }
    }

    // ---- epilogue (shared with the first layer): sums minus the padded positions, which all
    // counted as +1
    const int corr = 9 * CWP * 32 - g.k_bits;
    TilePos pos;
    pos.n = g.n; pos.h = g.h; pos.w = g.w; pos.c_out = g.c_out;
    pos.lth = g.lth; pos.ltw = g.ltw; pos.img0 = img0; pos.y0 = y0; pos.x0 = x0;
    auto getx = [&](int i, int j, int r) { return (int)acc[i][j][r] - corr; };
    if (ep.preact) conv_tile_store_preact<TM, TN>(getx, wm * TM * 32, o_blk + wn * TN * 32, l32, half, pos, ep.preact);
    if (ep.packed) {
        // bits -> LDS tile [output pixel][2*TN words] (reusing the weight buffer) -> coalesced stores
        constexpr int BW = 2 * TN;
        __syncthreads();                      // every wave is done with the weight chunk
        conv_tile_step_to_lds<TM, TN>(getx, wm * TM * 32, wn * TN, BW, l32, half, Ts + wn * TN * 32, sw, ep.pool,
                                      ep.pool_first != 0, Bs);
        __syncthreads();
        conv_tile_copy_out<BW>(Bs, 64 * TM, o_blk >> 5, pos, ep, t);
    }
}

ConvGeom make_geom(int n, int h, int w, int c_in, int c_out, int pixels, int bn)
{
    ConvGeom g;
    g.n = n; g.h = h; g.w = w;
    g.cw = (c_in + 31) / 32;
    g.c_out = c_out;
    g.k_bits = 9 * c_in;
    const TileShape ts = make_tile_shape(h, w, pixels);
    g.ltw = ts.ltw; g.lth = ts.lth; g.ni = ts.ni;
    g.tiles_x = ts.tiles_x; g.tiles_y = ts.tiles_y;
    g.n_co_tiles = (c_out + bn - 1) / bn;
    return g;
}

template <int TM, int TN, int WPH>
size_t smem_bytes(const ConvGeom &g)
{
    constexpr int V = WPH >= 4 ? 4 : WPH;
    constexpr int LSB = 2 * steps_per_chunk(WPH) + V;
    constexpr int NBUF = weights_resident(TM, TN, WPH) ? 9 * WPH / steps_per_chunk(WPH) : 1;
    const size_t patch = (size_t)g.ni * ((1 << g.lth) + 2) * ((1 << g.ltw) + 2) * (2 * WPH) * 4;
    return (size_t)NBUF * 64 * TN * LSB * 4 + 64 * TN * 4 + patch;
}

template <int TM, int TN, int WPH>
bnn_status launch_one(const uint32_t *in, const uint32_t *wt, int n, int h, int w, int c_in, int c_out,
                      const EpiArgs &ep, hipStream_t s)
{
    ConvGeom g = make_geom(n, h, w, c_in, c_out, 64 * TM, 64 * TN);
    const size_t smem = smem_bytes<TM, TN, WPH>(g);
    const int64_t blocks = (int64_t)g.n_co_tiles * g.tiles_x * g.tiles_y * ((n + g.ni - 1) / g.ni);
    if (smem > (size_t)MAX_SMEM || blocks > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((bconv_mfma<TM, TN, WPH>), dim3((unsigned)blocks), dim3(256), smem, s, in, wt, g, ep);
    return hip_result(hipGetLastError());
}

// Blocks a (64*TM pixels) x (64*TN channels) block tile would give, or -1 if its LDS
// footprint does not fit.
template <int TM, int TN, int WPH>
int64_t blocks_one(int n, int h, int w, int c_in, int c_out)
{
    ConvGeom g = make_geom(n, h, w, c_in, c_out, 64 * TM, 64 * TN);
    if (smem_bytes<TM, TN, WPH>(g) > (size_t)MAX_SMEM) return -1;
    return (int64_t)g.n_co_tiles * g.tiles_x * g.tiles_y * ((n + g.ni - 1) / g.ni);
}

// Largest block tile that fits LDS and still fills most of the 256 compute units.
template <int WPH>
bnn_status launch_wph(const uint32_t *in, const uint32_t *wt, int n, int h, int w, int c_in, int c_out,
                      const EpiArgs &ep, hipStream_t s)
{
    const int64_t want = 512;     // two resident blocks per compute unit
    if (blocks_one<4, 2, WPH>(n, h, w, c_in, c_out) >= want)
        return launch_one<4, 2, WPH>(in, wt, n, h, w, c_in, c_out, ep, s);
    if (blocks_one<2, 2, WPH>(n, h, w, c_in, c_out) >= want)
        return launch_one<2, 2, WPH>(in, wt, n, h, w, c_in, c_out, ep, s);
    return launch_one<1, 1, WPH>(in, wt, n, h, w, c_in, c_out, ep, s);
}

}  // namespace

}  // namespace bnn
#endif

// First layer for gfx950: int8 activations x +-1 (int8) weights, int32 accumulation.
//
// x[n,y,x,o] = sum_{i<kh, j<kw, c<c_in} a(n, y+i-pad, x+j-pad, c) * W[o,i,j,c]
// (paper Sec. II-A convolutional layer applied to the 8-bit input image; with
// kh = kw = h = w = 1 it is the fully-connected first layer of an MLP).
//
// Five kernels, picked by shape:
//   conv_first_small  at most 6144 tiles of 32 pixels x 32 channels, kernel height <= 4, kernel rows of <= 16 bytes:
//                     one wave per 32 pixels x 32 channels, operands straight from global
//                     memory, the step in registers (latency: batch 1 .. 8 of a small image).
//   conv_first_img    3x3, one ring of padding, <= 4 channels, power-of-two width: whole images
//                     in LDS, persistent blocks (throughput: large batches of small images).
//   conv_first_mfma   small kernels (kh * roundup16(kw*c_in) <= 128 bytes per pixel): the int8
//                     input patch and the block's weights live in LDS; each lane gathers 16
//                     contiguous patch bytes (one kernel row of one pixel) per MFMA operand
//                     and v_mfma_i32_32x32x32_i8 does the sums.  Pixels are window-major, the
//                     epilogue is the one of the binary convolution.
//   fc_first_mfma     1x1 kernels without padding and c_in % 16 == 0 (the MLP's first layer):
//                     an int8 GEMM whose operands are read straight from global memory
//                     (fc_first_small: the same with K split over a block's waves, for few rows).
//   conv_first_kernel any other shape: one lane = one output pixel x 32 output channels with
//                     v_dot4_i32_i8.
//
// conv_first_kernel: one lane = one output pixel x 32 output channels.  The flattened taps (i, j, c) are taken
// four at a time with v_dot4_i32_i8: the lane gathers its four activation bytes into a
// dword, the block keeps the weights of its 32 channels in LDS as [tap group][channel]
// dwords (zero beyond K), so every lane of a wave reads the same LDS address (broadcast).
// With pool == 2 lanes are ordered window-major: four neighbouring lanes hold the 2x2
// window and OR their bit words.
#include "bnn_internal.h"
#include "conv_epilogue.h"

namespace bnn {

namespace {

constexpr int K4C = 256;   // tap groups (of 4) per LDS chunk -> 32 KB of weights

struct FirstGeom {
    int n, h, w, c_in, c_out, kh, kw, pad, pad_value;
    int ho, wo, pool, k, k4;
};

// The launch's blocks zero, between them, the words a later launch of the same chain accumulates into.
__device__ __forceinline__ void clear_words(const ClearArgs &c)
{
    if (c.count > 0 && blockIdx.y == 0)
        for (int i = blockIdx.x * 256 + threadIdx.x; i < c.count; i += gridDim.x * 256) c.ptr[i] = 0;
}

__global__ __launch_bounds__(256) void conv_first_kernel(const int8_t *__restrict__ in,
                                                         const int8_t *__restrict__ wt, FirstGeom g,
                                                         EpiArgs ep, ClearArgs clr)
{
    __shared__ int W4[K4C][32];
    clear_words(clr);

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
        if (g.pool == 2 && ep.pool_first) {
            // pool the int32 pre-activations of the window (four neighbouring lanes) first
#pragma unroll
            for (int o = 0; o < 32; ++o) {
                int v = live ? acc[o] : INT32_MIN;
                v = max(v, __shfl_xor(v, 1));
                v = max(v, __shfl_xor(v, 2));
                acc[o] = v;
            }
        }
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

// ------------------------------------------------------------------ matrix-core kernels
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct FirstGeomM {
    int n, h, w, c_in, c_out, kh, kw, pad, pad_value;
    int ho, wo;
    int lth, ltw, ni, tiles_x, tiles_y, n_co_tiles, n_items;
    int sl, slp, kp;            // bytes of one kernel row, padded to 16, and padded K (multiple of 32)
    int patch_bytes;
    unsigned mg_cin, mg_pw, mg_ph, mg_kh;   // ceil(2^32 / d) for d = c_in, patch width / height, kh
    int step_grp, step_ty, step_tx;         // a grid's worth of items as an (image group, row, column) increment
    unsigned mg_tx, mg_ty;                  // magic_floor of tiles_x, tiles_y
};

// floor(n / d) for n, d < 2^16 with mg = ceil(2^32 / d) (mg == 0 stands for d == 1): one v_mul_hi_u32.
__device__ __forceinline__ int div_magic(int n, unsigned mg) { return mg ? (int)__umulhi((unsigned)n, mg) : n; }

// Block = 4 waves x 64 pixels (two 32-row tiles each) x NG groups of 64 channels, taken one
// group after the other; blocks are persistent (weights staged once, then a grid-stride
// walk over the pixel tiles).  Output bits go through an LDS tile and leave as one vector
// store per pixel.
// K is ordered [kernel row ti][tj*c_in + c], every kernel row zero-padded to slp bytes on
// the weight side; the activation bytes behind a short row are whatever follows in the
// patch and meet zero weights.
//
// PIPE (patch of at most 1024 bytes, i.e. four bytes per thread): the next tile's patch bytes
// are loaded into registers before the current tile is computed and stored to the second
// patch buffer afterwards, so their latency hides behind the tile and the block needs one
// barrier per tile.  Otherwise the patch is staged in place between two barriers.  Packed
// words go to one of two LDS output tiles and are copied out after the next barrier.
//
// NS > 0 (the launcher's choice for PIPE when a kernel row fits 16 bytes): the number of
// 32-wide K steps is the compile-time NS and a K step's two 16-byte halves are two kernel
// rows, so every LDS address of the tile loop is a per-lane base fixed at kernel start plus an
// immediate, and the pixel-tile and channel-group loops are straight-line code.
template <int NG, bool PIPE, int NS>
__global__ __launch_bounds__(256, NS > 0 ? 4 : 3) void conv_first_mfma(const int8_t *__restrict__ in,
                                                       const int8_t *__restrict__ wt, FirstGeomM g, EpiArgs ep,
                                                       ClearArgs clr)
{
    extern __shared__ __align__(16) unsigned char smem[];
    clear_words(clr);
    constexpr bool FAST = NS > 0;
    constexpr int NSA = FAST ? NS : 1;
    const int ws = FAST ? NS * 32 + 16 : g.kp + 16;             // weight row stride in bytes
    constexpr int TN = 2;                                       // 32-channel tiles per group
    constexpr int BW = 2 * NG;                                  // packed output words per pixel
    unsigned char *Wl = smem;                                   // [64*NG][ws]
    uint32_t *Ol = reinterpret_cast<uint32_t *>(smem + 64 * NG * ws);          // [2][256][BW]
    int *Tl = reinterpret_cast<int *>(smem + 64 * NG * ws + 2 * 256 * BW * 4);  // [64*NG] start values
    unsigned char *Pl = smem + 64 * NG * ws + 2 * 256 * BW * 4 + 64 * NG * 4;   // [1 or 2] x ([ni][ph][pw][c_in] + slack)

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, half = lane >> 5;

    const int co_tile = blockIdx.y;
    const int th = 1 << g.lth, tw = 1 << g.ltw;
    const int o_blk = co_tile * 64 * NG;
    const int pw = tw + g.kw - 1, ph = th + g.kh - 1;

    // ---- this lane's two pixels (window-major rows of the implicit GEMM)
    int pixbyte[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int p = wave * 64 + i * 32 + l32;
        const int wq = p >> 2, sub = p & 3;
        const int wx = wq & ((tw >> 1) - 1);
        const int wy = (wq >> (g.ltw - 1)) & ((th >> 1) - 1);
        const int il = wq >> (g.ltw - 1 + g.lth - 1);
        const int py = 2 * wy + (sub >> 1), px = 2 * wx + (sub & 1);
        pixbyte[i] = ((il * ph + py) * pw + px) * g.c_in;
    }
    const int u16 = g.slp >> 4;                  // 16-byte units per kernel row
    const int nsteps = FAST ? NS : g.kp >> 5;
    // FAST: dword index and byte shift of this lane's 16 operand bytes per (pixel tile, K step);
    // kernel rows past the last one read the patch start and meet zero weights
    int gd[2][NSA];
    unsigned gsh[2][NSA];
    if (FAST) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int ks = 0; ks < NSA; ++ks) {
                const int ti = 2 * ks + half;
                const int addr = ti < g.kh ? pixbyte[i] + ti * pw * g.c_in : 0;
                gd[i][ks] = addr >> 2;
                gsh[i][ks] = (unsigned)addr & 3u;
            }
    }
    const unsigned char *wlane = Wl + l32 * ws + half * 16;     // this lane's bytes of a weight row tile

    StepWords<TN> sw[NG];

    // ---- persistent loop over (image group, tile) work items
    struct Item { int grp, ty, tx; };                   // image group, tile row, tile column
    auto decode = [&](int item) {
        Item c;
        const int r1 = div_by(item, g.tiles_x, g.mg_tx);
        c.tx = item - r1 * g.tiles_x;
        c.grp = div_by(r1, g.tiles_y, g.mg_ty);
        c.ty = r1 - c.grp * g.tiles_y;
        return c;
    };
    // a step of gridDim.x items is a fixed (group, row, column) increment with carries
    Item step;
    step.grp = g.step_grp; step.ty = g.step_ty; step.tx = g.step_tx;
    auto advance = [&](Item &c) {
        c.tx += step.tx;
        if (c.tx >= g.tiles_x) { c.tx -= g.tiles_x; ++c.ty; }
        c.ty += step.ty;
        if (c.ty >= g.tiles_y) { c.ty -= g.tiles_y; ++c.grp; }
        c.grp += step.grp;
    };
    auto item_pos = [&](const Item &c) {
        TilePos pos;
        pos.n = g.n; pos.h = g.ho; pos.w = g.wo; pos.c_out = g.c_out;
        pos.lth = g.lth; pos.ltw = g.ltw; pos.img0 = c.grp * g.ni; pos.y0 = c.ty * th; pos.x0 = c.tx * tw;
        return pos;
    };
    // Patch bytes base + u*256 + t (u = 0..3) of an item: pad_value outside the image, zero in
    // the slack behind the patch.  Branch-free, so that the four loads are in flight together:
    // bytes that are not read from the image load the tensor's first byte instead.
    const int total = g.ni * ph * pw * g.c_in;
    auto load_bytes = [&](const Item &c, int base, int (&v)[4]) {
        const int img0 = c.grp * g.ni, y0 = c.ty * th, x0 = c.tx * tw;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = base + u * 256 + t;
            const int p0 = div_magic(idx, g.mg_cin), ch = idx - p0 * g.c_in;
            const int p1 = div_magic(p0, g.mg_pw), px = p0 - p1 * pw;
            const int il = div_magic(p1, g.mg_ph), py = p1 - il * ph;
            const int y = y0 + py - g.pad, x = x0 + px - g.pad, img = img0 + il;
            const bool inside = idx < total && img < g.n && y >= 0 && y < g.h && x >= 0 && x < g.w;
            const int8_t b = in[inside ? (((int64_t)img * g.h + y) * g.w + x) * g.c_in + ch : 0];
            v[u] = inside ? (int)b : (idx < total ? g.pad_value : 0);
        }
    };
    // PIPE: the position of a thread's four bytes inside the patch does not depend on the
    // item, so it is worked out once: image, row and column relative to the tile origin
    // (packed into one register) and the byte offset relative to the origin's address.
    int pk[4], rel[4];
    if (PIPE) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = u * 256 + t;
            const int p0 = div_magic(idx, g.mg_cin), ch = idx - p0 * g.c_in;
            const int p1 = div_magic(p0, g.mg_pw), px = p0 - p1 * pw;
            const int il = div_magic(p1, g.mg_ph), py = p1 - il * ph;
            // 12-bit signed fields: -1024 <= -pad <= ry, rx < patch extent - pad <= 1024 (the patch has
            // at most 1024 bytes and the interface caps pad at 1024); il < 64 keeps the sign bit clear
            const int ry = py - g.pad, rx = px - g.pad;
            pk[u] = idx < total ? ((il << 24) | ((ry & 0xfff) << 12) | (rx & 0xfff)) : -1;
            rel[u] = ((il * g.h + ry) * g.w + rx) * g.c_in + ch;
        }
    }
    auto load_bytes_pipe = [&](const Item &c, int (&v)[4]) {
        const int img0 = c.grp * g.ni, y0 = c.ty * th, x0 = c.tx * tw;
        const int8_t *origin = in + (((int64_t)img0 * g.h + y0) * g.w + x0) * g.c_in;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int y = y0 + ((pk[u] << 8) >> 20), x = x0 + ((pk[u] << 20) >> 20), img = img0 + (pk[u] >> 24);
            const bool in_patch = pk[u] >= 0;
            const bool inside = in_patch & (img < g.n) & ((unsigned)y < (unsigned)g.h) & ((unsigned)x < (unsigned)g.w);
            const int8_t b = inside ? origin[rel[u]] : in[0];
            v[u] = inside ? (int)b : (in_patch ? g.pad_value : 0);
        }
    };
    auto store_bytes = [&](unsigned char *P, int base, const int (&v)[4]) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = base + u * 256 + t;
            if (idx < g.patch_bytes) P[idx] = (unsigned char)(int8_t)v[u];
        }
    };

    int vn[4];
    Item cur = decode(blockIdx.x < (unsigned)g.n_items ? (int)blockIdx.x : 0), prev = cur, nxt = cur;
    const CopyLane copy_lane = make_copy_lane(256, item_pos(cur), ep.pool, t);
    // the first patch is requested before the weights, so that their latencies overlap
    if (PIPE && (int)blockIdx.x < g.n_items) load_bytes_pipe(cur, vn);

    // ---- weights of this block's channels in the K-padded layout, staged once per block.
    // One thread per (channel, kernel row): its sl source bytes are contiguous in memory and
    // land at the start of a slp-byte slot whose rest is zero; loads of a slot are issued
    // together.  The K padding behind the last kernel row is zeroed separately.
    {
        const int k_total = g.kh * g.sl;
        const int nrow = 64 * NG;
        // Bytes come through a buffer resource over the weight tensor: a channel past c_out
        // addresses past its end and reads zeros, so the loads need no predicate; the bytes
        // behind a short kernel row (the next row's weights) are masked off per dword.
        const __amdgpu_buffer_rsrc_t wr =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(wt), 0, g.c_out * k_total, 0x00020000);
        for (int pair = t; pair < nrow * g.kh; pair += 256) {
            const int row = div_magic(pair, g.mg_kh), ti = pair - row * g.kh;
            const int base = (o_blk + row) * k_total + ti * g.sl;
            unsigned char *dst = Wl + row * ws + ti * g.slp;
            for (int b0 = 0; b0 < g.slp; b0 += 16) {
                unsigned v[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) v[q] = __builtin_amdgcn_raw_buffer_load_b8(wr, base + b0 + q, 0, 0);
                unsigned w[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int nvalid = g.sl - b0 - 4 * k;          // weight bytes in this dword
                    const unsigned mask = nvalid >= 4 ? 0xffffffffu : (nvalid <= 0 ? 0u : (1u << (8 * nvalid)) - 1u);
                    w[k] = (v[4 * k] | (v[4 * k + 1] << 8) | (v[4 * k + 2] << 16) | (v[4 * k + 3] << 24)) & mask;
                }
                *reinterpret_cast<uint4 *>(dst + b0) = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
        // kp rounds kh * slp (a multiple of 16) up to a multiple of 32: the tail is 0 or 16 bytes
        const int tail0 = g.kh * g.slp;
        if (g.kp > tail0) {
            for (int row = t; row < nrow; row += 256)
                *reinterpret_cast<uint4 *>(Wl + row * ws + tail0) = make_uint4(0u, 0u, 0u, 0u);
        }
    }

    // per-channel step parameters, fetched once per block (the first barrier of the tile
    // loop publishes the accumulator start values; sums stay far below 2^30)
    if (ep.packed) {
#pragma unroll
        for (int grp = 0; grp < NG; ++grp) sw[grp] = load_step_words<TN>(ep, o_blk + grp * 64, l32, g.c_out);
    }
    stage_bias_i32(ep, o_blk, 64 * NG, g.c_out, 1 << 30, Tl, t);
    if (PIPE && (int)blockIdx.x < g.n_items) store_bytes(Pl, 0, vn);
    int it = 0;
    for (int item = blockIdx.x; item < g.n_items; item += gridDim.x, ++it) {
        const unsigned char *Pc = Pl + (PIPE ? (it & 1) * g.patch_bytes : 0);
        uint32_t *Oc = Ol + (it & 1) * (256 * BW);
        prev = cur;
        cur = nxt;
        advance(nxt);
        const int next_item = item + (int)gridDim.x;
        if (!PIPE) {
            __syncthreads();      // previous item's patch fully consumed
            for (int base = 0; base < g.patch_bytes; base += 256 * 4) {
                int v[4];
                load_bytes(cur, base, v);
                store_bytes(Pl, base, v);
            }
        }
        __syncthreads();          // patch (and, the first time, weights and start values) visible
        if (PIPE && next_item < g.n_items) load_bytes_pipe(nxt, vn);
        if (ep.packed && it > 0)
            conv_tile_copy_out<BW>(Ol + ((it - 1) & 1) * (256 * BW), copy_lane, o_blk >> 5, item_pos(prev), ep);
        const unsigned *P32 = reinterpret_cast<const unsigned *>(Pc);

        const TilePos pos = item_pos(cur);

        // one 32-pixel tile after the other (keeps the register footprint small enough for
        // three blocks per compute unit)
        constexpr int IU = FAST ? 2 : 1, GU = FAST ? NG : 1;
#pragma unroll IU
        for (int i = 0; i < 2; ++i) {
            // activation operands of all K steps (at most 4), gathered once per pixel tile:
            // 16 bytes from an arbitrary byte address = five aligned dwords, funnel-shifted
            v4i a[4];
            auto gather16 = [&](int ks, int d, unsigned sh) {
                const unsigned w0 = P32[d], w1 = P32[d + 1], w2 = P32[d + 2], w3 = P32[d + 3], w4 = P32[d + 4];
                a[ks][0] = (int)__builtin_amdgcn_alignbyte(w1, w0, sh);
                a[ks][1] = (int)__builtin_amdgcn_alignbyte(w2, w1, sh);
                a[ks][2] = (int)__builtin_amdgcn_alignbyte(w3, w2, sh);
                a[ks][3] = (int)__builtin_amdgcn_alignbyte(w4, w3, sh);
            };
            if constexpr (FAST) {
#pragma unroll
                for (int ks = 0; ks < NS; ++ks) gather16(ks, gd[i][ks], gsh[i][ks]);
            } else {
                const int pixb = i ? pixbyte[1] : pixbyte[0];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    if (ks >= nsteps) break;
                    const int k16 = 2 * ks + half;
                    const int ti = k16 / u16, off = (k16 - ti * u16) << 4;
                    const int addr = ti < g.kh ? pixb + ti * pw * g.c_in + off : 0;
                    gather16(ks, addr >> 2, (unsigned)addr & 3u);
                }
            }
            const int row0 = wave * 64 + i * 32;

#pragma unroll GU
            for (int grp = 0; grp < NG; ++grp) {
                __builtin_amdgcn_s_setprio(1);           // multiplies outrank other waves' epilogues
                // accumulators start at the channels' biases (see stage_bias_i32)
                const int *Tg = Tl + grp * 64;
                v16i acc[TN];
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[j] = load_bias16<v16i>(Tg + j * 32, half);
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    if (FAST ? ks >= NS : ks >= nsteps) break;
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const v4i b = *reinterpret_cast<const v4i *>(wlane + (grp * TN + j) * 32 * ws + ks * 32);
                        acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b, a[ks], acc[j], 0, 0, 0);   // rows = channels
                    }
                }
                __builtin_amdgcn_s_setprio(0);
                const int ch0 = o_blk + grp * 64;
                if (ep.preact) {
                    auto getx = [&](int, int j, int r) {
                        return acc[j][r] - Tg[j * 32 + (r >> 2) * 8 + half * 4 + (r & 3)];
                    };
                    conv_tile_store_preact<1, TN>(getx, row0, ch0, l32, half, pos, ep.preact);
                }
                if (ep.packed) {
                    // select this group's words without indexing the register array dynamically
                    StepWords<TN> cursw = sw[0];
#pragma unroll
                    for (int q = 1; q < NG; ++q)
                        if (grp == q) cursw = sw[q];
                    auto gets = [&](int, int j, int r) { return acc[j][r]; };
                    conv_tile_step_to_lds<1, TN>(gets, row0, grp * TN, BW, l32, half, cursw, ep.pool,
                                                 ep.pool_first != 0, Oc);
                }
                if (FAST) __builtin_amdgcn_sched_barrier(0);      // one group's registers at a time
            }
        }
        if (PIPE && next_item < g.n_items) store_bytes(Pl + ((it + 1) & 1) * g.patch_bytes, 0, vn);
    }
    if (ep.packed && it > 0) {
        __syncthreads();
        conv_tile_copy_out<BW>(Ol + ((it - 1) & 1) * (256 * BW), copy_lane, o_blk >> 5, item_pos(cur), ep);
    }
}

// ---- 3x3 kernels, one ring of padding, images of a few KB: whole images in LDS.
//
// conv_first_mfma stages, per 256-pixel tile, the tile's input patch byte by byte (every byte has
// its own bounds test); for the benchmark's first layers that staging, not the arithmetic, is
// most of the kernel.  Here a block copies whole images (contiguous in memory: 16-byte loads, no
// index arithmetic) into LDS slots and then takes the 256-pixel tiles of those images one after
// the other.  Rows above and below an image fall into the slot's pad regions, which are filled
// with pad_value once per block; the columns left and right of the image are patched into the
// gathered operand with a per-lane byte mask (a lane's pixel column does not change: a tile
// spans the whole image width).  Work unit = (image group, run of TPB consecutive tiles); the
// next unit's images are requested before the current unit is computed and stored to the other
// LDS buffer afterwards.  MFMA, epilogue and deferred copy-out are those of conv_first_mfma's
// straight-line variant: K = [kernel row][3 * c_in bytes, padded to 16], two kernel rows per
// K step (the second step's upper half meets zero weights).
struct FirstGeomI {
    int n, h, c_in, c_out, pad_value;
    int lth, ltw, ni;           // tile = (1 << lth) rows x (1 << ltw = image width) columns x ni images
    int tiles_y, tpb, cpg;      // tiles per image group, tiles per work unit, work units per image group
    int n_groups, n_units;
    int img_bytes;              // h * w * c_in, a multiple of 16
    int front, slot_bytes;      // pad bytes before an image in its LDS slot (multiple of 16) / slot size
    int buf_bytes;              // ni * slot_bytes
    unsigned mg_upi, mg_cpg;    // magic_floor of 16-byte units per image, of cpg
};

template <int NG, int NU>
__global__ __launch_bounds__(256, 4) void conv_first_img(const int8_t *__restrict__ in, const int8_t *__restrict__ wt,
                                                         FirstGeomI g, EpiArgs ep, ClearArgs clr)
{
    extern __shared__ __align__(16) unsigned char smem[];
    clear_words(clr);
    constexpr int NS = 2, TN = 2, BW = 2 * NG, WS = NS * 32 + 16;
    unsigned char *Wl = smem;                                                    // [64*NG][WS]
    uint32_t *Ol = reinterpret_cast<uint32_t *>(smem + 64 * NG * WS);            // [2][256][BW]
    int *Tl = reinterpret_cast<int *>(smem + 64 * NG * WS + 2 * 256 * BW * 4);   // [64*NG] start values
    unsigned char *Pl = smem + 64 * NG * WS + 2 * 256 * BW * 4 + 64 * NG * 4;    // [2][ni] image slots

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int o_blk = (int)blockIdx.y * 64 * NG;
    const int w = 1 << g.ltw, th = 1 << g.lth;
    const int row_bytes = w * g.c_in;

    // ---- work units: unit u = image group u / cpg, tiles [(u % cpg) * tpb, + tpb)
    auto group_of = [&](int u) { return div_by(u, g.cpg, g.mg_cpg); };
    // 16-byte units of a group's images: unit -> (image slot, offset); branch-free loads, a unit
    // beyond the last image of the batch reads the tensor's first bytes (never used: its pixels
    // are not stored)
    // (named registers, not an array: the loads sit inside a conditional and an array would be
    // kept in scratch memory)
    uint4 vn0, vn1;
    vn0 = vn1 = make_uint4(0u, 0u, 0u, 0u);
    auto load_unit = [&](int u, int64_t src, int valid) {
        const int byte = (u * 256 + t) * 16;
        return *reinterpret_cast<const uint4 *>(in + (byte < valid ? src + byte : (int64_t)0));
    };
    auto load_group = [&](int grp) {
        const int valid = min(g.ni, g.n - grp * g.ni) * g.img_bytes;
        const int64_t src = (int64_t)grp * g.ni * g.img_bytes;
        vn0 = load_unit(0, src, valid);
        if constexpr (NU > 1) vn1 = load_unit(1, src, valid);
    };
    auto store_unit = [&](int u, int buf, const uint4 &v) {
        const int upi = g.img_bytes >> 4;
        const int unit = u * 256 + t;
        const int il = div_by(unit, upi, g.mg_upi);
        if (il < g.ni)
            *reinterpret_cast<uint4 *>(Pl + buf * g.buf_bytes + il * g.slot_bytes + g.front + (unit - il * upi) * 16) = v;
    };
    auto store_group = [&](int buf) {
        store_unit(0, buf, vn0);
        if constexpr (NU > 1) store_unit(1, buf, vn1);
    };
    // ---- prologue.  Every global load of the prologue (first images, weights, thresholds, flips)
    // is issued before the first of them is waited for: one memory latency instead of four.
    const int first_unit = (int)blockIdx.x;
    if (first_unit < g.n_units) load_group(group_of(first_unit));

    // weights of this block's channels, K-padded: one thread per (channel, kernel row) slot of 16
    // bytes (3 * c_in source bytes, contiguous in memory) through a buffer resource over the weight
    // tensor: slots of channels past c_out, and of the rounds' unused threads, address past its end
    // and read zeros
    constexpr int NPAIR = 64 * NG * 3, NR = (NPAIR + 255) / 256;
    const int sl = 3 * g.c_in, k_total = 3 * sl;
    // (the range is rounded up to whole dwords: the last valid byte's dword must not be refused; the
    // at most three bytes behind the tensor share an aligned dword with it and are masked off)
    const __amdgpu_buffer_rsrc_t wr =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(wt), 0, (g.c_out * k_total + 3) & ~3, 0x00020000);
    unsigned wv[NR][4];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const int pair = t + 256 * r;
        const int row = pair / 3, ti = pair - row * 3;
        // the slot's 3 * c_in <= 12 source bytes lie in the four dwords from its start rounded down
        const int base = pair < NPAIR ? ((o_blk + row) * k_total + ti * sl) & ~3 : 0x7ffffff0;
#pragma unroll
        for (int q = 0; q < 4; ++q) wv[r][q] = __builtin_amdgcn_raw_buffer_load_b32(wr, base + 4 * q, 0, 0);
    }
    // threshold of channel t of the block (start value of its accumulators), flips
    int thr_t = 0;
    if (ep.packed && t < 64 * NG && o_blk + t < g.c_out) thr_t = ep.thr[o_blk + t];
    StepWords<TN> sw[NG];
    if (ep.packed) {
#pragma unroll
        for (int grp = 0; grp < NG; ++grp) sw[grp] = load_step_words<TN>(ep, o_blk + grp * 64, l32, g.c_out);
    }

    // ---- pad regions of every slot of both buffers, once per block
    {
        const unsigned pv = (unsigned)(uint8_t)(int8_t)g.pad_value * 0x01010101u;
        const int padw = (g.slot_bytes - g.img_bytes) >> 2, frontw = g.front >> 2;
        const unsigned mg = magic_floor(padw);
        for (int idx = t; idx < 2 * g.ni * padw; idx += 256) {
            const int slot = div_by(idx, padw, mg), j = idx - slot * padw;
            const int off = j < frontw ? j * 4 : g.img_bytes + j * 4;
            *reinterpret_cast<unsigned *>(Pl + slot * g.slot_bytes + off) = pv;
        }
    }

    // ---- this lane's two pixels (window-major rows of the implicit GEMM): where the 16 operand
    // bytes of (pixel tile i, K step ks) start inside an image buffer, relative to the unit's
    // first tile row, and the bytes of the operand that lie left or right of the image
    int gd[2][NS];
    unsigned gsh[2][NS], edge[2][3];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int p = wave * 64 + i * 32 + l32;
        const int wq = p >> 2, sub = p & 3;
        const int wx = wq & ((w >> 1) - 1);
        const int wy = (wq >> (g.ltw - 1)) & ((th >> 1) - 1);
        const int il = wq >> (g.ltw - 1 + g.lth - 1);
        const int py = 2 * wy + (sub >> 1), px = 2 * wx + (sub & 1);
#pragma unroll
        for (int ks = 0; ks < NS; ++ks) {
            const int ti = 2 * ks + half;
            const int addr = ti < 3 ? il * g.slot_bytes + g.front + (py + ti - 1) * row_bytes + (px - 1) * g.c_in : 0;
            gd[i][ks] = addr >> 2;
            gsh[i][ks] = (unsigned)addr & 3u;
        }
        // operand bytes [0, c_in) lie left of the image for px == 0, bytes [2 c_in, 3 c_in) right of it
        // for px == w - 1 (c_in <= 4: twelve operand bytes, three dwords)
        const unsigned __int128 field = ((unsigned __int128)1 << (8 * g.c_in)) - 1;
        const unsigned __int128 m = (px == 0 ? field : 0) | (px == w - 1 ? field << (16 * g.c_in) : 0);
        edge[i][0] = (unsigned)m; edge[i][1] = (unsigned)(m >> 32); edge[i][2] = (unsigned)(m >> 64);
    }
    const unsigned padv4 = (unsigned)(uint8_t)(int8_t)g.pad_value * 0x01010101u;
    const unsigned char *wlane = Wl + l32 * WS + half * 16;     // this lane's bytes of a weight row tile

    // ---- what was loaded goes to LDS: weight slots (the bytes behind a kernel row's 3 * c_in
    // belong to the next row and are masked off; the K padding behind the third row is zero),
    // accumulator start values -(threshold) - 1 (see stage_bias_i32), the first images
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const int pair = t + 256 * r;
        const int row = pair / 3, ti = pair - row * 3;
        const unsigned sh = (unsigned)((o_blk + row) * k_total + ti * sl) & 3u;
        unsigned wd[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int nvalid = sl - 4 * k;
            const unsigned mask = nvalid >= 4 ? 0xffffffffu : (nvalid <= 0 ? 0u : (1u << (8 * nvalid)) - 1u);
            wd[k] = (k < 3 ? __builtin_amdgcn_alignbyte(wv[r][k + 1], wv[r][k], sh) : 0u) & mask;
        }
        if (pair < NPAIR) *reinterpret_cast<uint4 *>(Wl + row * WS + ti * 16) = make_uint4(wd[0], wd[1], wd[2], wd[3]);
    }
    if (t < 64 * NG) {
        *reinterpret_cast<uint4 *>(Wl + t * WS + 48) = make_uint4(0u, 0u, 0u, 0u);
        int v = 0;
        if (ep.packed && o_blk + t < g.c_out) {
            const int bound = 1 << 30;
            v = thr_t > bound ? bound : (thr_t < -bound ? -bound : thr_t);
            v = -v - 1;
        }
        Tl[t] = v;
    }
    if (first_unit < g.n_units) store_group(0);

    auto tile_pos = [&](int grp, int ty) {
        TilePos pos;
        pos.n = g.n; pos.h = g.h; pos.w = w; pos.c_out = g.c_out;
        pos.lth = g.lth; pos.ltw = g.ltw; pos.img0 = grp * g.ni; pos.y0 = ty * th; pos.x0 = 0;
        return pos;
    };
    TilePos prev = tile_pos(0, 0);
    const CopyLane copy_lane = make_copy_lane(256, prev, ep.pool, t);

    int it = 0, ui = 0;
    for (int unit = first_unit; unit < g.n_units; unit += (int)gridDim.x, ++ui) {
        const int grp = group_of(unit);
        const int ty0 = (unit - grp * g.cpg) * g.tpb;
        const int next_unit = unit + (int)gridDim.x;
        const unsigned *P32 = reinterpret_cast<const unsigned *>(Pl + (ui & 1) * g.buf_bytes);
        for (int k = 0; k < g.tpb; ++k, ++it) {
            const int ty = ty0 + k;
            uint32_t *Oc = Ol + (it & 1) * (256 * BW);
            __syncthreads();      // the unit's images (first tile) / nothing reads the previous tile's words any more
            if (k == 0 && next_unit < g.n_units) load_group(group_of(next_unit));
            if (ep.packed && it > 0)
                conv_tile_copy_out<BW>(Ol + ((it - 1) & 1) * (256 * BW), copy_lane, o_blk >> 5, prev, ep);
            const TilePos pos = tile_pos(grp, ty);
            prev = pos;
            const int tile_dw = (ty * th * row_bytes) >> 2;       // a tile's rows are a multiple of four bytes
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                v4i a[NS];
#pragma unroll
                for (int ks = 0; ks < NS; ++ks) {
                    const int d = gd[i][ks] + tile_dw;
                    const unsigned sh = gsh[i][ks];
                    const unsigned w0 = P32[d], w1 = P32[d + 1], w2 = P32[d + 2], w3 = P32[d + 3], w4 = P32[d + 4];
                    const unsigned b0 = __builtin_amdgcn_alignbyte(w1, w0, sh), b1 = __builtin_amdgcn_alignbyte(w2, w1, sh);
                    const unsigned b2 = __builtin_amdgcn_alignbyte(w3, w2, sh), b3 = __builtin_amdgcn_alignbyte(w4, w3, sh);
                    a[ks][0] = (int)((b0 & ~edge[i][0]) | (padv4 & edge[i][0]));
                    a[ks][1] = (int)((b1 & ~edge[i][1]) | (padv4 & edge[i][1]));
                    a[ks][2] = (int)((b2 & ~edge[i][2]) | (padv4 & edge[i][2]));
                    a[ks][3] = (int)b3;
                }
                const int row0 = wave * 64 + i * 32;
#pragma unroll
                for (int cg = 0; cg < NG; ++cg) {
                    __builtin_amdgcn_s_setprio(1);           // multiplies outrank other waves' epilogues
                    const int *Tg = Tl + cg * 64;
                    v16i acc[TN];
#pragma unroll
                    for (int j = 0; j < TN; ++j) acc[j] = load_bias16<v16i>(Tg + j * 32, half);
#pragma unroll
                    for (int ks = 0; ks < NS; ++ks)
#pragma unroll
                        for (int j = 0; j < TN; ++j) {
                            const v4i b = *reinterpret_cast<const v4i *>(wlane + (cg * TN + j) * 32 * WS + ks * 32);
                            acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b, a[ks], acc[j], 0, 0, 0);   // rows = channels
                        }
                    __builtin_amdgcn_s_setprio(0);
                    const int ch0 = o_blk + cg * 64;
                    if (ep.preact) {
                        auto getx = [&](int, int j, int r) {
                            return acc[j][r] - Tg[j * 32 + (r >> 2) * 8 + half * 4 + (r & 3)];
                        };
                        conv_tile_store_preact<1, TN>(getx, row0, ch0, l32, half, pos, ep.preact);
                    }
                    if (ep.packed) {
                        StepWords<TN> cursw = sw[0];
#pragma unroll
                        for (int q = 1; q < NG; ++q)
                            if (cg == q) cursw = sw[q];
                        auto gets = [&](int, int j, int r) { return acc[j][r]; };
                        conv_tile_step_to_lds<1, TN>(gets, row0, cg * TN, BW, l32, half, cursw, ep.pool,
                                                     ep.pool_first != 0, Oc);
                    }
                    __builtin_amdgcn_sched_barrier(0);      // one group's registers at a time
                }
            }
        }
        // the other buffer was last read one unit ago, and every wave has passed a barrier since
        if (next_unit < g.n_units) store_group((ui + 1) & 1);
    }
    if (ep.packed && it > 0) {
        __syncthreads();
        conv_tile_copy_out<BW>(Ol + ((it - 1) & 1) * (256 * BW), copy_lane, o_blk >> 5, prev, ep);
    }
}

// 1x1, pad 0, c_in % 16 == 0: int8 GEMM  X[m][o] = sum_c A[m][c] * W[o][c];  m = pixel index.
// Block = 2 x 2 waves, one 32 x 32 tile each; operands are 16-byte global loads.
__global__ __launch_bounds__(256) void fc_first_mfma(const int8_t *__restrict__ A, const int8_t *__restrict__ Wt,
                                                     int64_t M, int N, int K, EpiArgs ep, ClearArgs clr)
{
    clear_words(clr);
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int nbn = (N + 63) / 64;
    const int64_t m0 = (int64_t)(blockIdx.x / nbn) * 64 + (wave >> 1) * 32;
    const int n0 = (blockIdx.x % nbn) * 64 + (wave & 1) * 32;
    const int64_t arow = (m0 + l32 < M) ? m0 + l32 : M - 1;
    const int brow = (n0 + l32 < N) ? n0 + l32 : N - 1;
    const int8_t *ap = A + arow * K;
    const int8_t *bp = Wt + (int64_t)brow * K;
    v16i acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0;
    const int nsteps = (K + 31) / 32;
    for (int ks = 0; ks < nsteps; ++ks) {
        const bool ok = ks * 32 + half * 16 < K;         // K % 16 == 0: a 16-byte slice is all in or all out
        const int koff = ok ? ks * 32 + half * 16 : 0;   // a slice past K re-reads the row's first one (in bounds)
        v4i a = *reinterpret_cast<const v4i *>(ap + koff);
        v4i b = *reinterpret_cast<const v4i *>(bp + koff);
        if (!ok) { a = v4i{0, 0, 0, 0}; b = v4i{0, 0, 0, 0}; }
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc, 0, 0, 0);
    }
    const int col = n0 + l32;
    const bool cok = col < N;
    if (ep.preact) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = m0 + (r >> 2) * 8 + half * 4 + (r & 3);
            if (row < M && cok) ep.preact[row * N + col] = acc[r];
        }
    }
    if (ep.packed) {
        const int nw = (N + 31) >> 5;
        const int thr = cok ? ep.thr[col] : 0;
        const bool flip = cok && ep.flip && ep.flip[col];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool bit = cok && ((acc[r] > thr) != flip);
            const unsigned long long mask = __ballot(bit);
            const unsigned word = half ? (unsigned)(mask >> 32) : (unsigned)mask;
            const int64_t row = m0 + (r >> 2) * 8 + half * 4 + (r & 3);
            if (l32 == 0 && row < M && (n0 >> 5) < nw) ep.packed[row * nw + (n0 >> 5)] = word;
        }
    }
}

// The same int8 GEMM when the 64 x 64 blocks above would leave most compute units idle (the MLP's
// first layer at batch 64: eight of them, each walking K = 784 alone with one load round trip per
// step): a block owns 32 x 32 outputs and its four waves split K, wave v taking the 32-byte steps
// v, v + 4, ... in rounds of up to eight with all loads of a round in flight; the partial sums
// (integers) meet in LDS and wave 0 runs the epilogue.
__global__ __launch_bounds__(256) void fc_first_small(const int8_t *__restrict__ A, const int8_t *__restrict__ Wt,
                                                      int64_t M, int N, int K, int nbn, EpiArgs ep, ClearArgs clr)
{
    clear_words(clr);
    constexpr int UR = 8;
    __shared__ int red[3][16][64];
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int64_t m0 = (int64_t)(blockIdx.x / nbn) * 32;
    const int n0 = (blockIdx.x % nbn) * 32;
    const int64_t arow = (m0 + l32 < M) ? m0 + l32 : M - 1;
    const int brow = (n0 + l32 < N) ? n0 + l32 : N - 1;
    const int8_t *ap = A + arow * K;
    const int8_t *bp = Wt + (int64_t)brow * K;
    v16i acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0;
    const int nsteps = (K + 31) / 32;
    for (int s0 = wave; s0 < nsteps; s0 += 4 * UR) {
        v4i a[UR], b[UR];
#pragma unroll
        for (int k = 0; k < UR; ++k) {
            const int ks = s0 + 4 * k;
            const bool ok = ks < nsteps && ks * 32 + half * 16 < K;   // K % 16 == 0: a slice is all in or all out
            const int koff = ok ? ks * 32 + half * 16 : 0;           // (else the row's first slice, zeroed)
            a[k] = *reinterpret_cast<const v4i *>(ap + koff);
            b[k] = *reinterpret_cast<const v4i *>(bp + koff);
            if (!ok) { a[k] = v4i{0, 0, 0, 0}; b[k] = v4i{0, 0, 0, 0}; }
        }
#pragma unroll
        for (int k = 0; k < UR; ++k)
            if (s0 + 4 * k < nsteps) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[k], b[k], acc, 0, 0, 0);
    }
    if (wave > 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wave - 1][r][lane] = acc[r];
    }
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] += red[0][r][lane] + red[1][r][lane] + red[2][r][lane];

    // register r of lane (l32, half): row m0 + 8 (r / 4) + 4 half + r % 4, column n0 + l32
    const int col = n0 + l32;
    const bool cok = col < N;
    if (ep.preact) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = m0 + (r >> 2) * 8 + half * 4 + (r & 3);
            if (row < M && cok) ep.preact[row * N + col] = acc[r];
        }
    }
    if (ep.packed) {
        const int nw = (N + 31) >> 5;
        const int thr = cok ? ep.thr[col] : 0;
        const bool flip = cok && ep.flip && ep.flip[col];
        unsigned mine = 0;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const unsigned long long mask = __ballot(cok && ((acc[r] > thr) != flip));
            const unsigned word = half ? (unsigned)(mask >> 32) : (unsigned)mask;
            if (l32 == r) mine = word;          // lane r of each half keeps the word of register r
        }
        const int64_t row = m0 + (l32 >> 2) * 8 + half * 4 + (l32 & 3);
        if (l32 < 16 && row < M) ep.packed[row * nw + (n0 >> 5)] = mine;
    }
}

// ---------------------------------------------------------------------------------------------
// A few thousand tiles of 32 pixels x 32 channels at most (small batches of a small image): latency is what counts.
// One wave = 32 output pixels x 32 output channels and nothing is staged: a lane half owns one
// kernel row (ti = 2 * K step + half; kernel height <= 4, a row's kw * c_in <= 16 bytes), reads
// the row's bytes of its pixel and of its channel's weights as five dwords around the unaligned
// start (buffer loads: dwords outside the tensor read as zero) and shifts them into place; bytes
// left or right of the image, and rows above or below it, become the pad value.  Two
// v_mfma_i32_32x32x32_i8 (rows = channels, columns = pixels), then the step in registers: a lane
// holds 16 of its pixel's 32 channel bits, the other half of the wave the rest; with pooling the
// four lanes of a 2x2 window (pixels are window-major then) combine their words or their sums.
struct FirstGeomS {
    int n, h, w, c_in, c_out, kh, kw, sl, pad, pad_value;
    int ho, wo, pool, npix;
    int w2, hw2;                 // output columns and pixels per image, in windows when pooling
    unsigned mg_w2, mg_hw2;
};

__device__ __forceinline__ unsigned bytes_below(int t)      // mask of the bytes b < t of a dword
{
    return t <= 0 ? 0u : (t >= 4 ? 0xffffffffu : (1u << (8 * t)) - 1u);
}

__global__ __launch_bounds__(64) void conv_first_small(const int8_t *__restrict__ in, const int8_t *__restrict__ wt,
                                                       FirstGeomS g, EpiArgs ep, ClearArgs clr)
{
    if (clr.count > 0 && blockIdx.y == 0)
        for (int i = blockIdx.x * 64 + threadIdx.x; i < clr.count; i += gridDim.x * 64) clr.ptr[i] = 0;

    const int lane = threadIdx.x;
    const int l32 = lane & 31, half = lane >> 5;
    const int o0 = blockIdx.y * 32;
    const int oc = o0 + l32;                                  // this lane's weight row

    // this lane's pixel
    const int p = blockIdx.x * 32 + l32;
    const bool pix_ok = p < g.npix;
    const int q = g.pool == 2 ? p >> 2 : p, sub = g.pool == 2 ? p & 3 : 0;
    const int img = div_by(q, g.hw2, g.mg_hw2);
    const int rem = q - img * g.hw2;
    const int wy = div_by(rem, g.w2, g.mg_w2), wx = rem - wy * g.w2;
    const int y = wy * g.pool + (sub >> 1), x = wx * g.pool + (sub & 1);

    // thresholds and flips of this lane's 16 channels (register r: channel 8 (r / 4) + 4 half + r % 4
    // of the tile), on their way early: one address per lane plus immediate offsets; channels
    // past c_out read as zero and are masked off at the end (the clamped flip of such a lane too)
    int thr[16];
    unsigned flipv = 0;                     // flip of channel o0 + l32: one per lane
    if (ep.packed) {
        const __amdgpu_buffer_rsrc_t tr =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(ep.thr), 0, g.c_out * 4, 0x00020000);
        const int tb = (o0 + half * 4) * 4;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            thr[r] = __builtin_amdgcn_raw_buffer_load_b32(tr, tb + ((r >> 2) * 8 + (r & 3)) * 4, 0, 0);
        if (ep.flip) flipv = ep.flip[oc < g.c_out ? oc : g.c_out - 1];
    }

    const __amdgpu_buffer_rsrc_t ir = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(in), 0, (g.n * g.h * g.w * g.c_in + 3) & ~3, 0x00020000);
    const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(wt), 0, (g.c_out * g.kh * g.sl + 3) & ~3, 0x00020000);

    unsigned xa[2][5], xw[2][5];
    int a_addr[2], w_addr[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int ti = 2 * ks + half;
        a_addr[ks] = ((img * g.h + (y + ti - g.pad)) * g.w + (x - g.pad)) * g.c_in;
        w_addr[ks] = (oc * g.kh + ti) * g.sl;
#pragma unroll
        for (int d = 0; d < 5; ++d) {
            // (a dword that starts below zero holds no image byte; its offset becomes one past every
            // tensor this kernel accepts, which reads as zero.  Weight offsets are never negative.)
            const unsigned ao = min((unsigned)((a_addr[ks] & ~3) + 4 * d), 0x7ffffff0u);
            xa[ks][d] = __builtin_amdgcn_raw_buffer_load_b32(ir, (int)ao, 0, 0);
            xw[ks][d] = __builtin_amdgcn_raw_buffer_load_b32(wr, (w_addr[ks] & ~3) + 4 * d, 0, 0);
        }
    }

    // bytes of a kernel row that lie left of the image (columns x - pad + tj < 0) or right of it
    const int lo = (g.pad - x > 0 ? g.pad - x : 0) * g.c_in;
    const int right = g.w + g.pad - x;
    const int hi = (right < g.kw ? (right > 0 ? right : 0) : g.kw) * g.c_in;
    const unsigned padv4 = (unsigned)(uint8_t)(int8_t)g.pad_value * 0x01010101u;
    unsigned outside[4], wkeep[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        outside[d] = bytes_below(lo - 4 * d) | ~bytes_below(hi - 4 * d);
        wkeep[d] = bytes_below(g.sl - 4 * d);                 // a weight row's own bytes; K padding is zero
    }

    v16i acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int ti = 2 * ks + half;
        const int yy = y + ti - g.pad;
        const bool row_in = pix_ok && yy >= 0 && yy < g.h;
        const bool w_ok = ti < g.kh && oc < g.c_out;
        const unsigned sa = (unsigned)a_addr[ks] & 3u, swt = (unsigned)w_addr[ks] & 3u;
        v4i av, wv;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const unsigned ad = __builtin_amdgcn_alignbyte(xa[ks][d + 1], xa[ks][d], sa);
            const unsigned wd = __builtin_amdgcn_alignbyte(xw[ks][d + 1], xw[ks][d], swt);
            av[d] = (int)(row_in ? ((ad & ~outside[d]) | (padv4 & outside[d])) : padv4);
            wv[d] = (int)(w_ok ? wd & wkeep[d] : 0u);
        }
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wv, av, acc, 0, 0, 0);
    }

    if (ep.preact && pix_ok) {
        int32_t *dst = ep.preact + ((int64_t)(img * g.ho + y) * g.wo + x) * g.c_out;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int o = o0 + (r >> 2) * 8 + half * 4 + (r & 3);
            if (o < g.c_out) dst[o] = acc[r];
        }
    }
    if (ep.packed) {
        if (g.pool == 2 && ep.pool_first != 0) {    // max over the window's four lanes, then the step
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int v = acc[r];
                v = max(v, __shfl_xor(v, 1));
                acc[r] = max(v, __shfl_xor(v, 2));
            }
        }
        // decision of register r in bit r: the sign of thr - x, shifted in from the right
        unsigned dec = 0;
#pragma unroll
        for (int r = 15; r >= 0; --r) {
            const int64_t diff = (int64_t)thr[r] - (int64_t)acc[r];          // negative iff x > thr
            dec = (dec << 1) | (unsigned)((uint64_t)diff >> 63);
        }
        // nibble r / 4 of the 16 bits goes to bits 8 (r / 4) + 4 half .. + 3 of the channel word
        unsigned bits = (dec & 0x000fu) | ((dec & 0x00f0u) << 4) | ((dec & 0x0f00u) << 8) | ((dec & 0xf000u) << 12);
        bits <<= 4 * half;
        unsigned word = bits | (unsigned)__shfl_xor((int)bits, 32);
        word ^= (unsigned)__ballot(flipv != 0);     // both wave halves hold the tile's 32 flips
        const int left = g.c_out - o0;              // channels of this tile that exist
        word &= left >= 32 ? 0xffffffffu : (1u << left) - 1u;
        if (g.pool == 2 && ep.pool_first == 0) {    // max of +-1 values = OR of the bits
            word |= (unsigned)__shfl_xor((int)word, 1);
            word |= (unsigned)__shfl_xor((int)word, 2);
        }
        const int nw = (g.c_out + 31) >> 5;
        if (half == 0 && pix_ok && sub == 0) ep.packed[(int64_t)q * nw + blockIdx.y] = word;
    }
}

bnn_status launch_first_small(const int8_t *in, const int8_t *wt, int n, int h, int w, int c_in, int c_out,
                              int kh, int kw, int pad, int pad_value, const EpiArgs &ep, const ClearArgs &clr,
                              hipStream_t s)
{
    FirstGeomS g;
    g.n = n; g.h = h; g.w = w; g.c_in = c_in; g.c_out = c_out; g.kh = kh; g.kw = kw; g.sl = kw * c_in;
    g.pad = pad; g.pad_value = pad_value;
    g.ho = h + 2 * pad - kh + 1; g.wo = w + 2 * pad - kw + 1;
    g.pool = ep.packed ? ep.pool : 1;
    const int64_t npix = (int64_t)n * g.ho * g.wo;
    // up to 6144 waves (pixel tiles x channel tiles): measured against the staged kernels on the two
    // benchmark models' first layers, it wins below that (batch 48 / 64) and ties there
    const int64_t waves = ((npix + 31) / 32) * ((c_out + 31) / 32);
    if (kh > 4 || g.sl > 16 || waves > 6144 || (int64_t)n * h * w * c_in > 0x7ffffff0LL ||
        (int64_t)c_out * kh * g.sl > 0x7ffffff0LL)
        return BNN_ERR_UNSUPPORTED;
    g.npix = (int)npix;
    g.w2 = g.wo / g.pool;
    g.hw2 = (g.ho / g.pool) * g.w2;
    g.mg_w2 = magic_floor(g.w2); g.mg_hw2 = magic_floor(g.hw2);
    const dim3 grid((unsigned)((npix + 31) / 32), (unsigned)((c_out + 31) / 32));
    hipLaunchKernelGGL(conv_first_small, grid, dim3(64), 0, s, in, wt, g, ep, clr);
    return hip_result(hipGetLastError());
}

template <int NG>
bnn_status launch_first_mfma(const int8_t *in, const int8_t *wt, FirstGeomM &g, const EpiArgs &ep,
                             const ClearArgs &clr, hipStream_t s)
{
    g.n_co_tiles = (g.c_out + 64 * NG - 1) / (64 * NG);
    // pipelined patch: four bytes per thread, each addressed by a 32-bit offset from the tile origin
    const bool pipe = g.patch_bytes <= 1024 && (int64_t)(g.ni + 1) * g.h * g.w * g.c_in < 0x7fffffffLL;
    const size_t smem = (size_t)64 * NG * (g.kp + 16) + 2 * 256 * 2 * NG * 4 + 64 * NG * 4 +
                        (size_t)(pipe ? 2 : 1) * g.patch_bytes;
    const int64_t items = (int64_t)g.tiles_x * g.tiles_y * ((g.n + g.ni - 1) / g.ni);
    if (smem > 64 * 1024 || items > 0x7fffffffLL || g.n_co_tiles > 65535) return BNN_ERR_UNSUPPORTED;
    g.n_items = (int)items;
    // persistent blocks: weights are staged once, then the block walks its share of the tiles
    const int ns = g.kp >> 5;
    const bool fast = pipe && g.slp == 16 && ns <= 2;           // the straight-line variants: four blocks per CU
    const int64_t cap = 256 * (fast ? 4 : 3);
    const unsigned bx = (unsigned)(items < cap ? items : cap);
    const dim3 grid(bx, (unsigned)g.n_co_tiles);
    {   // bx items as an (image group, tile row, tile column) increment
        const int r1 = (int)bx / g.tiles_x;
        g.step_tx = (int)bx - r1 * g.tiles_x;
        g.step_grp = r1 / g.tiles_y;
        g.step_ty = r1 - g.step_grp * g.tiles_y;
        g.mg_tx = magic_floor(g.tiles_x);
        g.mg_ty = magic_floor(g.tiles_y);
    }
    if (fast && ns == 1)
        hipLaunchKernelGGL((conv_first_mfma<NG, true, 1>), grid, dim3(256), smem, s, in, wt, g, ep, clr);
    else if (fast)
        hipLaunchKernelGGL((conv_first_mfma<NG, true, 2>), grid, dim3(256), smem, s, in, wt, g, ep, clr);
    else if (pipe)
        hipLaunchKernelGGL((conv_first_mfma<NG, true, 0>), grid, dim3(256), smem, s, in, wt, g, ep, clr);
    else
        hipLaunchKernelGGL((conv_first_mfma<NG, false, 0>), grid, dim3(256), smem, s, in, wt, g, ep, clr);
    return hip_result(hipGetLastError());
}

// Whole-image kernel: 3x3, one ring of padding, at most four input channels, image width a power
// of two that a 256-pixel tile spans, image groups of at most 8 KB.  BNN_ERR_UNSUPPORTED otherwise.
template <int NG>
bnn_status launch_first_img(const int8_t *in, const int8_t *wt, int n, int h, int w, int c_in, int c_out,
                            int pad_value, const EpiArgs &ep, const ClearArgs &clr, hipStream_t s)
{
    // a 256-pixel tile spans the whole image width (a power of two, 2 .. 128); it takes 256 / w rows
    // of one image, or whole images when they have fewer than 256 pixels (height a power of two then)
    auto log2_exact = [](int v) { int l = 0; while ((1 << l) < v) ++l; return (1 << l) == v ? l : -1; };
    const int ltw = log2_exact(w);
    if (ltw < 1 || ltw > 7) return BNN_ERR_UNSUPPORTED;
    int lth = 8 - ltw, ni = 1;
    if (h < (1 << lth)) {
        lth = log2_exact(h);
        if (lth < 1) return BNN_ERR_UNSUPPORTED;
        ni = 256 >> (ltw + lth);
    } else if (h % (1 << lth) != 0) {
        return BNN_ERR_UNSUPPORTED;
    }
    const int th = 1 << lth;
    FirstGeomI g;
    g.n = n; g.h = h; g.c_in = c_in; g.c_out = c_out; g.pad_value = pad_value;
    g.lth = lth; g.ltw = ltw; g.ni = ni;
    g.img_bytes = h * w * c_in;
    if ((g.img_bytes & 15) != 0 || (int64_t)g.ni * g.img_bytes > 8192) return BNN_ERR_UNSUPPORTED;
    const int row_bytes = w * c_in;
    g.front = (row_bytes + c_in + 15) & ~15;
    g.slot_bytes = (g.front + g.img_bytes + row_bytes + c_in + 32 + 15) & ~15;   // gathers read 20 bytes past a row's start
    g.buf_bytes = g.ni * g.slot_bytes;
    g.tiles_y = ni == 1 ? h / th : 1;
    g.n_groups = (n + g.ni - 1) / g.ni;
    const int n_co_tiles = (c_out + 64 * NG - 1) / (64 * NG);
    // tiles per work unit: as many as still leave four blocks for every compute unit
    g.tpb = 1;
    for (int d = g.tiles_y; d >= 1; --d)
        if (g.tiles_y % d == 0 && (int64_t)g.n_groups * (g.tiles_y / d) * n_co_tiles >= 1024) { g.tpb = d; break; }
    g.cpg = g.tiles_y / g.tpb;
    const int64_t units = (int64_t)g.n_groups * g.cpg;
    if (units > 0x3fffffffLL || n_co_tiles > 65535) return BNN_ERR_UNSUPPORTED;
    g.n_units = (int)units;
    g.mg_upi = magic_floor(g.img_bytes >> 4);
    g.mg_cpg = magic_floor(g.cpg);
    const size_t smem = (size_t)64 * NG * 80 + 2 * 256 * 2 * NG * 4 + 64 * NG * 4 + (size_t)2 * g.buf_bytes;
    if (smem > 40 * 1024) return BNN_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)(units < 1024 ? units : 1024), (unsigned)n_co_tiles);
    const int group_bytes = g.ni * g.img_bytes;
    if (group_bytes <= 4096)
        hipLaunchKernelGGL((conv_first_img<NG, 1>), grid, dim3(256), smem, s, in, wt, g, ep, clr);
    else
        hipLaunchKernelGGL((conv_first_img<NG, 2>), grid, dim3(256), smem, s, in, wt, g, ep, clr);
    return hip_result(hipGetLastError());
}

}  // namespace

bnn_status launch_conv_first_int8(const int8_t *in, int n, int h, int w, int c_in, const int8_t *wt,
                                  int c_out, int kh, int kw, int pad, int pad_value, const EpiArgs &ep,
                                  const ClearArgs &clr, hipStream_t s)
{
    if (n == 0) return BNN_OK;
    const int ho_ = h + 2 * pad - kh + 1, wo_ = w + 2 * pad - kw + 1;
    const int pool_ = ep.packed ? ep.pool : 1;
    // int8 GEMM straight from global memory
    if (kh == 1 && kw == 1 && pad == 0 && (c_in & 15) == 0 && pool_ == 1) {
        const int64_t M = (int64_t)n * h * w;
        const int64_t blocks = ceil_div64(M, 64) * ceil_div64(c_out, 64);
        if (blocks < 192) {
            const int nbn = (c_out + 31) / 32;
            const unsigned grid = (unsigned)(ceil_div64(M, 32) * nbn);
            hipLaunchKernelGGL(fc_first_small, dim3(grid), dim3(256), 0, s, in, wt, M, c_out, c_in, nbn, ep, clr);
            return hip_result(hipGetLastError());
        }
        if (blocks <= 0x7fffffffLL) {
            hipLaunchKernelGGL(fc_first_mfma, dim3((unsigned)blocks), dim3(256), 0, s, in, wt, M, c_out, c_in, ep, clr);
            return hip_result(hipGetLastError());
        }
    }
    // a few thousand pixels: one wave per 32 x 32 outputs, nothing staged
    {
        const bnn_status st = launch_first_small(in, wt, n, h, w, c_in, c_out, kh, kw, pad, pad_value, ep, clr, s);
        if (st != BNN_ERR_UNSUPPORTED) return st;
    }
    // 3x3 over small images: whole images in LDS
    if (kh == 3 && kw == 3 && pad == 1 && c_in <= 4 && (int64_t)n * h * w * c_in < 0x7fffffff00LL) {
        const TileShape ts = make_tile_shape(ho_, wo_, 256);
        const int64_t ptiles = (int64_t)ts.tiles_x * ts.tiles_y * ((n + ts.ni - 1) / ts.ni);
        const bool two_groups = c_out > 64 && ptiles * ((c_out + 127) / 128) >= 256;
        const bnn_status st = two_groups ? launch_first_img<2>(in, wt, n, h, w, c_in, c_out, pad_value, ep, clr, s)
                                         : launch_first_img<1>(in, wt, n, h, w, c_in, c_out, pad_value, ep, clr, s);
        if (st != BNN_ERR_UNSUPPORTED) return st;
    }
    // small kernels: patch + weights in LDS, matrix cores
    {
        FirstGeomM g;
        g.n = n; g.h = h; g.w = w; g.c_in = c_in; g.c_out = c_out;
        g.kh = kh; g.kw = kw; g.pad = pad; g.pad_value = pad_value;
        g.ho = ho_; g.wo = wo_;
        g.sl = kw * c_in;
        g.slp = (g.sl + 15) & ~15;
        g.kp = (kh * g.slp + 31) & ~31;
        const TileShape ts = make_tile_shape(ho_, wo_, 256);
        g.lth = ts.lth; g.ltw = ts.ltw; g.ni = ts.ni; g.tiles_x = ts.tiles_x; g.tiles_y = ts.tiles_y;
        const int64_t pbytes = (int64_t)g.ni * ((1 << g.lth) + kh - 1) * ((1 << g.ltw) + kw - 1) * c_in;
        g.patch_bytes = (int)((pbytes + 32 + 15) & ~15LL);       // slack: reads run past short rows
        auto magic = [](int d) { return d == 1 ? 0u : (unsigned)((0x100000000ULL + d - 1) / d); };
        g.mg_cin = magic(c_in);
        g.mg_pw = magic((1 << g.ltw) + kw - 1);
        g.mg_ph = magic((1 << g.lth) + kh - 1);
        g.mg_kh = magic(kh);
        // (the weight tensor is addressed with 32-bit byte offsets)
        if (g.kp <= 128 && pbytes <= 24 * 1024 && (int64_t)c_out * kh * g.sl < 0x7fffffffLL) {
            // two channel groups per block amortise the patch; with too few pixel tiles to fill
            // the chip (small batches) one group per block doubles the blocks instead
            const int64_t ptiles = (int64_t)g.tiles_x * g.tiles_y * ((n + g.ni - 1) / g.ni);
            const bool two_groups = c_out > 64 && ptiles * ((c_out + 127) / 128) >= 256;
            const bnn_status st = two_groups ? launch_first_mfma<2>(in, wt, g, ep, clr, s)
                                             : launch_first_mfma<1>(in, wt, g, ep, clr, s);
            if (st != BNN_ERR_UNSUPPORTED) return st;
        }
    }
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
    hipLaunchKernelGGL(conv_first_kernel, dim3((unsigned)bx, (unsigned)by), dim3(256), 0, s, in, wt, g, ep, clr);
    return hip_result(hipGetLastError());
}

}  // namespace bnn

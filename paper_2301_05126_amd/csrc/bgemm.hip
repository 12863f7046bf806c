// Binary fully-connected layer / binary GEMM for gfx950.
//
// C[r][o] = sum_t a[r][t] * b[o][t] over +-1 values stored one bit each
//         = 2*popcount(xnor) - #bits  (paper Sec. II-A neuron formula).
//
// Dense tiles run on the matrix cores: each 32-bit word of packed operand bits is expanded
// in registers into 32 FP4 (E2M1) values +-1.0 and fed to
// v_mfma_f32_32x32x64_f8f6f4 (the form without block scales).  Products are +-1 and partial sums are
// integers below 2^24, so the FP32 accumulators are exact.  Both operands use the same
// bit -> sign map (bit 1 -> -1.0) and the same permutation of K inside a word, neither of
// which changes a dot product.  Zero-filled words beyond K (and the zero tail bits of the
// last word) count as matches, a constant that the epilogue subtracts.
//
//   bgemm_mfma<TM,TN>  block = 2x2 waves, wave tile (32*TM) x (32*TN), K streamed through
//                      LDS as packed words in chunks of 16 .. 64 words.
//   bgemm_small        few 64 x 64 tiles: 32 x 32 outputs per block, K split over its four waves,
//                      operands straight from global memory.
//   bgemv_rows         m <= 8: bandwidth-bound, xor + popcount on the VALU, four output rows of
//                      B per wave, halving-butterfly reduction over the 64 lanes.
// All end in the same epilogue: optional int32 store, optional threshold/flip/bit-pack.  The two
// small-problem kernels can also carry the model's last layer (TAIL): each block adds the share
// of its 32-bit output words to the logits.
#include "bnn_internal.h"

namespace bnn {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// Packed k-words per LDS chunk: small tiles take long chunks (fewer barriers per MFMA, their
// launches are latency-bound), the 256 x 256 tile short ones (registers).
constexpr int chunk_words(int tm, int tn) { return tm * tn >= 16 ? 16 : (tm * tn >= 4 ? 32 : 64); }


template <int VEC>
__device__ __forceinline__ uint4 load_row_words(const uint32_t *__restrict__ base, int64_t row,
                                                int64_t rows, int kw_total, int kpos)
{
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (row < rows) {
        const uint32_t *p = base + row * (int64_t)kw_total + kpos;
        if (VEC == 4) {
            if (kpos < kw_total) v = *reinterpret_cast<const uint4 *>(p);
        } else if (VEC == 2) {
            if (kpos < kw_total) { uint2 t = *reinterpret_cast<const uint2 *>(p); v.x = t.x; v.y = t.y; }
            if (kpos + 2 < kw_total) { uint2 t = *reinterpret_cast<const uint2 *>(p + 2); v.z = t.x; v.w = t.y; }
        } else {
            if (kpos < kw_total) v.x = p[0];
            if (kpos + 1 < kw_total) v.y = p[1];
            if (kpos + 2 < kw_total) v.z = p[2];
            if (kpos + 3 < kw_total) v.w = p[3];
        }
    }
    return v;
}

// The same four words without branches, so that many such loads can be in flight together: a
// word that does not exist reads the tensor's first word and is zeroed afterwards.
template <int VEC>
__device__ __forceinline__ uint4 load_row_words_nb(const uint32_t *__restrict__ base, int64_t row,
                                                   int64_t rows, int kw_total, int kpos)
{
    const bool row_ok = row < rows;
    const int64_t at = row * (int64_t)kw_total + kpos;
    uint4 v;
    if (VEC == 4) {
        const bool ok = row_ok && kpos < kw_total;
        v = *reinterpret_cast<const uint4 *>(base + (ok ? at : 0));
        v.x = ok ? v.x : 0u; v.y = ok ? v.y : 0u; v.z = ok ? v.z : 0u; v.w = ok ? v.w : 0u;
    } else if (VEC == 2) {
        const bool ok0 = row_ok && kpos < kw_total, ok1 = row_ok && kpos + 2 < kw_total;
        const uint2 lo = *reinterpret_cast<const uint2 *>(base + (ok0 ? at : 0));
        const uint2 hi = *reinterpret_cast<const uint2 *>(base + (ok1 ? at + 2 : 0));
        v = make_uint4(ok0 ? lo.x : 0u, ok0 ? lo.y : 0u, ok1 ? hi.x : 0u, ok1 ? hi.y : 0u);
    } else {
        uint32_t w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool ok = row_ok && kpos + q < kw_total;
            const uint32_t x = base[ok ? at + q : 0];
            w[q] = ok ? x : 0u;
        }
        v = make_uint4(w[0], w[1], w[2], w[3]);
    }
    return v;
}

// 32 packed bits -> 32 FP4 values in the low four dwords of an MFMA operand.
// FP4 E2M1: 0b0010 = +1.0, 0b1010 = -1.0; bit b of the word lands in nibble b/4 of dword 3 - b%4.
// sgn / one hold 0x88888888 / 0x22222222 in registers so that each dword is one v_and_or_b32.
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

__device__ __forceinline__ uint32_t word_of(const uint4 &v, int q)
{
    return q == 0 ? v.x : (q == 1 ? v.y : (q == 2 ? v.z : v.w));
}

// Where a block's tile lies and when the block starts.
struct GemmWalk {
    int nbm, nbn;            // tiles along M and N
    unsigned stagger_ticks;  // start delays of the first 256 blocks are spread over this many 100 MHz ticks
};

// One block per tile.  Tile numbers run column-major inside bands of eight tile rows, and the
// blocks that hardware deals to one XCD (ids equal modulo 8) take neighbouring numbers, so the
// tiles in flight on one L2 form a patch that shares rows of A and of B.
template <int TM, int TN, int VEC>
__global__ __launch_bounds__(256, 1) void bgemm_mfma(const uint32_t *__restrict__ A,
                                                      const uint32_t *__restrict__ B, int64_t M, int64_t N,
                                                      int Kw, int K, GemmWalk gw, EpiArgs ep)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;     // 2 x 2 waves
    constexpr int KC = chunk_words(TM, TN);
    constexpr int LS = KC + 4;    // LDS row stride in words; LS/4 odd -> 16-byte reads of
                                  // consecutive rows fall into distinct bank groups
    constexpr int UPR = KC / 4, SA = BM * UPR / 256, SB = BN * UPR / 256;   // staging units
    constexpr int NG = KC / 8, NST = KC / 2;      // 8-word groups and MFMA steps per chunk
    __shared__ __align__(16) uint32_t As[BM * LS];
    __shared__ __align__(16) uint32_t Bs[BN * LS];

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, half = lane >> 5;

    const int nblk = (int)gridDim.x;
    int tile = (int)blockIdx.x;
    if ((nblk & 7) == 0) tile = (int)(blockIdx.x & 7) * (nblk >> 3) + (int)(blockIdx.x >> 3);
    int64_t m0, n0;
    {
        const int band = tile / (8 * gw.nbn);
        const int rows_in_band = min(8, gw.nbm - band * 8);
        const int idx = tile - band * 8 * gw.nbn;
        const int nb = idx / rows_in_band;
        m0 = (int64_t)(band * 8 + (idx - nb * rows_in_band)) * BM;
        n0 = (int64_t)nb * BN;
    }

    // staging: a chunk of a tile is (rows x UPR) 16-byte units; SA units of A, SB of B per thread
    uint4 pa[SA], pb[SB];
    auto prefetch = [&](int k0) {
#pragma unroll
        for (int r = 0; r < SA; ++r) {
            const int idx = t + 256 * r;
            pa[r] = load_row_words<VEC>(A, m0 + idx / UPR, M, Kw, k0 + (idx % UPR) * 4);
        }
#pragma unroll
        for (int r = 0; r < SB; ++r) {
            const int idx = t + 256 * r;
            pb[r] = load_row_words<VEC>(B, n0 + idx / UPR, N, Kw, k0 + (idx % UPR) * 4);
        }
    };
    prefetch(0);

    // Several rounds of 256 x 256 tiles (one block per compute unit at a time): the first round's
    // blocks start spread over a few microseconds.  Every later block starts when a compute unit
    // falls free, so tiles keep ending at different times on different compute units for the whole
    // run, and the tiles' stores (256 KB each) do not all meet in the memory system at once.
    // (Bounded wait on the free-running 100 MHz counter.)
    if (gw.stagger_ticks && blockIdx.x < 256u) {
        const unsigned long long wait = (unsigned long long)blockIdx.x * gw.stagger_ticks / 256u;
        const long long t0 = wall_clock64();
        while ((unsigned long long)(wall_clock64() - t0) < wait) __builtin_amdgcn_s_sleep(16);
    }

    // VALU instructions to place behind each MFMA: 7 per expanded word, (TM+TN) words per step
    constexpr int VPM = (7 * (TM + TN) + TM * TN - 1) / (TM * TN);
    uint32_t sgn = 0x88888888u, one = 0x22222222u;
    asm volatile("" : "+s"(sgn));     // keep both masks in registers (v_and_or_b32 takes no literals)
    asm volatile("" : "+v"(one));

    const int nchunks = (Kw + KC - 1) / KC;
    const int corr = nchunks * KC * 32 - K;      // padded positions all counted as +1
    const uint32_t *a_rd = As + (wm * TM * 32 + l32) * LS + half * 4;
    const uint32_t *b_rd = Bs + (wn * TN * 32 + l32) * LS + half * 4;

    {
        v16f acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        for (int kc = 0; kc < nchunks; ++kc) {
            __syncthreads();
#pragma unroll
            for (int r = 0; r < SA; ++r) {
                const int idx = t + 256 * r;
                *reinterpret_cast<uint4 *>(As + (idx / UPR) * LS + (idx % UPR) * 4) = pa[r];
            }
#pragma unroll
            for (int r = 0; r < SB; ++r) {
                const int idx = t + 256 * r;
                *reinterpret_cast<uint4 *>(Bs + (idx / UPR) * LS + (idx % UPR) * 4) = pb[r];
            }
            __syncthreads();
            if (kc + 1 < nchunks) prefetch((kc + 1) * KC);

            // a chunk = NG groups of 8 words; lane half h owns words [8g + 4h, 8g + 4h + 4).
            // Operands of step s+1 are expanded on the VALU while the matrix core runs step s.
            uint4 wa[NG][TM], wb[NG][TN];
#pragma unroll
            for (int g = 0; g < NG; ++g) {
#pragma unroll
                for (int i = 0; i < TM; ++i) wa[g][i] = *reinterpret_cast<const uint4 *>(a_rd + i * 32 * LS + g * 8);
#pragma unroll
                for (int j = 0; j < TN; ++j) wb[g][j] = *reinterpret_cast<const uint4 *>(b_rd + j * 32 * LS + g * 8);
            }
            v8i a[2][TM], b[2][TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[0][i] = expand_fp4(wa[0][i].x, sgn, one);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[0][j] = expand_fp4(wb[0][j].x, sgn, one);
#pragma unroll
            for (int st = 0; st < NST; ++st) {
                const int cur = st & 1, nxt = cur ^ 1;
                if (st + 1 < NST) {
                    const int g = (st + 1) >> 2, q = (st + 1) & 3;
#pragma unroll
                    for (int i = 0; i < TM; ++i) a[nxt][i] = expand_fp4(word_of(wa[g][i], q), sgn, one);
#pragma unroll
                    for (int j = 0; j < TN; ++j) b[nxt][j] = expand_fp4(word_of(wb[g][j], q), sgn, one);
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                            a[cur][i], b[cur][j], acc[i][j], 4, 4, 0, 0, 0, 0);
                // interleave: one MFMA, then its share of the next step's VALU work
#pragma unroll
                for (int k = 0; k < TM * TN; ++k) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, VPM, 0);
                }
            }
        }

        // ---- epilogue.  Accumulator register r of lane (l32, half) in tile (i, j) is
        // row 32i + 8(r/4) + 4*half + r%4, column 32j + l32.
        const int64_t rbase = m0 + wm * TM * 32 + half * 4;
        const int64_t cbase = n0 + wn * TN * 32 + l32;
        if (ep.preact) {
            if (TM * TN >= 16 && m0 + BM <= M && n0 + BN <= N && (int64_t)(BM - 1) * N + BN <= 0x1fffffffLL) {
                // A whole tile inside C: the stores go through a buffer resource over the tile's
                // part of C, so that a store is one conversion and one instruction -- the lane's part
                // of the address is fixed, the row of a register is a scalar offset, the column tile
                // an immediate.  Streaming stores: C is not read again by this kernel.
                const __amdgpu_buffer_rsrc_t crs = __builtin_amdgcn_make_buffer_rsrc(
                    ep.preact + (m0 * N + n0), 0, (int)(((int64_t)(BM - 1) * N + BN) * 4), 0x00020000);
                const unsigned row_bytes = (unsigned)N * 4u;
                const unsigned c_voff = (unsigned)(((wm * TM * 32 + half * 4) * (unsigned)N + wn * TN * 32 + l32) * 4u);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const unsigned soff = (unsigned)(i * 32 + (r >> 2) * 8 + (r & 3)) * row_bytes;
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            __builtin_amdgcn_raw_buffer_store_b32((int)acc[i][j][r] - corr, crs, c_voff + j * 128, soff,
                                                                  2 /* nontemporal */);
                    }
            } else {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const int64_t col = cbase + j * 32;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int64_t row = rbase + i * 32 + (r >> 2) * 8 + (r & 3);
                            if (row < M && col < N) ep.preact[row * N + col] = (int)acc[i][j][r] - corr;
                        }
                    }
            }
        }
        if (ep.packed) {
            // A ballot over the 32 columns of a tile is the packed word of one row (one per lane
            // half).  Lane r of each half keeps the word of register r, so that a tile's 32 words
            // leave with one store instruction per row block instead of one per word.
            const int64_t nw = (N + 31) >> 5;
            int thr[TN];
            bool flip[TN], cok[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t col = cbase + j * 32;
                cok[j] = col < N;
                thr[j] = cok[j] ? ep.thr[col] : 0;
                flip[j] = cok[j] && ep.flip && ep.flip[col];
            }
            const int64_t wi0 = (n0 + wn * TN * 32) >> 5;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                unsigned mine[TN];
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    mine[j] = 0;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int x = (int)acc[i][j][r] - corr;
                        const bool bit = cok[j] && ((x > thr[j]) != flip[j]);
                        const unsigned long long mask = __ballot(bit);
                        const unsigned word = half ? (unsigned)(mask >> 32) : (unsigned)mask;
                        if (l32 == r) mine[j] = word;
                    }
                }
                const int64_t row = rbase + i * 32 + (l32 >> 2) * 8 + (l32 & 3);
                if (l32 < 16 && row < M) {
                    uint32_t *dst = ep.packed + row * nw + wi0;
                    if (TN == 2 && (nw & 1) == 0 && wi0 + 1 < nw) {
                        *reinterpret_cast<uint2 *>(dst) = make_uint2(mine[0], mine[TN - 1]);
                    } else if (TN == 4 && (nw & 3) == 0 && wi0 + 3 < nw) {
                        *reinterpret_cast<uint4 *>(dst) = make_uint4(mine[0], mine[1 % TN], mine[2 % TN], mine[3 % TN]);
                    } else {
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            if (wi0 + j < nw) dst[j] = mine[j];
                    }
                }
            }
        }
    }
}

// Small dense problems (the 64 x 64 tiling would leave most compute units idle): a block owns
// 32 x 32 outputs and its four waves split K in units of four MFMA steps (eight packed words per
// row; lane half h owns words [8u + 4h, 8u + 4h + 4) of unit u, one 16-byte load per operand, lane
// and unit).  Wave v takes the units v, v + 4, ... in rounds of up to eight units with all loads
// of a round in flight together, straight from global memory (no staging, no barrier before the
// MFMAs); the partial sums meet in LDS and wave 0 runs the epilogue.  Latency, not throughput:
// with a quarter of K per wave and four times the blocks, a batch-256 FC layer of K = 8192 takes
// half the time of the 64 x 64 tile.
//
// TAIL (see bgemv_rows): the block's 32 output words, one per row, each give their share of at
// most 16 logits per row; thread t adds those of row t % 32 and classes t / 32 and t / 32 + 8.
template <int VEC, bool TAIL>
__global__ __launch_bounds__(256) void bgemm_small(const uint32_t *__restrict__ A, const uint32_t *__restrict__ B,
                                                   int64_t M, int64_t N, int Kw, int K, int nbn, EpiArgs ep,
                                                   FcTailArgs tail)
{
    constexpr int UR = 8;                   // units per wave and round
    __shared__ float red[3][16][64];        // partial sums of waves 1..3
    __shared__ uint32_t out_word[32];
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int64_t m0 = (int64_t)(blockIdx.x / nbn) * 32;
    const int64_t n0 = (int64_t)(blockIdx.x % nbn) * 32;
    const int units = (Kw + 7) >> 3;

    uint32_t w_tail[2] = {0u, 0u};          // on their way while the dot products run
    if (TAIL) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int j = (t >> 5) + 8 * i;
            if (j < tail.n_out) w_tail[i] = tail.w[(int64_t)j * ((N + 31) >> 5) + (n0 >> 5)];
        }
    }

    uint32_t sgn = 0x88888888u, one = 0x22222222u;
    asm volatile("" : "+s"(sgn));
    asm volatile("" : "+v"(one));
    v16f acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    for (int u0 = wave; u0 < units; u0 += 4 * UR) {
        uint4 wa[UR], wb[UR];
#pragma unroll
        for (int k = 0; k < UR; ++k) {
            const int u = u0 + 4 * k;
            // (a unit or a row past the end gives zeros)
            wa[k] = load_row_words_nb<VEC>(A, m0 + l32, M, Kw, u * 8 + half * 4);
            wb[k] = load_row_words_nb<VEC>(B, n0 + l32, N, Kw, u * 8 + half * 4);
        }
#pragma unroll
        for (int k = 0; k < UR; ++k) {
            if (u0 + 4 * k < units) {       // uniform per wave
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        expand_fp4(word_of(wa[k], q), sgn, one), expand_fp4(word_of(wb[k], q), sgn, one), acc, 4, 4,
                        0, 0, 0, 0);
            }
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wave - 1][r][lane] = acc[r];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
#pragma unroll
            for (int v = 0; v < 3; ++v) acc[r] += red[v][r][lane];      // small integers: exact in any order

        // ---- epilogue of one 32 x 32 tile: register r of lane (l32, half) is row 8(r/4) + 4*half + r%4, column l32
        const int corr = units * 8 * 32 - K;        // zero words and tail bits all counted as +1
        const int64_t rbase = m0 + half * 4, col = n0 + l32;
        const bool cok = col < N;
        if (ep.preact) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = rbase + (r >> 2) * 8 + (r & 3);
                if (row < M && cok) ep.preact[row * N + col] = (int)acc[r] - corr;
            }
        }
        if (ep.packed) {
            const int64_t nw = (N + 31) >> 5;
            const int thr = cok ? ep.thr[col] : 0;
            const bool flip = cok && ep.flip && ep.flip[col];
            unsigned mine = 0;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int x = (int)acc[r] - corr;
                const unsigned long long mask = __ballot(cok && ((x > thr) != flip));
                const unsigned word = half ? (unsigned)(mask >> 32) : (unsigned)mask;
                if (l32 == r) mine = word;          // lane r of each half keeps the word of register r
            }
            const int64_t row = rbase + (l32 >> 2) * 8 + (l32 & 3);
            if (l32 < 16 && row < M) ep.packed[row * nw + (n0 >> 5)] = mine;
            if (TAIL && l32 < 16) out_word[half * 4 + (l32 >> 2) * 8 + (l32 & 3)] = mine;
        }
    }
    if (TAIL) {
        __syncthreads();
        const int r = t & 31;
        const int64_t left = N - n0;                        // output bits the block's words hold
        const int valid = left < 32 ? (int)left : 32;
        const uint32_t mask = valid < 32 ? ((1u << valid) - 1u) : 0xffffffffu;
        const uint32_t wd = out_word[r];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int j = (t >> 5) + 8 * i;
            if (j < tail.n_out && m0 + r < M)
                atomicAdd(&tail.logits[(m0 + r) * tail.n_out + j],
                          valid - 2 * __builtin_popcount((wd ^ w_tail[i]) & mask));
        }
    }
}

// m <= MT rows of A (batch 1 .. 8): bandwidth / latency bound, on the VALU.
// Block = 8 waves = 32 consecutive outputs (one packed word); wave w owns outputs 4w..4w+3
// and streams their B rows with all loads of a K slice in flight at once.  Lanes stride K
// (16 bytes per lane when VEC == 4), accumulate popcount(a ^ b), then a halving butterfly
// reduces the 4 partial sums per lane over the 64 lanes with 2 + 1 + 4 shuffles per row.
//
// TAIL: the layer after this one is the model's last, which has no step and is therefore linear
// in this layer's output bits.  A block holds one whole 32-bit word of every output row, so it
// adds that word's share of each logit, valid - 2 popcount((word ^ w) & mask), to the logits with
// integer atomics (exact and independent of the order of arrival); the logits must be zero when
// the launch starts.  One thread per (row, logit): M * n_out <= 512.
template <int MT, int VEC, bool TAIL>
__global__ __launch_bounds__(512) void bgemv_rows(const uint32_t *__restrict__ A,
                                                  const uint32_t *__restrict__ B, int M, int64_t N, int Kw,
                                                  int K, EpiArgs ep, FcTailArgs tail)
{
    __shared__ int xs[MT][32];
    __shared__ uint32_t out_word[MT];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t o_base = (int64_t)blockIdx.x * 32;

    // this thread's word of the last layer's weights, on its way while the dot products run
    uint32_t w_tail = 0;
    int tail_r = 0, tail_j = 0;
    const bool tail_on = TAIL && (int)threadIdx.x < M * tail.n_out;
    if (tail_on) {
        tail_r = (int)threadIdx.x / tail.n_out;
        tail_j = (int)threadIdx.x - tail_r * tail.n_out;
        w_tail = tail.w[(int64_t)tail_j * ((N + 31) >> 5) + blockIdx.x];
    }

    int acc[MT][4];
#pragma unroll
    for (int r = 0; r < MT; ++r)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[r][q] = 0;

    const uint32_t *brow[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t o = o_base + wave * 4 + q;
        brow[q] = B + (o < N ? o : N - 1) * (int64_t)Kw;      // rows past N are computed, never stored
    }
    if (VEC == 4) {
        for (int kb = lane * 4; kb < Kw; kb += 256) {
            uint4 b[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) b[q] = *reinterpret_cast<const uint4 *>(brow[q] + kb);
#pragma unroll
            for (int r = 0; r < MT; ++r) {
                if (r < M) {
                    const uint4 a = *reinterpret_cast<const uint4 *>(A + (int64_t)r * Kw + kb);
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        acc[r][q] += __builtin_popcount(a.x ^ b[q].x) + __builtin_popcount(a.y ^ b[q].y) +
                                     __builtin_popcount(a.z ^ b[q].z) + __builtin_popcount(a.w ^ b[q].w);
                }
            }
        }
    } else {
        for (int kb = lane; kb < Kw; kb += 64) {
            uint32_t b[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) b[q] = brow[q][kb];
#pragma unroll
            for (int r = 0; r < MT; ++r) {
                if (r < M) {
                    const uint32_t a = A[(int64_t)r * Kw + kb];
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc[r][q] += __builtin_popcount(a ^ b[q]);
                }
            }
        }
    }

    // halving butterfly: after the exchanges with lane^32 and lane^16 a lane keeps the sum of
    // output q = 2*bit5 + bit4; the remaining four exchanges finish the sum over 16 lanes.
#pragma unroll
    for (int r = 0; r < MT; ++r) {
        if (r >= M) break;
        const bool hi5 = (lane & 32) != 0, hi4 = (lane & 16) != 0;
        const int s0 = hi5 ? acc[r][0] : acc[r][2], s1 = hi5 ? acc[r][1] : acc[r][3];   // what the partner keeps
        const int k0 = hi5 ? acc[r][2] : acc[r][0], k1 = hi5 ? acc[r][3] : acc[r][1];   // what this lane keeps
        const int t0 = k0 + __shfl_xor(s0, 32), t1 = k1 + __shfl_xor(s1, 32);
        int v = (hi4 ? t1 : t0) + __shfl_xor(hi4 ? t0 : t1, 16);
        v += __shfl_xor(v, 8);
        v += __shfl_xor(v, 4);
        v += __shfl_xor(v, 2);
        v += __shfl_xor(v, 1);
        if ((lane & 15) == 0) xs[r][wave * 4 + (lane >> 4)] = K - 2 * v;
    }
    __syncthreads();

    const int tid = threadIdx.x;
    if (tid < 256) {                // 8 rows x 32 outputs; waves 0..3 are entirely inside
        const int r = tid >> 5;
        const int ol = tid & 31;
        const int64_t o = o_base + ol;
        const bool ok = (r < MT) && (r < M) && (o < N);
        const int x = ok ? xs[r < MT ? r : 0][ol] : 0;
        if (ep.preact && ok) ep.preact[(int64_t)r * N + o] = x;
        if (ep.packed) {
            bool bit = false;
            if (ok) {
                bit = x > ep.thr[o];
                if (ep.flip && ep.flip[o]) bit = !bit;
            }
            const unsigned long long mask = __ballot(bit);   // lanes 0-31: row r, 32-63: row r+1
            const unsigned word = (lane < 32) ? (unsigned)(mask & 0xffffffffull) : (unsigned)(mask >> 32);
            const int64_t nw = (N + 31) >> 5;
            if (ol == 0 && r < M && r < MT) {
                ep.packed[(int64_t)r * nw + blockIdx.x] = word;
                if (TAIL) out_word[r] = word;
            }
        }
    }
    if (TAIL) {
        __syncthreads();
        if (tail_on) {
            const int64_t left = N - o_base;                 // output bits this block's word holds
            const int valid = left < 32 ? (int)left : 32;
            const uint32_t mask = valid < 32 ? ((1u << valid) - 1u) : 0xffffffffu;
            const int part = valid - 2 * __builtin_popcount((out_word[tail_r] ^ w_tail) & mask);
            atomicAdd(&tail.logits[(int64_t)tail_r * tail.n_out + tail_j], part);
        }
    }
}

template <int TM, int TN>
bnn_status launch_mfma(const uint32_t *a, int64_t m, int64_t k, const uint32_t *b, int64_t n, int kw,
                       const EpiArgs &ep, hipStream_t s)
{
    GemmWalk gw;
    const int64_t nbm = ceil_div64(m, 64 * TM), nbn = ceil_div64(n, 64 * TN);
    const int64_t blocks = nbm * nbn;
    if (blocks > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
    gw.nbm = (int)nbm; gw.nbn = (int)nbn;
    // two or more rounds of the 256 x 256 tile: the first round starts spread over 10 us
    gw.stagger_ticks = (TM * TN >= 16 && blocks >= 512) ? 1000 : 0;
    dim3 grid((unsigned)blocks);
    if ((kw & 3) == 0)
        hipLaunchKernelGGL((bgemm_mfma<TM, TN, 4>), grid, dim3(256), 0, s, a, b, m, n, kw, (int)k, gw, ep);
    else if ((kw & 1) == 0)
        hipLaunchKernelGGL((bgemm_mfma<TM, TN, 2>), grid, dim3(256), 0, s, a, b, m, n, kw, (int)k, gw, ep);
    else
        hipLaunchKernelGGL((bgemm_mfma<TM, TN, 1>), grid, dim3(256), 0, s, a, b, m, n, kw, (int)k, gw, ep);
    return hip_result(hipGetLastError());
}

// more than 8 rows, too few tiles for any of the three block tiles
bool fc_takes_small_kernel(int64_t m, int64_t n)
{
    return m > 8 && ceil_div64(m, 64) * ceil_div64(n, 64) < 192;
}

template <bool TAIL>
bnn_status launch_small(const uint32_t *a, int64_t m, int64_t k, const uint32_t *b, int64_t n, int kw,
                        const EpiArgs &ep, const FcTailArgs &tail, hipStream_t s)
{
    const int nbn = (int)ceil_div64(n, 32);
    const dim3 grid((unsigned)(nbn * ceil_div64(m, 32)));
    if ((kw & 3) == 0)
        hipLaunchKernelGGL((bgemm_small<4, TAIL>), grid, dim3(256), 0, s, a, b, m, n, kw, (int)k, nbn, ep, tail);
    else if ((kw & 1) == 0)
        hipLaunchKernelGGL((bgemm_small<2, TAIL>), grid, dim3(256), 0, s, a, b, m, n, kw, (int)k, nbn, ep, tail);
    else
        hipLaunchKernelGGL((bgemm_small<1, TAIL>), grid, dim3(256), 0, s, a, b, m, n, kw, (int)k, nbn, ep, tail);
    return hip_result(hipGetLastError());
}

// m <= 8 rows; the kernel is instantiated for 1, 2, 4 and 8 rows (a batch-1 launch is bound by its
// own instruction count, and the 8-row code is four times as long).
template <bool TAIL>
bnn_status launch_gemv(const uint32_t *a, int64_t m, int64_t k, const uint32_t *b, int64_t n, int kw,
                       const EpiArgs &ep, const FcTailArgs &tail, hipStream_t s)
{
    const dim3 grid((unsigned)ceil_div64(n, 32));
    const bool v4 = (kw & 3) == 0;
#define BNN_GEMV(MT)                                                                                          \
    do {                                                                                                      \
        if (v4)                                                                                               \
            hipLaunchKernelGGL((bgemv_rows<MT, 4, TAIL>), grid, dim3(512), 0, s, a, b, (int)m, n, kw, (int)k, ep, tail); \
        else                                                                                                  \
            hipLaunchKernelGGL((bgemv_rows<MT, 1, TAIL>), grid, dim3(512), 0, s, a, b, (int)m, n, kw, (int)k, ep, tail); \
    } while (0)
    if (m == 1) BNN_GEMV(1);
    else if (m == 2) BNN_GEMV(2);
    else if (m <= 4) BNN_GEMV(4);
    else BNN_GEMV(8);
#undef BNN_GEMV
    return hip_result(hipGetLastError());
}

}  // namespace

bnn_status launch_fc_binary(const uint32_t *a, int64_t m, int64_t k, const uint32_t *b, int64_t n,
                            const EpiArgs &ep, hipStream_t s)
{
    if (m == 0) return BNN_OK;
    const int kw = (int)((k + 31) / 32);
    if (m <= 8) {
        const FcTailArgs none = {nullptr, nullptr, 0};
        return launch_gemv<false>(a, m, k, b, n, kw, ep, none, s);
    }
    // largest tile that still fills most of the 256 compute units
    const int64_t want = 192;
    if (ceil_div64(m, 256) * ceil_div64(n, 256) >= want) return launch_mfma<4, 4>(a, m, k, b, n, kw, ep, s);
    if (ceil_div64(m, 128) * ceil_div64(n, 128) >= want) return launch_mfma<2, 2>(a, m, k, b, n, kw, ep, s);
    // fewer than that many 64 x 64 tiles: 32 x 32 tiles with K split over the block's waves
    if (fc_takes_small_kernel(m, n)) {
        const FcTailArgs none = {nullptr, nullptr, 0};
        return launch_small<false>(a, m, k, b, n, kw, ep, none, s);
    }
    return launch_mfma<1, 1>(a, m, k, b, n, kw, ep, s);
}

bool fc_binary_tail_qualifies(int64_t m, int64_t n, int64_t n_out)
{
    if (m < 1 || n_out < 1) return false;
    // Every logit receives one atomic per 32 outputs of this layer, and additions to one address
    // queue up behind each other: beyond these widths (measured: hidden layers of 512 .. 32768
    // outputs, with and without the tail) a launch of its own for the last layer is faster.
    if (m <= 8) return m * n_out <= 512 && n <= 8192;       // bgemv_rows: one thread per (row, class)
    return fc_takes_small_kernel(m, n) && n_out <= 16 &&    // bgemm_small: two classes per thread
           n <= 1024 && m * n_out <= FC_TAIL_MAX_LOGITS;
}

bnn_status launch_fc_binary_tail(const uint32_t *a, int64_t m, int64_t k, const uint32_t *b, int64_t n,
                                 const EpiArgs &ep, const FcTailArgs &tail, hipStream_t s)
{
    if (!fc_binary_tail_qualifies(m, n, tail.n_out) || !ep.packed || !tail.w || !tail.logits)
        return BNN_ERR_UNSUPPORTED;
    const int kw = (int)((k + 31) / 32);
    if (m > 8) return launch_small<true>(a, m, k, b, n, kw, ep, tail, s);
    return launch_gemv<true>(a, m, k, b, n, kw, ep, tail, s);
}

}  // namespace bnn

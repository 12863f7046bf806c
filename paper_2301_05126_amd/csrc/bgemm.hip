// Binary fully-connected layer / binary GEMM for gfx950.
//
// C[r][o] = K - 2 * sum_w popcount(A[r][w] ^ B[o][w])   (paper Sec. II-A neuron formula,
// 2*popcount(xnor) - #bits, rewritten with xor so that zero tail bits contribute nothing).
//
// Two kernels:
//   bgemm_tile   128x128 output tile per 256-thread block, 8x8 accumulators per lane,
//                K streamed through LDS in 32-word chunks; inner loop is
//                v_xor_b32 + v_bcnt_u32_b32 (the popcount instruction adds its accumulator).
//   bgemv_rows   for m <= 8: one block per 32 outputs, each wave streams whole B rows and
//                reduces across its 64 lanes.
// Both end in the same epilogue: optional int32 store, optional threshold/flip/bit-pack.
#include "bnn_internal.h"

namespace bnn {

namespace {

constexpr int BM = 128;      // rows of A per block
constexpr int BN = 128;      // rows of B (outputs) per block
constexpr int KC = 32;       // k-words per LDS chunk
constexpr int KU = KC / 4;   // 16-byte units per LDS row

// 16-byte LDS unit of (row, c4): rows are 8 units long; the unit column is xor-swizzled
// with bits of row/8 so that the 8 (or 16) lanes that differ in row/8 hit distinct banks.
__device__ __forceinline__ int lds_unit(int row, int c4) { return row * KU + (c4 ^ ((row >> 3) & (KU - 1))); }

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

__device__ __forceinline__ int popc_xor4(const uint4 &a, const uint4 &b, int acc)
{
    acc += __builtin_popcount(a.x ^ b.x);
    acc += __builtin_popcount(a.y ^ b.y);
    acc += __builtin_popcount(a.z ^ b.z);
    acc += __builtin_popcount(a.w ^ b.w);
    return acc;
}

// Epilogue shared by the tile kernel: lane (tx, ty) owns rows r0..r0+7 and the 8
// contiguous outputs o0..o0+7; acc holds popcounts.  Four neighbouring lanes (tx & 3)
// own the four bytes of one packed output word.
__device__ __forceinline__ void tile_epilogue(const int (&acc)[8][8], int64_t r0, int64_t o0, int tx,
                                              int64_t M, int64_t N, int K, const EpiArgs &ep)
{
    if (ep.preact) {
        const bool vec_ok = ((N & 3) == 0) && (o0 + 8 <= N);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int64_t r = r0 + i;
            if (r >= M) continue;
            int32_t *dst = ep.preact + r * N + o0;
            if (vec_ok) {
                int4 v0 = make_int4(K - 2 * acc[i][0], K - 2 * acc[i][1], K - 2 * acc[i][2], K - 2 * acc[i][3]);
                int4 v1 = make_int4(K - 2 * acc[i][4], K - 2 * acc[i][5], K - 2 * acc[i][6], K - 2 * acc[i][7]);
                *reinterpret_cast<int4 *>(dst) = v0;
                *reinterpret_cast<int4 *>(dst + 4) = v1;
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (o0 + j < N) dst[j] = K - 2 * acc[i][j];
            }
        }
    }
    if (ep.packed) {
        int thr[8];
        unsigned flipmask = 0, valid = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool ok = (o0 + j) < N;
            thr[j] = ok ? ep.thr[o0 + j] : 0;
            if (ok) valid |= 1u << j;
            if (ok && ep.flip && ep.flip[o0 + j]) flipmask |= 1u << j;
        }
        const int64_t nw = (N + 31) >> 5;
        const int64_t word_idx = o0 >> 5;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            unsigned byte = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) byte |= ((K - 2 * acc[i][j]) > thr[j] ? 1u : 0u) << j;
            byte = (byte ^ flipmask) & valid;
            unsigned word = byte << (8 * (tx & 3));
            word |= __shfl_xor(word, 1);
            word |= __shfl_xor(word, 2);
            const int64_t r = r0 + i;
            if ((tx & 3) == 0 && r < M && word_idx < nw) ep.packed[r * nw + word_idx] = word;
        }
    }
}

template <int VEC>
__global__ __launch_bounds__(256, 2) void bgemm_tile(const uint32_t *__restrict__ A,
                                                      const uint32_t *__restrict__ B, int64_t M, int64_t N,
                                                      int Kw, int K, int nbn, EpiArgs ep)
{
    __shared__ uint4 As[BM * KU];
    __shared__ uint4 Bs[BN * KU];

    const int t = threadIdx.x;
    const int tx = t & 15;
    const int ty = t >> 4;
    // 1-D grid: consecutive blocks walk the output tiles of one row block of A
    const int64_t m0 = (int64_t)(blockIdx.x / nbn) * BM;
    const int64_t n0 = (int64_t)(blockIdx.x % nbn) * BN;

    int acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0;

    // staging assignment: 4 units of A and 4 of B per thread per chunk
    int srow[4], sc4[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int idx = t + 256 * r;
        srow[r] = idx >> 3;
        sc4[r] = idx & 7;
    }

    uint4 pa[4], pb[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        pa[r] = load_row_words<VEC>(A, m0 + srow[r], M, Kw, sc4[r] * 4);
        pb[r] = load_row_words<VEC>(B, n0 + srow[r], N, Kw, sc4[r] * 4);
    }

    const int nchunks = (Kw + KC - 1) / KC;
    for (int kc = 0; kc < nchunks; ++kc) {
        __syncthreads();   // previous chunk fully consumed
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            As[lds_unit(srow[r], sc4[r])] = pa[r];
            Bs[lds_unit(srow[r], sc4[r])] = pb[r];
        }
        __syncthreads();
        if (kc + 1 < nchunks) {
            const int k0 = (kc + 1) * KC;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                pa[r] = load_row_words<VEC>(A, m0 + srow[r], M, Kw, k0 + sc4[r] * 4);
                pb[r] = load_row_words<VEC>(B, n0 + srow[r], N, Kw, k0 + sc4[r] * 4);
            }
        }
#pragma unroll
        for (int c4 = 0; c4 < KU; ++c4) {
            uint4 a[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) a[i] = As[lds_unit(ty * 8 + i, c4)];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint4 b = Bs[lds_unit(tx * 8 + j, c4)];
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i][j] = popc_xor4(a[i], b, acc[i][j]);
            }
        }
    }

    tile_epilogue(acc, m0 + ty * 8, n0 + tx * 8, tx, M, N, K, ep);
}

// m <= MT rows of A.  Block = 4 waves, 32 consecutive outputs (one packed word); wave w
// takes outputs 8w..8w+7 one after another, lanes stride the K words, then a butterfly
// reduction over the 64 lanes.
template <int MT>
__global__ __launch_bounds__(256) void bgemv_rows(const uint32_t *__restrict__ A,
                                                  const uint32_t *__restrict__ B, int M, int64_t N, int Kw,
                                                  int K, EpiArgs ep)
{
    __shared__ int xs[MT][32];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t o_base = (int64_t)blockIdx.x * 32;

    for (int q = 0; q < 8; ++q) {
        const int ol = wave * 8 + q;
        const int64_t o = o_base + ol;
        int acc[MT];
#pragma unroll
        for (int r = 0; r < MT; ++r) acc[r] = 0;
        if (o < N) {
            const uint32_t *brow = B + o * (int64_t)Kw;
            for (int w = lane; w < Kw; w += 64) {
                const uint32_t b = brow[w];
#pragma unroll
                for (int r = 0; r < MT; ++r)
                    if (r < M) acc[r] += __builtin_popcount(A[(int64_t)r * Kw + w] ^ b);
            }
        }
#pragma unroll
        for (int r = 0; r < MT; ++r) {
            int v = acc[r];
#pragma unroll
            for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s);
            if (lane == 0) xs[r][ol] = K - 2 * v;
        }
    }
    __syncthreads();

    const int tid = threadIdx.x;
    const int r = tid >> 5;       // 8 rows x 32 outputs = 256 threads
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
        if (ol == 0 && r < M && r < MT) ep.packed[(int64_t)r * nw + blockIdx.x] = word;
    }
}

}  // namespace

bnn_status launch_fc_binary(const uint32_t *a, int64_t m, int64_t k, const uint32_t *b, int64_t n,
                            const EpiArgs &ep, hipStream_t s)
{
    if (m == 0) return BNN_OK;
    const int kw = (int)((k + 31) / 32);
    if (m <= 8) {
        dim3 grid((unsigned)ceil_div64(n, 32));
        hipLaunchKernelGGL(bgemv_rows<8>, grid, dim3(256), 0, s, a, b, (int)m, n, kw, (int)k, ep);
        return hip_result(hipGetLastError());
    }
    const int nbn = (int)ceil_div64(n, BN);
    dim3 grid((unsigned)(nbn * ceil_div64(m, BM)));
    if ((kw & 3) == 0)
        hipLaunchKernelGGL(bgemm_tile<4>, grid, dim3(256), 0, s, a, b, m, n, kw, (int)k, nbn, ep);
    else if ((kw & 1) == 0)
        hipLaunchKernelGGL(bgemm_tile<2>, grid, dim3(256), 0, s, a, b, m, n, kw, (int)k, nbn, ep);
    else
        hipLaunchKernelGGL(bgemm_tile<1>, grid, dim3(256), 0, s, a, b, m, n, kw, (int)k, nbn, ep);
    return hip_result(hipGetLastError());
}

}  // namespace bnn

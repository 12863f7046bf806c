// Binary 3x3 convolution (stride 1, pad 1 with -1) for gfx950, im2col-free.
//
// x[n,y,x,o] = K - 2 * sum_{tap, w} popcount(in[n, y+i-1, x+j-1, w] ^ W[o, tap, w]),  K = 9*c_in
// (paper Sec. II-A: convolutional layer of binarized neurons).  Out-of-image taps read
// zero words, i.e. -1 activations, so every output sums exactly K products.
//
// One 256-thread block computes 128 pixels x 128 output channels.  The 128 pixels are
// `ni` images x (th x tw) spatial tile; the input patch with its halo is staged once in LDS
// and all 9 taps are read from it with shifted addresses.  Weights stream through LDS in
// 32-word chunks of the [c_out][9*cw] matrix.  Each lane owns a 2x4 pixel patch x 8
// contiguous channels, so a 2x2 pool is an OR inside the lane and the 8 channel bits are
// one byte of the packed output word.
#include "bnn_internal.h"

namespace bnn {

namespace {

constexpr int BN = 128;          // output channels per block
constexpr int KC = 32;           // weight k-words per LDS chunk
constexpr int MAX_PATCH_BYTES = 48 * 1024;

struct ConvGeom {
    int n, h, w, cw;             // input: images, height, width, words per pixel
    int c_out, k_bits, kwt;      // outputs, K = 9*c_in, weight words per output = 9*cw
    int th, tw, ni;              // tile: th x tw pixels of ni images (th*tw*ni == 128)
    int tiles_x, tiles_y, n_co_tiles;
};

template <int V> struct WordVec;
template <> struct WordVec<4> { using type = uint4; };
template <> struct WordVec<2> { using type = uint2; };
template <> struct WordVec<1> { using type = uint32_t; };

__device__ __forceinline__ int popc_acc(uint4 a, uint4 b, int acc)
{
    acc += __builtin_popcount(a.x ^ b.x);
    acc += __builtin_popcount(a.y ^ b.y);
    acc += __builtin_popcount(a.z ^ b.z);
    acc += __builtin_popcount(a.w ^ b.w);
    return acc;
}
__device__ __forceinline__ int popc_acc(uint2 a, uint2 b, int acc)
{
    acc += __builtin_popcount(a.x ^ b.x);
    acc += __builtin_popcount(a.y ^ b.y);
    return acc;
}
__device__ __forceinline__ int popc_acc(uint32_t a, uint32_t b, int acc)
{
    return acc + __builtin_popcount(a ^ b);
}

template <int V> __device__ __forceinline__ typename WordVec<V>::type zero_vec();
template <> __device__ __forceinline__ uint4 zero_vec<4>() { return make_uint4(0, 0, 0, 0); }
template <> __device__ __forceinline__ uint2 zero_vec<2>() { return make_uint2(0, 0); }
template <> __device__ __forceinline__ uint32_t zero_vec<1>() { return 0u; }

// V = words per LDS/global access (4, 2 or 1); cw % V == 0.
template <int V>
__global__ __launch_bounds__(256, 2) void bconv3x3_tile(const uint32_t *__restrict__ in,
                                                         const uint32_t *__restrict__ wt, ConvGeom g,
                                                         EpiArgs ep)
{
    using vec_t = typename WordVec<V>::type;
    constexpr int UPR = KC / V;                       // units per weight row in a chunk
    extern __shared__ __align__(16) unsigned char smem[];
    vec_t *Bs = reinterpret_cast<vec_t *>(smem);                       // [BN][UPR], swizzled
    vec_t *Ps = reinterpret_cast<vec_t *>(smem + BN * KC * 4);         // patch, [pixel][cw/V]

    const int t = threadIdx.x;
    const int tx = t & 15;
    const int ty = t >> 4;

    // block -> (channel tile, spatial tile, image group); channel tiles of one patch adjacent
    int bid = blockIdx.x;
    const int co_tile = bid % g.n_co_tiles; bid /= g.n_co_tiles;
    const int tile_x = bid % g.tiles_x;     bid /= g.tiles_x;
    const int tile_y = bid % g.tiles_y;     bid /= g.tiles_y;
    const int img0 = bid * g.ni;
    const int y0 = tile_y * g.th, x0 = tile_x * g.tw;
    const int o_blk = co_tile * BN;

    const int pw = g.tw + 2, ph = g.th + 2;
    const int cwu = g.cw / V;                         // units per pixel

    // ---- stage the input patch (halo included; outside the image = zero words = -1)
    {
        const int total = g.ni * ph * pw * cwu;
        for (int idx = t; idx < total; idx += 256) {
            const int u = idx % cwu;
            int p = idx / cwu;
            const int px = p % pw; p /= pw;
            const int py = p % ph;
            const int il = p / ph;
            const int y = y0 + py - 1, x = x0 + px - 1, img = img0 + il;
            vec_t v = zero_vec<V>();
            if (img < g.n && y >= 0 && y < g.h && x >= 0 && x < g.w)
                v = *reinterpret_cast<const vec_t *>(in + (((int64_t)img * g.h + y) * g.w + x) * g.cw + u * V);
            Ps[idx] = v;
        }
    }

    // ---- this lane's 2x4 pixel patch
    const int ppr = g.tw >> 2;                        // lane patches per tile row
    const int ppi = (g.th >> 1) * ppr;                // lane patches per image
    const int il = ty / ppi;
    const int pid = ty % ppi;
    const int prow = pid / ppr, pcol = pid % ppr;
    const int pix0 = ((il * ph + prow * 2) * pw + pcol * 4) * cwu;    // unit offset of tap (0,0) of pixel (0,0)

    int acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0;

    // weight staging: BN rows x UPR units per chunk
    constexpr int STG = BN * UPR / 256;               // units per thread per chunk
    vec_t pb[STG];
    auto load_w = [&](int k0) {
#pragma unroll
        for (int r = 0; r < STG; ++r) {
            const int idx = t + 256 * r;
            const int row = idx / UPR, u = idx % UPR;
            const int kpos = k0 + u * V;
            const int o = o_blk + row;
            vec_t v = zero_vec<V>();
            if (o < g.c_out && kpos < g.kwt)
                v = *reinterpret_cast<const vec_t *>(wt + (int64_t)o * g.kwt + kpos);
            pb[r] = v;
        }
    };
    load_w(0);

    const int nchunks = (g.kwt + KC - 1) / KC;
    for (int kc = 0; kc < nchunks; ++kc) {
        __syncthreads();
#pragma unroll
        for (int r = 0; r < STG; ++r) {
            const int idx = t + 256 * r;
            const int row = idx / UPR, u = idx % UPR;
            Bs[row * UPR + (u ^ ((row >> 3) & (UPR - 1)))] = pb[r];
        }
        __syncthreads();
        if (kc + 1 < nchunks) load_w((kc + 1) * KC);

        const int k0 = kc * KC;
        const int ucount = min(KC, g.kwt - k0) / V;   // kwt % V == 0
        int kk = k0;
        int tap = kk / g.cw;
        int cwpos = kk - tap * g.cw;
        for (int u = 0; u < ucount; ++u) {
            const int ti = tap / 3, tj = tap - ti * 3;
            const int aoff = pix0 + (ti * pw + tj) * cwu + cwpos / V;
            vec_t a[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) a[i] = Ps[aoff + ((i >> 2) * pw + (i & 3)) * cwu];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int row = tx * 8 + j;
                const vec_t b = Bs[row * UPR + (u ^ ((row >> 3) & (UPR - 1)))];
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i][j] = popc_acc(a[i], b, acc[i][j]);
            }
            cwpos += V;
            if (cwpos == g.cw) { cwpos = 0; ++tap; }
        }
    }

    // ---- epilogue
    const int img = img0 + il;
    const int yb = y0 + prow * 2, xb = x0 + pcol * 4;
    const int o0 = o_blk + tx * 8;
    const int K = g.k_bits;
    if (ep.preact) {
        const bool vec_ok = ((g.c_out & 3) == 0) && (o0 + 8 <= g.c_out);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int y = yb + (i >> 2), x = xb + (i & 3);
            if (img >= g.n || y >= g.h || x >= g.w) continue;
            int32_t *dst = ep.preact + (((int64_t)img * g.h + y) * g.w + x) * g.c_out + o0;
            if (vec_ok) {
                *reinterpret_cast<int4 *>(dst) =
                    make_int4(K - 2 * acc[i][0], K - 2 * acc[i][1], K - 2 * acc[i][2], K - 2 * acc[i][3]);
                *reinterpret_cast<int4 *>(dst + 4) =
                    make_int4(K - 2 * acc[i][4], K - 2 * acc[i][5], K - 2 * acc[i][6], K - 2 * acc[i][7]);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (o0 + j < g.c_out) dst[j] = K - 2 * acc[i][j];
            }
        }
    }
    if (ep.packed) {
        int thr[8];
        unsigned flipmask = 0, valid = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool ok = (o0 + j) < g.c_out;
            thr[j] = ok ? ep.thr[o0 + j] : 0;
            if (ok) valid |= 1u << j;
            if (ok && ep.flip && ep.flip[o0 + j]) flipmask |= 1u << j;
        }
        unsigned bytes[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            unsigned b = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) b |= ((K - 2 * acc[i][j]) > thr[j] ? 1u : 0u) << j;
            bytes[i] = (b ^ flipmask) & valid;
        }
        const int cwo = (g.c_out + 31) >> 5;
        const int wi = o0 >> 5;
        const int sh = 8 * (tx & 3);
        if (ep.pool == 2) {
            const int ho = g.h >> 1, wo = g.w >> 1;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                unsigned b = bytes[2 * q] | bytes[2 * q + 1] | bytes[4 + 2 * q] | bytes[4 + 2 * q + 1];
                unsigned word = b << sh;
                word |= __shfl_xor(word, 1);
                word |= __shfl_xor(word, 2);
                const int yo = yb >> 1, xo = (xb >> 1) + q;
                if ((tx & 3) == 0 && img < g.n && yo < ho && xo < wo && wi < cwo)
                    ep.packed[(((int64_t)img * ho + yo) * wo + xo) * cwo + wi] = word;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                unsigned word = bytes[i] << sh;
                word |= __shfl_xor(word, 1);
                word |= __shfl_xor(word, 2);
                const int y = yb + (i >> 2), x = xb + (i & 3);
                if ((tx & 3) == 0 && img < g.n && y < g.h && x < g.w && wi < cwo)
                    ep.packed[(((int64_t)img * g.h + y) * g.w + x) * cwo + wi] = word;
            }
        }
    }
}

int pow2_ceil(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

ConvGeom make_geom(int n, int h, int w, int c_in, int c_out)
{
    ConvGeom g;
    g.n = n; g.h = h; g.w = w;
    g.cw = (c_in + 31) / 32;
    g.c_out = c_out;
    g.k_bits = 9 * c_in;
    g.kwt = 9 * g.cw;
    int tw = pow2_ceil(w);
    tw = tw < 4 ? 4 : (tw > 16 ? 16 : tw);
    int th = pow2_ceil(h);
    const int th_max = 128 / tw;
    th = th < 2 ? 2 : (th > th_max ? th_max : th);
    g.tw = tw; g.th = th; g.ni = 128 / (th * tw);
    g.tiles_x = (w + tw - 1) / tw;
    g.tiles_y = (h + th - 1) / th;
    g.n_co_tiles = (c_out + BN - 1) / BN;
    return g;
}

size_t patch_bytes(const ConvGeom &g) { return (size_t)g.ni * (g.th + 2) * (g.tw + 2) * g.cw * 4; }

}  // namespace

bool conv_binary_supported(int h, int w, int c_in)
{
    ConvGeom g = make_geom(1, h, w, c_in, 1);
    return patch_bytes(g) <= (size_t)MAX_PATCH_BYTES;
}

bnn_status launch_conv_binary(const uint32_t *in, int n, int h, int w, int c_in, const uint32_t *wt,
                              int c_out, const EpiArgs &ep, hipStream_t s)
{
    if (n == 0) return BNN_OK;
    ConvGeom g = make_geom(n, h, w, c_in, c_out);
    const size_t smem = (size_t)BN * KC * 4 + patch_bytes(g);
    const int64_t blocks = (int64_t)g.n_co_tiles * g.tiles_x * g.tiles_y * ((n + g.ni - 1) / g.ni);
    if (blocks > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
    dim3 grid((unsigned)blocks);
    if ((g.cw & 3) == 0)
        hipLaunchKernelGGL(bconv3x3_tile<4>, grid, dim3(256), smem, s, in, wt, g, ep);
    else if ((g.cw & 1) == 0)
        hipLaunchKernelGGL(bconv3x3_tile<2>, grid, dim3(256), smem, s, in, wt, g, ep);
    else
        hipLaunchKernelGGL(bconv3x3_tile<1>, grid, dim3(256), smem, s, in, wt, g, ep);
    return hip_result(hipGetLastError());
}

}  // namespace bnn

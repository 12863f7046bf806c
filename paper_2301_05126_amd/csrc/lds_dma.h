// Helpers shared by the matrix-core kernels for gfx950: global -> LDS transfers that bypass
// the vector registers, and the expansion of packed bits into FP4 operands.
#ifndef BNN_LDS_DMA_H
#define BNN_LDS_DMA_H
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bnn {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

// Buffer resource over `bytes` bytes at `base` (raw buffer, offsets past the end read zeros).
__device__ __forceinline__ v4i make_raw_rsrc(const void *base, unsigned bytes)
{
    const unsigned long long a = (unsigned long long)base;
    v4i r;
    r[0] = (int)(unsigned)a;
    r[1] = (int)(unsigned)((a >> 32) & 0xffffu);       // stride 0
    r[2] = (int)bytes;
    r[3] = 0x00020000;
    return r;
}

// One wave-wide copy global -> LDS without touching vector registers: lane l's 16 (or 4)
// bytes at byte offset voff of the buffer land at LDS byte address lds_base + 16*l (4*l).
// Written as inline assembly so that the compiler does not serialise the transfer against
// the LDS reads of the tile being multiplied; completion is awaited explicitly
// (s_waitcnt vmcnt(0)) before the barrier that publishes the buffer.  lds_base is wave-uniform.
// Each statement overwrites M0 and says so in its clobber list, so the compiler's own uses of M0
// are re-initialised after it (it warns that M0 is a reserved register; that warning is silenced
// for these four statements only).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_dma16(v4i rsrc, unsigned lds_base, unsigned voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(rsrc) : "memory", "m0");
}
// the same with a scalar byte offset added to the address
__device__ __forceinline__ void lds_dma16_soff(v4i rsrc, unsigned lds_base, unsigned voff, unsigned soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}
__device__ __forceinline__ void lds_dma4_soff(v4i rsrc, unsigned lds_base, unsigned voff, unsigned soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}
__device__ __forceinline__ void lds_dma4(v4i rsrc, unsigned lds_base, unsigned voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(rsrc) : "memory", "m0");
}

#pragma clang diagnostic pop

typedef int v8i __attribute__((ext_vector_type(8)));

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

// Dword `part` (0..3) of expand_fp4.
__device__ __forceinline__ uint32_t expand_part(uint32_t w, int part, uint32_t sgn, uint32_t one)
{
    return part == 3 ? ((w & sgn) | one) : (((w << (3 - part)) & sgn) | one);
}

// The same for two words at once, the words of two consecutive MFMA steps held in a 64-bit
// register pair: one 64-bit shift moves both (the bits that cross from the low word into the
// high one land below each nibble's sign position, where the mask drops them), so a pair costs
// three shifts instead of six.  The two steps split the pair's dwords by shift amount, not by
// word: step 0 takes the dwords shifted by 3 and 2 of both words, step 1 those shifted by 1 and
// 0.  Both MFMA operands are built this way, so every bit still meets its partner exactly once
// over the two steps.  expand_pair_half returns dwords 2*dp and 2*dp+1 of step q's operand.
// (The shift is written as assembly: the compiler would split it back into 32-bit shifts.)
__device__ __forceinline__ uint2 shift_pair_half(uint2 w, int q, int dp)
{
    const int sh = (q == 0 ? 3 : 1) - dp;
    if (sh > 0) {
        const uint64_t p = (uint64_t)w.x | ((uint64_t)w.y << 32);
        uint64_t r;
        asm("v_lshlrev_b64 %0, %1, %2" : "=v"(r) : "n"(sh), "v"(p));
        w = make_uint2((uint32_t)r, (uint32_t)(r >> 32));
    }
    return w;
}
__device__ __forceinline__ uint2 mask_pair(uint2 w, uint32_t sgn, uint32_t one)
{
    return make_uint2((w.x & sgn) | one, (w.y & sgn) | one);
}
__device__ __forceinline__ uint2 expand_pair_half(uint2 w, int q, int dp, uint32_t sgn, uint32_t one)
{
    return mask_pair(shift_pair_half(w, q, dp), sgn, one);
}

}  // namespace

}  // namespace bnn
#endif

// Device-side building blocks shared by the LoRDS kernels (gfx950 only).
//
//  - bit-unpacking of 2/3/4-bit codes held in registers,
//  - bf16 helpers,
//  - the wave-level tile mapping used by the fused kernels, and
//  - access to the (possibly fp32) rank-r factors as bf16 MFMA operands.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lords {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

// ---------------------------------------------------------------------------
// A group of 32 consecutive codes of one row occupies BITS dwords.
// code e (0..31) sits at bits [BITS*e, BITS*e+BITS) of that little-endian string.
// `e` is a compile-time constant after unrolling, so this becomes one v_bfe_u32
// (plus a v_alignbit_b32 for the two 3-bit codes that straddle a dword).
// ---------------------------------------------------------------------------
template <int BITS>
__device__ __forceinline__ uint32_t code_at(const uint32_t (&w)[BITS], int e)
{
    const int o = BITS * e, d = o >> 5, s = o & 31;
    uint32_t v = w[d] >> s;
    if (s + BITS > 32) v |= w[(d + 1) < BITS ? d + 1 : d] << (32 - s);
    return v & ((1u << BITS) - 1u);
}

// Load the BITS dwords of one 32-code group (4-byte aligned address).
template <int BITS>
__device__ __forceinline__ void load_group(const uint8_t *p, uint32_t (&w)[BITS])
{
    const uint32_t *q = reinterpret_cast<const uint32_t *>(p);
#pragma unroll
    for (int i = 0; i < BITS; ++i) w[i] = q[i];
}

__device__ __forceinline__ uint16_t bf16_bits(float x)
{
    __bf16 h = (__bf16)x;                      // v_cvt_pk_bf16_f32, round-to-nearest-even
    return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b)
{
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}

// ---------------------------------------------------------------------------
// The rank-r factors as bf16 MFMA operands.
//
// bf16 factors are used as they are (contraction length r).  fp32 factors are
// split x = hi + lo with hi = bf16(x), lo = bf16(x - hi) and the scale is formed
// as  B A ~= Bhi Ahi + Bhi Alo + Blo Ahi,  i.e. one contraction of length 3r
// over the concatenated operands  B' = [Bhi | Bhi | Blo],  A' = [Ahi ; Alo ; Ahi].
// Every product of two bf16 values is exact in the fp32 accumulator, and the
// dropped Blo Alo term is below 2^-16 relative.
// ---------------------------------------------------------------------------
struct Factors {
    const void *B;   // N x r
    const void *A;   // r x K
    int N, K, r;
    int f32;         // 0: bf16 factors, 1: fp32 factors
    int r_eff;       // r (bf16) or 3r (fp32)
};

__device__ __forceinline__ uint16_t factorA_bits(const Factors &f, int jj, int k)
{
    if (jj >= f.r_eff || k >= f.K) return 0;
    if (!f.f32) return reinterpret_cast<const uint16_t *>(f.A)[(size_t)jj * f.K + k];
    const int seg = jj / f.r, j = jj - seg * f.r;
    const float x = reinterpret_cast<const float *>(f.A)[(size_t)j * f.K + k];
    const uint16_t hi = bf16_bits(x);
    return seg == 1 ? bf16_bits(x - bf16_to_f32(hi)) : hi;
}

// Same as factorA_bits for the product A[j][k] * x (one-token path: the activation is folded
// into the A tile).  fp32 factors: the fp32 product is split hi/lo like a factor.
__device__ __forceinline__ uint16_t factorAx_bits(const Factors &f, int jj, int k, float x)
{
    if (jj >= f.r_eff || k >= f.K) return 0;
    if (!f.f32) return bf16_bits(bf16_to_f32(reinterpret_cast<const uint16_t *>(f.A)[(size_t)jj * f.K + k]) * x);
    const int seg = jj / f.r, j = jj - seg * f.r;
    const float p = reinterpret_cast<const float *>(f.A)[(size_t)j * f.K + k] * x;
    const uint16_t hi = bf16_bits(p);
    return seg == 1 ? bf16_bits(p - bf16_to_f32(hi)) : hi;
}

__device__ __forceinline__ uint16_t factorB_bits(const Factors &f, int n, int jj)
{
    if (jj >= f.r_eff || n >= f.N) return 0;
    if (!f.f32) return reinterpret_cast<const uint16_t *>(f.B)[(size_t)n * f.r + jj];
    const int seg = jj / f.r, j = jj - seg * f.r;
    const float x = reinterpret_cast<const float *>(f.B)[(size_t)n * f.r + j];
    const uint16_t hi = bf16_bits(x);
    return seg == 2 ? bf16_bits(x - bf16_to_f32(hi)) : hi;
}

// fp32 sums that pass from one workgroup to another through memory: 16-byte stores and loads at
// agent scope (sc1: written through to, and read from, the level all XCDs share), so that the hand-over
// needs no write-back or invalidation of a whole L2.  Written as assembly because the language
// offers agent-scope atomic accesses of at most 8 bytes; the waits are placed by hand.
__device__ __forceinline__ void store16_agent(float *p, f32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1" :: "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ f32x4 load16_agent(const float *p)
{
    f32x4 v;
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
    return v;
}

}  // namespace lords

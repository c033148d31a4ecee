// Pieces shared by the small-M (decode) kernels: arguments, the transposing LDS read that
// turns a row-major A tile into scale-MFMA operands, and the code-pair look-up addressing.
#pragma once
#include "lords_device.h"
#include "lords_launch.h"

namespace lords {

constexpr int kNS = 8;       // max slabs (of 16 rows) per workgroup
constexpr int kDepth = 2;    // slabs whose loads are in flight ahead of the one computed

struct DecodeArgs {
    const uint16_t *X;
    const uint8_t *codes;
    const float *codebook;
    Factors f;
    void *Y;
    float *partial;        // [splits][M][N] fp32, used when splits > 1
    unsigned *counters;    // one ticket per slab chunk (gridDim.x), zero between calls
    int M, N, K;
    int y_f32;
    int row_bytes;
    int nslabs;            // ceil(N / 16)
    int ns;                // slabs per workgroup, <= kNS
    int splits;            // gridDim.z
    int b_vec_ok;
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4_t;
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

template <int AST>
__device__ __forceinline__ bf16x8 tr_read_pair_d(const uint16_t *tile, int row, int col)
{
    const uint16_t *p0 = tile + row * AST + col;
    const uint16_t *p1 = p0 + 4 * AST;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)p0);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)p1);
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
    s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// LDS byte address of the table entry of code pair p (codes 2p, 2p+1) of a 32-code group.
template <int BITS>
__device__ __forceinline__ uint32_t pair_addr(const uint32_t (&w)[BITS], int p, uint32_t laneoff)
{
    if (BITS == 4) {
        // result byte1 = byte (p&3) of dword p>>2, byte0 = laneoff, bytes 2,3 = 0
        return __builtin_amdgcn_perm(w[p >> 2], laneoff, 0x0C0C0000u | ((4u + (p & 3)) << 8));
    }
    const int o = 2 * BITS * p, d = o >> 5, s = o & 31;
    uint32_t v = w[d] >> s;
    if (s + 2 * BITS > 32) v |= w[(d + 1) < BITS ? d + 1 : d] << (32 - s);
    return ((v & ((1u << (2 * BITS)) - 1u)) << 8) | laneoff;
}

__device__ __forceinline__ uint32_t lds_load_u32(uint32_t byte_addr)
{
    // The kernels below declare no static LDS, so their dynamic LDS starts at address 0 and
    // a table offset is an LDS address.
    return *reinterpret_cast<const __attribute__((address_space(3))) uint32_t *>((uintptr_t)byte_addr);
}


}  // namespace lords

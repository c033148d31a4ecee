// Quantisation side of the path (the inverse of lords_dequant), streaming kernels:
//
//   lords_quantize  : Alg. 1 step 2.1.  For every element, the level index
//                     q = argmin_i (S * C[i] - W)^2 with S = sum_j B[n][j] A[j][k], packed to `bits` bits.
//   lords_block_init: the block-wise scale that Alg. 1 step 1 starts from (ComputeScale with block
//                     size K/r, read as symmetric absmax scaling, Sec. 3.1), written directly as
//                     factors: B = block scales (N x r), A = 0/1 block indicator (r x K), so that
//                     B A is that piecewise-constant scale matrix (rank <= r).
//
// The index is an integer decided by floating point, so the arithmetic is fixed operation by
// operation (all fp32, each correctly rounded):
//   S    = fma(B[n][r-1], A[r-1][k], ... fma(B[n][0], A[0][k], 0) ...)      j increasing
//   d_i  = fma(S, C[i], -W),  e_i = d_i * d_i,  q = the lowest i with minimal e_i
//   block scale = max|W_block| / max_i |C[i]|
#include "lords_device.h"
#include "lords_launch.h"

namespace lords {

// One thread per group of 32 consecutive elements of one row: 32 scales, 32 searches, BITS dwords out.
// The 128 threads of a workgroup take the SAME 32 columns of 128 consecutive rows, so the A values
// of a step of the j loop are the same for every lane (scalar loads, operands straight from scalar
// registers) and only B is read per lane.
template <int BITS, bool F32FACT, bool F32W>
__global__ __launch_bounds__(128) void quantize_kernel(const void *__restrict__ Wv, const float *__restrict__ codebook,
                                                       const void *__restrict__ Bv, const void *__restrict__ Av,
                                                       uint8_t *__restrict__ codes, int N, int K, int r)
{
    constexpr int NL = 1 << BITS;
    __shared__ float lut[NL];
    if (threadIdx.x < NL) lut[threadIdx.x] = codebook[threadIdx.x];
    __syncthreads();
    const int gpr = K / 32;                                  // groups per row
    const int grp = blockIdx.y;
    const int row = blockIdx.x * 128 + threadIdx.x;
    const int n = row < N ? row : N - 1;                     // rows >= N: recomputed, never stored
    const int k0 = grp * 32;

    float s[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) s[e] = 0.f;
    for (int j = 0; j < r; ++j) {
        float b;
        if (F32FACT) b = reinterpret_cast<const float *>(Bv)[(size_t)n * r + j];
        else b = bf16_to_f32(reinterpret_cast<const uint16_t *>(Bv)[(size_t)n * r + j]);
        if (F32FACT) {
            const f32x4 *a = reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(Av) + (size_t)j * K + k0);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const f32x4 v = a[q];
#pragma unroll
                for (int e = 0; e < 4; ++e) s[4 * q + e] = __builtin_fmaf(b, v[e], s[4 * q + e]);
            }
        } else {
            const u32x4 *a = reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(Av) + (size_t)j * K + k0);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u32x4 v = a[q];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    s[8 * q + 2 * e] = __builtin_fmaf(b, __builtin_bit_cast(float, v[e] << 16), s[8 * q + 2 * e]);
                    s[8 * q + 2 * e + 1] = __builtin_fmaf(b, __builtin_bit_cast(float, v[e] & 0xFFFF0000u), s[8 * q + 2 * e + 1]);
                }
            }
        }
    }

    float w[32];
    if (F32W) {
        const f32x4 *p = reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(Wv) + (size_t)n * K + k0);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const f32x4 v = p[q];
#pragma unroll
            for (int e = 0; e < 4; ++e) w[4 * q + e] = v[e];
        }
    } else {
        const u32x4 *p = reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(Wv) + (size_t)n * K + k0);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const u32x4 v = p[q];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                w[8 * q + 2 * e] = __builtin_bit_cast(float, v[e] << 16);
                w[8 * q + 2 * e + 1] = __builtin_bit_cast(float, v[e] & 0xFFFF0000u);
            }
        }
    }

    uint32_t out[BITS];
#pragma unroll
    for (int d = 0; d < BITS; ++d) out[d] = 0u;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        uint32_t best = 0u;
        float ebest;
        {
            const float d0 = __builtin_fmaf(s[e], lut[0], -w[e]);
            ebest = d0 * d0;
        }
#pragma unroll
        for (int i = 1; i < NL; ++i) {
            const float d = __builtin_fmaf(s[e], lut[i], -w[e]);
            const float err = d * d;
            const bool better = err < ebest;               // strict: ties keep the lower index
            best = better ? (uint32_t)i : best;
            ebest = better ? err : ebest;
        }
        const int o = BITS * e, dw = o >> 5, sh = o & 31;
        out[dw] |= best << sh;
        if (sh + BITS > 32) out[dw + 1 < BITS ? dw + 1 : dw] |= best >> (32 - sh);
    }
    if (row >= N) return;
    uint32_t *dst = reinterpret_cast<uint32_t *>(codes + ((size_t)n * gpr + grp) * (4 * BITS));
#pragma unroll
    for (int d = 0; d < BITS; ++d) dst[d] = out[d];
}

// One wave per block of g = K/r consecutive columns of a row: coalesced reads, max over the lanes
// (a maximum does not depend on the order it is taken in).
template <bool F32W, bool F32FACT>
__global__ __launch_bounds__(256) void block_scale_kernel(const void *__restrict__ Wv, const float *__restrict__ codebook,
                                                          void *__restrict__ Bv, int N, int K, int r, int nl)
{
    const int lane = threadIdx.x & 63;
    const long blk = (long)blockIdx.x * 4 + (threadIdx.x >> 6);      // block index n * r + j
    if (blk >= (long)N * r) return;
    const int n = (int)(blk / r), j = (int)(blk % r), g = K / r;
    float cmax = 0.f;
    for (int i = 0; i < nl; ++i) cmax = fmaxf(cmax, fabsf(codebook[i]));
    float m = 0.f;
    for (int k = lane; k < g; k += 64) {
        const size_t at = (size_t)n * K + (size_t)j * g + k;
        const float v = F32W ? reinterpret_cast<const float *>(Wv)[at]
                             : bf16_to_f32(reinterpret_cast<const uint16_t *>(Wv)[at]);
        m = fmaxf(m, fabsf(v));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if (lane == 0) {
        const float sc = m / cmax;
        if (F32FACT) reinterpret_cast<float *>(Bv)[blk] = sc;
        else reinterpret_cast<uint16_t *>(Bv)[blk] = bf16_bits(sc);
    }
}

// The same for block sizes g that divide 256 (and are multiples of 4): W is read as one flat stream of
// 4-element vectors, kU vectors per lane in flight; a block is g/4 neighbouring lanes of one vector row,
// its maximum taken by cross-lane steps within that group.  Blocks are consecutive in the flat order
// (K = r g), so block b is elements b g .. b g + g - 1 and its scale is entry b of B.
constexpr int kBsU = 8;
template <bool F32W, bool F32FACT>
__global__ __launch_bounds__(256) void block_scale_vec_kernel(const void *__restrict__ Wv, const float *__restrict__ codebook,
                                                              void *__restrict__ Bv, long nvec, int g, int nl)
{
    const int lane = threadIdx.x & 63;
    const long wave = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long v0 = wave * (64 * kBsU) + lane;                       // this lane's first vector
    if (wave * (64 * kBsU) >= nvec) return;
    float cmax = 0.f;
    for (int i = 0; i < nl; ++i) cmax = fmaxf(cmax, fabsf(codebook[i]));
    float m[kBsU];
#pragma unroll
    for (int u = 0; u < kBsU; ++u) {
        const long v = v0 + 64 * u;
        const long vc = v < nvec ? v : nvec - 1;                      // past the end: a copy of the last vector, never stored
        float x0, x1, x2, x3;
        if (F32W) {
            const f32x4 t = reinterpret_cast<const f32x4 *>(Wv)[vc];
            x0 = t[0]; x1 = t[1]; x2 = t[2]; x3 = t[3];
        } else {
            typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
            const u32x2 t = reinterpret_cast<const u32x2 *>(Wv)[vc];
            x0 = __builtin_bit_cast(float, t[0] << 16); x1 = __builtin_bit_cast(float, t[0] & 0xFFFF0000u);
            x2 = __builtin_bit_cast(float, t[1] << 16); x3 = __builtin_bit_cast(float, t[1] & 0xFFFF0000u);
        }
        m[u] = fmaxf(fmaxf(fabsf(x0), fabsf(x1)), fmaxf(fabsf(x2), fabsf(x3)));
    }
    const int lpb = g >> 2;                                           // lanes per block: 1, 2, 4, ... 64
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        if (off < lpb) {
#pragma unroll
            for (int u = 0; u < kBsU; ++u) m[u] = fmaxf(m[u], __shfl_xor(m[u], off));
        }
    }
    if ((lane & (lpb - 1)) == 0) {
#pragma unroll
        for (int u = 0; u < kBsU; ++u) {
            const long v = v0 + 64 * u;
            if (v >= nvec) continue;
            const long blk = v / lpb;
            const float sc = m[u] / cmax;
            if (F32FACT) reinterpret_cast<float *>(Bv)[blk] = sc;
            else reinterpret_cast<uint16_t *>(Bv)[blk] = bf16_bits(sc);
        }
    }
}

template <bool F32FACT>
__global__ __launch_bounds__(256) void block_indicator_kernel(void *__restrict__ Av, int K, int r)
{
    const long id = (long)blockIdx.x * 256 + threadIdx.x;
    if (id >= (long)r * K) return;
    const int j = (int)(id / K), k = (int)(id % K), g = K / r;
    const float v = (k / g == j) ? 1.f : 0.f;
    if (F32FACT) reinterpret_cast<float *>(Av)[id] = v;
    else reinterpret_cast<uint16_t *>(Av)[id] = bf16_bits(v);
}

template <int BITS>
static hipError_t launch_quantize_bits(const void *W, const float *codebook, const void *B, const void *A, void *codes,
                                       int N, int K, int r, bool f32w, bool f32fact, hipStream_t st)
{
    const dim3 grid((unsigned)((N + 127) / 128), (unsigned)(K / 32)), block(128);
#define LORDS_QCASE(FF_, FW_) \
    hipLaunchKernelGGL((quantize_kernel<BITS, FF_, FW_>), grid, block, 0, st, W, codebook, B, A, (uint8_t *)codes, N, K, r)
    if (f32fact) { if (f32w) LORDS_QCASE(true, true); else LORDS_QCASE(true, false); }
    else { if (f32w) LORDS_QCASE(false, true); else LORDS_QCASE(false, false); }
#undef LORDS_QCASE
    return hipGetLastError();
}

hipError_t launch_quantize(const void *W, const float *codebook, const void *B, const void *A, void *codes,
                           int N, int K, int r, int bits, bool f32w, bool f32fact, hipStream_t st)
{
    switch (bits) {
        case 2: return launch_quantize_bits<2>(W, codebook, B, A, codes, N, K, r, f32w, f32fact, st);
        case 3: return launch_quantize_bits<3>(W, codebook, B, A, codes, N, K, r, f32w, f32fact, st);
        default: return launch_quantize_bits<4>(W, codebook, B, A, codes, N, K, r, f32w, f32fact, st);
    }
}

hipError_t launch_block_init(const void *W, const float *codebook, void *B, void *A,
                             int N, int K, int r, int bits, bool f32w, bool f32fact, hipStream_t st)
{
    const long nblk = (long)N * r;
    const dim3 g1((unsigned)((nblk + 3) / 4)), g2((unsigned)(((long)r * K + 255) / 256));
    const int nl = 1 << bits;
    const int g = K / r;
    if ((g % 4) == 0 && (256 % g) == 0) {
        const long nvec = (long)N * K / 4;
        const dim3 gv((unsigned)((nvec + 4 * 64 * kBsU - 1) / (4 * 64 * kBsU)));
#define LORDS_BCASE(FW_, FF_) \
    hipLaunchKernelGGL((block_scale_vec_kernel<FW_, FF_>), gv, dim3(256), 0, st, W, codebook, B, nvec, g, nl)
        if (f32w) { if (f32fact) LORDS_BCASE(true, true); else LORDS_BCASE(true, false); }
        else { if (f32fact) LORDS_BCASE(false, true); else LORDS_BCASE(false, false); }
#undef LORDS_BCASE
    } else if (f32w) {
        if (f32fact) hipLaunchKernelGGL((block_scale_kernel<true, true>), g1, dim3(256), 0, st, W, codebook, B, N, K, r, nl);
        else hipLaunchKernelGGL((block_scale_kernel<true, false>), g1, dim3(256), 0, st, W, codebook, B, N, K, r, nl);
    } else {
        if (f32fact) hipLaunchKernelGGL((block_scale_kernel<false, true>), g1, dim3(256), 0, st, W, codebook, B, N, K, r, nl);
        else hipLaunchKernelGGL((block_scale_kernel<false, false>), g1, dim3(256), 0, st, W, codebook, B, N, K, r, nl);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (f32fact) hipLaunchKernelGGL((block_indicator_kernel<true>), g2, dim3(256), 0, st, A, K, r);
    else hipLaunchKernelGGL((block_indicator_kernel<false>), g2, dim3(256), 0, st, A, K, r);
    return hipGetLastError();
}

}  // namespace lords

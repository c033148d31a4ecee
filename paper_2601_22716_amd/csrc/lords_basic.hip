// Stand-alone unpack and dequantise kernels (the parity artefacts of the path).
//
//   lords_unpack : packed codes -> one uint8 index per element
//   lords_dequant: W_hat = C[q] (.) (B A), written to device memory
//
// Both are streaming kernels bound by their output writes; the fused
// lords_matmul kernels never call them.
#include "lords_device.h"
#include "lords_launch.h"

namespace lords {

// One thread per group of 32 codes: BITS dwords in, 32 bytes out.
template <int BITS>
__global__ __launch_bounds__(256) void unpack_kernel(const uint8_t *__restrict__ codes,
                                                     uint8_t *__restrict__ idx, long groups)
{
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= groups) return;
    uint32_t w[BITS];
    load_group<BITS>(codes + gid * (4 * BITS), w);
    uint32_t out[8];
#pragma unroll
    for (int d = 0; d < 8; ++d) {
        out[d] = code_at<BITS>(w, 4 * d) | (code_at<BITS>(w, 4 * d + 1) << 8) |
                 (code_at<BITS>(w, 4 * d + 2) << 16) | (code_at<BITS>(w, 4 * d + 3) << 24);
    }
    u32x4 *o = reinterpret_cast<u32x4 *>(idx + gid * 32);
    o[0] = u32x4{out[0], out[1], out[2], out[3]};
    o[1] = u32x4{out[4], out[5], out[6], out[7]};
}

// One thread per group of 32 codes of one row.  The scale is summed over j in
// increasing order with fp32 FMAs (exact products for bf16 factors).
template <int BITS, bool F32FACT, bool F32OUT>
__global__ __launch_bounds__(128) void dequant_kernel(const uint8_t *__restrict__ codes,
                                                      const float *__restrict__ codebook,
                                                      const void *__restrict__ Bv,
                                                      const void *__restrict__ Av,
                                                      void *__restrict__ Wv, int N, int K, int r)
{
    __shared__ float lut[1 << BITS];
    if (threadIdx.x < (1 << BITS)) lut[threadIdx.x] = codebook[threadIdx.x];
    __syncthreads();
    const int gpr = K / 32;                                  // groups per row
    const int blocks_per_row = (gpr + 127) / 128;
    const int n = blockIdx.x / blocks_per_row;
    const int grp = (blockIdx.x % blocks_per_row) * 128 + threadIdx.x;
    if (grp >= gpr) return;
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
    uint32_t w[BITS];
    load_group<BITS>(codes + ((size_t)n * gpr + grp) * (4 * BITS), w);
    if (F32OUT) {
        f32x4 *o = reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(Wv) + (size_t)n * K + k0);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            f32x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = lut[code_at<BITS>(w, 4 * q + e)] * s[4 * q + e];
            o[q] = v;
        }
    } else {
        u32x4 *o = reinterpret_cast<u32x4 *>(reinterpret_cast<uint16_t *>(Wv) + (size_t)n * K + k0);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t lo = bf16_bits(lut[code_at<BITS>(w, 8 * q + 2 * e)] * s[8 * q + 2 * e]);
                const uint32_t hi = bf16_bits(lut[code_at<BITS>(w, 8 * q + 2 * e + 1)] * s[8 * q + 2 * e + 1]);
                v[e] = lo | (hi << 16);
            }
            o[q] = v;
        }
    }
}

template <int BITS>
static hipError_t launch_unpack_bits(const void *codes, uint8_t *idx, int N, int K, hipStream_t st)
{
    const long groups = (long)N * (K / 32);
    const long blocks = (groups + 255) / 256;
    hipLaunchKernelGGL(unpack_kernel<BITS>, dim3((unsigned)blocks), dim3(256), 0, st,
                       (const uint8_t *)codes, idx, groups);
    return hipGetLastError();
}

// Slab-tile layout of the codes (see lords_repack in the header): one thread per 32-code chunk of the
// tiled buffer, chunks in storage order, so the writes are contiguous; chunks beyond the matrix are zero.
template <int BITS>
__global__ __launch_bounds__(256) void repack_kernel(const uint8_t *__restrict__ codes, uint8_t *__restrict__ tiled,
                                                     int N, int K, int nct, long chunks)
{
    const long id = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= chunks) return;
    const long tile = id >> 6;
    const int ch = (int)(id & 63), g = ch >> 4, c = ch & 15;
    const long s = tile / nct;
    const int t = (int)(tile - s * nct);
    const long n = s * 16 + c;
    const int grp = 4 * t + g;
    uint32_t w[BITS];
#pragma unroll
    for (int e = 0; e < BITS; ++e) w[e] = 0u;
    if (n < N && grp < (K >> 5)) load_group<BITS>(codes + (size_t)n * (K / 8 * BITS) + (size_t)grp * (4 * BITS), w);
    uint32_t *o = reinterpret_cast<uint32_t *>(tiled + (size_t)id * (4 * BITS));
#pragma unroll
    for (int e = 0; e < BITS; ++e) o[e] = w[e];
}

template <int BITS>
static hipError_t launch_repack_bits(const void *codes, void *tiled, int N, int K, hipStream_t st)
{
    const int nct = (K + 127) / 128;
    const long chunks = (long)((N + 15) / 16) * nct * 64;
    hipLaunchKernelGGL(repack_kernel<BITS>, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st,
                       (const uint8_t *)codes, (uint8_t *)tiled, N, K, nct, chunks);
    return hipGetLastError();
}

hipError_t launch_repack(const void *codes, void *tiled, int N, int K, int bits, hipStream_t st)
{
    switch (bits) {
        case 2: return launch_repack_bits<2>(codes, tiled, N, K, st);
        case 3: return launch_repack_bits<3>(codes, tiled, N, K, st);
        default: return launch_repack_bits<4>(codes, tiled, N, K, st);
    }
}

hipError_t launch_unpack(const void *codes, uint8_t *idx, int N, int K, int bits, hipStream_t st)
{
    switch (bits) {
        case 2: return launch_unpack_bits<2>(codes, idx, N, K, st);
        case 3: return launch_unpack_bits<3>(codes, idx, N, K, st);
        default: return launch_unpack_bits<4>(codes, idx, N, K, st);
    }
}

template <int BITS, bool F32FACT, bool F32OUT>
static hipError_t launch_dequant_t(const void *codes, const float *codebook, const void *B, const void *A,
                                   void *W, int N, int K, int r, hipStream_t st)
{
    const long blocks_per_row = (K / 32 + 127) / 128;
    hipLaunchKernelGGL((dequant_kernel<BITS, F32FACT, F32OUT>), dim3((unsigned)(blocks_per_row * N)), dim3(128), 0, st,
                       (const uint8_t *)codes, codebook, B, A, W, N, K, r);
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_dequant_bits(const void *codes, const float *codebook, const void *B, const void *A,
                                      void *W, int N, int K, int r, bool f32fact, bool f32out, hipStream_t st)
{
    if (f32fact) return f32out ? launch_dequant_t<BITS, true, true>(codes, codebook, B, A, W, N, K, r, st)
                               : launch_dequant_t<BITS, true, false>(codes, codebook, B, A, W, N, K, r, st);
    return f32out ? launch_dequant_t<BITS, false, true>(codes, codebook, B, A, W, N, K, r, st)
                  : launch_dequant_t<BITS, false, false>(codes, codebook, B, A, W, N, K, r, st);
}

hipError_t launch_dequant(const void *codes, const float *codebook, const void *B, const void *A, void *W,
                          int N, int K, int r, int bits, bool f32fact, bool f32out, hipStream_t st)
{
    switch (bits) {
        case 2: return launch_dequant_bits<2>(codes, codebook, B, A, W, N, K, r, f32fact, f32out, st);
        case 3: return launch_dequant_bits<3>(codes, codebook, B, A, W, N, K, r, f32fact, f32out, st);
        default: return launch_dequant_bits<4>(codes, codebook, B, A, W, N, K, r, f32fact, f32out, st);
    }
}

// h = silu(g) * u on fp32 inputs, one rounding at the store (the gate of a SwiGLU MLP when the two
// products could not be combined inside the matmul kernel).  Four elements per thread.
template <bool F32OUT>
__global__ __launch_bounds__(256) void silu_mul_kernel(const float *__restrict__ G, const float *__restrict__ U,
                                                       void *__restrict__ H, long count)
{
    const long i0 = ((long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i0 >= count) return;
    float g[4], u[4];
    if (i0 + 4 <= count) {
        const f32x4 gv = *reinterpret_cast<const f32x4 *>(G + i0), uv = *reinterpret_cast<const f32x4 *>(U + i0);
#pragma unroll
        for (int e = 0; e < 4; ++e) { g[e] = gv[e]; u[e] = uv[e]; }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const long i = i0 + e < count ? i0 + e : count - 1;
            g[e] = G[i];
            u[e] = U[i];
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (i0 + e >= count) break;
        const float h = g[e] / (1.0f + __expf(-g[e])) * u[e];
        if (F32OUT) reinterpret_cast<float *>(H)[i0 + e] = h;
        else reinterpret_cast<uint16_t *>(H)[i0 + e] = bf16_bits(h);
    }
}

hipError_t launch_silu_mul(const float *G, const float *U, void *H, long count, bool f32out, hipStream_t st)
{
    if (count <= 0) return hipSuccess;
    const long threads = (count + 3) / 4;
    const unsigned blocks = (unsigned)((threads + 255) / 256);
    if (f32out) hipLaunchKernelGGL(silu_mul_kernel<true>, dim3(blocks), dim3(256), 0, st, G, U, H, count);
    else hipLaunchKernelGGL(silu_mul_kernel<false>, dim3(blocks), dim3(256), 0, st, G, U, H, count);
    return hipGetLastError();
}

}  // namespace lords

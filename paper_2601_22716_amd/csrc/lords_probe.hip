// Measurement aids (not part of the method): two kernels that measure what this GPU delivers to
// ANY kernel, so that the benchmark can quote a kernel's rate against a measured ceiling beside
// the vendor's peak.
//   lords_probe_stream_read: a read-only pass over a buffer (16-byte loads, eight in flight per
//                            lane, every line touched once, one contiguous span per workgroup) -> achievable HBM read bandwidth.
//   lords_probe_mfma_bf16:   register-resident v_mfma_f32_16x16x32_bf16 chains, no memory traffic
//                            -> achievable dense bf16 matrix rate; with operands of ones and small
//                            integers, or with operands that differ in every lane and element (the
//                            sustained rate depends on the data: the chip lowers its clock under the
//                            switching activity of real operands).
#include "../../include/lords.h"
#include "lords_device.h"

namespace lords {

__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4 *__restrict__ src, size_t n16, uint32_t *sink)
{
    // a workgroup reads one contiguous span, 4 KB per step and eight steps in flight
    const size_t span = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t lo = span * blockIdx.x, hi = lo + span < n16 ? lo + span : n16;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t i = lo + threadIdx.x; i < hi; i += 8 * 256) {
        u32x4 v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const size_t j = i + (size_t)q * 256;
            v[q] = j < hi ? src[j] : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) acc ^= v[q];
    }
    // (the sum is stored only for a value that random data never gives: the loads cannot be dropped)
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u && acc[0] == 0x7F4A7C15u) sink[0] = acc[1];
}

__global__ __launch_bounds__(512) void probe_mfma_kernel(int iters, int pattern, float *sink)
{
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) {
        if (pattern == 0) { a[e] = (__bf16)(float)(threadIdx.x & 3); b[e] = (__bf16)1.0f; }       // few bits set, few bits toggling
        else {                                                                                  // every lane and element different
            uint32_t h = (threadIdx.x * 8u + e + 1u) * 2654435761u;
            a[e] = (__bf16)(((int)(h >> 8 & 0xFFFF) - 32768) * (1.0f / 32768.0f));
            b[e] = (__bf16)(((int)(h >> 3 & 0xFFFF) - 32768) * (1.0f / 65536.0f));
        }
    }
    f32x4 acc[8];
    for (int c = 0; c < 8; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.f;
    for (int c = 0; c < 8; ++c) s += acc[c][0] + acc[c][1] + acc[c][2] + acc[c][3];
    if (s == 12345.678f) sink[0] = s;
}

}  // namespace lords

extern "C" {

int lords_probe_stream_read(const void *buffer, size_t bytes, void *sink, void *stream)
{
    if (!buffer || !sink) return LORDS_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(buffer) & 15u) != 0) return LORDS_ERR_ALIGN;
    const size_t n16 = bytes / 16;
    if (n16 == 0) return LORDS_OK;
    // eight workgroups per CU, sixteen for large buffers; no more than the buffer has 4 KB pieces
    const size_t want = bytes >= ((size_t)256 << 20) ? 4096 : 2048;
    size_t wgs = n16 / 256 < want ? (n16 + 255) / 256 : want;
    hipLaunchKernelGGL(lords::probe_read_kernel, dim3((unsigned)wgs), dim3(256), 0, (hipStream_t)stream,
                       (const lords::u32x4 *)buffer, n16, (uint32_t *)sink);
    return hipGetLastError() == hipSuccess ? LORDS_OK : LORDS_ERR_LAUNCH;
}

int lords_probe_mfma_bf16(int iterations, int pattern, void *sink, double *flop_per_launch, void *stream)
{
    if (!sink) return LORDS_ERR_NULL;
    if (iterations < 1 || pattern < 0 || pattern > 1) return LORDS_ERR_SHAPE;
    const int wgs = 256 * 2, waves = 4;                     // two workgroups of four waves per CU
    if (flop_per_launch) *flop_per_launch = (double)wgs * waves * iterations * 8 * (2.0 * 16 * 16 * 32);
    hipLaunchKernelGGL(lords::probe_mfma_kernel, dim3(wgs), dim3(64 * waves), 0, (hipStream_t)stream, iterations, pattern, (float *)sink);
    return hipGetLastError() == hipSuccess ? LORDS_OK : LORDS_ERR_LAUNCH;
}

}  // extern "C"

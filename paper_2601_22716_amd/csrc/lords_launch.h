// Host-side launch functions of the kernel translation units (internal; the
// public boundary is include/lords.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lords {

hipError_t launch_unpack(const void *codes, uint8_t *idx, int N, int K, int bits, hipStream_t st);

hipError_t launch_dequant(const void *codes, const float *codebook, const void *B, const void *A, void *W,
                          int N, int K, int r, int bits, bool f32fact, bool f32out, hipStream_t st);

struct MatmulProblem {
    const void *X;          // M x K bf16
    const void *codes;      // N x K*bits/8
    const float *codebook;  // 2^bits
    const void *B;          // N x r
    const void *A;          // r x K
    void *Y;                // M x N
    int M, N, K, r, bits;
    bool f32fact, f32out;
};

// Bytes of fp32 workspace the decode path needs for this problem (0 if none).
size_t decode_workspace_bytes(const MatmulProblem &p);
// Small-M path.  `workspace` must hold decode_workspace_bytes(p) bytes (may be null if 0).
hipError_t launch_decode(const MatmulProblem &p, void *workspace, hipStream_t st);
// MFMA GEMM path for large M.
hipError_t launch_prefill(const MatmulProblem &p, hipStream_t st);

}  // namespace lords

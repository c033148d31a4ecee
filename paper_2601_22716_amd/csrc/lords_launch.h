// Host-side launch functions of the kernel translation units (internal; the
// public boundary is include/lords.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lords {

// A kernel that asks for more dynamic LDS than the default limit must be told so once PER DEVICE
// (the attribute belongs to the function on the device that is current).  One of these, static,
// per kernel instantiation; a repeated call from two threads does the same thing twice.
struct LdsOptIn {
    bool done[16] = {};
};
inline hipError_t allow_dynamic_lds(LdsOptIn &state, const void *func, size_t bytes)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 16) return hipErrorInvalidDevice;
    if (!state.done[dev]) {
        e = hipFuncSetAttribute(func, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return e;
        state.done[dev] = true;
    }
    return hipSuccess;
}

hipError_t launch_unpack(const void *codes, uint8_t *idx, int N, int K, int bits, hipStream_t st);
hipError_t launch_repack(const void *codes, void *tiled, int N, int K, int bits, hipStream_t st);

hipError_t launch_dequant(const void *codes, const float *codebook, const void *B, const void *A, void *W,
                          int N, int K, int r, int bits, bool f32fact, bool f32out, hipStream_t st);

// H = silu(G) * U, element by element, fp32 in (lords_basic.hip).
hipError_t launch_silu_mul(const float *G, const float *U, void *H, long count, bool f32out, hipStream_t st);

// Quantisation side (lords_quant.hip).
hipError_t launch_quantize(const void *W, const float *codebook, const void *B, const void *A, void *codes,
                           int N, int K, int r, int bits, bool f32w, bool f32fact, hipStream_t st);
hipError_t launch_block_init(const void *W, const float *codebook, void *B, void *A,
                             int N, int K, int r, int bits, bool f32w, bool f32fact, hipStream_t st);

// Backward side (lords_backward.hip).  codes_t: the packed codes with the roles of rows and columns
// swapped (K rows of N codes); N must be a multiple of 32.
hipError_t launch_transpose_codes(const void *codes, void *codes_t, int N, int K, int bits, hipStream_t st);
hipError_t launch_transpose_factor(const void *in, void *out, int rows, int cols, bool f32, hipStream_t st);
// dB (N x r) and dA (r x K), fp32, from dY (M x N) and X (M x K), both bf16.  `workspace` must hold
// factor_grad_workspace_bytes(N, K, r) bytes (fp32 partial results per tile, added in a fixed order).
bool factor_grad_supported(int N, int K, int r);
size_t factor_grad_workspace_bytes(int N, int K, int r);
hipError_t launch_factor_grad(const void *dY, const void *X, const void *codes, const float *codebook, const void *B,
                              const void *A, float *dB, float *dA, int M, int N, int K, int r, int bits, bool f32fact,
                              void *workspace, hipStream_t st);

struct MatmulProblem {
    const void *X;          // M x K bf16
    const void *codes;      // N x K*bits/8
    const float *codebook;  // 2^bits
    const void *B;          // N x r
    const void *A;          // r x K
    void *Y;                // M x N
    int M, N, K, r, bits;
    bool f32fact, f32out;
    bool tiled = false;     // `codes` is in the slab-tile layout (lords_repack): tile (slab s, column tile t) at
                            // (s * ceil(K/128) + t) * 256 * bits bytes, chunk (row c, group g) at (16 g + c) * 4 * bits inside
};

// The front of the per-device workspace is reserved for arrival tickets (always zero between calls).
constexpr size_t kTicketBytes = 16384;

// Exchange slots of the one-/two-token kernel (lords_gemv.hip): a region that is zero between calls.
constexpr size_t kZeroBytes = 4u << 20;

// One- and two-token path (lords_gemv.hip), bf16 factors, ranks up to 64 (one token) / 32 (two).
// `zeroed`: kZeroBytes of device memory, zero when handed over and left at zero (used only when the
// layer is wider than one workgroup's column range).
bool decode_gemv_supported(const MatmulProblem &p);
hipError_t launch_decode_gemv(const MatmulProblem &p, void *zeroed, hipStream_t st);

// Several matrices applied to the SAME activations in a single launch: same K, rank, code width, level
// table and factor type (bf16), own N.  act: matrices 0 and 1 (same N) are a
// gate/up pair and Y[0] receives silu(gate) * up; Y[1] is not written.
constexpr int kMaxBatch = 8;
struct BatchedProblem {
    const void *X;
    const float *codebook;
    const void *codes[kMaxBatch];
    const void *B[kMaxBatch];
    const void *A[kMaxBatch];
    void *Y[kMaxBatch];
    int N[kMaxBatch];
    int L, M, K, r, bits;
    bool f32fact, f32out, act;
    bool tiled = false;     // every codes[l] is in the slab-tile layout (see MatmulProblem)
};
// One and two tokens, bf16 factors (lords_gemv.hip): all matrices in one launch; `zeroed` as for the single matrix.
bool decode_gemv_batched_supported(const BatchedProblem &p);
hipError_t launch_decode_gemv_batched(const BatchedProblem &p, void *zeroed, hipStream_t st);
// The same for 2..16 tokens, ranks up to 64 (lords_decode_mx.hip); same workspace convention as below.
bool decode_mx_batched_supported(const BatchedProblem &p);
size_t decode_mx_batched_workspace_bytes(const BatchedProblem &p);
hipError_t launch_decode_mx_batched(const BatchedProblem &p, void *workspace, hipStream_t st);

// Few-token path (2..16 tokens per pass), bf16 factors, ranks up to 64 (lords_decode_mx.hip); same
// workspace convention.
bool decode_mx_supported(const MatmulProblem &p);
size_t decode_mx_workspace_bytes(const MatmulProblem &p);
hipError_t launch_decode_mx(const MatmulProblem &p, void *workspace, hipStream_t st);

// Small-M path, ranks up to 128 contraction columns (lords_decode.hip).  The workspace holds
// the arrival tickets (zero when handed over, left at zero) followed by fp32 partial sums.
bool decode_fast_supported(const MatmulProblem &p);
size_t decode_fast_workspace_bytes(const MatmulProblem &p);
hipError_t launch_decode_fast(const MatmulProblem &p, void *workspace, hipStream_t st);

// Small-M path for any rank (lords_fused.hip): K split over workgroups, partial sums added
// by a second kernel.  `workspace` must hold decode_workspace_bytes(p) bytes.
size_t decode_workspace_bytes(const MatmulProblem &p);
hipError_t launch_decode(const MatmulProblem &p, void *workspace, hipStream_t st);
// MFMA GEMM path for large M: bf16 factors up to 128 rank columns (lords_prefill.hip) ...
bool prefill_fast_supported(const MatmulProblem &p);
// Scratch the kernel would like for the parts of tiles that two or more workgroups share (at most `limit`; with
// less it plans for less, down to 0 = one whole tile per workgroup), and the launch: `part`/`part_bytes` that
// scratch, `zeroed` kZeroBytes of device memory that are zero when handed over and left at zero.
size_t prefill_fast_workspace_bytes(const MatmulProblem &p, size_t limit);
hipError_t launch_prefill_fast(const MatmulProblem &p, void *part, size_t part_bytes, void *zeroed, hipStream_t st);
// ... and the general variant (fp32 factors, any rank; lords_fused.hip).
hipError_t launch_prefill(const MatmulProblem &p, hipStream_t st);

}  // namespace lords

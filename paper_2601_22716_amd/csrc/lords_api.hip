// C ABI of the library (include/lords.h): argument checks, path choice, launches.
// No arithmetic of the method lives here.
#include "../../include/lords.h"
#include "lords_launch.h"

#include <mutex>

namespace lords {
bool fused_rank_supported(int r, bool f32fact);
}

namespace {

constexpr int kVersion = 100;   // 0.1.0
constexpr int kMaxDevices = 16;

// Per-device fp32 workspace for the split-K partial sums of the small-M path.
// Grown on demand, never shrunk, released only at process exit by the runtime.
struct Workspace {
    void *ptr = nullptr;
    size_t bytes = 0;
};
Workspace g_ws[kMaxDevices];
std::mutex g_ws_mutex;

int get_workspace(size_t need, void **out)
{
    *out = nullptr;
    if (need == 0) return LORDS_OK;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LORDS_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    Workspace &w = g_ws[dev];
    if (w.bytes < need) {
        // Work already queued may still read the old buffer: wait for it before freeing.
        if (w.ptr) {
            if (hipDeviceSynchronize() != hipSuccess) return LORDS_ERR_LAUNCH;
            (void)hipFree(w.ptr);
            w.ptr = nullptr;
            w.bytes = 0;
        }
        size_t want = need < (size_t)(8u << 20) ? (size_t)(8u << 20) : need;
        if (hipMalloc(&w.ptr, want) != hipSuccess) { w.ptr = nullptr; return LORDS_ERR_LAUNCH; }
        // arrival tickets at the front of the buffer must start at zero; kernels leave them at zero
        if (hipMemset(w.ptr, 0, want) != hipSuccess || hipDeviceSynchronize() != hipSuccess) return LORDS_ERR_LAUNCH;
        w.bytes = want;
    }
    *out = w.ptr;
    return LORDS_OK;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline bool bad_bits(int bits) { return bits != 2 && bits != 3 && bits != 4; }
inline bool bad_dtype(int d) { return d != LORDS_BF16 && d != LORDS_F32; }
inline bool bad_nk(int N, int K) { return N < 1 || K < 32 || (K % 32) != 0; }

}  // namespace

extern "C" {

int lords_version(void) { return kVersion; }

const char *lords_status_string(int status)
{
    switch (status) {
        case LORDS_OK: return "ok";
        case LORDS_ERR_NULL: return "a required pointer is NULL";
        case LORDS_ERR_BITS: return "bits must be 2, 3 or 4";
        case LORDS_ERR_SHAPE: return "bad shape: need N >= 1, r >= 1, M >= 0, K a positive multiple of 32";
        case LORDS_ERR_ALIGN: return "a pointer is not 16-byte aligned";
        case LORDS_ERR_DTYPE: return "unknown dtype or path value";
        case LORDS_ERR_LAUNCH: return "the HIP runtime refused a launch or an allocation";
        case LORDS_ERR_UNSUPPORTED: return "this shape is not supported by the requested path";
        default: return "unknown status";
    }
}

size_t lords_row_bytes(int K, int bits)
{
    if (bad_bits(bits) || K < 32 || (K % 32) != 0) return 0;
    return (size_t)K / 8 * (size_t)bits;
}

long lords_equivalent_rank(long N, long K, long group)
{
    if (N < 1 || K < 1 || group < 1) return -1;
    const long long num = (long long)N * (long long)K;
    const long long den = (long long)group * ((long long)N + (long long)K);
    return (long)(num / den);
}

int lords_unpack(const void *codes, uint8_t *idx, int N, int K, int bits, void *stream)
{
    if (!codes || !idx) return LORDS_ERR_NULL;
    if (bad_bits(bits)) return LORDS_ERR_BITS;
    if (bad_nk(N, K)) return LORDS_ERR_SHAPE;
    if (misaligned(codes) || misaligned(idx)) return LORDS_ERR_ALIGN;
    return lords::launch_unpack(codes, idx, N, K, bits, (hipStream_t)stream) == hipSuccess ? LORDS_OK : LORDS_ERR_LAUNCH;
}

int lords_dequant(const void *codes, const float *codebook, const void *B, const void *A, void *W,
                  int N, int K, int r, int bits, lords_dtype factor_dtype, lords_dtype w_dtype, void *stream)
{
    if (!codes || !codebook || !B || !A || !W) return LORDS_ERR_NULL;
    if (bad_bits(bits)) return LORDS_ERR_BITS;
    if (bad_nk(N, K) || r < 1) return LORDS_ERR_SHAPE;
    if (misaligned(codes) || misaligned(codebook) || misaligned(B) || misaligned(A) || misaligned(W)) return LORDS_ERR_ALIGN;
    if (bad_dtype((int)factor_dtype) || bad_dtype((int)w_dtype)) return LORDS_ERR_DTYPE;
    return lords::launch_dequant(codes, codebook, B, A, W, N, K, r, bits, factor_dtype == LORDS_F32,
                                 w_dtype == LORDS_F32, (hipStream_t)stream) == hipSuccess ? LORDS_OK : LORDS_ERR_LAUNCH;
}

int lords_quantize(const void *W, const float *codebook, const void *B, const void *A, void *codes,
                   int N, int K, int r, int bits, lords_dtype w_dtype, lords_dtype factor_dtype, void *stream)
{
    if (!W || !codebook || !B || !A || !codes) return LORDS_ERR_NULL;
    if (bad_bits(bits)) return LORDS_ERR_BITS;
    if (bad_nk(N, K) || r < 1) return LORDS_ERR_SHAPE;
    if (misaligned(W) || misaligned(codebook) || misaligned(B) || misaligned(A) || misaligned(codes)) return LORDS_ERR_ALIGN;
    if (bad_dtype((int)w_dtype) || bad_dtype((int)factor_dtype)) return LORDS_ERR_DTYPE;
    return lords::launch_quantize(W, codebook, B, A, codes, N, K, r, bits, w_dtype == LORDS_F32,
                                  factor_dtype == LORDS_F32, (hipStream_t)stream) == hipSuccess ? LORDS_OK : LORDS_ERR_LAUNCH;
}

int lords_block_init(const void *W, const float *codebook, void *B, void *A,
                     int N, int K, int r, int bits, lords_dtype w_dtype, lords_dtype factor_dtype, void *stream)
{
    if (!W || !codebook || !B || !A) return LORDS_ERR_NULL;
    if (bad_bits(bits)) return LORDS_ERR_BITS;
    if (bad_nk(N, K) || r < 1 || (K % r) != 0) return LORDS_ERR_SHAPE;
    if (misaligned(W) || misaligned(codebook) || misaligned(B) || misaligned(A)) return LORDS_ERR_ALIGN;
    if (bad_dtype((int)w_dtype) || bad_dtype((int)factor_dtype)) return LORDS_ERR_DTYPE;
    return lords::launch_block_init(W, codebook, B, A, N, K, r, bits, w_dtype == LORDS_F32,
                                    factor_dtype == LORDS_F32, (hipStream_t)stream) == hipSuccess ? LORDS_OK : LORDS_ERR_LAUNCH;
}

int lords_matmul_ex(const void *X, const void *codes, const float *codebook, const void *B, const void *A, void *Y,
                    int M, int N, int K, int r, int bits, lords_dtype factor_dtype, lords_dtype y_dtype,
                    void *stream, lords_path path)
{
    if (!X || !codes || !codebook || !B || !A || !Y) return LORDS_ERR_NULL;
    if (bad_bits(bits)) return LORDS_ERR_BITS;
    if (bad_nk(N, K) || r < 1 || M < 0) return LORDS_ERR_SHAPE;
    if (misaligned(X) || misaligned(codes) || misaligned(codebook) || misaligned(B) || misaligned(A) || misaligned(Y))
        return LORDS_ERR_ALIGN;
    if (bad_dtype((int)factor_dtype) || bad_dtype((int)y_dtype)) return LORDS_ERR_DTYPE;
    if (path != LORDS_PATH_AUTO && path != LORDS_PATH_DECODE && path != LORDS_PATH_PREFILL) return LORDS_ERR_DTYPE;
    if (M == 0) return LORDS_OK;
    const bool f32fact = factor_dtype == LORDS_F32;
    if (!lords::fused_rank_supported(r, f32fact)) return LORDS_ERR_UNSUPPORTED;

    lords::MatmulProblem p{X, codes, codebook, B, A, Y, M, N, K, r, bits, f32fact, y_dtype == LORDS_F32};
    if (path == LORDS_PATH_AUTO) path = (M <= 32) ? LORDS_PATH_DECODE : LORDS_PATH_PREFILL;   // measured cross-over
    hipError_t e;
    if (path == LORDS_PATH_DECODE) {
        void *ws = nullptr;
        const bool one = lords::decode_m1_supported(p);
        const bool few = !one && M > 1 && lords::decode_mx_supported(p);
        const bool fast = !one && !few && lords::decode_fast_supported(p);
        const size_t need = one ? lords::decode_m1_workspace_bytes(p)
                          : few ? lords::decode_mx_workspace_bytes(p)
                          : fast ? lords::decode_fast_workspace_bytes(p)
                                 : lords::kTicketBytes + lords::decode_workspace_bytes(p);
        const int rc = get_workspace(need, &ws);
        if (rc != LORDS_OK) return rc;
        if (one) e = lords::launch_decode_m1(p, ws, (hipStream_t)stream);
        else if (few) e = lords::launch_decode_mx(p, ws, (hipStream_t)stream);
        else if (fast) e = lords::launch_decode_fast(p, ws, (hipStream_t)stream);
        else e = lords::launch_decode(p, ws ? (unsigned char *)ws + lords::kTicketBytes : nullptr, (hipStream_t)stream);
    } else {
        e = lords::prefill_fast_supported(p) ? lords::launch_prefill_fast(p, (hipStream_t)stream)
                                             : lords::launch_prefill(p, (hipStream_t)stream);
    }
    return e == hipSuccess ? LORDS_OK : LORDS_ERR_LAUNCH;
}

int lords_matmul(const void *X, const void *codes, const float *codebook, const void *B, const void *A, void *Y,
                 int M, int N, int K, int r, int bits, lords_dtype factor_dtype, lords_dtype y_dtype, void *stream)
{
    return lords_matmul_ex(X, codes, codebook, B, A, Y, M, N, K, r, bits, factor_dtype, y_dtype, stream, LORDS_PATH_AUTO);
}

}  // extern "C"

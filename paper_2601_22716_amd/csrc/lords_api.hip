// C ABI of the library (include/lords.h): argument checks, path choice, launches.
// No arithmetic of the method lives here.
#include "../../include/lords.h"
#include "lords_launch.h"

#include <mutex>

namespace lords {
bool fused_rank_supported(int r, bool f32fact);
}

namespace {

constexpr int kVersion = 200;   // 0.2.0
constexpr int kMaxDevices = 16;

// Layout of a workspace, the library's own or a caller's:
//   [0, kZeroBytes)                         exchange slots of the one-/two-token kernel   } zero when handed over,
//   [kZeroBytes, kZeroBytes + kTicketBytes) arrival tickets of the few-token kernels      } left at zero by every call
//   [kFront, ...)                           fp32 partial sums and other scratch, contents of no interest between calls
constexpr size_t kFront = lords::kZeroBytes + lords::kTicketBytes;

struct WsView {
    unsigned char *base = nullptr;     // start of the zero region
    size_t bytes = 0;
    void *zeroed() const { return base; }
    void *tickets() const { return base ? base + lords::kZeroBytes : nullptr; }    // what the few-token kernels call "workspace"
    void *scratch() const { return base ? base + kFront : nullptr; }
};

// The library's own per-device workspace (convenience entry points).  A block that has been handed
// out is never freed or moved: work already queued, and HIP graphs captured earlier, keep using it.
// When a call needs more, a new block is allocated (and its front zeroed, which waits for the
// device); while the stream is being captured that is refused instead.
struct OwnWorkspace {
    unsigned char *ptr = nullptr;
    size_t bytes = 0;
};
OwnWorkspace g_ws[kMaxDevices];
std::mutex g_ws_mutex;

int get_workspace(size_t need, void *stream, WsView *out)
{
    *out = WsView{};
    if (need < kFront) need = kFront;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LORDS_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    OwnWorkspace &w = g_ws[dev];
    if (w.bytes < need) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing((hipStream_t)stream, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return LORDS_ERR_LAUNCH;
        size_t want = need < (size_t)(16u << 20) ? (size_t)(16u << 20) : need + need / 2;
        unsigned char *fresh = nullptr;
        if (hipMalloc((void **)&fresh, want) != hipSuccess) return LORDS_ERR_LAUNCH;
        if (hipMemset(fresh, 0, kFront) != hipSuccess || hipDeviceSynchronize() != hipSuccess) return LORDS_ERR_LAUNCH;
        w.ptr = fresh;          // (the previous block stays allocated: it may still be in use)
        w.bytes = want;
    }
    out->base = w.ptr;
    out->bytes = w.bytes;
    return LORDS_OK;
}

// One token: the regrouped kernel of lords_gemv.hip wherever it takes the shape.  Two tokens: the same,
// except at ranks above 32 on layers above 32 M weights with at least as many rows as columns, where the
// few-token kernel measured faster (us, regrouped / few-token: 14336 x 4096 rank 48 20.9 / 19.6,
// 28672 x 8192 rank 64 85 / 66; against 14336 x 4096 rank 32 14.7 / 15.4, 4096 x 14336 rank 32 16.7 / 17.8,
// rank 48 22.3 / 24.6, 4096 x 4096 8.3 / 10.2, 6144 x 4096 10.1 / 11.1).
bool use_gemv(const lords::MatmulProblem &p, lords_path path)
{
    if (path == LORDS_PATH_SMALLM) return false;
    if (path == LORDS_PATH_GEMV) return lords::decode_gemv_supported(p);
    if (p.M == 2 && p.r > 32 && (long)p.N * p.K > (32L << 20) && p.N >= p.K) return false;
    return lords::decode_gemv_supported(p);
}

// Which few-token kernel takes a problem, and the scratch it asks for behind the tickets.
enum DecodeKind { kFew, kFast, kGeneral };
DecodeKind decode_kind(const lords::MatmulProblem &p)
{
    if (p.M > 1 && lords::decode_mx_supported(p)) return kFew;
    if (lords::decode_fast_supported(p)) return kFast;
    return kGeneral;
}
size_t decode_scratch(const lords::MatmulProblem &p)
{
    size_t with_tickets;
    switch (decode_kind(p)) {
        case kFew: with_tickets = lords::decode_mx_workspace_bytes(p); break;
        case kFast: with_tickets = lords::decode_fast_workspace_bytes(p); break;
        default: return lords::decode_workspace_bytes(p);
    }
    return with_tickets > lords::kTicketBytes ? with_tickets - lords::kTicketBytes : 0;
}
inline bool is_decode(lords_path path) { return path == LORDS_PATH_DECODE || path == LORDS_PATH_GEMV || path == LORDS_PATH_SMALLM; }
// Measured cross-over.  Up to 16 tokens the few-token kernels win (28672 x 8192, rank 64: 68 / 80 us at
// 8 / 16 tokens against 87-90 us for the large-M kernel; 4096 x 14336, rank 48: 25 / 31 us against 50 us),
// except at ranks 65..128, which the few-token family serves with its oldest kernel: there the large-M
// kernel wins from two tokens on (28672 x 8192, rank 128: 219 against 117 us at two tokens, 235 against
// 117 us at eight; 14336 x 4096: 71 against 48 us at two; one token: 124 against 117 us and 42 against 48 us).
inline lords_path resolve_path(lords_path path, const lords::MatmulProblem &p)
{
    if (path != LORDS_PATH_AUTO) return path;
    if (p.M > 16) return LORDS_PATH_PREFILL;
    if (p.M >= 2 && p.r > 64 && lords::prefill_fast_supported(p)) return LORDS_PATH_PREFILL;
    return LORDS_PATH_DECODE;
}

// Bytes of workspace (front included) one checked problem needs on `path` (already resolved).  The
// large-M kernel takes what it is given: with `limit` bytes or more it shares tiles between
// workgroups, with less it falls back to whole tiles and needs none.
constexpr size_t kNoLimit = ~(size_t)0;
size_t matmul_need(const lords::MatmulProblem &p, lords_path path, size_t limit = kNoLimit)
{
    size_t scratch = 0;
    if (is_decode(path)) scratch = use_gemv(p, path) ? 0 : decode_scratch(p);
    else if (lords::prefill_fast_supported(p)) scratch = lords::prefill_fast_workspace_bytes(p, limit > kFront ? limit - kFront : 0);
    return kFront + ((scratch + 255) & ~(size_t)255);
}

int launch_matmul(const lords::MatmulProblem &p, lords_path path, const WsView &ws, void *stream)
{
    hipError_t e;
    if (is_decode(path)) {
        if (use_gemv(p, path)) e = lords::launch_decode_gemv(p, ws.zeroed(), (hipStream_t)stream);
        else if (path == LORDS_PATH_GEMV) return LORDS_ERR_UNSUPPORTED;
        else switch (decode_kind(p)) {
            case kFew: e = lords::launch_decode_mx(p, ws.tickets(), (hipStream_t)stream); break;
            case kFast: e = lords::launch_decode_fast(p, ws.tickets(), (hipStream_t)stream); break;
            default: e = lords::launch_decode(p, ws.scratch(), (hipStream_t)stream);
        }
    } else {
        e = lords::prefill_fast_supported(p)
                ? lords::launch_prefill_fast(p, ws.scratch(), ws.bytes > kFront ? ws.bytes - kFront : 0, ws.zeroed(), (hipStream_t)stream)
                : lords::launch_prefill(p, (hipStream_t)stream);
    }
    return e == hipSuccess ? LORDS_OK : LORDS_ERR_LAUNCH;
}

// Workspace for one checked problem on `path` (already resolved), plus `extra` bytes behind it that
// are left to the caller (*extra_ptr).
int plan_workspace(const lords::MatmulProblem &p, lords_path path, size_t extra, void *stream, WsView *ws, void **extra_ptr)
{
    const size_t own = matmul_need(p, path);
    const int rc = get_workspace(own + extra, stream, ws);
    if (rc == LORDS_OK && extra_ptr) *extra_ptr = ws->base + own;
    return rc;
}

int run_matmul(const lords::MatmulProblem &p, lords_path path, void *stream)
{
    path = resolve_path(path, p);
    if (path == LORDS_PATH_GEMV && !use_gemv(p, path)) return LORDS_ERR_UNSUPPORTED;
    WsView ws;
    const int rc = plan_workspace(p, path, 0, stream, &ws, nullptr);
    return rc != LORDS_OK ? rc : launch_matmul(p, path, ws, stream);
}

// Several matrices in ONE launch, if a kernel takes the case: a status, or -1 if none does.
int run_batched(const lords::BatchedProblem &bp, void *stream)
{
    if (lords::decode_gemv_batched_supported(bp)) {
        WsView ws;
        const int rc = get_workspace(kFront, stream, &ws);
        if (rc != LORDS_OK) return rc;
        return lords::launch_decode_gemv_batched(bp, ws.zeroed(), (hipStream_t)stream) == hipSuccess ? LORDS_OK : LORDS_ERR_LAUNCH;
    }
    if (!lords::decode_mx_batched_supported(bp)) return -1;
    WsView ws;
    const int rc = get_workspace(lords::kZeroBytes + lords::decode_mx_batched_workspace_bytes(bp), stream, &ws);
    if (rc != LORDS_OK) return rc;
    return lords::launch_decode_mx_batched(bp, ws.tickets(), (hipStream_t)stream) == hipSuccess ? LORDS_OK : LORDS_ERR_LAUNCH;
}

// ---- the entry point that allocates nothing: its scratch is this array, one copy per GPU ----
constexpr size_t kStaticBytes = (size_t)24 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];
unsigned char *g_static_ptr[kMaxDevices] = {};
std::mutex g_static_mutex;

int static_workspace(WsView *out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LORDS_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        // the array's name is a host-side stand-in: its device address on THIS GPU is asked for once
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LORDS_ERR_LAUNCH;
        g_static_ptr[dev] = (unsigned char *)ptr;
    }
    out->base = g_static_ptr[dev];
    out->bytes = kStaticBytes;
    return LORDS_OK;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline bool bad_bits(int bits) { return bits != 2 && bits != 3 && bits != 4; }
inline bool bad_dtype(int d) { return d != LORDS_BF16 && d != LORDS_F32; }
inline bool bad_nk(int N, int K) { return N < 1 || K < 32 || (K % 32) != 0; }
inline bool bad_path(int p) { return p < LORDS_PATH_AUTO || p > LORDS_PATH_SMALLM; }

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
        case LORDS_ERR_WORKSPACE: return "the workspace is missing or too small";
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

int lords_mixed_schedule(int n_layers, double fraction_first, int bits_first, int bits_rest,
                         int *layer_bits, double *avg_bits)
{
    if (!layer_bits) return LORDS_ERR_NULL;
    if (bad_bits(bits_first) || bad_bits(bits_rest)) return LORDS_ERR_BITS;
    if (n_layers < 1 || !(fraction_first >= 0.0)) return LORDS_ERR_SHAPE;
    const double x = fraction_first * (double)n_layers + 0.5;
    const int n_first = x >= (double)n_layers ? n_layers : (int)x;      // x >= 0: truncation is the floor
    long sum = 0;
    for (int l = 0; l < n_layers; ++l) {
        layer_bits[l] = l < n_first ? bits_first : bits_rest;
        sum += layer_bits[l];
    }
    if (avg_bits) *avg_bits = (double)sum / (double)n_layers;
    return LORDS_OK;
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
    if (bad_path((int)path)) return LORDS_ERR_DTYPE;
    if (M == 0) return LORDS_OK;
    const bool f32fact = factor_dtype == LORDS_F32;
    if (!lords::fused_rank_supported(r, f32fact)) return LORDS_ERR_UNSUPPORTED;

    lords::MatmulProblem p{X, codes, codebook, B, A, Y, M, N, K, r, bits, f32fact, y_dtype == LORDS_F32};
    return run_matmul(p, path, stream);
}

size_t lords_workspace_zero_bytes(void) { return kFront; }

size_t lords_workspace_bytes(int M, int N, int K, int r, int bits, lords_dtype factor_dtype, lords_path path)
{
    if (bad_bits(bits) || bad_nk(N, K) || r < 1 || M < 0 || bad_dtype((int)factor_dtype) || bad_path((int)path)) return 0;
    const bool f32fact = factor_dtype == LORDS_F32;
    if (!lords::fused_rank_supported(r, f32fact)) return 0;
    if (M == 0) return kFront;
    lords::MatmulProblem p{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, M, N, K, r, bits, f32fact, true};
    return matmul_need(p, resolve_path(path, p));
}

namespace {
int matmul_in(const void *X, const void *codes, const float *codebook, const void *B, const void *A, void *Y,
              int M, int N, int K, int r, int bits, lords_dtype factor_dtype, lords_dtype y_dtype, void *stream,
              lords_path path, const WsView &ws, bool ws_given, bool tiled = false)
{
    if (!X || !codes || !codebook || !B || !A || !Y) return LORDS_ERR_NULL;
    if (bad_bits(bits)) return LORDS_ERR_BITS;
    if (bad_nk(N, K) || r < 1 || M < 0) return LORDS_ERR_SHAPE;
    if (misaligned(X) || misaligned(codes) || misaligned(codebook) || misaligned(B) || misaligned(A) || misaligned(Y))
        return LORDS_ERR_ALIGN;
    if (ws_given && (reinterpret_cast<uintptr_t>(ws.base) & 255u) != 0) return LORDS_ERR_ALIGN;
    if (bad_dtype((int)factor_dtype) || bad_dtype((int)y_dtype)) return LORDS_ERR_DTYPE;
    if (bad_path((int)path)) return LORDS_ERR_DTYPE;
    if (M == 0) return LORDS_OK;
    const bool f32fact = factor_dtype == LORDS_F32;
    if (!lords::fused_rank_supported(r, f32fact)) return LORDS_ERR_UNSUPPORTED;
    lords::MatmulProblem p{X, codes, codebook, B, A, Y, M, N, K, r, bits, f32fact, y_dtype == LORDS_F32};
    p.tiled = tiled;
    path = resolve_path(path, p);
    if (path == LORDS_PATH_GEMV && !use_gemv(p, path)) return LORDS_ERR_UNSUPPORTED;
    if (tiled) {
        // the slab-tile layout is read by the one-/two-token, the few-token and the large-M kernel only
        const bool ok = is_decode(path) ? (use_gemv(p, path) || decode_kind(p) == kFew) : lords::prefill_fast_supported(p);
        if (!ok) return LORDS_ERR_UNSUPPORTED;
    }
    // (a caller's workspace must have the size the query gives; the static one is used as far as it goes)
    if (!ws.base || ws.bytes < matmul_need(p, path, ws_given ? kNoLimit : ws.bytes)) return LORDS_ERR_WORKSPACE;
    return launch_matmul(p, path, ws, stream);
}
}  // namespace

int lords_matmul_ws(const void *X, const void *codes, const float *codebook, const void *B, const void *A, void *Y,
                    int M, int N, int K, int r, int bits, lords_dtype factor_dtype, lords_dtype y_dtype,
                    void *stream, lords_path path, void *workspace, size_t workspace_bytes)
{
    WsView ws;
    ws.base = (unsigned char *)workspace;
    ws.bytes = workspace_bytes;
    return matmul_in(X, codes, codebook, B, A, Y, M, N, K, r, bits, factor_dtype, y_dtype, stream, path, ws, true);
}

size_t lords_repack_bytes(int N, int K, int bits)
{
    if (bad_bits(bits) || bad_nk(N, K)) return 0;
    return (size_t)((N + 15) / 16) * (size_t)((K + 127) / 128) * 256u * (size_t)bits;
}

int lords_repack(const void *codes, void *codes_tiled, int N, int K, int bits, void *stream)
{
    if (!codes || !codes_tiled) return LORDS_ERR_NULL;
    if (bad_bits(bits)) return LORDS_ERR_BITS;
    if (bad_nk(N, K)) return LORDS_ERR_SHAPE;
    if (misaligned(codes) || misaligned(codes_tiled)) return LORDS_ERR_ALIGN;
    return lords::launch_repack(codes, codes_tiled, N, K, bits, (hipStream_t)stream) == hipSuccess ? LORDS_OK : LORDS_ERR_LAUNCH;
}

int lords_matmul_repacked(const void *X, const void *codes_tiled, const float *codebook, const void *B, const void *A, void *Y,
                          int M, int N, int K, int r, int bits, lords_dtype factor_dtype, lords_dtype y_dtype,
                          void *stream, lords_path path)
{
    // argument checks first (no workspace is touched for a bad call), then the library's own workspace
    WsView none;
    const int rc0 = matmul_in(X, codes_tiled, codebook, B, A, Y, M, N, K, r, bits, factor_dtype, y_dtype, stream, path, none, false, true);
    if (rc0 != LORDS_ERR_WORKSPACE) return rc0;          // LORDS_OK only for M == 0
    const bool f32fact = factor_dtype == LORDS_F32;
    lords::MatmulProblem p{X, codes_tiled, codebook, B, A, Y, M, N, K, r, bits, f32fact, y_dtype == LORDS_F32};
    p.tiled = true;
    WsView ws;
    const int rc = plan_workspace(p, resolve_path(path, p), 0, stream, &ws, nullptr);
    if (rc != LORDS_OK) return rc;
    return matmul_in(X, codes_tiled, codebook, B, A, Y, M, N, K, r, bits, factor_dtype, y_dtype, stream, path, ws, false, true);
}

size_t lords_noalloc_limit(void) { return kStaticBytes; }

int lords_matmul_noalloc(const void *X, const void *codes, const float *codebook, const void *B, const void *A, void *Y,
                         int M, int N, int K, int r, int bits, lords_dtype factor_dtype, lords_dtype y_dtype, void *stream)
{
    WsView ws;
    const int rc = static_workspace(&ws);
    if (rc != LORDS_OK) return rc;
    return matmul_in(X, codes, codebook, B, A, Y, M, N, K, r, bits, factor_dtype, y_dtype, stream, LORDS_PATH_AUTO, ws, false);
}

int lords_matmul_batched(const void *X, const void *const *codes, const float *codebook, const void *const *B,
                         const void *const *A, void *const *Y, const int *N, int L, int M, int K, int r, int bits,
                         lords_dtype factor_dtype, lords_dtype y_dtype, void *stream)
{
    if (!X || !codes || !codebook || !B || !A || !Y || !N) return LORDS_ERR_NULL;
    if (L < 1 || L > lords::kMaxBatch) return LORDS_ERR_SHAPE;
    for (int l = 0; l < L; ++l)
        if (!codes[l] || !B[l] || !A[l] || !Y[l]) return LORDS_ERR_NULL;
    if (bad_bits(bits)) return LORDS_ERR_BITS;
    if (K < 32 || (K % 32) != 0 || r < 1 || M < 0) return LORDS_ERR_SHAPE;
    for (int l = 0; l < L; ++l)
        if (N[l] < 1) return LORDS_ERR_SHAPE;
    if (misaligned(X) || misaligned(codebook)) return LORDS_ERR_ALIGN;
    for (int l = 0; l < L; ++l)
        if (misaligned(codes[l]) || misaligned(B[l]) || misaligned(A[l]) || misaligned(Y[l])) return LORDS_ERR_ALIGN;
    if (bad_dtype((int)factor_dtype) || bad_dtype((int)y_dtype)) return LORDS_ERR_DTYPE;
    if (M == 0) return LORDS_OK;
    const bool f32fact = factor_dtype == LORDS_F32;
    if (!lords::fused_rank_supported(r, f32fact)) return LORDS_ERR_UNSUPPORTED;

    lords::BatchedProblem bp;
    bp.X = X; bp.codebook = codebook;
    for (int l = 0; l < lords::kMaxBatch; ++l) {
        const int s = l < L ? l : 0;
        bp.codes[l] = codes[s]; bp.B[l] = B[s]; bp.A[l] = A[s]; bp.Y[l] = Y[s]; bp.N[l] = N[s];
    }
    bp.L = L; bp.M = M; bp.K = K; bp.r = r; bp.bits = bits;
    bp.f32fact = f32fact; bp.f32out = y_dtype == LORDS_F32; bp.act = false;
    if (L > 1) {
        const int rc = run_batched(bp, stream);
        if (rc >= 0) return rc;
    }
    // more than one token (or a case the one-launch kernel does not take): matrix by matrix
    for (int l = 0; l < L; ++l) {
        lords::MatmulProblem p{X, codes[l], codebook, B[l], A[l], Y[l], M, N[l], K, r, bits, f32fact, y_dtype == LORDS_F32};
        const int rc = run_matmul(p, LORDS_PATH_AUTO, stream);
        if (rc != LORDS_OK) return rc;
    }
    return LORDS_OK;
}

int lords_gate_up(const void *X, const void *codes_gate, const void *B_gate, const void *A_gate,
                  const void *codes_up, const void *B_up, const void *A_up, const float *codebook, void *H,
                  int M, int N, int K, int r, int bits, lords_dtype factor_dtype, lords_dtype h_dtype, void *stream)
{
    if (!X || !codes_gate || !B_gate || !A_gate || !codes_up || !B_up || !A_up || !codebook || !H) return LORDS_ERR_NULL;
    if (bad_bits(bits)) return LORDS_ERR_BITS;
    if (bad_nk(N, K) || r < 1 || M < 0) return LORDS_ERR_SHAPE;
    if (misaligned(X) || misaligned(codes_gate) || misaligned(B_gate) || misaligned(A_gate) || misaligned(codes_up) ||
        misaligned(B_up) || misaligned(A_up) || misaligned(codebook) || misaligned(H))
        return LORDS_ERR_ALIGN;
    if (bad_dtype((int)factor_dtype) || bad_dtype((int)h_dtype)) return LORDS_ERR_DTYPE;
    if (M == 0) return LORDS_OK;
    const bool f32fact = factor_dtype == LORDS_F32, f32out = h_dtype == LORDS_F32;
    if (!lords::fused_rank_supported(r, f32fact)) return LORDS_ERR_UNSUPPORTED;

    lords::BatchedProblem bp;
    bp.X = X; bp.codebook = codebook;
    for (int l = 0; l < lords::kMaxBatch; ++l) {
        const bool up = l == 1;
        bp.codes[l] = up ? codes_up : codes_gate; bp.B[l] = up ? B_up : B_gate; bp.A[l] = up ? A_up : A_gate;
        bp.Y[l] = H; bp.N[l] = N;
    }
    bp.L = 2; bp.M = M; bp.K = K; bp.r = r; bp.bits = bits;
    bp.f32fact = f32fact; bp.f32out = f32out; bp.act = true;
    {
        const int rc = run_batched(bp, stream);
        if (rc >= 0) return rc;
    }
    // Otherwise: both products in fp32 into the workspace, at most kChunk tokens at a time, then one
    // element-wise pass.  The arithmetic is the same: fp32 sums, silu(gate) * up in fp32, one rounding.
    constexpr int kChunk = 1024;
    const size_t esz = f32out ? 4 : 2;
    for (int m0 = 0; m0 < M; m0 += kChunk) {
        const int mc = M - m0 < kChunk ? M - m0 : kChunk;
        const size_t tmp_bytes = (size_t)2 * mc * N * sizeof(float);
        const void *Xc = (const unsigned char *)X + (size_t)m0 * K * 2;
        lords::MatmulProblem pg{Xc, codes_gate, codebook, B_gate, A_gate, nullptr, mc, N, K, r, bits, f32fact, true};
        const lords_path path = resolve_path(LORDS_PATH_AUTO, pg);
        WsView ws;
        void *tmp = nullptr;
        int rc = plan_workspace(pg, path, tmp_bytes, stream, &ws, &tmp);
        if (rc != LORDS_OK) return rc;
        float *G = (float *)tmp, *U = G + (size_t)mc * N;
        pg.Y = G;
        lords::MatmulProblem pu{Xc, codes_up, codebook, B_up, A_up, U, mc, N, K, r, bits, f32fact, true};
        rc = launch_matmul(pg, path, ws, stream);
        if (rc != LORDS_OK) return rc;
        rc = launch_matmul(pu, path, ws, stream);
        if (rc != LORDS_OK) return rc;
        if (lords::launch_silu_mul(G, U, (unsigned char *)H + (size_t)m0 * N * esz, (long)mc * N, f32out,
                                   (hipStream_t)stream) != hipSuccess)
            return LORDS_ERR_LAUNCH;
    }
    return LORDS_OK;
}

int lords_transpose_codes(const void *codes, void *codes_t, int N, int K, int bits, void *stream)
{
    if (!codes || !codes_t) return LORDS_ERR_NULL;
    if (bad_bits(bits)) return LORDS_ERR_BITS;
    if (bad_nk(N, K) || (N % 32) != 0) return LORDS_ERR_SHAPE;
    if (misaligned(codes) || misaligned(codes_t)) return LORDS_ERR_ALIGN;
    return lords::launch_transpose_codes(codes, codes_t, N, K, bits, (hipStream_t)stream) == hipSuccess ? LORDS_OK : LORDS_ERR_LAUNCH;
}

int lords_backward_input(const void *dY, const void *codes_t, const float *codebook, const void *B, const void *A, void *dX,
                         int M, int N, int K, int r, int bits, lords_dtype factor_dtype, lords_dtype dx_dtype, void *stream)
{
    if (!dY || !codes_t || !codebook || !B || !A || !dX) return LORDS_ERR_NULL;
    if (bad_bits(bits)) return LORDS_ERR_BITS;
    if (bad_nk(N, K) || (N % 32) != 0 || r < 1 || M < 0) return LORDS_ERR_SHAPE;
    if (misaligned(dY) || misaligned(codes_t) || misaligned(codebook) || misaligned(B) || misaligned(A) || misaligned(dX))
        return LORDS_ERR_ALIGN;
    if (bad_dtype((int)factor_dtype) || bad_dtype((int)dx_dtype)) return LORDS_ERR_DTYPE;
    if (M == 0) return LORDS_OK;
    const bool f32fact = factor_dtype == LORDS_F32;
    if (!lords::fused_rank_supported(r, f32fact)) return LORDS_ERR_UNSUPPORTED;
    // The transposed layer: rows = the K in-features, columns = the N out-features, factors A^T (K x r)
    // and B^T (r x N); its forward product applied to dY is dX.
    const size_t esz = f32fact ? 4 : 2;
    const size_t at_bytes = ((size_t)K * r * esz + 255) & ~(size_t)255, bt_bytes = ((size_t)r * N * esz + 255) & ~(size_t)255;
    lords::MatmulProblem p{dY, codes_t, codebook, nullptr, nullptr, dX, M, K, N, r, bits, f32fact, dx_dtype == LORDS_F32};
    const lords_path path = resolve_path(LORDS_PATH_AUTO, p);
    WsView ws;
    void *extra = nullptr;
    const int rc = plan_workspace(p, path, at_bytes + bt_bytes, stream, &ws, &extra);
    if (rc != LORDS_OK) return rc;
    void *At = extra, *Bt = (unsigned char *)extra + at_bytes;
    if (lords::launch_transpose_factor(A, At, r, K, f32fact, (hipStream_t)stream) != hipSuccess) return LORDS_ERR_LAUNCH;
    if (lords::launch_transpose_factor(B, Bt, N, r, f32fact, (hipStream_t)stream) != hipSuccess) return LORDS_ERR_LAUNCH;
    p.B = At;
    p.A = Bt;
    return launch_matmul(p, path, ws, stream);
}

int lords_backward_factors(const void *dY, const void *X, const void *codes, const float *codebook, const void *B,
                           const void *A, float *dB, float *dA, int M, int N, int K, int r, int bits,
                           lords_dtype factor_dtype, void *stream)
{
    if (!dY || !X || !codes || !codebook || !B || !A || !dB || !dA) return LORDS_ERR_NULL;
    if (bad_bits(bits)) return LORDS_ERR_BITS;
    if (bad_nk(N, K) || r < 1 || M < 0) return LORDS_ERR_SHAPE;
    if (misaligned(dY) || misaligned(X) || misaligned(codes) || misaligned(codebook) || misaligned(B) || misaligned(A) ||
        misaligned(dB) || misaligned(dA))
        return LORDS_ERR_ALIGN;
    if (bad_dtype((int)factor_dtype)) return LORDS_ERR_DTYPE;
    if (!lords::factor_grad_supported(N, K, r)) return LORDS_ERR_UNSUPPORTED;
    WsView ws;
    const int rc = get_workspace(kFront + lords::factor_grad_workspace_bytes(N, K, r), stream, &ws);
    if (rc != LORDS_OK) return rc;
    return lords::launch_factor_grad(dY, X, codes, codebook, B, A, dB, dA, M, N, K, r, bits, factor_dtype == LORDS_F32,
                                     ws.scratch(), (hipStream_t)stream) == hipSuccess
               ? LORDS_OK : LORDS_ERR_LAUNCH;
}

int lords_matmul(const void *X, const void *codes, const float *codebook, const void *B, const void *A, void *Y,
                 int M, int N, int K, int r, int bits, lords_dtype factor_dtype, lords_dtype y_dtype, void *stream)
{
    return lords_matmul_ex(X, codes, codebook, B, A, Y, M, N, K, r, bits, factor_dtype, y_dtype, stream, LORDS_PATH_AUTO);
}

}  // extern "C"

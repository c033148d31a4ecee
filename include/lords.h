/*
 * lords.h -- C ABI of the MI355X (gfx950) LoRDS inference library.
 *
 * LoRDS ("low-rank decomposed scaling", arXiv 2601.22716) stores a weight matrix
 * W_hat (N out-features x K in-features) as
 *      W_hat = C[Q] (.) S ,   S = B A                         (Sec. 3.2 Eq. 3; Sec. 3.3)
 * where Q holds one k-bit level index per element (k = 2, 3 or 4), C is the
 * 2^k-entry look-up table of the target data type (Alg. 1, "Require"), and the
 * element-wise scale S is the product of the rank-r factors B (N x r) and
 * A (r x K).  S and W_hat are regenerated per tile inside the kernels and are
 * never written to device memory by lords_matmul.
 *
 * Conventions common to every entry point
 *  - Every data pointer is a DEVICE pointer owned by the caller, at least 16-byte
 *    aligned, to a dense row-major array.  The library neither keeps nor frees
 *    them.  `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *    Calls enqueue work on `stream` and return without synchronising.
 *  - Packed code rows: row n starts at byte n*K*bits/8; a row is a little-endian
 *    bit string (bit b of the row is bit b%8 of byte b/8) and code k occupies bits
 *    [bits*k, bits*k+bits).  4 bits: two codes per byte, low nibble first; 2 bits:
 *    four per byte from the low end; 3 bits: 32 codes per 12 bytes.
 *  - K must be a multiple of 32 (whole 12-byte groups at 3 bits, whole 16-byte
 *    loads at 4 bits).  N >= 1 and M >= 0 are otherwise arbitrary; ranks r >= 1 up to 6144 (bf16
 *    factors) or 2048 (fp32 factors) run (LORDS_ERR_UNSUPPORTED beyond).  Calls with further
 *    restrictions say so: lords_transpose_codes / lords_backward_input (N % 32 == 0),
 *    lords_backward_factors (N % 8 == 0, r <= 64), lords_block_init (K % r == 0).
 *  - The level table is narrowed to 16 bits inside the multiplying kernels (bf16 at one and two
 *    tokens, fp16 otherwise): levels must lie within fp16 range (|c| <= 65504, not below 6e-8
 *    unless zero); the tables of the paper (Sec. 3.1: INT4, NF4) are far inside it.
 *  - Factors B and A are both bf16 or both fp32 (`factor_dtype`); X is bf16.
 *  - Outputs are overwritten entirely (no accumulate).
 *  - Errors are returned, never thrown.  Arguments are checked in the fixed order
 *    NULL -> BITS -> SHAPE -> ALIGN -> DTYPE before anything is launched, so a bad
 *    call touches no memory.  A launch failure reported by the runtime gives
 *    LORDS_ERR_LAUNCH.
 *  - Workspace.  Some kernels meet through device memory (exchange slots, arrival tickets, fp32
 *    partial sums).  lords_matmul_ws takes that memory from the caller and then neither allocates,
 *    frees nor synchronises; lords_matmul_noalloc uses an array built into the library.  The other
 *    multiplying entry points (lords_matmul, lords_matmul_ex, lords_matmul_batched, lords_gate_up,
 *    lords_backward_*) use a per-device workspace of the library's own: allocated on first need;
 *    when a call needs more, a larger block is allocated (its front is zeroed, which waits for the
 *    device once) and the old one is kept, so that work already queued and HIP graphs captured
 *    earlier stay valid; it is released when the process ends.  Such a growth is refused with
 *    LORDS_ERR_LAUNCH while `stream` is being captured: warm a shape up once before capturing it.
 *    Calls that share one workspace and overlap in time on one device race; issue them from one
 *    stream (or give every stream its own workspace through lords_matmul_ws).  The library keeps no
 *    other state; entry points may be called from several host threads.
 */
#ifndef LORDS_H
#define LORDS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LORDS_OK = 0,
    LORDS_ERR_NULL = 1,    /* a required pointer is NULL */
    LORDS_ERR_BITS = 2,    /* bits is not 2, 3 or 4 */
    LORDS_ERR_SHAPE = 3,   /* N < 1, r < 1, M < 0, K < 32, K % 32 != 0, or a size overflows int */
    LORDS_ERR_ALIGN = 4,   /* a pointer is not 16-byte aligned */
    LORDS_ERR_DTYPE = 5,   /* unknown lords_dtype / lords_path value */
    LORDS_ERR_LAUNCH = 6,  /* the HIP runtime refused the launch or a workspace allocation */
    LORDS_ERR_UNSUPPORTED = 7, /* the forced path cannot run this shape */
    LORDS_ERR_WORKSPACE = 8   /* lords_matmul_ws / lords_matmul_noalloc: workspace missing or too small */
} lords_status;

typedef enum { LORDS_BF16 = 0, LORDS_F32 = 1 } lords_dtype;

/* Which kernel family lords_matmul_ex runs.  AUTO picks by M (up to 16 tokens: DECODE). */
typedef enum {
    LORDS_PATH_AUTO = 0,
    LORDS_PATH_DECODE = 1,   /* memory-bound small-M family, the kernel picked by M: GEMV where it applies, else SMALLM */
    LORDS_PATH_PREFILL = 2,  /* bf16 MFMA GEMM with the dequantised tile as operand */
    LORDS_PATH_MFMA = 2,     /* (the same) */
    LORDS_PATH_GEMV = 3,     /* the one-/two-token kernel alone: M <= 2, bf16 factors, rank <= 64,
                                LORDS_ERR_UNSUPPORTED otherwise */
    LORDS_PATH_SMALLM = 4    /* the few-token kernels alone (16 tokens per pass over the codes), any M */
} lords_path;

/* Library version: major*10000 + minor*100 + patch. */
int lords_version(void);

/* Static, NUL-terminated description of a lords_status value. */
const char *lords_status_string(int status);

/* Bytes of one packed row of K codes (K*bits/8); 0 if bits or K is invalid. */
size_t lords_row_bytes(int K, int bits);

/* Rank whose factor budget r(N+K) matches a block-wise scale budget NK/group:
 * floor(NK / (group (N+K)))  (Sec. 3.2; Appendix A, Table 7).  -1 on bad input. */
long lords_equivalent_rank(long N, long K, long group);

/* Code width of every layer of a mixed-precision stack (Sec. 4.2, ultra-low-bit setting; Table 3):
 * the first floor(fraction_first * n_layers + 1/2) layers use bits_first, the remaining ones
 * bits_rest.  With 4 and 2 bits, fractions 1/2, 1/4 and 1/8 give the 3-, 2.5- and 2.25-bit
 * configurations.  Host-side only: the widths are then passed, layer by layer, as the `bits` of
 * the other calls (the matrices of one lords_matmul_batched / lords_gate_up call belong to one
 * layer and share one width).
 *   layer_bits  out  host array of n_layers ints, caller-owned
 *   avg_bits    out  host, may be NULL: mean width over the layers (layers of equal size)
 * Errors: LORDS_ERR_NULL (layer_bits), LORDS_ERR_BITS (either width not 2, 3 or 4),
 * LORDS_ERR_SHAPE (n_layers < 1, fraction_first negative or not a number; fractions above 1
 * mean every layer). */
int lords_mixed_schedule(int n_layers, double fraction_first, int bits_first, int bits_rest,
                         int *layer_bits, double *avg_bits);

/* Bit-unpack only: idx[n*K + k] = code k of row n.  (The storage side of Q; Alg. 1's
 * quantised matrix holds one level per element.)
 *   codes  in   N x K*bits/8 bytes
 *   idx    out  N x K uint8
 */
int lords_unpack(const void *codes, uint8_t *idx, int N, int K, int bits, void *stream);

/* Dequantise: W[n*K + k] = codebook[q[n][k]] * sum_j B[n][j] A[j][k]
 * (W_hat = Q (.) (BA), Sec. 3.3; scale absorbed into dequantisation, Fig. 1b).
 *   codebook  in   2^bits fp32
 *   B, A      in   N x r and r x K, dtype `factor_dtype`
 *   W         out  N x K, dtype `w_dtype`; the scale is accumulated in fp32 and the
 *                  product rounded once on store.
 * A parity artefact: the fast path (lords_matmul) never writes W.
 */
int lords_dequant(const void *codes, const float *codebook, const void *B, const void *A,
                  void *W, int N, int K, int r, int bits,
                  lords_dtype factor_dtype, lords_dtype w_dtype, void *stream);

/* Quantise (the inverse of lords_dequant; Alg. 1, step 2.1): for every element the index of the level
 * that minimises (S v - W)^2 over the table, S = sum_j B[n][j] A[j][k]; ties go to the lowest index.
 * The decision is taken in fp32: S by fused multiply-adds in increasing j, d = fma(S, C[i], -W), d*d compared.
 *   W      in   N x K, dtype `w_dtype`
 *   codes  out  N x K*bits/8 bytes, packed as described at the top
 */
int lords_quantize(const void *W, const float *codebook, const void *B, const void *A, void *codes,
                   int N, int K, int r, int bits, lords_dtype w_dtype, lords_dtype factor_dtype, void *stream);

/* Block-wise starting point of Alg. 1 (step 1, ComputeScale with block size K/r, read as symmetric absmax
 * scaling, Sec. 3.1) written as factors: B[n][j] = max |W[n][jg .. jg+g)| / max_i |C[i]|, g = K/r, and
 * A[j][k] = 1 if k/g == j else 0, so that B A is the piecewise-constant block scale (rank <= r).
 * K must be a multiple of r (LORDS_ERR_SHAPE otherwise).
 *   B      out  N x r,  A  out  r x K, dtype `factor_dtype` (bf16: the fp32 value rounded to nearest even)
 */
int lords_block_init(const void *W, const float *codebook, void *B, void *A,
                     int N, int K, int r, int bits, lords_dtype w_dtype, lords_dtype factor_dtype, void *stream);

/* Fused dequantise-and-multiply: Y[m*N + n] = sum_k X[m][k] * W_hat[n][k]
 * (the linear layer the paper's inference kernel replaces, Sec. 4.4; Fig. 1b).
 *   X   in   M x K bf16
 *   Y   out  M x N, dtype `y_dtype`; accumulation is fp32.
 * M == 0 returns LORDS_OK without launching.  M <= 16 takes the memory-bound
 * decode kernels (one pass over the codes for all tokens; at one and two tokens the
 * regrouped sum y = rowsum(B (.) (C[Q] (A (.) x)^T)), which never forms the scale per
 * element), larger M the MFMA GEMM
 * (which cuts K into up to four ranges, added in a fixed order, when there are too
 * few tiles to fill the chip); results are run-to-run deterministic.
 */
int lords_matmul(const void *X, const void *codes, const float *codebook,
                 const void *B, const void *A, void *Y,
                 int M, int N, int K, int r, int bits,
                 lords_dtype factor_dtype, lords_dtype y_dtype, void *stream);

/* Same, with the kernel family forced (for cross-over sweeps and tests). */
int lords_matmul_ex(const void *X, const void *codes, const float *codebook,
                    const void *B, const void *A, void *Y,
                    int M, int N, int K, int r, int bits,
                    lords_dtype factor_dtype, lords_dtype y_dtype, void *stream,
                    lords_path path);

/* ---- Workspace owned by the caller ----
 * lords_workspace_bytes: bytes lords_matmul_ws needs for this problem on `path` (the front region
 *   included); 0 if an argument is invalid or the rank unsupported.  Host-side only, no GPU call.
 * lords_workspace_zero_bytes: the leading bytes of a workspace that must be ZERO when it is first
 *   handed over (exchange slots and arrival tickets).  Every call leaves them at zero; the rest of
 *   the workspace is scratch whose contents do not matter.  If a launch ever fails or a kernel is
 *   aborted, zero them again before the next call.
 * lords_matmul_ws: lords_matmul_ex with the workspace passed in.  It performs no allocation, no
 *   free and no synchronisation (safe under stream capture; a captured graph refers to the caller's
 *   buffer).  `workspace` is a device pointer, 256-byte aligned, of at least
 *   lords_workspace_bytes(...) bytes (LORDS_ERR_WORKSPACE if NULL or smaller; a workspace sized for
 *   the largest problem serves them all).  Two calls that overlap in time must not share one.
 */
size_t lords_workspace_bytes(int M, int N, int K, int r, int bits, lords_dtype factor_dtype, lords_path path);
size_t lords_workspace_zero_bytes(void);
int lords_matmul_ws(const void *X, const void *codes, const float *codebook,
                    const void *B, const void *A, void *Y,
                    int M, int N, int K, int r, int bits,
                    lords_dtype factor_dtype, lords_dtype y_dtype, void *stream,
                    lords_path path, void *workspace, size_t workspace_bytes);

/* For callers that cannot allocate at all (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): lords_matmul (path AUTO) with its scratch in a fixed array that
 * is part of the library image, lords_noalloc_limit() = 24 MiB per GPU, held until the process
 * ends.  Calls neither hipMalloc nor hipFree nor any allocating routine, and does not synchronise.
 * A problem whose lords_workspace_bytes(...) exceeds the limit is refused with LORDS_ERR_WORKSPACE
 * (every decode shape of the Llama-3-8B/70B layers fits; large prefill shapes whose K range is cut
 * may not).  All calls on one GPU share the array: calls that overlap in time on one GPU race.  Its
 * front (slots and tickets) starts at zero and every call leaves it at zero.
 */
size_t lords_noalloc_limit(void);
int lords_matmul_noalloc(const void *X, const void *codes, const float *codebook,
                         const void *B, const void *A, void *Y,
                         int M, int N, int K, int r, int bits,
                         lords_dtype factor_dtype, lords_dtype y_dtype, void *stream);

/* Slab-tile layout of the codes: an offline re-ordering of the packed matrix matched to the lane map of
 * the matrix-core kernels (the paper's kernels are only said to be fused, Sec. 4.4; the layout is this
 * build's).  The matrix is cut into slabs of 16 rows and column tiles of 128 columns; tile (s, t) is
 * stored whole at byte (s * ceil(K/128) + t) * 256 * bits, and inside it the 32-code chunk (4 * bits
 * bytes, as in the canonical row) of row 16 s + c, group 4 t + g sits at (16 g + c) * 4 * bits.  A wave
 * that wants 16 rows x 128 columns then reads ONE contiguous piece in lane order, instead of 16 row
 * segments two KB apart (measured on the one-token kernel: 13.6 -> 12.95 us on 14336 x 4096).  Rows
 * >= N and groups >= K/32 of the last tiles are zero bytes.  Codes, levels and scales are unchanged.
 *   lords_repack_bytes     size of the tiled buffer (host only; 0 for invalid arguments).
 *   lords_repack           codes (N x K*bits/8, canonical) -> codes_tiled (device, lords_repack_bytes).
 *   lords_matmul_repacked  lords_matmul_ex on a tiled matrix; same arguments, results and error order.
 *                          Served by the one-/two-token, the few-token and the large-M kernel (bf16
 *                          factors, rank <= 128); LORDS_ERR_UNSUPPORTED where a call would need one of
 *                          the fallback kernels.  Uses the library's own workspace (see the preamble).
 */
size_t lords_repack_bytes(int N, int K, int bits);
int lords_repack(const void *codes, void *codes_tiled, int N, int K, int bits, void *stream);
int lords_matmul_repacked(const void *X, const void *codes_tiled, const float *codebook,
                          const void *B, const void *A, void *Y,
                          int M, int N, int K, int r, int bits,
                          lords_dtype factor_dtype, lords_dtype y_dtype, void *stream, lords_path path);

/* Several quantised matrices applied to the SAME activations: Y[l] = X W_hat[l]^T for l = 0 .. L-1.
 * Every linear layer of a transformer block carries its own codes and factors (Sec. 4.3; module
 * list of Table 7), and the query/key/value projections (and gate/up) read one input; at one token a
 * layer is a few microseconds of memory traffic, so the end-to-end decode rate (Sec. 4.4, Table 6)
 * is set by per-launch overheads that one launch for all of them pays once.
 *   codes, B, A, Y, N   in   HOST arrays of L entries: device pointers (Y[l] is written: M x N[l],
 *                            dtype `y_dtype`) and row counts.  The arrays are read before the call
 *                            returns.
 *   K, r, bits, codebook, factor_dtype are shared by all L matrices.  1 <= L <= 8 (LORDS_ERR_SHAPE).
 * With M <= 16 and bf16 factors of rank <= 64 all matrices are served by one kernel launch;
 * other cases run matrix by matrix.  Each Y[l] is the same sum lords_matmul computes for that matrix
 * (bit-identical from three tokens on; at one and two tokens the single-matrix call may run another
 * kernel, with another rounding of the same sum).
 */
int lords_matmul_batched(const void *X, const void *const *codes, const float *codebook,
                         const void *const *B, const void *const *A, void *const *Y, const int *N,
                         int L, int M, int K, int r, int bits,
                         lords_dtype factor_dtype, lords_dtype y_dtype, void *stream);

/* Gate and up projection of a gated MLP block (the Gate and Up modules of Table 7, both N x K, same
 * input) with the block's activation applied on the way out:
 *      H[m][n] = silu(G[m][n]) * U[m][n],   G = X W_hat_gate^T,  U = X W_hat_up^T,
 *      silu(g) = g / (1 + exp(-g)).
 * G and U are summed in fp32 and never rounded or written out on their own; the product is formed in
 * fp32 and rounded once to `h_dtype`.  With M <= 16 (bf16 factors, rank <= 64) this is one launch; larger
 * M multiplies at most 1024 tokens at a time into an fp32 workspace and combines them in one pass.
 *   H   out  M x N
 */
int lords_gate_up(const void *X, const void *codes_gate, const void *B_gate, const void *A_gate,
                  const void *codes_up, const void *B_up, const void *A_up, const float *codebook,
                  void *H, int M, int N, int K, int r, int bits,
                  lords_dtype factor_dtype, lords_dtype h_dtype, void *stream);

/* ---- Backward of the layer, for fine-tuning the scale factors (Sec. 3.4: B and A are trained, the
 * codes stay fixed).  With Y = X W_hat^T and dY the gradient of a scalar loss with respect to Y:
 *      dX = dY W_hat,     G = dY^T X,   P = C[q] (.) G,     dB = P A^T,     dA = B^T P.
 * G and P (N x K) are never written to device memory. ---- */

/* The packed codes with rows and columns swapped: codes_t has K rows of N codes, code n of row k
 * being code k of row n of `codes`.  Made once per layer (the codes do not change during this kind of
 * fine-tuning) and handed to lords_backward_input.  N must be a multiple of 32 (LORDS_ERR_SHAPE).
 *   codes    in   N x K*bits/8 bytes
 *   codes_t  out  K x N*bits/8 bytes
 */
int lords_transpose_codes(const void *codes, void *codes_t, int N, int K, int bits, void *stream);

/* dX[m][k] = sum_n dY[m][n] W_hat[n][k]: the forward product of the transposed layer
 * W_hat^T = C[Q^T] (.) (A^T B^T), run by the kernels of lords_matmul (same arithmetic, same accuracy).
 *   dY       in   M x N bf16
 *   codes_t  in   from lords_transpose_codes
 *   B, A     in   N x r and r x K (NOT transposed: the library transposes them into its workspace)
 *   dX       out  M x K, dtype `dx_dtype`
 * N must be a multiple of 32.
 */
int lords_backward_input(const void *dY, const void *codes_t, const float *codebook, const void *B, const void *A,
                         void *dX, int M, int N, int K, int r, int bits,
                         lords_dtype factor_dtype, lords_dtype dx_dtype, void *stream);

/* dB[n][j] = sum_k C[q[n][k]] G[n][k] A[j][k],  dA[j][k] = sum_n B[n][j] C[q[n][k]] G[n][k],
 * G = dY^T X accumulated in fp32 over the tokens.  P = C[q] (.) G is rounded once to bf16 and fp32
 * factors are rounded to bf16 as MFMA operands; the sums are fp32 and run-to-run identical.
 *   dY, X    in   M x N and M x K, bf16
 *   dB, dA   out  N x r and r x K, fp32 (overwritten, not accumulated into)
 * Needs N % 8 == 0 and r <= 64 (LORDS_ERR_UNSUPPORTED otherwise); M == 0 gives zeros.
 * Uses the library's per-device workspace: (2 ceil(K/256) N r + ceil(N/256) r K) * 4 bytes of partial results.
 */
int lords_backward_factors(const void *dY, const void *X, const void *codes, const float *codebook,
                           const void *B, const void *A, float *dB, float *dA,
                           int M, int N, int K, int r, int bits, lords_dtype factor_dtype, void *stream);

/* ---- Measurement aids (not part of the method; used by the benchmark for measured ceilings) ----
 * lords_probe_stream_read: one read-only pass over `bytes` bytes at `buffer` (device, 16-byte aligned)
 *   with 16-byte loads, every cache line touched once, nothing written (`sink`: 4 device bytes that
 *   stay untouched for any real data).  Bytes / time is the HBM read rate this GPU gives to a kernel
 *   that does nothing else.
 * lords_probe_mfma_bf16: `iterations` rounds of eight independent v_mfma_f32_16x16x32_bf16 per wave,
 *   operands in registers, on eight waves per CU; *flop_per_launch (host, may be NULL) receives the
 *   floating-point operations of one launch.  Flop / time is the dense bf16 matrix rate this GPU
 *   sustains, clock under load included.  `pattern` 0: operands of ones and small integers (few bits
 *   toggle); 1: operands that differ in every lane and element, as real weights and activations do.
 */
int lords_probe_stream_read(const void *buffer, size_t bytes, void *sink, void *stream);
int lords_probe_mfma_bf16(int iterations, int pattern, void *sink, double *flop_per_launch, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LORDS_H */

/*
 * CPU oracle for the LoRDS inference path in plain C, fp64.  TEST INFRASTRUCTURE ONLY.
 *
 * A second, library-free statement of the same definitions as lords_oracle.py
 * (no BLAS, no blocking, no reordering: every sum runs over its index in
 * increasing order).  It exists so that (a) full-size layers can be checked in
 * seconds and (b) the benchmark can time "the oracle on the host cores" beside
 * the GPU.  Rows of W_hat are independent, so they are handed to OpenMP
 * threads; nothing else is parallel.  It shares no code with the HIP path and
 * the product never links it.
 *
 *   q[n][k]   = bits [bits*k, bits*k+bits) of packed row n, the row being a
 *               little-endian bit string (bit b = bit b%8 of byte b/8)
 *   S[n][k]   = sum_j B[n][j] * A[j][k]                 (paper Sec. 3.2, Eq. 3)
 *   W[n][k]   = C[q[n][k]] * S[n][k]                    (paper Sec. 3.3 objective,
 *               W_hat = Q (.) (BA) with Q_ij a level of the look-up table)
 *   Y[m][n]   = sum_k X[m][k] * W[n][k]                 (the linear layer, Sec. 4.4)
 *
 * Inputs are float (bf16-exact where the layer stores bf16) and are widened to
 * double before use.  Return value: 0 on success, -1 on a bad argument.
 *
 * The quantisation side (Alg. 1 step 2.1 and the block-wise scale of step 1) is stated here in
 * fp32, because there floating point decides an integer and both sides of a parity test have to
 * take that decision in the same precision.  Every operation below is one correctly rounded fp32
 * operation (fmaf, *, /, comparisons), in the order written; the file is compiled with
 * -ffp-contract=off so that nothing else gets fused:
 *   S[n][k]   = fmaf(B[n][r-1], A[r-1][k], ... fmaf(B[n][0], A[0][k], 0) ...)    j increasing
 *   q[n][k]   = the lowest i minimising e_i = d_i * d_i,  d_i = fmaf(S[n][k], C[i], -W[n][k])
 *   scale of a block = (max over the block of |W|) / (max over the levels of |C|)
 * The fp64 statement of the same definitions is in lords_oracle.py; tests pin the two together.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int code_at(const uint8_t *row, long k, int bits)
{
    int q = 0;
    for (int b = 0; b < bits; ++b) {
        long bit = (long)bits * k + b;
        q |= ((row[bit >> 3] >> (bit & 7)) & 1) << b;
    }
    return q;
}

static int bad_shape(long N, long K, long r, int bits)
{
    return N < 0 || K < 0 || r < 0 || (bits != 2 && bits != 3 && bits != 4) || ((K * bits) % 8) != 0;
}

int lords_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int lords_oracle_unpack(const uint8_t *codes, uint8_t *q, long N, long K, int bits)
{
    if (!codes || !q || bad_shape(N, K, 0, bits)) return -1;
    const long rb = K * bits / 8;
#pragma omp parallel for schedule(static)
    for (long n = 0; n < N; ++n)
        for (long k = 0; k < K; ++k)
            q[n * K + k] = (uint8_t)code_at(codes + n * rb, k, bits);
    return 0;
}

/* one row of W_hat into w[0..K) */
static void dequant_row(const uint8_t *row, const float *codebook, const float *Brow,
                        const float *A, double *w, long K, long r, int bits)
{
    for (long k = 0; k < K; ++k) {
        double s = 0.0;
        for (long j = 0; j < r; ++j)
            s += (double)Brow[j] * (double)A[j * K + k];
        w[k] = (double)codebook[code_at(row, k, bits)] * s;
    }
}

int lords_oracle_dequant(const uint8_t *codes, const float *codebook, const float *B,
                         const float *A, double *W, long N, long K, long r, int bits)
{
    if (!codes || !codebook || !B || !A || !W || bad_shape(N, K, r, bits)) return -1;
    const long rb = K * bits / 8;
#pragma omp parallel for schedule(static)
    for (long n = 0; n < N; ++n)
        dequant_row(codes + n * rb, codebook, B + n * r, A, W + n * K, K, r, bits);
    return 0;
}

/* Y[m][i] for the out-features rows[i] (rows == NULL: all N rows, i == n).
 * Y is M x nrows, row-major. */
int lords_oracle_matmul_rows(const float *X, const uint8_t *codes, const float *codebook,
                             const float *B, const float *A, double *Y,
                             long M, long N, long K, long r, int bits,
                             const long *rows, long nrows)
{
    if (!X || !codes || !codebook || !B || !A || !Y || M < 0 || bad_shape(N, K, r, bits)) return -1;
    if (!rows) nrows = N;
    for (long i = 0; rows && i < nrows; ++i)
        if (rows[i] < 0 || rows[i] >= N) return -1;
    const long rb = K * bits / 8;
    int failed = 0;
#pragma omp parallel
    {
        double *w = (double *)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
        if (!w) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (long i = 0; i < nrows; ++i) {
            if (!w) continue;
            const long n = rows ? rows[i] : i;
            dequant_row(codes + n * rb, codebook, B + n * r, A, w, K, r, bits);
            for (long m = 0; m < M; ++m) {
                double acc = 0.0;
                for (long k = 0; k < K; ++k)
                    acc += (double)X[m * K + k] * w[k];
                Y[m * nrows + i] = acc;
            }
        }
        free(w);
    }
    return failed ? -1 : 0;
}

int lords_oracle_matmul(const float *X, const uint8_t *codes, const float *codebook,
                        const float *B, const float *A, double *Y,
                        long M, long N, long K, long r, int bits)
{
    return lords_oracle_matmul_rows(X, codes, codebook, B, A, Y, M, N, K, r, bits, (const long *)0, N);
}

/* ---- quantisation side, fp32 (see the header) --------------------------------------------- */

int lords_oracle_pack(const uint8_t *q, uint8_t *codes, long N, long K, int bits)
{
    if (!q || !codes || bad_shape(N, K, 0, bits)) return -1;
    const long rb = K * bits / 8;
    for (long n = 0; n < N; ++n) {
        uint8_t *row = codes + n * rb;
        for (long b = 0; b < rb; ++b) row[b] = 0;
        for (long k = 0; k < K; ++k) {
            const int v = q[n * K + k];
            if (v >> bits) return -1;
            for (int b = 0; b < bits; ++b) {
                const long bit = (long)bits * k + b;
                row[bit >> 3] |= (uint8_t)(((v >> b) & 1) << (bit & 7));
            }
        }
    }
    return 0;
}

int lords_oracle_quantize_f32(const float *W, const float *codebook, const float *B, const float *A,
                              uint8_t *q, long N, long K, long r, int bits)
{
    if (!W || !codebook || !B || !A || !q || bad_shape(N, K, r, bits)) return -1;
    const int nl = 1 << bits;
#pragma omp parallel for schedule(static)
    for (long n = 0; n < N; ++n)
        for (long k = 0; k < K; ++k) {
            float s = 0.0f;
            for (long j = 0; j < r; ++j) s = fmaf(B[n * r + j], A[j * K + k], s);
            const float w = W[n * K + k];
            int best = 0;
            float ebest = 0.0f;
            for (int i = 0; i < nl; ++i) {
                const float d = fmaf(s, codebook[i], -w);
                const float e = d * d;
                if (i == 0 || e < ebest) { best = i; ebest = e; }
            }
            q[n * K + k] = (uint8_t)best;
        }
    return 0;
}

int lords_oracle_block_init_f32(const float *W, const float *codebook, float *B, float *A,
                                long N, long K, long r, int bits)
{
    if (!W || !codebook || !B || !A || bad_shape(N, K, r, bits) || r < 1 || (K % r) != 0) return -1;
    const long g = K / r;
    float cmax = 0.0f;
    for (int i = 0; i < (1 << bits); ++i)
        if (fabsf(codebook[i]) > cmax) cmax = fabsf(codebook[i]);
    for (long n = 0; n < N; ++n)
        for (long j = 0; j < r; ++j) {
            float m = 0.0f;
            for (long k = j * g; k < (j + 1) * g; ++k)
                if (fabsf(W[n * K + k]) > m) m = fabsf(W[n * K + k]);
            B[n * r + j] = m / cmax;
        }
    for (long j = 0; j < r; ++j)
        for (long k = 0; k < K; ++k)
            A[j * K + k] = (k / g == j) ? 1.0f : 0.0f;
    return 0;
}

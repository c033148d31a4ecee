// Fused dequantise-and-multiply kernels:  Y = X (C[Q] (.) (B A))^T  on gfx950.
//
// One kernel body serves the memory-bound small-M path (MB = 1, X read straight
// from global memory, K split across workgroups) and the MFMA GEMM path for
// large M (X staged in LDS, MB blocks of 16 tokens per workgroup).
//
// Wave-level tile mapping (everything is built on v_mfma_f32_16x16x32_bf16,
// D[i][j] held by lane l as j = l%16, i = 4*(l/16)+{0..3}):
//
//   lane l = (c = l%16, g = l/16) owns, for weight row n0+c, the 32-code groups
//   k in [kb + 32*(G*g+v), +32), v = 0..G-1: BITS dwords per group, loaded straight
//   into registers and unpacked there.
//
//   Scale tile.  For group v the wave issues 8 "S" MFMAs per 32 columns of the
//   padded rank:  D[i][j] with j <-> weight row n0+j and i <-> column
//   k = kb + 32*(G*(i/4)+v) + 4t + i%4  (t = 0..7 is the MFMA number).  The
//   b-operand is 8 consecutive rank entries of row n0+c of B (kept in registers
//   for the whole K range); the a-operand is 8 consecutive rank entries of one
//   column of A, fetched from the row-major A tile in LDS with the transposing
//   ds_read_b64_tr_b16.  Lane (c,g) therefore receives exactly the 32 scales of
//   the 32 codes it holds: S-MFMA t, accumulator i <-> code 4t+i of the group.
//
//   Dequantise in registers: w = C[code] * S, rounded once to bf16.
//
//   Product.  Four "Y" MFMAs per group contract those 32 columns:
//   a-operand = the lane's own dequantised row slice (8 values per MFMA),
//   b-operand = 8 activations X[m = c][same 8 columns]; D[i][j] with i <-> weight
//   row, j <-> token.  Accumulators stay in registers over the whole K range.
#include "lords_device.h"
#include "lords_launch.h"

namespace lords {

struct FusedArgs {
    const uint16_t *X;
    const uint8_t *codes;
    const float *codebook;
    Factors f;
    void *Y;           // M x N (used when splits == 1)
    float *partial;    // [splits][M][N] fp32 (used when splits > 1)
    int M, N, K;
    int y_f32;
    int row_bytes;
    int ntiles;           // ceil(K / KT)
    int tiles_per_split;
    int splits;
    int b_vec_ok;      // bf16 factors, r % 8 == 0: 16-byte operand loads of B are legal
};

constexpr int kG = 2;               // 32-code groups per lane per K tile
constexpr int kKT = 128 * kG;       // columns per K tile
constexpr int kAST = kKT + 8;       // LDS row stride (elements) of the A and X tiles

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ __forceinline__ bf16x8 tr_read_pair(const uint16_t *tile, int row, int col)
{
    // two transposing reads: rank entries row..row+3 and row+4..row+7 (per 16-lane block)
    const uint16_t *p0 = tile + row * kAST + col;
    const uint16_t *p1 = p0 + 4 * kAST;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p0);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p1);
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
    s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// Stage rank rows [jbase, jbase + RP) of the A tile (RP x kKT, row-major, zero padded).
template <int RP>
__device__ __forceinline__ void stage_A_tile(const FusedArgs &a, uint16_t *As, int jbase, int kb, int tid)
{
    if (!a.f.f32) {
        for (int id = tid; id < RP * (kKT / 8); id += 256) {
            const int jl = id / (kKT / 8), kc = id % (kKT / 8), k = kb + 8 * kc, jj = jbase + jl;
            u32x4 v = u32x4{0u, 0u, 0u, 0u};
            if (jj < a.f.r && k < a.K)
                v = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(a.f.A) + (size_t)jj * a.K + k);
            *reinterpret_cast<u32x4 *>(As + jl * kAST + 8 * kc) = v;
        }
    } else {
        for (int id = tid; id < RP * kKT; id += 256) {
            const int jl = id / kKT, kk = id % kKT;
            As[jl * kAST + kk] = factorA_bits(a.f, jbase + jl, kb + kk);
        }
    }
}

// 8 consecutive rank entries jj0.. of row n of B as an MFMA operand.
__device__ __forceinline__ bf16x8 load_B_operand(const FusedArgs &a, int n, int jj0)
{
    if (a.b_vec_ok && n < a.N && jj0 + 8 <= a.f.r)
        return *reinterpret_cast<const bf16x8 *>(reinterpret_cast<const uint16_t *>(a.f.B) + (size_t)n * a.f.r + jj0);
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
    s16x8 t;
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = (short)factorB_bits(a.f, n, jj0 + e);
    return __builtin_bit_cast(bf16x8, t);
}

// MULTI = false: the whole padded rank (32*SS) is staged at once and the B operands
// live in registers.  MULTI = true (ranks beyond 128 columns): the rank is walked in
// chunks of 32*SS, each staged in turn, B operands re-read from global memory.
template <int BITS, int SS, int R, int MB, bool XLDS, bool MULTI>
__global__ __launch_bounds__(256) void fused_kernel(FusedArgs a)
{
    constexpr int RP = 32 * SS;            // rank columns staged at a time
    constexpr int NL = 1 << BITS;
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t *As = reinterpret_cast<uint16_t *>(smem);                 // [RP][kAST]
    uint16_t *Xs = As + RP * kAST;                                     // [16*MB][kAST] when XLDS
    float *lut = reinterpret_cast<float *>(Xs + (XLDS ? 16 * MB * kAST : 0));

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int n_wave = (blockIdx.x * 4 + wave) * (16 * R);
    const int m_blk = blockIdx.y * (16 * MB);
    const int kt0 = blockIdx.z * a.tiles_per_split;
    const int kt1 = min(kt0 + a.tiles_per_split, a.ntiles);
    const int N = a.N, K = a.K, M = a.M;
    const int nchunks = MULTI ? (a.f.r_eff + RP - 1) / RP : 1;

    if (tid < NL) lut[tid] = a.codebook[tid];

    bf16x8 Bop[R][SS];
    if (!MULTI) {
#pragma unroll
        for (int rho = 0; rho < R; ++rho)
#pragma unroll
            for (int s = 0; s < SS; ++s) Bop[rho][s] = load_B_operand(a, n_wave + 16 * rho + c, 32 * s + 8 * g);
    }

    f32x4 acc[R][MB];
#pragma unroll
    for (int rho = 0; rho < R; ++rho)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[rho][mb] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int kt = kt0; kt < kt1; ++kt) {
        const int kb = kt * kKT;
        f32x4 S[kG][R][8];
#pragma unroll
        for (int v = 0; v < kG; ++v)
#pragma unroll
            for (int rho = 0; rho < R; ++rho)
#pragma unroll
                for (int t = 0; t < 8; ++t) S[v][rho][t] = f32x4{0.f, 0.f, 0.f, 0.f};

        for (int ch = 0; ch < nchunks; ++ch) {
            __syncthreads();                       // everyone is done with the previous tiles
            stage_A_tile<RP>(a, As, ch * RP, kb, tid);
            if (XLDS && ch == 0) {
                for (int id = tid; id < 16 * MB * (kKT / 8); id += 256) {
                    const int mm = id / (kKT / 8), kc = id % (kKT / 8), k = kb + 8 * kc, gm = m_blk + mm;
                    u32x4 v = u32x4{0u, 0u, 0u, 0u};
                    if (gm < M && k < K) v = *reinterpret_cast<const u32x4 *>(a.X + (size_t)gm * K + k);
                    *reinterpret_cast<u32x4 *>(Xs + mm * kAST + 8 * kc) = v;
                }
            }
            __syncthreads();
            if (MULTI) {
#pragma unroll
                for (int rho = 0; rho < R; ++rho)
#pragma unroll
                    for (int s = 0; s < SS; ++s)
                        Bop[rho][s] = load_B_operand(a, n_wave + 16 * rho + c, ch * RP + 32 * s + 8 * g);
            }
            // ---- scale tile: 8 S-MFMAs per group and 32 rank columns, shared by the R slabs ----
#pragma unroll
            for (int v = 0; v < kG; ++v)
#pragma unroll
                for (int s = 0; s < SS; ++s)
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        const bf16x8 Aop = tr_read_pair(As, 32 * s + 8 * g + (c >> 2), 32 * (kG * (c & 3) + v) + 4 * t);
#pragma unroll
                        for (int rho = 0; rho < R; ++rho)
                            S[v][rho][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aop, Bop[rho][s], S[v][rho][t], 0, 0, 0);
                    }
        }

#pragma unroll
        for (int v = 0; v < kG; ++v) {
            const int kgrp = kb + 32 * (kG * g + v);     // first column of this lane's group
            // ---- unpack, look up, scale, round to bf16 --------------------------------------
            bf16x8 Wop[R][4];
#pragma unroll
            for (int rho = 0; rho < R; ++rho) {
                const int n = min(n_wave + 16 * rho + c, N - 1);
                uint32_t w[BITS];
                if (kgrp < K) {
                    load_group<BITS>(a.codes + (size_t)n * a.row_bytes + (size_t)(kgrp >> 5) * (4 * BITS), w);
                } else {
#pragma unroll
                    for (int i = 0; i < BITS; ++i) w[i] = 0u;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float cv = lut[code_at<BITS>(w, 8 * u + e)];
                        Wop[rho][u][e] = (__bf16)(cv * S[v][rho][2 * u + (e >> 2)][e & 3]);
                    }
                }
            }
            // ---- product: 4 Y-MFMAs per slab and 16-token block ----------------------------
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                bf16x8 Xop[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (XLDS) {
                        Xop[u] = *reinterpret_cast<const bf16x8 *>(Xs + (16 * mb + c) * kAST + 32 * (kG * g + v) + 8 * u);
                    } else {
                        const int m = m_blk + 16 * mb + c;
                        u32x4 t = u32x4{0u, 0u, 0u, 0u};
                        if (m < M && kgrp < K) t = *reinterpret_cast<const u32x4 *>(a.X + (size_t)m * K + kgrp + 8 * u);
                        Xop[u] = __builtin_bit_cast(bf16x8, t);
                    }
                }
#pragma unroll
                for (int rho = 0; rho < R; ++rho)
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        acc[rho][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Wop[rho][u], Xop[u], acc[rho][mb], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: lane (c,g) holds token m = c, rows n = 4g + e of each slab --------------
#pragma unroll
    for (int rho = 0; rho < R; ++rho) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int m = m_blk + 16 * mb + c;
            if (m >= M) continue;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int n = n_wave + 16 * rho + 4 * g + e;
                if (n >= N) continue;
                const float val = acc[rho][mb][e];
                if (a.splits > 1) {
                    a.partial[((size_t)blockIdx.z * M + m) * N + n] = val;
                } else if (a.y_f32) {
                    reinterpret_cast<float *>(a.Y)[(size_t)m * N + n] = val;
                } else {
                    reinterpret_cast<uint16_t *>(a.Y)[(size_t)m * N + n] = bf16_bits(val);
                }
            }
        }
    }
}

// Y = sum over splits of partial, in increasing split order (deterministic).
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ partial, void *__restrict__ Y,
                                                              long MN, int splits, int y_f32)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= MN) return;
    float s = 0.f;
    for (int z = 0; z < splits; ++z) s += partial[(long)z * MN + i];
    if (y_f32) reinterpret_cast<float *>(Y)[i] = s;
    else reinterpret_cast<uint16_t *>(Y)[i] = bf16_bits(s);
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
constexpr int kDecodeR = 2;      // 16-row slabs per wave, small-M path
constexpr int kPrefillR = 2;
constexpr int kPrefillMB = 8;    // 16-token blocks per workgroup, MFMA GEMM path

static int pick_ss(int r_eff)
{
    const int rp = (r_eff + 31) / 32;
    if (rp <= 1) return 1;
    if (rp <= 2) return 2;
    if (rp <= 4) return 4;
    return 0;                     // beyond 128 rank columns: walked in chunks of 128
}

static int decode_splits(const MatmulProblem &p, int *tiles_per_split)
{
    const int ntiles = (p.K + kKT - 1) / kKT;
    const int rowblocks = (p.N + 64 * kDecodeR - 1) / (64 * kDecodeR);
    int want = (1024 + rowblocks - 1) / rowblocks;        // aim for about 4 workgroups per CU
    if (want > ntiles) want = ntiles;
    if (want < 1) want = 1;
    const int tps = (ntiles + want - 1) / want;
    *tiles_per_split = tps;
    return (ntiles + tps - 1) / tps;
}

size_t decode_workspace_bytes(const MatmulProblem &p)
{
    int tps;
    const int splits = decode_splits(p, &tps);
    if (splits <= 1) return 0;
    const int mchunk = p.M < 16 ? p.M : 16;
    return (size_t)splits * mchunk * p.N * sizeof(float);
}

static FusedArgs make_args(const MatmulProblem &p)
{
    FusedArgs a;
    a.X = (const uint16_t *)p.X;
    a.codes = (const uint8_t *)p.codes;
    a.codebook = p.codebook;
    a.f.B = p.B; a.f.A = p.A; a.f.N = p.N; a.f.K = p.K; a.f.r = p.r;
    a.f.f32 = p.f32fact ? 1 : 0;
    a.f.r_eff = p.f32fact ? 3 * p.r : p.r;
    a.Y = p.Y; a.partial = nullptr;
    a.M = p.M; a.N = p.N; a.K = p.K;
    a.y_f32 = p.f32out ? 1 : 0;
    a.row_bytes = p.K / 8 * p.bits;
    a.ntiles = (p.K + kKT - 1) / kKT;
    a.tiles_per_split = a.ntiles;
    a.splits = 1;
    a.b_vec_ok = (!p.f32fact && (p.r % 8) == 0) ? 1 : 0;
    return a;
}

template <int BITS, int SS, int R, int MB, bool XLDS, bool MULTI>
static hipError_t launch_fused(const FusedArgs &a, dim3 grid, hipStream_t st)
{
    const size_t smem = (size_t)(32 * SS) * kAST * 2 + (XLDS ? (size_t)16 * MB * kAST * 2 : 0) + 16 * sizeof(float);
    static LdsOptIn lds_opt_in;
    if (smem > 48 * 1024) {
        const hipError_t e = allow_dynamic_lds(lds_opt_in, reinterpret_cast<const void *>(&fused_kernel<BITS, SS, R, MB, XLDS, MULTI>), smem);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((fused_kernel<BITS, SS, R, MB, XLDS, MULTI>), grid, dim3(256), smem, st, a);
    return hipGetLastError();
}

template <int R, int MB, bool XLDS>
static hipError_t dispatch_fused(const FusedArgs &a, int bits, int ss, dim3 grid, hipStream_t st)
{
#define LORDS_CASE(B_, S_) \
    if (bits == B_ && ss == S_) return launch_fused<B_, S_, R, MB, XLDS, false>(a, grid, st);
    LORDS_CASE(2, 1) LORDS_CASE(2, 2) LORDS_CASE(2, 4)
    LORDS_CASE(3, 1) LORDS_CASE(3, 2) LORDS_CASE(3, 4)
    LORDS_CASE(4, 1) LORDS_CASE(4, 2) LORDS_CASE(4, 4)
#undef LORDS_CASE
    if (ss == 0) {
        if (bits == 2) return launch_fused<2, 4, R, MB, XLDS, true>(a, grid, st);
        if (bits == 3) return launch_fused<3, 4, R, MB, XLDS, true>(a, grid, st);
        if (bits == 4) return launch_fused<4, 4, R, MB, XLDS, true>(a, grid, st);
    }
    return hipErrorInvalidValue;
}

// The contraction length (r, or 3r for fp32 factors) must stay addressable in 32-bit tile arithmetic.
bool fused_rank_supported(int r, bool f32fact) { return r >= 1 && r <= (f32fact ? 2048 : 6144); }

hipError_t launch_decode(const MatmulProblem &p, void *workspace, hipStream_t st)
{
    const int ss = pick_ss(p.f32fact ? 3 * p.r : p.r);
    int tps;
    const int splits = decode_splits(p, &tps);
    const int rowblocks = (p.N + 64 * kDecodeR - 1) / (64 * kDecodeR);
    for (int m0 = 0; m0 < p.M; m0 += 16) {
        MatmulProblem q = p;
        q.M = (p.M - m0) < 16 ? (p.M - m0) : 16;
        q.X = (const uint16_t *)p.X + (size_t)m0 * p.K;
        q.Y = p.f32out ? (void *)((float *)p.Y + (size_t)m0 * p.N) : (void *)((uint16_t *)p.Y + (size_t)m0 * p.N);
        FusedArgs a = make_args(q);
        a.tiles_per_split = tps;
        a.splits = splits;
        a.partial = (float *)workspace;
        hipError_t e = dispatch_fused<kDecodeR, 1, false>(a, p.bits, ss, dim3(rowblocks, 1, splits), st);
        if (e != hipSuccess) return e;
        if (splits > 1) {
            const long MN = (long)q.M * q.N;
            hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((MN + 255) / 256)), dim3(256), 0, st,
                               (const float *)workspace, q.Y, MN, splits, a.y_f32);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

hipError_t launch_prefill(const MatmulProblem &p, hipStream_t st)
{
    const int ss = pick_ss(p.f32fact ? 3 * p.r : p.r);
    FusedArgs a = make_args(p);
    const int rowblocks = (p.N + 64 * kPrefillR - 1) / (64 * kPrefillR);
    const int mblocks = (p.M + 16 * kPrefillMB - 1) / (16 * kPrefillMB);
    return dispatch_fused<kPrefillR, kPrefillMB, true>(a, p.bits, ss, dim3(rowblocks, mblocks, 1), st);
}

}  // namespace lords

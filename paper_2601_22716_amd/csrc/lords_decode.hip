// Small-M (decode) kernel of  Y = X (C[Q] (.) (B A))^T  on gfx950: memory-bound,
// every packed code is read from HBM exactly once.
//
// Work split.  A wave owns one block of KT = 128*G columns and streams down a
// chunk of 16-row slabs; the four waves of a workgroup own four consecutive
// column blocks and the same slabs, so their partial sums meet in LDS.  Column
// blocks beyond four per row (K > 4*KT) are spread over gridDim.z workgroups
// whose partial sums meet in a workspace; the last workgroup to arrive (an atomic
// ticket per slab chunk) adds them in a fixed order, so results are
// run-to-run identical.
//
// Per wave, once:  the A columns of its block go through a wave-private LDS tile
// and come back, transposed by ds_read_b64_tr_b16, as the a-operands of the scale
// MFMAs; they and the activations (b-operands of the product MFMAs) then stay in
// registers for the whole row loop.  Per slab: two things are loaded, the lane's
// G*32 packed codes of row n0+c and 8 rank entries of that row of B.
//
// Lane mapping (v_mfma_f32_16x16x32_bf16; lane l = (c = l%16, g = l/16)):
//   scale MFMA t of group v:  D[i][j],  j <-> row n0+j,
//                             i <-> column kb + 32*(G*(i/4)+v) + 4t + i%4,
//   so lane (c,g) gets, in accumulator i of MFMA t, the scale of code 4t+i of the
//   32-code group it holds (columns kb + 32*(G*g+v) ...).
//   product MFMA u of group v: a-operand = the lane's 8 dequantised weights
//   8u..8u+7 of the group, b-operand = X[c][the same 8 columns]; D[i][j] with
//   i <-> row, j <-> token.
//
// Level look-up.  Two codes (2*BITS bits) index an LDS table of fp16 pairs; the
// table is replicated 64 times (one dword column per lane: address =
// index*256 + lane*4) so no two lanes ever meet in a bank, and at 4 bits the
// address is formed by a single v_perm_b32 (the code byte lands in address bits
// 8..15).  v_fma_mix_f32 multiplies the fp16 level by the fp32 scale directly;
// the product is rounded once to bf16 for the MFMA.  fp16 holds the levels of
// the NF / INT tables to 2^-12 relative; levels must lie within fp16 range.
#include "lords_decode_common.h"

namespace lords {

// M1 = true : one token.  The activations are folded into the A tile (A[j][k] * x[k], rounded
//             to bf16) so the scale MFMAs deliver S[n][k] * x[k]; the product with the level
//             is then accumulated per lane in fp32 (v_fma_mix_f32) and the lanes are summed in
//             LDS at the end.  No product MFMA, no bf16 rounding of the weights.
// M1 = false: 2..16 tokens, product MFMAs as described at the top of the file.
// BVEC      : bf16 factors with r % 8 == 0, so 8 rank entries of a row of B are one 16-byte load.
template <int BITS, int SS, int G, bool BVEC, bool M1>
__global__ __launch_bounds__(256) void decode_kernel(DecodeArgs a)
{
    constexpr int KT = 128 * G, AST = KT + 8, NL = 1 << BITS, NE = 1 << (2 * BITS);
    constexpr int A_BYTES = 4 * 32 * AST * 2, LUT_BYTES = NE * 256, RED_BYTES = 4 * kNS * 64 * 16;
    constexpr int R0 = A_BYTES > LUT_BYTES ? (A_BYTES > RED_BYTES ? A_BYTES : RED_BYTES)
                                           : (LUT_BYTES > RED_BYTES ? LUT_BYTES : RED_BYTES);
    extern __shared__ __align__(16) unsigned char smem[];
    float *cb = reinterpret_cast<float *>(smem + R0);          // [16]
    int *flag = reinterpret_cast<int *>(smem + R0 + 64);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int kb = (blockIdx.z * 4 + wave) * KT;               // first column of this wave's block
    const int slab0 = blockIdx.x * a.ns;
    const int ns = min(a.ns, a.nslabs - slab0);
    const int N = a.N, K = a.K, M = a.M;
    const uint32_t laneoff = (uint32_t)lane * 4u;

    // Loads of slab i.  Branch-free on purpose: every address is clamped into the arrays, so the
    // loads can be issued kDepth slabs ahead without a wait in between.  Codes fetched for
    // columns >= K are never used (the A tile is zero there, so the scale is zero), rank entries
    // >= r of B meet zero rows of the A tile, rows >= N are dropped at the store.
    uint32_t cw[kNS][G][BITS];
    bf16x8 Bop[kNS][SS];
    const int ngroups = K >> 5;
    auto issue = [&](int i) {
        const int n = min((slab0 + i) * 16 + c, N - 1);
#pragma unroll
        for (int v = 0; v < G; ++v) {
            const int grp = min((kb >> 5) + G * g + v, ngroups - 1);
            load_group<BITS>(a.codes + (size_t)n * a.row_bytes + (size_t)grp * (4 * BITS), cw[i][v]);
        }
        if (BVEC) {
#pragma unroll
            for (int s = 0; s < SS; ++s) {
                const int jj0 = 32 * s + 8 * g;
                Bop[i][s] = *reinterpret_cast<const bf16x8 *>(
                    reinterpret_cast<const uint16_t *>(a.f.B) + (size_t)n * a.f.r + (jj0 + 8 <= a.f.r ? jj0 : 0));
            }
        }
    };
    // Factors that cannot be read as 16-byte operands (fp32, or a rank that is not a multiple
    // of 8) are gathered element by element at the point of use: the slow, general variant.
    auto gather_B = [&](int i) {
        const int row = (slab0 + i) * 16 + c;
#pragma unroll
        for (int s = 0; s < SS; ++s) {
            typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
            s16x8 t;
#pragma unroll
            for (int e = 0; e < 8; ++e) t[e] = (short)factorB_bits(a.f, row, 32 * s + 8 * g + e);
            Bop[i][s] = __builtin_bit_cast(bf16x8, t);
        }
    };

    // ---- 0. first loads of the row stream go out before any set-up --------------------------
#pragma unroll
    for (int i = 0; i < kDepth; ++i) issue(i);

    if (tid < NL) cb[tid] = a.codebook[tid];

    // ---- 1. A columns of this wave's block -> a-operands of the scale MFMAs ------------------
    bf16x8 Aop[G][SS][8];
    {
        uint16_t *Aw = reinterpret_cast<uint16_t *>(smem) + wave * (32 * AST);    // wave-private tile
        constexpr int CPR = KT / 8;                   // 16-byte chunks per tile row
        constexpr int NCH = 32 * CPR / 64;            // chunks per lane; lane's column chunk is lane % CPR for all
        const int kc = lane % CPR, k0 = kb + 8 * kc;
        float xk[8];
        if (M1) {
            u32x4 xv = u32x4{0u, 0u, 0u, 0u};
            if (k0 < K) xv = *reinterpret_cast<const u32x4 *>(a.X + k0);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                xk[2 * e] = __builtin_bit_cast(float, xv[e] << 16);
                xk[2 * e + 1] = __builtin_bit_cast(float, xv[e] & 0xFFFF0000u);
            }
        }
#pragma unroll
        for (int s = 0; s < SS; ++s) {
            __syncthreads();
            if (!a.f.f32) {
                u32x4 tmp[NCH];                       // all loads first, then the stores
#pragma unroll
                for (int q = 0; q < NCH; ++q) {
                    const int jj = 32 * s + (lane + 64 * q) / CPR;
                    tmp[q] = u32x4{0u, 0u, 0u, 0u};
                    if (jj < a.f.r && k0 < K)
                        tmp[q] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(a.f.A) + (size_t)jj * K + k0);
                }
#pragma unroll
                for (int q = 0; q < NCH; ++q) {
                    const int jl = (lane + 64 * q) / CPR;
                    u32x4 o = tmp[q];
                    if (M1) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float lo = __builtin_bit_cast(float, o[e] << 16) * xk[2 * e];
                            const float hi = __builtin_bit_cast(float, o[e] & 0xFFFF0000u) * xk[2 * e + 1];
                            o[e] = (uint32_t)bf16_bits(lo) | ((uint32_t)bf16_bits(hi) << 16);
                        }
                    }
                    *reinterpret_cast<u32x4 *>(Aw + jl * AST + 8 * kc) = o;
                }
            } else {
                for (int id = lane; id < 32 * KT; id += 64) {
                    const int jl = id / KT, kk = id % KT;
                    uint16_t v;
                    if (M1) {
                        const float x = (kb + kk < K) ? bf16_to_f32(a.X[kb + kk]) : 0.f;
                        v = factorAx_bits(a.f, 32 * s + jl, kb + kk, x);
                    } else {
                        v = factorA_bits(a.f, 32 * s + jl, kb + kk);
                    }
                    Aw[jl * AST + kk] = v;
                }
            }
            __syncthreads();
#pragma unroll
            for (int v = 0; v < G; ++v)
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    Aop[v][s][t] = tr_read_pair_d<AST>(Aw, 8 * g + (c >> 2), 32 * (G * (c & 3) + v) + 4 * t);
        }
    }

    // ---- 2. level table: entry idx = (code_hi << BITS) | code_lo, 64 copies ------------------
    __syncthreads();
    {
        uint32_t *lut32 = reinterpret_cast<uint32_t *>(smem);
        for (int id = tid; id < NE * 16; id += 256) {
            const int idx = id >> 4, q = id & 15;
            f16x2 h;
            h[0] = (_Float16)cb[idx & (NL - 1)];
            h[1] = (_Float16)cb[idx >> BITS];
            const uint32_t pv = __builtin_bit_cast(uint32_t, h);
            *reinterpret_cast<u32x4 *>(lut32 + idx * 64 + 4 * q) = u32x4{pv, pv, pv, pv};
        }
    }
    __syncthreads();

    // ---- 3. activations of this block: b-operands of the product MFMAs -----------------------
    bf16x8 Xop[M1 ? 1 : G][4];
    if (!M1) {
#pragma unroll
        for (int v = 0; v < G; ++v) {
            const int kgrp = kb + 32 * (G * g + v);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                u32x4 t = u32x4{0u, 0u, 0u, 0u};
                if (c < M && kgrp < K) t = *reinterpret_cast<const u32x4 *>(a.X + (size_t)c * K + kgrp + 8 * u);
                Xop[v][u] = __builtin_bit_cast(bf16x8, t);
            }
        }
    }

    // ---- 4. the row stream ---------------------------------------------------------------------
    f32x4 acc[M1 ? 1 : kNS];      // product-MFMA accumulators (rows x tokens)
    float acc1[M1 ? kNS : 1];     // one token: the lane's partial dot product of row n0+c
#pragma unroll
    for (int i = 0; i < kNS; ++i) {
        if (M1) acc1[i] = 0.f; else acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (i < ns) {
            if (i + kDepth < kNS) issue(i + kDepth);
            __builtin_amdgcn_sched_barrier(0);     // keep the prefetch ahead of this slab's arithmetic
            if (!BVEC) gather_B(i);
            float p0 = 0.f, p1 = 0.f, p2 = 0.f, p3 = 0.f;
#pragma unroll
            for (int v = 0; v < G; ++v) {
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {       // half a group: scale MFMAs 4hh .. 4hh+3
                    f32x4 S[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) S[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < SS; ++s)
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            S[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aop[v][s][4 * hh + t], Bop[i][s], S[t], 0, 0, 0);
#pragma unroll
                    for (int uu = 0; uu < 2; ++uu) {
                        const int u = 2 * hh + uu;
                        bf16x8 W;
#pragma unroll
                        for (int pp = 0; pp < 4; ++pp) {
                            const uint32_t ad = pair_addr<BITS>(cw[i][v], 4 * u + pp, laneoff);
                            const f16x2 h = __builtin_bit_cast(f16x2, lds_load_u32(ad));
                            const int e0 = 2 * pp, e1 = 2 * pp + 1;
                            const float s0 = S[2 * uu + (e0 >> 2)][e0 & 3], s1 = S[2 * uu + (e1 >> 2)][e1 & 3];
                            if (M1) {
                                if (pp & 1) { p2 = __builtin_fmaf((float)h[0], s0, p2); p3 = __builtin_fmaf((float)h[1], s1, p3); }
                                else        { p0 = __builtin_fmaf((float)h[0], s0, p0); p1 = __builtin_fmaf((float)h[1], s1, p1); }
                            } else {
                                W[e0] = (__bf16)__builtin_fmaf((float)h[0], s0, 0.0f);
                                W[e1] = (__bf16)__builtin_fmaf((float)h[1], s1, 0.0f);
                            }
                        }
                        if (!M1) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(W, Xop[v][u], acc[i], 0, 0, 0);
                    }
                }
            }
            if (M1) acc1[i] = (p0 + p1) + (p2 + p3);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- 5. add the four column blocks of this workgroup (fixed order) -------------------------
    __syncthreads();                               // the table is dead from here on
    if (M1) {
        float *red = reinterpret_cast<float *>(smem);  // [4][kNS][64]
#pragma unroll
        for (int i = 0; i < kNS; ++i)
            if (i < ns) red[(wave * kNS + i) * 64 + lane] = acc1[i];
        __syncthreads();
        for (int q = tid; q < ns * 16; q += 256) {
            const int i = q >> 4, row = q & 15, n = (slab0 + i) * 16 + row;
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w)
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) s += red[(w * kNS + i) * 64 + gg * 16 + row];
            if (n >= N) continue;
            if (a.splits > 1)
                __hip_atomic_store(&a.partial[(size_t)blockIdx.z * N + n], s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else if (a.y_f32) reinterpret_cast<float *>(a.Y)[n] = s;
            else reinterpret_cast<uint16_t *>(a.Y)[n] = bf16_bits(s);
        }
    } else {
        f32x4 *red = reinterpret_cast<f32x4 *>(smem);  // [4][kNS][64]
#pragma unroll
        for (int i = 0; i < kNS; ++i)
            if (i < ns) red[(wave * kNS + i) * 64 + lane] = acc[i];
        __syncthreads();
        for (int q = tid; q < ns * 64; q += 256) {
            const int i = q >> 6, l = q & 63, m = l & 15, gl = l >> 4;
            if (m >= M) continue;
            f32x4 s = red[(0 * kNS + i) * 64 + l];
#pragma unroll
            for (int w = 1; w < 4; ++w) {
                const f32x4 t = red[(w * kNS + i) * 64 + l];
                s[0] += t[0]; s[1] += t[1]; s[2] += t[2]; s[3] += t[3];
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int n = (slab0 + i) * 16 + 4 * gl + e;
                if (n >= N) continue;
                if (a.splits > 1)
                    __hip_atomic_store(&a.partial[((size_t)blockIdx.z * M + m) * N + n], s[e], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                else if (a.y_f32) reinterpret_cast<float *>(a.Y)[(size_t)m * N + n] = s[e];
                else reinterpret_cast<uint16_t *>(a.Y)[(size_t)m * N + n] = bf16_bits(s[e]);
            }
        }
    }

    // ---- 6. column blocks held by other workgroups: the last one to arrive adds them -----------
    if (a.splits > 1) {
        // The partial sums were written with device-coherent (write-through) stores, so waiting
        // for them to complete is enough to publish them; no L2 write-back or invalidate is needed.
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (tid == 0) {
            const unsigned old = __hip_atomic_fetch_add(&a.counters[blockIdx.x], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int last = (old == (unsigned)(a.splits - 1));
            // every other workgroup of this chunk has already passed: hand the ticket back at zero
            if (last) __hip_atomic_store(&a.counters[blockIdx.x], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *flag = last;
        }
        __syncthreads();
        if (*flag) {
            const int rows = ns * 16;
            for (int q = tid; q < M * rows; q += 256) {
                const int m = q / rows, n = slab0 * 16 + (q % rows);
                if (n >= N) continue;
                float s = 0.f;
                for (int z = 0; z < a.splits; ++z)
                    s += __hip_atomic_load(&a.partial[((size_t)z * M + m) * N + n], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (a.y_f32) reinterpret_cast<float *>(a.Y)[(size_t)m * N + n] = s;
                else reinterpret_cast<uint16_t *>(a.Y)[(size_t)m * N + n] = bf16_bits(s);
            }
        }
    }
}


// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
constexpr size_t kCounterBytes = kTicketBytes;     // tickets: 4096 slab chunks

static int decode_ss(const MatmulProblem &p)
{
    const int r_eff = p.f32fact ? 3 * p.r : p.r;
    const int rp = (r_eff + 31) / 32;
    return rp <= 1 ? 1 : rp <= 2 ? 2 : rp <= 4 ? 4 : 0;
}

struct DecodePlan {
    int ss, G, KT, splits, ns, chunks;
};

static DecodePlan decode_plan(const MatmulProblem &p)
{
    DecodePlan d;
    d.ss = decode_ss(p);
    d.G = d.ss == 1 ? 2 : 1;
    d.KT = 128 * d.G;
    const int kblocks = (p.K + d.KT - 1) / d.KT;
    d.splits = (kblocks + 3) / 4;
    const int nslabs = (p.N + 15) / 16;
    int want_chunks = 512 / d.splits;                  // about two resident workgroups per CU
    if (want_chunks < 1) want_chunks = 1;
    int ns = (nslabs + want_chunks - 1) / want_chunks;
    if (ns > kNS) ns = kNS;
    if (ns < 1) ns = 1;
    d.ns = ns;
    d.chunks = (nslabs + ns - 1) / ns;
    return d;
}

bool decode_fast_supported(const MatmulProblem &p)
{
    if (decode_ss(p) == 0) return false;
    const DecodePlan d = decode_plan(p);
    return (size_t)d.chunks * sizeof(unsigned) <= kCounterBytes;
}

size_t decode_fast_workspace_bytes(const MatmulProblem &p)
{
    const DecodePlan d = decode_plan(p);
    if (d.splits <= 1) return 0;
    const int mchunk = p.M < 16 ? p.M : 16;
    return kCounterBytes + (size_t)d.splits * mchunk * p.N * sizeof(float);
}

template <int BITS, int SS, int G, bool BVEC, bool M1>
static hipError_t launch_decode_t(const DecodeArgs &a, dim3 grid, hipStream_t st)
{
    constexpr int KT = 128 * G, AST = KT + 8;
    constexpr size_t A_BYTES = 4 * 32 * AST * 2, LUT_BYTES = (size_t)(1 << (2 * BITS)) * 256, RED_BYTES = 4 * kNS * 64 * 16;
    constexpr size_t R0 = A_BYTES > LUT_BYTES ? (A_BYTES > RED_BYTES ? A_BYTES : RED_BYTES)
                                              : (LUT_BYTES > RED_BYTES ? LUT_BYTES : RED_BYTES);
    const size_t smem = R0 + 128;
    static LdsOptIn lds_opt_in;
    if (smem > 48 * 1024) {
        const hipError_t e = allow_dynamic_lds(lds_opt_in, reinterpret_cast<const void *>(&decode_kernel<BITS, SS, G, BVEC, M1>), smem);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((decode_kernel<BITS, SS, G, BVEC, M1>), grid, dim3(256), smem, st, a);
    return hipGetLastError();
}

// `workspace` must be zero-filled when first handed over (tickets) and hold
// decode_fast_workspace_bytes(p) bytes; the kernel leaves the tickets at zero again.
hipError_t launch_decode_fast(const MatmulProblem &p, void *workspace, hipStream_t st)
{
    const DecodePlan d = decode_plan(p);
    for (int m0 = 0; m0 < p.M; m0 += 16) {
        DecodeArgs a;
        a.M = (p.M - m0) < 16 ? (p.M - m0) : 16;
        a.X = (const uint16_t *)p.X + (size_t)m0 * p.K;
        a.Y = p.f32out ? (void *)((float *)p.Y + (size_t)m0 * p.N) : (void *)((uint16_t *)p.Y + (size_t)m0 * p.N);
        a.codes = (const uint8_t *)p.codes;
        a.codebook = p.codebook;
        a.f.B = p.B; a.f.A = p.A; a.f.N = p.N; a.f.K = p.K; a.f.r = p.r;
        a.f.f32 = p.f32fact ? 1 : 0;
        a.f.r_eff = p.f32fact ? 3 * p.r : p.r;
        a.counters = (unsigned *)workspace;
        a.partial = workspace ? (float *)((unsigned char *)workspace + kCounterBytes) : nullptr;
        a.N = p.N; a.K = p.K;
        a.y_f32 = p.f32out ? 1 : 0;
        a.row_bytes = p.K / 8 * p.bits;
        a.nslabs = (p.N + 15) / 16;
        a.ns = d.ns;
        a.splits = d.splits;
        a.b_vec_ok = (!p.f32fact && (p.r % 8) == 0) ? 1 : 0;
        const dim3 grid(d.chunks, 1, d.splits);
        hipError_t e = hipErrorInvalidValue;
#define LORDS_DCASE(B_, S_, G_) \
    if (p.bits == B_ && d.ss == S_) \
        e = a.b_vec_ok ? (a.M == 1 ? launch_decode_t<B_, S_, G_, true, true>(a, grid, st)   \
                                   : launch_decode_t<B_, S_, G_, true, false>(a, grid, st)) \
                       : (a.M == 1 ? launch_decode_t<B_, S_, G_, false, true>(a, grid, st)  \
                                   : launch_decode_t<B_, S_, G_, false, false>(a, grid, st));
        LORDS_DCASE(2, 1, 2) LORDS_DCASE(2, 2, 1) LORDS_DCASE(2, 4, 1)
        LORDS_DCASE(3, 1, 2) LORDS_DCASE(3, 2, 1) LORDS_DCASE(3, 4, 1)
        LORDS_DCASE(4, 1, 2) LORDS_DCASE(4, 2, 1) LORDS_DCASE(4, 4, 1)
#undef LORDS_DCASE
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace lords

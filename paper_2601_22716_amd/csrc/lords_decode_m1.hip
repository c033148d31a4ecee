// One-token (M = 1) decode kernel of  y = (C[Q] (.) (B A)) x  on gfx950: the GEMV.
//
// Work split.  A workgroup of eight waves owns ONE block of KT = 128*G columns and a chunk of
// 8*ns slabs of 16 rows; wave w streams down slabs w*ns .. w*ns+ns-1 of the chunk.  Because the
// eight waves share the column block, the A tile of the block is staged once per workgroup:
// A[j][k] * x[k] (the activation folded in, rounded to bf16) goes row-major into LDS, and each
// wave fetches its scale-MFMA a-operands from it with the transposing ds_read_b64_tr_b16 and
// keeps them in registers for the whole row stream.  The scale MFMAs then deliver S[n][k]*x[k];
// the lane multiplies by the level of its code (v_fma_mix_f32, fp16 level x fp32 scale) and
// accumulates its partial dot product of row n0+c in fp32.  Nothing is rounded to bf16 after the
// A tile.  At the end of a chunk the four lanes of a row are added with two cross-lane
// shuffles and the column blocks (gridDim.z of them) meet in a workspace: device-coherent
// stores, one arrival ticket per chunk, the last workgroup adds the blocks in increasing order,
// so results are run-to-run identical.
//
// Lane mapping and look-up table: as in lords_decode.hip (lane (c,g) holds the G*32 codes of
// row n0+c at columns kb + 32*(G*g+v); scale MFMA t, accumulator i <-> code 4t+i).
#include "lords_decode_common.h"

namespace lords {

#ifndef LORDS_M1_WAVES
#define LORDS_M1_WAVES 8
#endif
constexpr int kM1Waves = LORDS_M1_WAVES;
constexpr int kM1Threads = 64 * kM1Waves;

struct M1Args {
    const uint16_t *X;
    const uint8_t *codes;
    const float *codebook;
    Factors f;
    void *Y;
    float *partial;        // [kblocks][N] fp32, used when kblocks > 1
    unsigned *counters;    // one ticket per chunk, zero between calls
    int N, K;
    int y_f32;
    int row_bytes;
    int nslabs;            // ceil(N / 16)
    int ns;                // slabs per wave per chunk, <= kNS
    int nchunks;           // chunks of 8*ns slabs
    int kblocks;           // gridDim.z
};

template <int BITS, int SS, int G, bool BVEC>
__global__ __launch_bounds__(kM1Threads) void decode_m1_kernel(M1Args a)
{
    constexpr int KT = 128 * G, AST = KT + 8, NL = 1 << BITS, NE = 1 << (2 * BITS), CPR = KT / 8;
    constexpr int LUT_BYTES = NE * 256, A_BYTES = SS * 32 * AST * 2;
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t *As = reinterpret_cast<uint16_t *>(smem + LUT_BYTES);        // [SS*32][AST]
    int *flag = reinterpret_cast<int *>(smem + LUT_BYTES + A_BYTES);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int kb = blockIdx.z * KT;
    const int N = a.N, K = a.K;
    const uint32_t laneoff = (uint32_t)lane * 4u;
    const int ngroups = K >> 5;

    LORDS_STAMP(0);
    // Loads of slab i of the current chunk, branch-free (addresses clamped into the arrays) so that
    // they can run kDepth slabs ahead: codes of columns >= K meet zero scales, rank entries >= r of
    // B meet zero rows of the A tile, rows >= N are dropped at the store.
    int chunk = blockIdx.x;
    int slab0 = (chunk * kM1Waves + wave) * a.ns;                    // this wave's first slab
    uint32_t cw[kNS][G][BITS];
    bf16x8 Bop[kNS][SS];
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
    LORDS_STAMP_WG(0);
    LORDS_STAMP_ALL(8, atomicMin);
    LORDS_STAMP_ALL(9, atomicMax);
    // ---- 1. set-up loads (A tile of this column block, activations, levels: all L2-resident) go
    //         out FIRST, the first slabs of the row stream (HBM) right behind them.  A wave's loads
    //         return in order, so the other way round the set-up would wait for HBM. --------------
    constexpr int NCH = SS * 32 * CPR / kM1Threads;           // 16-byte chunks of the A tile per thread
    constexpr int NIT = (NE * 16 + kM1Threads - 1) / kM1Threads;
    const int kc = tid % CPR, k0 = kb + 8 * kc;               // the thread's column chunk is fixed
    u32x4 xv = u32x4{0u, 0u, 0u, 0u};
    u32x4 tmp[NCH];
    float lo[NIT], hi[NIT];
    if (!a.f.f32) {
        if (k0 < K) xv = *reinterpret_cast<const u32x4 *>(a.X + k0);
#pragma unroll
        for (int q = 0; q < NCH; ++q) {
            const int jj = (tid + kM1Threads * q) / CPR;
            tmp[q] = u32x4{0u, 0u, 0u, 0u};
            if (jj < a.f.r && k0 < K)
                tmp[q] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(a.f.A) + (size_t)jj * K + k0);
        }
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int id = tid + kM1Threads * it, idx = (id >> 4) & (NE - 1);
        lo[it] = a.codebook[idx & (NL - 1)];
        hi[it] = a.codebook[idx >> BITS];
    }
    __builtin_amdgcn_sched_barrier(0);
#ifdef LORDS_M1_SETUP_FIRST
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
    for (int i = 0; i < kDepth; ++i) issue(i);
    __builtin_amdgcn_sched_barrier(0);

    // ---- 2. the A tile, activations folded in: A[j][k] * x[k] rounded to bf16 ------------------
    if (!a.f.f32) {
#pragma unroll
        for (int q = 0; q < NCH; ++q) {
            const int jj = (tid + kM1Threads * q) / CPR;
            u32x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float l = __builtin_bit_cast(float, tmp[q][e] << 16) * __builtin_bit_cast(float, xv[e] << 16);
                const float h = __builtin_bit_cast(float, tmp[q][e] & 0xFFFF0000u) * __builtin_bit_cast(float, xv[e] & 0xFFFF0000u);
                o[e] = (uint32_t)bf16_bits(l) | ((uint32_t)bf16_bits(h) << 16);
            }
            *reinterpret_cast<u32x4 *>(As + jj * AST + 8 * kc) = o;
        }
    } else {
        for (int id = tid; id < SS * 32 * KT; id += kM1Threads) {
            const int jj = id / KT, kk = id % KT;
            const float x = (kb + kk < K) ? bf16_to_f32(a.X[kb + kk]) : 0.f;
            As[jj * AST + kk] = factorAx_bits(a.f, jj, kb + kk, x);
        }
    }
    // ---- 3. level table: entry idx = (code_hi << BITS) | code_lo, one dword column per lane ----
    {
        uint32_t *lut32 = reinterpret_cast<uint32_t *>(smem);
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int id = tid + kM1Threads * it, idx = id >> 4, q = id & 15;
            if (idx < NE) {
                f16x2 h;
                h[0] = (_Float16)lo[it];
                h[1] = (_Float16)hi[it];
                const uint32_t pv = __builtin_bit_cast(uint32_t, h);
                *reinterpret_cast<u32x4 *>(lut32 + idx * 64 + 4 * q) = u32x4{pv, pv, pv, pv};
            }
        }
    }
    __syncthreads();
    LORDS_STAMP(1);
    LORDS_STAMP_WG(1);
    bf16x8 Aop[G][SS][8];
#pragma unroll
    for (int s = 0; s < SS; ++s)
#pragma unroll
        for (int v = 0; v < G; ++v)
#pragma unroll
            for (int t = 0; t < 8; ++t)
                Aop[v][s][t] = tr_read_pair_d<AST>(As, 32 * s + 8 * g + (c >> 2), 32 * (G * (c & 3) + v) + 4 * t);
    LORDS_STAMP(2);
    LORDS_STAMP_WG(2);

    // ---- 3. the row stream, chunk by chunk ------------------------------------------------------
    for (; chunk < a.nchunks; chunk += gridDim.x) {
        if (chunk != (int)blockIdx.x) {
            slab0 = (chunk * kM1Waves + wave) * a.ns;
#pragma unroll
            for (int i = 0; i < kDepth; ++i) issue(i);
        }
        const int nsw = max(0, min(a.ns, a.nslabs - slab0));


        float acc1[kNS];
#pragma unroll
        for (int i = 0; i < kNS; ++i) {
            acc1[i] = 0.f;
            if (i < nsw) {
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
                        for (int pq = 0; pq < 8; ++pq) {   // code pairs 8hh .. 8hh+7 of the group
                            const uint32_t ad = pair_addr<BITS>(cw[i][v], 8 * hh + pq, laneoff);
                            const f16x2 h = __builtin_bit_cast(f16x2, lds_load_u32(ad));
                            const float s0 = S[pq >> 1][(2 * pq) & 3], s1 = S[pq >> 1][(2 * pq + 1) & 3];
                            if (pq & 1) { p2 = __builtin_fmaf((float)h[0], s0, p2); p3 = __builtin_fmaf((float)h[1], s1, p3); }
                            else        { p0 = __builtin_fmaf((float)h[0], s0, p0); p1 = __builtin_fmaf((float)h[1], s1, p1); }
                        }
                    }
                }
                acc1[i] = (p0 + p1) + (p2 + p3);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        LORDS_STAMP(3);
    LORDS_STAMP_WG(3);

        // ---- 4. add the four lanes of each row (two cross-lane steps, each issued for all slabs
        //         before its results are used), hand the row sums over -------------------------------
        float t16[kNS];
#pragma unroll
        for (int i = 0; i < kNS; ++i) t16[i] = __shfl_xor(acc1[i], 16);
#pragma unroll
        for (int i = 0; i < kNS; ++i) acc1[i] += t16[i];
#pragma unroll
        for (int i = 0; i < kNS; ++i) t16[i] = __shfl_xor(acc1[i], 32);
#pragma unroll
        for (int i = 0; i < kNS; ++i) {
            if (i < nsw) {
                const float v = acc1[i] + t16[i];
                const int n = (slab0 + i) * 16 + c;
                if (g == 0 && n < N) {
                    if (a.kblocks > 1)
                        __hip_atomic_store(&a.partial[(size_t)blockIdx.z * N + n], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    else if (a.y_f32) reinterpret_cast<float *>(a.Y)[n] = v;
                    else reinterpret_cast<uint16_t *>(a.Y)[n] = bf16_bits(v);
                }
            }
        }
        LORDS_STAMP(4);
    LORDS_STAMP_WG(4);
        // ---- 5. other column blocks: the last workgroup to arrive adds them in order --------------
        if (a.kblocks > 1) {
            // The partial sums went out as device-coherent (write-through) stores: once they have
            // completed they are visible to every workgroup, without an L2 write-back or invalidate.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            if (tid == 0) {
                const unsigned old = __hip_atomic_fetch_add(&a.counters[chunk], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const int last = (old == (unsigned)(a.kblocks - 1));
                // every other workgroup of this chunk has passed: hand the ticket back at zero
                if (last) __hip_atomic_store(&a.counters[chunk], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                *flag = last;
            }
            __syncthreads();
            if (*flag) {
                const int row0 = chunk * kM1Waves * a.ns * 16, rows = kM1Waves * a.ns * 16;
                // two rows per thread and pass, all their loads in flight at once; blocks added in order
                for (int q = tid; q < rows; q += 2 * kM1Threads) {
                    const int n0 = min(row0 + q, N - 1), n1 = min(row0 + q + kM1Threads, N - 1);
                    float s0 = 0.f, s1 = 0.f;
                    for (int z0 = 0; z0 < a.kblocks; z0 += 16) {
                        float t0[16], t1[16];
#pragma unroll
                        for (int u = 0; u < 16; ++u) {
                            const int z = min(z0 + u, a.kblocks - 1);
                            t0[u] = __hip_atomic_load(&a.partial[(size_t)z * N + n0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            t1[u] = __hip_atomic_load(&a.partial[(size_t)z * N + n1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
#pragma unroll
                        for (int u = 0; u < 16; ++u)
                            if (z0 + u < a.kblocks) { s0 += t0[u]; s1 += t1[u]; }
                    }
                    if (row0 + q < N && q < rows) {
                        if (a.y_f32) reinterpret_cast<float *>(a.Y)[n0] = s0;
                        else reinterpret_cast<uint16_t *>(a.Y)[n0] = bf16_bits(s0);
                    }
                    if (row0 + q + kM1Threads < N && q + kM1Threads < rows) {
                        if (a.y_f32) reinterpret_cast<float *>(a.Y)[n1] = s1;
                        else reinterpret_cast<uint16_t *>(a.Y)[n1] = bf16_bits(s1);
                    }
                }
            }
        }
        LORDS_STAMP(5);
    LORDS_STAMP_WG(5);
    }
    LORDS_STAMP(6);
    LORDS_STAMP_WG(6);
    LORDS_STAMP_ALL(10, atomicMin);
    LORDS_STAMP_ALL(11, atomicMax);
}

#ifdef LORDS_PHASE_TIMING
extern "C" int lords_debug_phase_times(unsigned long long *out)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(lords_phase_times), sizeof(unsigned long long) * 32);
}
extern "C" int lords_debug_wg_times(unsigned long long *out)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(lords_wg_times), sizeof(unsigned long long) * 4096 * 8);
}
extern "C" int lords_debug_reset()
{
    unsigned long long init[32];
    for (int i = 0; i < 32; ++i) init[i] = 0ull;
    init[16 + 8] = ~0ull; init[16 + 10] = ~0ull;
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(lords_phase_times), init, sizeof(init));
}
#endif

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct M1Plan {
    int ss, G, KT, kblocks, ns, nchunks, gx;
};

static int m1_ss(const MatmulProblem &p)
{
    const int r_eff = p.f32fact ? 3 * p.r : p.r;
    const int rp = (r_eff + 31) / 32;
    return rp <= 1 ? 1 : rp <= 2 ? 2 : rp <= 4 ? 4 : 0;
}

static M1Plan m1_plan(const MatmulProblem &p)
{
    M1Plan d;
    d.ss = m1_ss(p);
    d.G = d.ss == 1 ? 2 : 1;
    d.KT = 128 * d.G;
    d.kblocks = (p.K + d.KT - 1) / d.KT;
    const int nslabs = (p.N + 15) / 16;
    int gx = 256 / d.kblocks;                          // one resident workgroup per CU
    if (gx < 1) gx = 1;
    int ns = (nslabs + kM1Waves * gx - 1) / (kM1Waves * gx);
    if (ns > kNS) ns = kNS;
    if (ns < 1) ns = 1;
    d.ns = ns;
    d.nchunks = (nslabs + kM1Waves * ns - 1) / (kM1Waves * ns);
    d.gx = gx < d.nchunks ? gx : d.nchunks;
    return d;
}

bool decode_m1_supported(const MatmulProblem &p)
{
    if (p.M != 1 || m1_ss(p) == 0) return false;
    const M1Plan d = m1_plan(p);
    return (size_t)d.nchunks * sizeof(unsigned) <= kTicketBytes && d.kblocks <= 65535;
}

size_t decode_m1_workspace_bytes(const MatmulProblem &p)
{
    const M1Plan d = m1_plan(p);
    if (d.kblocks <= 1) return 0;
    return kTicketBytes + (size_t)d.kblocks * p.N * sizeof(float);
}

template <int BITS, int SS, int G, bool BVEC>
static hipError_t launch_m1_t(const M1Args &a, dim3 grid, hipStream_t st)
{
    constexpr int KT = 128 * G, AST = KT + 8;
    const size_t smem = (size_t)(1 << (2 * BITS)) * 256 + (size_t)SS * 32 * AST * 2 + 64;
    static bool attr_set = false;
    if (!attr_set && smem > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&decode_m1_kernel<BITS, SS, G, BVEC>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((decode_m1_kernel<BITS, SS, G, BVEC>), grid, dim3(kM1Threads), smem, st, a);
    return hipGetLastError();
}

hipError_t launch_decode_m1(const MatmulProblem &p, void *workspace, hipStream_t st)
{
    const M1Plan d = m1_plan(p);
    M1Args a;
    a.X = (const uint16_t *)p.X;
    a.codes = (const uint8_t *)p.codes;
    a.codebook = p.codebook;
    a.f.B = p.B; a.f.A = p.A; a.f.N = p.N; a.f.K = p.K; a.f.r = p.r;
    a.f.f32 = p.f32fact ? 1 : 0;
    a.f.r_eff = p.f32fact ? 3 * p.r : p.r;
    a.Y = p.Y;
    a.counters = (unsigned *)workspace;
    a.partial = workspace ? (float *)((unsigned char *)workspace + kTicketBytes) : nullptr;
    a.N = p.N; a.K = p.K;
    a.y_f32 = p.f32out ? 1 : 0;
    a.row_bytes = p.K / 8 * p.bits;
    a.nslabs = (p.N + 15) / 16;
    a.ns = d.ns;
    a.nchunks = d.nchunks;
    a.kblocks = d.kblocks;
    const bool bvec = !p.f32fact && (p.r % 8) == 0;
    const dim3 grid(d.gx, 1, d.kblocks);
    hipError_t e = hipErrorInvalidValue;
#define LORDS_M1CASE(B_, S_, G_) \
    if (p.bits == B_ && d.ss == S_) e = bvec ? launch_m1_t<B_, S_, G_, true>(a, grid, st) : launch_m1_t<B_, S_, G_, false>(a, grid, st);
    LORDS_M1CASE(2, 1, 2) LORDS_M1CASE(2, 2, 1) LORDS_M1CASE(2, 4, 1)
    LORDS_M1CASE(3, 1, 2) LORDS_M1CASE(3, 2, 1) LORDS_M1CASE(3, 4, 1)
    LORDS_M1CASE(4, 1, 2) LORDS_M1CASE(4, 2, 1) LORDS_M1CASE(4, 4, 1)
#undef LORDS_M1CASE
    return e;
}

}  // namespace lords

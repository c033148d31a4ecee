// One-token (M = 1) decode kernel of  y = (C[Q] (.) (B A)) x  on gfx950: the GEMV.
//
// Arithmetic.  With one activation vector the scale never has to be formed per element:
//      y[n] = sum_k C[q[n][k]] * (sum_j B[n][j] A[j][k]) * x[k]
//           = sum_j B[n][j] * T[n][j],      T = C[Q] (A (.) x)^T        (Sec. 3.3, regrouped)
// T is a dense N x K by K x r contraction, so it runs on the matrix cores: the b-operand is the
// looked-up level of each code (bf16), the a-operand the A tile with the activation folded in
// (A[j][k] * x[k], bf16; fp32 factors: the fp32 product split into a bf16 hi and a lo tile).
// The only per-element vector work left is the table look-up itself; the B factor enters once
// per row and rank entry, in fp32, on the fp32 accumulator.
//
// Work split.  A workgroup of eight waves owns ONE block of KT = 128*G columns and a chunk of
// 8*ns slabs of 16 rows; wave w streams down slabs w*ns .. w*ns+ns-1 of the chunk.  Because the
// eight waves share the column block, the folded A tile is staged once per workgroup, row-major
// in LDS, with coalesced loads; each wave then reads its MFMA a-operands from it (lane (i, g)
// needs eight consecutive columns of tile row i, the layout the MFMA wants) and keeps them in
// registers for the whole row stream.  Memory instructions are the scarce resource of this
// kernel (a wave-level load occupies the address unit for at least 16 cycles, far longer when
// its lanes touch many cache lines), so every stream load is a full 16 bytes per lane: G loads
// of codes and one of B per slab.
//
// Rank order.  Tile row i of a-operand tile t stands for rank entry j = QW*(i/4) + 4*t + i%4
// (QW = rank entries per lane group), so that accumulator lane (c, g) ends up with T[n0+c][j]
// for the CONTIGUOUS run j = QW*g .. QW*g+QW-1 and its share of B[n0+c][.] is one vector load.
//
// At the end of a chunk the four lanes of a row are added with two cross-lane steps and the
// column blocks (gridDim.z of them) meet in a workspace: device-coherent stores, one arrival
// ticket per chunk, the last workgroup adds the blocks in increasing order, so results are
// run-to-run identical.
//
// Lane mapping and look-up table: lane (c, g) = (lane % 16, lane / 16) holds the G 32-code
// groups of row n0+c at columns kb + 32*(G*g+v); MFMA (v, u) contracts codes 8u..8u+7 of group
// v of all four lane groups.  Table entry (code_hi << BITS) | code_lo holds the two levels as a
// bf16 pair, replicated once per lane (address = entry*256 + lane*4: no bank conflicts).
#include "lords_decode_common.h"

namespace lords {

constexpr int kM1Waves = 8;
constexpr int kM1Threads = 64 * kM1Waves;
constexpr int kM1Tickets = 64;        // chunks whose tickets are taken at once
constexpr int kM1Depth = kDepth;      // slabs whose loads are in flight ahead of the one computed (deeper measured slower)

constexpr int kM1MaxLayers = kMaxBatch;   // matrices one batched launch can hold

// One weight matrix.  A batched launch (several matrices applied to the same activation vector)
// gives each matrix a contiguous range of blockIdx.x.
struct M1Layer {
    const uint8_t *codes;
    const void *A;         // r x K
    const void *B;         // N x r
    void *Y;
    float *partial;        // [kblocks][N] fp32, used when the column blocks meet in the workspace
    unsigned *counters;    // one ticket per chunk, zero between calls
    int N;
    int nslabs;            // ceil(N / 16)
    int ns;                // slabs per wave per chunk, <= kNS
    int nchunks;           // chunks of 8*ns slabs
    int gx0, gxn;          // first blockIdx.x of this matrix and how many it has
};

template <int NLAYERS>
struct M1ArgsT {
    const uint16_t *X;
    const float *codebook;
    int K, r;
    int y_f32;
    int row_bytes;
    int kblocks;           // gridDim.z
    int L;                 // matrices in this launch
    int act;               // 1: matrices 0 and 1 are a gate/up pair, Y of matrix 0 receives silu(gate) * up
    M1Layer layer[NLAYERS];
};
typedef M1ArgsT<1> M1Args;
typedef M1ArgsT<kM1MaxLayers> M1MultiArgs;

// BITS: code width.  JT: 16-row a-operand tiles (bf16 factors: one per 16 rank entries, 2 or 4;
// fp32 factors: the hi tiles, then as many lo tiles).  G: 32-code groups per lane.  BVEC: the B
// run of a lane can be read with 16-byte loads.  F32: fp32 factors.  MULTI: batched launch.
template <int BITS, int JT, int G, bool BVEC, bool F32, bool MULTI = false>
__global__ __launch_bounds__(kM1Threads) __attribute__((amdgpu_waves_per_eu(2, 2))) void decode_m1_kernel(M1ArgsT<MULTI ? kM1MaxLayers : 1> a)
{
    constexpr int CBW = G == 1 ? 4 : 1, NSG = kM1Waves / CBW;        // column blocks per workgroup, waves per block
    constexpr int KT = 128 * G, WK = CBW * KT, AST = WK + 8, NL = 1 << BITS, NE = 1 << (2 * BITS), CPR = WK / 8;
    constexpr int JR = F32 ? JT / 2 : JT;                   // tiles of the rank itself
    constexpr int QW = 4 * JR;                              // rank entries per lane group
    constexpr int BW = F32 ? QW : QW / 2;                   // dwords of B per lane and slab
    constexpr int LUT_BYTES = NE * 256, A_BYTES = JT * 16 * AST * 2;
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t *As = reinterpret_cast<uint16_t *>(smem + LUT_BYTES);        // [JT*16][AST]; later the block sums
    int *flag = reinterpret_cast<int *>(smem + LUT_BYTES + A_BYTES);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int cb = wave % CBW, sg = wave / CBW;                // this wave's column block and slab group
    const int kw = blockIdx.z * WK;                            // first column of the workgroup
    const int kb = kw + cb * KT;                               // first column of this wave
    // the matrix this workgroup works on (wave-uniform), its index among that matrix's workgroups
    int li = 0;
    if (MULTI)
        while (li + 1 < a.L && (int)blockIdx.x >= a.layer[li + 1].gx0) ++li;
    const M1Layer ly = a.layer[MULTI ? li : 0];
    const int bx = MULTI ? (int)blockIdx.x - ly.gx0 : (int)blockIdx.x;
    const int gxl = MULTI ? ly.gxn : (int)gridDim.x;
    const bool meet = a.kblocks > 1 || (MULTI && a.act);      // column blocks (and a gate/up pair) meet in the workspace
    const int N = ly.N, K = a.K, r = a.r;
    const uint32_t laneoff = (uint32_t)lane * 4u;
    const int ngroups = K >> 5;

    // Loads of slab i of the current chunk, branch-free (addresses clamped into the arrays) so that
    // they can run kM1Depth slabs ahead: codes of columns >= K meet zero a-operands, rank entries
    // >= r meet zero rows of the A tile (their B entries are read from the front of the row, or set to
    // zero by the entry-wise gather), rows >= N are dropped at the store.
    int chunk = bx;
    int slab0 = (chunk * NSG + sg) * ly.ns;                           // this wave's first slab
    uint32_t cw[kNS][G][BITS];
    uint32_t Bq[kNS][BW];
    // (a request past the wave's last slab `last` repeats that slab: same cache lines, no new traffic)
    auto issue = [&](int i, int first, int last) __attribute__((always_inline)) {
        const int n = min(min(first + i, last) * 16 + c, N - 1);
#pragma unroll
        for (int v = 0; v < G; ++v) {
            const int grp = min((kb >> 5) + G * g + v, ngroups - 1);
            load_group<BITS>(ly.codes + (size_t)n * a.row_bytes + (size_t)grp * (4 * BITS), cw[i][v]);
        }
        if (BVEC) {
#pragma unroll
            for (int h = 0; h < BW / 4; ++h) {
                const int j0 = QW * g + (F32 ? 4 : 8) * h;
                const int jc = j0 < r ? j0 : 0;
                u32x4 t;
                if (F32) t = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const float *>(ly.B) + (size_t)n * r + jc);
                else t = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(ly.B) + (size_t)n * r + jc);
#pragma unroll
                for (int e = 0; e < 4; ++e) Bq[i][4 * h + e] = t[e];
            }
        }
    };
    // B run of a lane when it cannot be read as vectors: entry by entry, zero beyond the rank
    auto gather_B = [&](int i) __attribute__((always_inline)) {
        const int n = min((slab0 + i) * 16 + c, N - 1);
        uint32_t t[QW];
#pragma unroll
        for (int e = 0; e < QW; ++e) {
            const int j = QW * g + e, jc = j < r ? j : 0;
            const uint32_t raw = F32 ? reinterpret_cast<const uint32_t *>(ly.B)[(size_t)n * r + jc]
                                     : (uint32_t)reinterpret_cast<const uint16_t *>(ly.B)[(size_t)n * r + jc];
            t[e] = j < r ? raw : 0u;
        }
#pragma unroll
        for (int e = 0; e < BW; ++e) Bq[i][e] = F32 ? t[e % QW] : (t[(2 * e) % QW] | (t[(2 * e + 1) % QW] << 16));
    };

    // ---- 1. set-up loads (A tile of this column block, activations, levels) go out FIRST, the
    //         first slabs of the row stream right behind them.  A wave's loads return in order,
    //         so the other way round the set-up would wait for the stream. --------------------------
    constexpr int NCH = JT * 16 * CPR / kM1Threads;           // 16-byte chunks of the A tile per thread
    constexpr int NIT = (NE * 16 + kM1Threads - 1) / kM1Threads;
    const int kc = tid % CPR, k0 = kw + 8 * kc;               // the thread's column chunk is fixed
    u32x4 xv = u32x4{0u, 0u, 0u, 0u};
    u32x4 tmp[F32 ? 1 : NCH];
    float lo[NIT], hi[NIT];
    if (!F32) {
        if (k0 < K) xv = *reinterpret_cast<const u32x4 *>(a.X + k0);
#pragma unroll
        for (int q = 0; q < NCH; ++q) {
            const int jj = (tid + kM1Threads * q) / CPR, t = jj >> 4, i = jj & 15;
            const int j = QW * (i >> 2) + 4 * t + (i & 3);
            tmp[q] = u32x4{0u, 0u, 0u, 0u};
            if (j < r && k0 < K)
                tmp[q] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(ly.A) + (size_t)j * K + k0);
        }
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int id = tid + kM1Threads * it, idx = (id >> 4) & (NE - 1);
        lo[it] = a.codebook[idx & (NL - 1)];
        hi[it] = a.codebook[idx >> BITS];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < kM1Depth; ++i) issue(i, slab0, max(slab0, min(slab0 + ly.ns, ly.nslabs) - 1));
    __builtin_amdgcn_sched_barrier(0);

    // ---- 2. the A tile, activations folded in: A[j][k] * x[k] rounded to bf16 ------------------
    if (!F32) {
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
        // fp32 factors (not the fast case): the fp32 product, split into a bf16 hi and lo tile
        for (int id = tid; id < JR * 16 * WK; id += kM1Threads) {
            const int jj = id / WK, kk = id % WK, t = jj >> 4, i = jj & 15;
            const int j = QW * (i >> 2) + 4 * t + (i & 3);
            float p = 0.f;
            if (j < r && kw + kk < K)
                p = reinterpret_cast<const float *>(ly.A)[(size_t)j * K + kw + kk] * bf16_to_f32(a.X[kw + kk]);
            const uint16_t ph = bf16_bits(p);
            As[jj * AST + kk] = ph;
            As[(JR * 16 + jj) * AST + kk] = bf16_bits(p - bf16_to_f32(ph));
        }
    }
    // ---- 3. level table ------------------------------------------------------------------------
    {
        uint32_t *lut32 = reinterpret_cast<uint32_t *>(smem);
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int id = tid + kM1Threads * it, idx = id >> 4, q = id & 15;
            if (idx < NE) {
                const uint32_t pv = (uint32_t)bf16_bits(lo[it]) | ((uint32_t)bf16_bits(hi[it]) << 16);
                *reinterpret_cast<u32x4 *>(lut32 + idx * 64 + 4 * q) = u32x4{pv, pv, pv, pv};
            }
        }
    }
    __syncthreads();
    bf16x8 Aop[G][4][JT];
#pragma unroll
    for (int v = 0; v < G; ++v)
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int t = 0; t < JT; ++t)
                Aop[v][u][t] = *reinterpret_cast<const bf16x8 *>(As + (16 * t + c) * AST + cb * KT + 32 * (G * g + v) + 8 * u);
    if (CBW > 1) __syncthreads();                          // every wave has its operands: the tile region may be reused

    // ---- 4. the row stream, chunk by chunk ------------------------------------------------------
    for (; chunk < ly.nchunks; chunk += gxl) {
        slab0 = (chunk * NSG + sg) * ly.ns;                  // (its first kM1Depth slabs are on their way)
        const int nsw = max(0, min(ly.ns, ly.nslabs - slab0));

        float ysum[kNS];
#pragma unroll
        for (int i = 0; i < kNS; ++i) {
            ysum[i] = 0.f;
            if (i < nsw) {
                if (i + kM1Depth < kNS) issue(i + kM1Depth, slab0, slab0 + nsw - 1);
                __builtin_amdgcn_sched_barrier(0);     // keep the prefetch ahead of this slab's arithmetic
                if (!BVEC) gather_B(i);
                // one accumulator per tile, first MFMA on a literal zero; the two tiles (and the
                // other wave of the SIMD) hide the latency of the dependent chain
                // one accumulator chain per (group, tile): independent chains keep the matrix pipe busy
                f32x4 acc[G][JT];
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int v = 0; v < G; ++v) {
                        u32x4 w;
#pragma unroll
                        for (int d = 0; d < 4; ++d) w[d] = lds_load_u32(pair_addr<BITS>(cw[i][v], 4 * u + d, laneoff));
                        const bf16x8 Wop = __builtin_bit_cast(bf16x8, w);
#pragma unroll
                        for (int t = 0; t < JT; ++t)
                            acc[v][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aop[v][u][t], Wop,
                                                                                u == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[v][t], 0, 0, 0);
                    }
                // accumulator element e of tile t is T[n][QW*g + 4t + e]: weigh with the lane's B run
                float y0 = 0.f, y1 = 0.f;
#pragma unroll
                for (int t = 0; t < JR; ++t)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float s = acc[0][t][e];
                        if (G == 2) s += acc[G - 1][t][e];
                        if (F32) {
                            s += acc[0][JT - JR + t][e];
                            if (G == 2) s += acc[G - 1][JT - JR + t][e];
                        }
                        const int q = 4 * t + e;                       // position in the lane's run
                        const uint32_t raw = F32 ? Bq[i][q % BW] : ((q & 1) ? (Bq[i][(q >> 1) % BW] & 0xFFFF0000u) : (Bq[i][(q >> 1) % BW] << 16));
                        float b = __builtin_bit_cast(float, raw);
                        // (a vector-loaded run beyond the rank holds the row's first entries, finite
                        //  values, and meets s = 0 exactly: those rows of the A tile are zero)
                        if (e & 1) y1 = __builtin_fmaf(s, b, y1);
                        else y0 = __builtin_fmaf(s, b, y0);
                    }
                ysum[i] = y0 + y1;
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        // The first slabs of the next chunk are requested before this chunk's sums are handed over
        // (their registers are free), so the stream does not drain in between.  Outside the slab
        // loop on purpose: inside it every load is unconditional, which lets the compiler count
        // exactly how many are in flight at each use.
        if (chunk + gxl < ly.nchunks) {
            const int next0 = ((chunk + gxl) * NSG + sg) * ly.ns;
#pragma unroll
            for (int i = 0; i < kM1Depth; ++i) issue(i, next0, max(next0, min(next0 + ly.ns, ly.nslabs) - 1));
        }

        // ---- 5. add the four lanes of each row (two cross-lane steps, each issued for all slabs
        //         before its results are used), hand the row sums over -------------------------------
        float t16[kNS];
#pragma unroll
        for (int i = 0; i < kNS; ++i) t16[i] = __shfl_xor(ysum[i], 16);
#pragma unroll
        for (int i = 0; i < kNS; ++i) ysum[i] += t16[i];
#pragma unroll
        for (int i = 0; i < kNS; ++i) t16[i] = __shfl_xor(ysum[i], 32);
        if (CBW == 1) {
#pragma unroll
            for (int i = 0; i < kNS; ++i) {
                if (i < nsw) {
                    const float v = ysum[i] + t16[i];
                    const int n = (slab0 + i) * 16 + c;
                    if (g == 0 && n < N) {
                        if (meet)
                            __hip_atomic_store(&ly.partial[(size_t)blockIdx.z * N + n], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        else if (a.y_f32) reinterpret_cast<float *>(ly.Y)[n] = v;
                        else reinterpret_cast<uint16_t *>(ly.Y)[n] = bf16_bits(v);
                    }
                }
            }
        } else {
            // the column blocks of this workgroup meet in LDS (the A tile is dead) and are added in block order
            float *red = reinterpret_cast<float *>(As);                  // [kM1Waves][kNS*16]
            if (g == 0) {
#pragma unroll
                for (int i = 0; i < kNS; ++i) red[wave * (kNS * 16) + i * 16 + c] = ysum[i] + t16[i];
            }
            __syncthreads();
            const int rows_sg = ly.ns * 16;                               // rows of one slab group
            if (tid < NSG * rows_sg) {
                const int sgr = tid / rows_sg, rem = tid - sgr * rows_sg;
                float v = 0.f;
#pragma unroll
                for (int w = 0; w < CBW; ++w) v += red[(sgr * CBW + w) * (kNS * 16) + rem];
                const int n = (chunk * NSG + sgr) * rows_sg + rem;
                if (n < N) {
                    if (meet)
                        __hip_atomic_store(&ly.partial[(size_t)blockIdx.z * N + n], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    else if (a.y_f32) reinterpret_cast<float *>(ly.Y)[n] = v;
                    else reinterpret_cast<uint16_t *>(ly.Y)[n] = bf16_bits(v);
                }
            }
            __syncthreads();                                             // the sums are rewritten by the next chunk
        }
    }

    // ---- 6. other column blocks: for every chunk this workgroup streamed, the last workgroup to
    //         arrive adds the blocks in order.  Done once, after the last chunk, so that the two
    //         dependent round trips (stores acknowledged, then the ticket) are paid once.  The
    //         partial sums went out as device-coherent (write-through) stores: once they have
    //         completed they are visible to every workgroup, without an L2 write-back or invalidate.
    if (meet) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        // a gate/up pair shares its tickets (same chunking): the last of both matrices' workgroups finishes
        const bool pair = MULTI && a.act;
        const unsigned arrivals = (unsigned)a.kblocks * (pair ? 2u : 1u);
        const float *Pg = pair ? a.layer[0].partial : ly.partial;
        const float *Pu = pair ? a.layer[MULTI ? 1 : 0].partial : nullptr;
        void *Yout = pair ? a.layer[0].Y : ly.Y;
        const int niter = (ly.nchunks - bx + gxl - 1) / gxl;
        for (int base = 0; base < niter; base += kM1Tickets) {
            const int nt = min(kM1Tickets, niter - base);
            if (tid < nt) {
                const int ch = bx + (base + tid) * gxl;
                const unsigned old = __hip_atomic_fetch_add(&ly.counters[ch], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const int last = (old == arrivals - 1u);
                // every other workgroup of this chunk has passed: hand the ticket back at zero
                if (last) __hip_atomic_store(&ly.counters[ch], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                flag[tid] = last;
            }
            __syncthreads();
            for (int t = 0; t < nt; ++t) {
                if (!flag[t]) continue;
                const int ch = bx + (base + t) * gxl;
                const int row0 = ch * NSG * ly.ns * 16, rows = NSG * ly.ns * 16;
                // two rows per thread and pass, all their loads in flight at once; blocks added in order
                for (int q = tid; q < rows; q += 2 * kM1Threads) {
                    const int n0 = min(row0 + q, N - 1), n1 = min(row0 + q + kM1Threads, N - 1);
                    float s0 = 0.f, s1 = 0.f;
                    auto add_blocks = [&](const float *P, float &r0, float &r1) __attribute__((always_inline)) {
                        for (int z0 = 0; z0 < a.kblocks; z0 += 16) {
                            float t0[16], t1[16];
#pragma unroll
                            for (int u = 0; u < 16; ++u) {
                                const int z = min(z0 + u, a.kblocks - 1);
                                t0[u] = __hip_atomic_load(&P[(size_t)z * N + n0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                t1[u] = __hip_atomic_load(&P[(size_t)z * N + n1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            }
#pragma unroll
                            for (int u = 0; u < 16; ++u)
                                if (z0 + u < a.kblocks) { r0 += t0[u]; r1 += t1[u]; }
                        }
                    };
                    add_blocks(Pg, s0, s1);
                    if (pair) {
                        // SwiGLU gate: silu(gate) * up on the fp32 sums, one rounding at the store
                        float u0 = 0.f, u1 = 0.f;
                        add_blocks(Pu, u0, u1);
                        s0 = s0 / (1.0f + __expf(-s0)) * u0;
                        s1 = s1 / (1.0f + __expf(-s1)) * u1;
                    }
                    if (row0 + q < N && q < rows) {
                        if (a.y_f32) reinterpret_cast<float *>(Yout)[n0] = s0;
                        else reinterpret_cast<uint16_t *>(Yout)[n0] = bf16_bits(s0);
                    }
                    if (row0 + q + kM1Threads < N && q + kM1Threads < rows) {
                        if (a.y_f32) reinterpret_cast<float *>(Yout)[n1] = s1;
                        else reinterpret_cast<uint16_t *>(Yout)[n1] = bf16_bits(s1);
                    }
                }
            }
            __syncthreads();                               // the flags are rewritten by the next batch
        }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct M1Plan {
    int jt, G, KT, kblocks, ns, nchunks, gx;
};

// a-operand tiles: bf16 factors need ceil(r/16), fp32 factors twice that (hi and lo); 2 or 4 are built
static int m1_jt(const MatmulProblem &p)
{
    const int tiles = (p.r + 15) / 16 * (p.f32fact ? 2 : 1);
    return tiles <= 2 ? 2 : tiles <= 4 ? 4 : 0;
}

// Slabs per wave and chunk when `nslabs` slabs are shared by `lanes` waves (all workgroups of a
// column block): a wave's share is cut into the fewest passes of at most kNS slabs, all equally long.
static int m1_slabs_per_chunk(long nslabs, long lanes)
{
    long share = (nslabs + lanes - 1) / lanes;
    if (share < 1) share = 1;
    const long passes = (share + kNS - 1) / kNS;
    return (int)((share + passes - 1) / passes);
}

static M1Plan m1_plan(const MatmulProblem &p)
{
    M1Plan d;
    d.jt = m1_jt(p);
    d.G = d.jt == 2 ? 2 : 1;
    d.KT = 128 * d.G;
    const int cbw = d.G == 1 ? 4 : 1, nsg = kM1Waves / cbw;      // as in the kernel
    d.kblocks = (p.K + cbw * d.KT - 1) / (cbw * d.KT);
    const int nslabs = (p.N + 15) / 16;
    int gx = 256 / d.kblocks;                          // one resident workgroup per CU
    if (gx < 1) gx = 1;
    d.ns = m1_slabs_per_chunk(nslabs, nsg * gx);
    d.nchunks = (nslabs + nsg * d.ns - 1) / (nsg * d.ns);
    d.gx = gx < d.nchunks ? gx : d.nchunks;
    return d;
}

bool decode_m1_supported(const MatmulProblem &p)
{
    if (p.M != 1 || m1_jt(p) == 0) return false;
    const M1Plan d = m1_plan(p);
    return (size_t)d.nchunks * sizeof(unsigned) <= kTicketBytes && d.kblocks <= 65535;
}

size_t decode_m1_workspace_bytes(const MatmulProblem &p)
{
    const M1Plan d = m1_plan(p);
    if (d.kblocks <= 1) return 0;
    return kTicketBytes + (size_t)d.kblocks * p.N * sizeof(float);
}

template <int BITS, int JT, int G, bool BVEC, bool F32, bool MULTI>
static hipError_t launch_m1_t(const M1ArgsT<MULTI ? kM1MaxLayers : 1> &a, dim3 grid, hipStream_t st)
{
    constexpr int KT = 128 * G, AST = (G == 1 ? 4 : 1) * KT + 8;
    const size_t smem = (size_t)(1 << (2 * BITS)) * 256 + (size_t)JT * 16 * AST * 2 + kM1Tickets * sizeof(int);
    static LdsOptIn lds_opt_in;
    if (smem > 48 * 1024) {
        const hipError_t e = allow_dynamic_lds(lds_opt_in, reinterpret_cast<const void *>(&decode_m1_kernel<BITS, JT, G, BVEC, F32, MULTI>), smem);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((decode_m1_kernel<BITS, JT, G, BVEC, F32, MULTI>), grid, dim3(kM1Threads), smem, st, a);
    return hipGetLastError();
}

template <int BITS, int JT, int G>
static hipError_t launch_m1_b(const M1Args &a, dim3 grid, bool bvec, bool f32, hipStream_t st)
{
    if (f32) return bvec ? launch_m1_t<BITS, JT, G, true, true, false>(a, grid, st) : launch_m1_t<BITS, JT, G, false, true, false>(a, grid, st);
    return bvec ? launch_m1_t<BITS, JT, G, true, false, false>(a, grid, st) : launch_m1_t<BITS, JT, G, false, false, false>(a, grid, st);
}

hipError_t launch_decode_m1(const MatmulProblem &p, void *workspace, hipStream_t st)
{
    const M1Plan d = m1_plan(p);
    M1Args a;
    a.X = (const uint16_t *)p.X;
    a.codebook = p.codebook;
    a.K = p.K; a.r = p.r;
    a.y_f32 = p.f32out ? 1 : 0;
    a.row_bytes = p.K / 8 * p.bits;
    a.kblocks = d.kblocks;
    a.L = 1;
    a.act = 0;
    M1Layer &ly = a.layer[0];
    ly.codes = (const uint8_t *)p.codes;
    ly.A = p.A;
    ly.B = p.B;
    ly.Y = p.Y;
    ly.counters = (unsigned *)workspace;
    ly.partial = workspace ? (float *)((unsigned char *)workspace + kTicketBytes) : nullptr;
    ly.N = p.N;
    ly.nslabs = (p.N + 15) / 16;
    ly.ns = d.ns;
    ly.nchunks = d.nchunks;
    ly.gx0 = 0;
    ly.gxn = d.gx;
    // 16-byte loads of a lane's B run: the run starts at a multiple of 8 (bf16) or 4 (fp32) entries
    const bool bvec = p.f32fact ? (p.r % 4) == 0 : (p.r % 8) == 0;
    const dim3 grid(d.gx, 1, d.kblocks);
    hipError_t e = hipErrorInvalidValue;
#define LORDS_M1CASE(B_, J_, G_) \
    if (p.bits == B_ && d.jt == J_) e = launch_m1_b<B_, J_, G_>(a, grid, bvec, p.f32fact, st);
    LORDS_M1CASE(2, 2, 2) LORDS_M1CASE(2, 4, 1)
    LORDS_M1CASE(3, 2, 2) LORDS_M1CASE(3, 4, 1)
    LORDS_M1CASE(4, 2, 2) LORDS_M1CASE(4, 4, 1)
#undef LORDS_M1CASE
    return e;
}

// ---------------------------------------------------------------------------------------------
// batched launch: several matrices, one activation vector
// ---------------------------------------------------------------------------------------------
struct M1BatchPlan {
    int jt, G, kblocks, total_gx;
    int ns[kM1MaxLayers], nchunks[kM1MaxLayers], gx0[kM1MaxLayers], gxn[kM1MaxLayers];
    size_t ticket0[kM1MaxLayers], partial0[kM1MaxLayers];     // offsets in tickets / floats
    size_t tickets, partial_floats;
};

static bool m1_batch_plan(const BatchedProblem &p, M1BatchPlan &d)
{
    if (p.M != 1 || p.f32fact || p.L < 1 || p.L > kM1MaxLayers) return false;
    if (p.act && (p.L != 2 || p.N[0] != p.N[1])) return false;
    const int tiles = (p.r + 15) / 16;
    d.jt = tiles <= 2 ? 2 : tiles <= 4 ? 4 : 0;
    if (d.jt == 0) return false;
    d.G = d.jt == 2 ? 2 : 1;
    const int cbw = d.G == 1 ? 4 : 1, nsg = kM1Waves / cbw, wk = cbw * 128 * d.G;
    d.kblocks = (p.K + wk - 1) / wk;
    if (d.kblocks > 65535) return false;
    // workgroups per matrix: one resident workgroup per CU in total, shared out by row count
    int budget = 256 / d.kblocks;
    if (budget < p.L) budget = p.L;
    long nslabs[kM1MaxLayers], sum = 0;
    for (int l = 0; l < p.L; ++l) { nslabs[l] = (p.N[l] + 15) / 16; sum += nslabs[l]; }
    int gx[kM1MaxLayers], used = 0;
    for (int l = 0; l < p.L; ++l) {
        gx[l] = p.act ? budget / 2 : (int)((long)budget * nslabs[l] / sum);
        if (gx[l] < 1) gx[l] = 1;
        used += gx[l];
    }
    // what rounding down left over goes to the matrices with the most slabs per workgroup
    while (!p.act && used < budget) {
        int best = 0;
        for (int l = 1; l < p.L; ++l)
            if (nslabs[l] * gx[best] > nslabs[best] * gx[l]) best = l;
        ++gx[best];
        ++used;
    }
    d.tickets = 0;
    d.partial_floats = 0;
    int x0 = 0;
    for (int l = 0; l < p.L; ++l) {
        const int ns = m1_slabs_per_chunk(nslabs[l], (long)nsg * gx[l]);
        d.ns[l] = ns;
        d.nchunks[l] = (int)((nslabs[l] + nsg * ns - 1) / (nsg * ns));
        d.gxn[l] = gx[l] < d.nchunks[l] ? gx[l] : d.nchunks[l];
        d.gx0[l] = x0;
        x0 += d.gxn[l];
        d.ticket0[l] = (p.act && l == 1) ? d.ticket0[0] : d.tickets;
        if (!(p.act && l == 1)) d.tickets += (size_t)d.nchunks[l];
        d.partial0[l] = d.partial_floats;
        d.partial_floats += (size_t)d.kblocks * p.N[l];
    }
    d.total_gx = x0;
    return d.tickets * sizeof(unsigned) <= kTicketBytes;
}

bool decode_m1_batched_supported(const BatchedProblem &p)
{
    M1BatchPlan d;
    return m1_batch_plan(p, d);
}

size_t decode_m1_batched_workspace_bytes(const BatchedProblem &p)
{
    M1BatchPlan d;
    if (!m1_batch_plan(p, d)) return 0;
    return kTicketBytes + d.partial_floats * sizeof(float);
}

hipError_t launch_decode_m1_batched(const BatchedProblem &p, void *workspace, hipStream_t st)
{
    M1BatchPlan d;
    if (!m1_batch_plan(p, d) || !workspace) return hipErrorInvalidValue;
    M1MultiArgs a;
    a.X = (const uint16_t *)p.X;
    a.codebook = p.codebook;
    a.K = p.K; a.r = p.r;
    a.y_f32 = p.f32out ? 1 : 0;
    a.row_bytes = p.K / 8 * p.bits;
    a.kblocks = d.kblocks;
    a.L = p.L;
    a.act = p.act ? 1 : 0;
    for (int l = 0; l < kM1MaxLayers; ++l) {
        const int s = l < p.L ? l : 0;                      // unused entries: copies of the first
        M1Layer &ly = a.layer[l];
        ly.codes = (const uint8_t *)p.codes[s];
        ly.A = p.A[s];
        ly.B = p.B[s];
        ly.Y = p.Y[s];
        ly.counters = (unsigned *)workspace + d.ticket0[s];
        ly.partial = (float *)((unsigned char *)workspace + kTicketBytes) + d.partial0[s];
        ly.N = p.N[s];
        ly.nslabs = (p.N[s] + 15) / 16;
        ly.ns = d.ns[s];
        ly.nchunks = d.nchunks[s];
        ly.gx0 = d.gx0[s];
        ly.gxn = d.gxn[s];
    }
    const bool bvec = (p.r % 8) == 0;
    const dim3 grid(d.total_gx, 1, d.kblocks);
    hipError_t e = hipErrorInvalidValue;
#define LORDS_M1CASE(B_, J_, G_)                                                                  \
    if (p.bits == B_ && d.jt == J_)                                                                \
        e = bvec ? launch_m1_t<B_, J_, G_, true, false, true>(a, grid, st)                         \
                 : launch_m1_t<B_, J_, G_, false, false, true>(a, grid, st);
    LORDS_M1CASE(2, 2, 2) LORDS_M1CASE(2, 4, 1)
    LORDS_M1CASE(3, 2, 2) LORDS_M1CASE(3, 4, 1)
    LORDS_M1CASE(4, 2, 2) LORDS_M1CASE(4, 4, 1)
#undef LORDS_M1CASE
    return e;
}

}  // namespace lords

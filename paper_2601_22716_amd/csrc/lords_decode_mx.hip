// Few-token (2 <= M <= 16 per pass) decode kernel of  Y = X (C[Q] (.) (B A))^T  on gfx950,
// bf16 factors, contraction length up to 64.  Memory-bound by design: every packed code is read
// from HBM exactly once per pass and shared by the (up to) 16 tokens.
//
// Work split.  A workgroup of eight waves owns 4*KT consecutive columns (KT = 128*G) and a chunk
// of 2*ns slabs of 16 rows.  Wave w owns column block w%4 and the slabs of half w/4, so two waves
// per SIMD share the register file (256 VGPRs each, all MFMAs in VGPR form).  The A tile of the
// 4*KT columns is staged ONCE per workgroup, row-major in LDS, with coalesced loads; each wave
// reads its scale-MFMA a-operands from it with the transposing ds_read_b64_tr_b16.  The X tile
// (16 tokens x 4*KT columns) then goes through the same LDS region and comes back as the
// b-operands of the product MFMAs.  Both operand sets stay in registers for the whole row stream.
//
// Per slab a wave loads the lane's G*32 packed codes and 8*SS rank entries of its row of B (all
// 16-byte loads), forms the scales S = B A of its 16 x KT block with G*8*SS scale MFMAs, looks up
// the fp16 level pair of every two codes (replicated LDS table, one dword column per lane),
// multiplies level and scale (v_fma_mix_f32), rounds the product once to bf16 and feeds G*4 product
// MFMAs (rows x tokens).  The four column blocks of a workgroup meet in LDS and are added in block
// order; column blocks of other workgroups (gridDim.z of them) meet in a workspace: device-coherent
// stores, one arrival ticket per chunk, the last workgroup adds the blocks in increasing order.
// Results are run-to-run identical.
//
// Lane mapping (v_mfma_f32_16x16x32_bf16; lane l = (c = l%16, g = l/16)):
//   scale MFMA t of group v:  D[i][j],  j <-> row n0+j,
//                             i <-> column kb + 32*(G*(i/4)+v) + 4t + i%4,
//   so lane (c,g) gets, in accumulator i of MFMA t, the scale of code 4t+i of the 32-code group
//   it holds (columns kb + 32*(G*g+v) ...).
//   product MFMA u of group v: a-operand = the lane's 8 dequantised weights 8u..8u+7 of the
//   group, b-operand = X[c][the same 8 columns]; D[i][j] with i <-> row, j <-> token.
#include <type_traits>
#include "lords_decode_common.h"

namespace lords {

constexpr int kMxWaves = 8;
constexpr int kMxThreads = 64 * kMxWaves;
constexpr int kMxTickets = 64;        // chunks whose tickets are taken at once

// One weight matrix.  A batched launch (several matrices applied to the same activations) gives
// each matrix a contiguous range of blockIdx.x.
struct MxLayer {
    const uint8_t *codes;
    const uint16_t *A;     // r x K bf16
    const uint16_t *B;     // N x r bf16
    void *Y;
    float *partial;        // [splits][M][N] fp32, used when the column blocks meet in the workspace
    unsigned *counters;    // `parts` tickets per chunk, zero between calls
    int N;
    int nslabs;            // ceil(N / 16)
    int ns;                // slabs per wave per chunk, <= kNS
    int nchunks;           // chunks of 2*ns slabs
    int gx0, gxn;          // first blockIdx.x of this matrix and how many it has
};

template <int NLAYERS>
struct MxArgsT {
    const uint16_t *X;     // M x K bf16, M <= 16
    const float *codebook;
    int M, K, r;
    int y_f32;
    int row_bytes;
    int splits;            // gridDim.z
    int L;                 // matrices in this launch
    int act;               // 1: matrices 0 and 1 are a gate/up pair, Y of matrix 0 receives silu(gate) * up
    int tiled;             // codes in the slab-tile layout (16 rows x 128 columns per tile, chunk 16 g + c of 4 * BITS bytes)
    int nct;               // column tiles per slab, ceil(K / 128)
    int parts;             // tickets per chunk: the chunk's outputs are read back in `parts` shares, each with a ticket of its own
    MxLayer layer[NLAYERS];
};
typedef MxArgsT<1> MxArgs;
typedef MxArgsT<kMaxBatch> MxMultiArgs;

template <int BITS, int SS, int G, bool BVEC, bool MULTI = false>
__global__ __launch_bounds__(kMxThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void decode_mx_kernel(MxArgsT<MULTI ? kMaxBatch : 1> a)
{
    // QUAD (2-bit codes): the table is indexed by a byte of four codes and holds four fp16 levels per entry, 32
    // copies of 8 bytes (lanes l and l + 32 share a copy; an 8-byte read serves them in different cycles): half the
    // address operations and LDS reads per weight of a pair table.
    constexpr bool QUAD = BITS == 2;
    constexpr int KT = 128 * G, WK = 4 * KT, AST = WK + 8, NL = 1 << BITS, NE = QUAD ? 256 : 1 << (2 * BITS), CPR = WK / 8;
    constexpr int LUT_BYTES = NE * 256, A_BYTES = SS * 32 * AST * 2;
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t *As = reinterpret_cast<uint16_t *>(smem + LUT_BYTES);        // [SS*32][AST], then X [16][AST], then sums

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int cb = wave & 3, half = wave >> 2;
    const int kw = blockIdx.z * WK;                            // first column of the workgroup
    const int kb = kw + cb * KT;                               // first column of this wave's block
    // the matrix this workgroup works on (wave-uniform), its index among that matrix's workgroups
    int li = 0;
    if (MULTI)
        while (li + 1 < a.L && (int)blockIdx.x >= a.layer[li + 1].gx0) ++li;
    const MxLayer ly = a.layer[MULTI ? li : 0];
    const int bx = MULTI ? (int)blockIdx.x - ly.gx0 : (int)blockIdx.x;
    const int gxl = MULTI ? ly.gxn : (int)gridDim.x;
    const bool meet = a.splits > 1 || (MULTI && a.act);       // column blocks (and a gate/up pair) meet in the workspace
    const int N = ly.N, K = a.K, M = a.M, r = a.r;
    const uint32_t laneoff = QUAD ? (uint32_t)(lane & 31) * 8u : (uint32_t)lane * 4u;
    const int ngroups = K >> 5;

    // Loads of slab i of the current chunk, branch-free (addresses clamped into the arrays) so that
    // they can run kDepth slabs ahead: codes of columns >= K meet zero scales, rank entries >= r of
    // B meet zero rows of the A tile, rows >= N are dropped at the store.
    int chunk = bx;
    int slab0 = (chunk * 2 + half) * ly.ns;                    // this wave's first slab
    uint32_t cw[kNS][G][BITS];
    bf16x8 Bop[kNS][SS];
    // (a request past the wave's last slab `last` repeats that slab: same cache lines, no new traffic)
    // Byte offset of the lane's group v inside its row (canonical rows) or inside its slab's run of tiles
    // (slab-tile layout: tile grp / 4, chunk 16 * (grp % 4) + row); and the step from slab to slab.
    uint32_t voff[G];
#pragma unroll
    for (int v = 0; v < G; ++v) {
        const int grp = min((kb >> 5) + G * g + v, ngroups - 1);
        voff[v] = a.tiled ? (uint32_t)(((grp >> 2) * 64 + (grp & 3) * 16 + c) * (4 * BITS)) : (uint32_t)grp * (4 * BITS);
    }
    const size_t slab_bytes = a.tiled ? (size_t)a.nct * 64 * (4 * BITS) : 0;
    auto issue = [&](int i, int first, int last) __attribute__((always_inline)) {
        const int slab = min(first + i, last);
        const int n = min(slab * 16 + c, N - 1);
        const uint8_t *rowp = a.tiled ? ly.codes + (size_t)slab * slab_bytes : ly.codes + (size_t)n * a.row_bytes;
#pragma unroll
        for (int v = 0; v < G; ++v) load_group<BITS>(rowp + voff[v], cw[i][v]);
        if (BVEC) {
#pragma unroll
            for (int s = 0; s < SS; ++s) {
                const int jj0 = 32 * s + 8 * g;
                Bop[i][s] = *reinterpret_cast<const bf16x8 *>(ly.B + (size_t)n * r + (jj0 + 8 <= r ? jj0 : 0));
            }
        }
    };
    // rank not a multiple of 8: the B operand is gathered entry by entry at the point of use
    auto gather_B = [&](int i) __attribute__((always_inline)) {
        const int n = min((slab0 + i) * 16 + c, N - 1);
#pragma unroll
        for (int s = 0; s < SS; ++s) {
            typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
            s16x8 t;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = 32 * s + 8 * g + e;
                t[e] = j < r ? (short)ly.B[(size_t)n * r + j] : (short)0;
            }
            Bop[i][s] = __builtin_bit_cast(bf16x8, t);
        }
    };

    // ---- 1. set-up loads (A tile, X tile, levels) go out FIRST, the first slabs of the row
    //         stream right behind them: a wave's loads return in order ---------------------------
    constexpr int NCA = SS * 32 * CPR / kMxThreads;           // 16-byte chunks of the A tile per thread
    constexpr int NCX = (16 * CPR + kMxThreads - 1) / kMxThreads;
    constexpr int NIT = (NE * 16 + kMxThreads - 1) / kMxThreads;
    const int kc = tid % CPR, k0 = kw + 8 * kc;               // the thread's column chunk is fixed
    u32x4 ta[NCA], tx[NCX];
    float lo[NIT], hi[NIT];
#pragma unroll
    for (int q = 0; q < NCA; ++q) {
        const int jj = (tid + kMxThreads * q) / CPR;
        ta[q] = u32x4{0u, 0u, 0u, 0u};
        if (jj < r && k0 < K) ta[q] = *reinterpret_cast<const u32x4 *>(ly.A + (size_t)jj * K + k0);
    }
#pragma unroll
    for (int q = 0; q < NCX; ++q) {
        const int m = (tid + kMxThreads * q) / CPR;
        tx[q] = u32x4{0u, 0u, 0u, 0u};
        if (m < M && k0 < K) tx[q] = *reinterpret_cast<const u32x4 *>(a.X + (size_t)m * K + k0);
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int id = tid + kMxThreads * it, idx = (id >> 4) & (NE - 1);
        // (QUAD: levels of codes 0, 1 of the entry's four here, of codes 2, 3 below)
        lo[it] = a.codebook[QUAD ? (idx & 3) : (idx & (NL - 1))];
        hi[it] = a.codebook[QUAD ? ((idx >> 2) & 3) : (idx >> BITS)];
    }
    float lo2[QUAD ? NIT : 1], hi2[QUAD ? NIT : 1];
    if constexpr (QUAD) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int id = tid + kMxThreads * it, idx = (id >> 4) & (NE - 1);
            lo2[it] = a.codebook[(idx >> 4) & 3];
            hi2[it] = a.codebook[idx >> 6];
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < kDepth; ++i) issue(i, slab0, max(slab0, min(slab0 + ly.ns, ly.nslabs) - 1));
    __builtin_amdgcn_sched_barrier(0);

    // ---- 2. A tile and level table into LDS; scale a-operands back, transposed -----------------
#pragma unroll
    for (int q = 0; q < NCA; ++q) {
        const int jj = (tid + kMxThreads * q) / CPR;
        *reinterpret_cast<u32x4 *>(As + jj * AST + 8 * kc) = ta[q];
    }
    {
        uint32_t *lut32 = reinterpret_cast<uint32_t *>(smem);
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int id = tid + kMxThreads * it, idx = id >> 4, q = id & 15;
            if (idx < NE) {
                f16x2 h;
                h[0] = (_Float16)lo[it];
                h[1] = (_Float16)hi[it];
                const uint32_t pv = __builtin_bit_cast(uint32_t, h);
                if constexpr (QUAD) {
                    f16x2 h2;
                    h2[0] = (_Float16)lo2[it];
                    h2[1] = (_Float16)hi2[it];
                    const uint32_t pv2 = __builtin_bit_cast(uint32_t, h2);
                    *reinterpret_cast<u32x4 *>(lut32 + idx * 64 + 4 * q) = u32x4{pv, pv2, pv, pv2};     // copies 2q, 2q + 1
                } else
                *reinterpret_cast<u32x4 *>(lut32 + idx * 64 + 4 * q) = u32x4{pv, pv, pv, pv};
            }
        }
    }
    __syncthreads();
    bf16x8 Aop[G][SS][8];
#pragma unroll
    for (int s = 0; s < SS; ++s)
#pragma unroll
        for (int v = 0; v < G; ++v)
#pragma unroll
            for (int t = 0; t < 8; ++t)
                Aop[v][s][t] = tr_read_pair_d<AST>(As + cb * KT, 32 * s + 8 * g + (c >> 2), 32 * (G * (c & 3) + v) + 4 * t);
    __syncthreads();                                       // every wave has its A operands

    // ---- 3. X tile through the same region; product b-operands back ----------------------------
#pragma unroll
    for (int q = 0; q < NCX; ++q) {
        const int m = (tid + kMxThreads * q) / CPR;
        if (m < 16) *reinterpret_cast<u32x4 *>(As + m * AST + 8 * kc) = tx[q];
    }
    __syncthreads();
    bf16x8 Xop[G][4];
#pragma unroll
    for (int v = 0; v < G; ++v)
#pragma unroll
        for (int u = 0; u < 4; ++u)
            Xop[v][u] = *reinterpret_cast<const bf16x8 *>(As + c * AST + cb * KT + 32 * (G * g + v) + 8 * u);
    __syncthreads();                                       // the region now takes the block sums

    f32x4 *red = reinterpret_cast<f32x4 *>(As);            // [8 waves][kNS][64 lanes]

    // ---- 4. the row stream, chunk by chunk ------------------------------------------------------
    for (; chunk < ly.nchunks; chunk += gxl) {
        slab0 = (chunk * 2 + half) * ly.ns;                // (its first kDepth slabs are on their way)
        const int nsw = max(0, min(ly.ns, ly.nslabs - slab0));
#pragma unroll
        for (int i = 0; i < kNS; ++i) {
            if (i < nsw) {
                if (i + kDepth < kNS) issue(i + kDepth, slab0, slab0 + nsw - 1);
                __builtin_amdgcn_sched_barrier(0);     // keep the prefetch ahead of this slab's arithmetic
                if (!BVEC) gather_B(i);
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int v = 0; v < G; ++v) {
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {       // half a group: scale MFMAs 4hh .. 4hh+3
                        f32x4 S[4];
#pragma unroll
                        for (int s = 0; s < SS; ++s)
#pragma unroll
                            for (int t = 0; t < 4; ++t)
                                S[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aop[v][s][4 * hh + t], Bop[i][s],
                                                                               s == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : S[t], 0, 0, 0);
#pragma unroll
                        for (int uu = 0; uu < 2; ++uu) {
                            const int u = 2 * hh + uu;
                            bf16x8 W;
                            if constexpr (QUAD) {
#pragma unroll
                                for (int q2 = 0; q2 < 2; ++q2) {               // bytes 2u, 2u + 1 of the group's eight: codes 8u .. 8u + 7
                                    const int b = 2 * u + q2;
                                    const uint32_t ad = __builtin_amdgcn_perm(cw[i][v][b >> 2], laneoff, 0x0C0C0000u | ((4u + (b & 3)) << 8));
                                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                                    const u32x2 t = *reinterpret_cast<const __attribute__((address_space(3))) u32x2 *>((uintptr_t)ad);
#pragma unroll
                                    for (int hq = 0; hq < 2; ++hq) {
                                        // (the word is picked by name: a bit cast of the subscripted element t[hq]
                                        // compiled to element 0 for both)
                                        const f16x2 h = __builtin_bit_cast(f16x2, hq == 0 ? t.x : t.y);
                                        const int e0 = 4 * q2 + 2 * hq, e1 = e0 + 1;
                                        const float s0 = S[2 * uu + (e0 >> 2)][e0 & 3], s1 = S[2 * uu + (e1 >> 2)][e1 & 3];
                                        W[e0] = (__bf16)__builtin_fmaf((float)h[0], s0, 0.0f);
                                        W[e1] = (__bf16)__builtin_fmaf((float)h[1], s1, 0.0f);
                                    }
                                }
                            } else
#pragma unroll
                            for (int pp = 0; pp < 4; ++pp) {
                                const uint32_t ad = pair_addr<BITS>(cw[i][v], 4 * u + pp, laneoff);
                                const f16x2 h = __builtin_bit_cast(f16x2, lds_load_u32(ad));
                                const int e0 = 2 * pp, e1 = 2 * pp + 1;
                                const float s0 = S[2 * uu + (e0 >> 2)][e0 & 3], s1 = S[2 * uu + (e1 >> 2)][e1 & 3];
                                W[e0] = (__bf16)__builtin_fmaf((float)h[0], s0, 0.0f);
                                W[e1] = (__bf16)__builtin_fmaf((float)h[1], s1, 0.0f);
                            }
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(W, Xop[v][u], acc, 0, 0, 0);
                        }
                    }
                }
                red[(wave * kNS + i) * 64 + lane] = acc;
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // The first slabs of the next chunk are requested before this chunk's sums are handed over
        // (their registers are free), so the stream does not drain in between.  Outside the slab
        // loop on purpose: inside it every load is unconditional, which lets the compiler count
        // exactly how many are in flight at each use.
        if (chunk + gxl < ly.nchunks) {
            const int next0 = ((chunk + gxl) * 2 + half) * ly.ns;
#pragma unroll
            for (int i = 0; i < kDepth; ++i) issue(i, next0, max(next0, min(next0 + ly.ns, ly.nslabs) - 1));
        }
        __syncthreads();

        // ---- 5. add the four column blocks (fixed order); lane (m, gl) of a slab holds rows 4gl..4gl+3
        const int rows = 2 * ly.ns * 16;                   // rows of the chunk
        const int row0 = chunk * rows;
        for (int q = tid; q < 2 * ly.ns * 64; q += kMxThreads) {
            const int hf = q / (ly.ns * 64), rem = q - hf * (ly.ns * 64), i = rem >> 6, l = rem & 63;
            const int m = l & 15, gl = l >> 4;
            f32x4 s = red[((hf * 4 + 0) * kNS + i) * 64 + l];
#pragma unroll
            for (int w = 1; w < 4; ++w) {
                const f32x4 t = red[((hf * 4 + w) * kNS + i) * 64 + l];
                s[0] += t[0]; s[1] += t[1]; s[2] += t[2]; s[3] += t[3];
            }
            if (m >= M) continue;
            if (meet && (N & 3) == 0) {
                // the lane's four sums are four neighbouring rows of one token: one 16-byte store
                const int nb = row0 + (hf * ly.ns + i) * 16 + 4 * gl;
                if (nb < N) store16_agent(ly.partial + ((size_t)blockIdx.z * M + m) * N + nb, s);
                continue;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int n = row0 + (hf * ly.ns + i) * 16 + 4 * gl + e;
                if (n >= N) continue;
                if (meet)
                    __hip_atomic_store(&ly.partial[((size_t)blockIdx.z * M + m) * N + n], s[e], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                else if (a.y_f32) reinterpret_cast<float *>(ly.Y)[(size_t)m * N + n] = s[e];
                else reinterpret_cast<uint16_t *>(ly.Y)[(size_t)m * N + n] = bf16_bits(s[e]);
            }
        }
        __syncthreads();                                   // the sums are rewritten by the next chunk
    }

    // ---- 6. column blocks held by other workgroups: for every chunk this workgroup streamed, the
    //         last workgroup to arrive adds them in order.  Done once, after the last chunk, so that
    //         the two dependent round trips (stores acknowledged, then the ticket) are paid once.
    //         The partial sums went out as device-coherent (write-through) stores: once they have
    //         completed they are visible to every workgroup, without an L2 write-back or invalidate.
    if (meet) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        // a gate/up pair shares its tickets (same chunking): the last of both matrices' workgroups finishes
        const bool pair = MULTI && a.act;
        const unsigned arrivals = (unsigned)a.splits * (pair ? 2u : 1u);
        const float *Pg = pair ? a.layer[0].partial : ly.partial;
        const float *Pu = pair ? a.layer[MULTI ? 1 : 0].partial : nullptr;
        void *Yout = pair ? a.layer[0].Y : ly.Y;
        const int rows = 2 * ly.ns * 16;
        const int niter = (ly.nchunks - bx + gxl - 1) / gxl;
        // Who reads the sums back.  The outputs of a chunk are cut into P shares with a ticket each, and share p
        // belongs to the workgroups of rank p (mod P) among those that meet in the chunk.  A workgroup first takes
        // the tickets of the shares of others, and only then, one round trip later, those of its own: workgroups that
        // end at about the same time thus each arrive last at their own shares, and the read-back (which runs at
        // the rate of one CU's device-coherent loads) is spread over all of them instead of falling to the slowest
        // alone.  Whatever the timing, every ticket is taken exactly once by each workgroup and the last taker reads
        // the share back: a workgroup that is late inherits the shares of those that have left.
        const int P = a.parts;
        const int rank = (int)blockIdx.z + ((pair && li == 1) ? a.splits : 0);
        const int mine = rank % P;
        const bool vec = (N & 3) == 0;
        const int T = vec ? M * (rows / 4) : M * rows;            // outputs (of four rows, or of one) per chunk
        const int ipp = (T + P - 1) / P;                          // the largest share
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        i32x4 *ent = reinterpret_cast<i32x4 *>(As);               // one entry per ticket of a batch (the sums' region is free now)
        for (int phase = 0; phase < 2; ++phase) {
            const int np = phase == 0 ? P - 1 : 1;                // shares per chunk in this phase
            const int ntot = niter * np;
            for (int base = 0; base < ntot; base += kMxTickets) {
                const int nt = min(kMxTickets, ntot - base);
                if (tid < nt) {
                    const int idx = base + tid, it = idx / np, pi = idx - it * np;
                    const int part = phase == 0 ? (pi < mine ? pi : pi + 1) : mine;
                    unsigned *tk = &ly.counters[(size_t)(bx + it * gxl) * P + part];
                    const unsigned old = __hip_atomic_fetch_add(tk, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const int last = (old == arrivals - 1u);
                    // every other workgroup of this chunk has passed: hand the ticket back at zero
                    if (last) __hip_atomic_store(tk, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    // (won, first output of the share, one past its last, first row of the chunk; 32-bit quotients)
                    ent[tid] = i32x4{last, (int)((unsigned)(part * T) / (unsigned)P), (int)((unsigned)((part + 1) * T) / (unsigned)P),
                                     (bx + it * gxl) * rows};
                }
                __syncthreads();
                // output q of a chunk whose first row is row0: the column blocks added in order, Y written
                auto reduce_item = [&](int q, int row0) __attribute__((always_inline)) {
                    if (vec) {
                        // four neighbouring rows, 16-byte loads, up to eight column blocks in flight
                        const int m = q / (rows / 4), n = row0 + 4 * (q - m * (rows / 4));
                        if (n >= N) return;
                        // ZB column blocks in one round trip, added in order.  Straight-line code per count: blocks
                        // beyond the last are not loaded at all (every device-coherent load costs its full price,
                        // also when it repeats an address), and no load's target register is merged with another
                        // value before the wait.
                        auto add_batch = [&](const float *Pp, int z0, auto zb, f32x4 &acc) __attribute__((always_inline)) {
                            constexpr int ZB = decltype(zb)::value;
                            f32x4 tz[ZB];
#pragma unroll
                            for (int u = 0; u < ZB; ++u) tz[u] = load16_agent(Pp + ((size_t)(z0 + u) * M + m) * N + n);
                            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
                            for (int u = 0; u < ZB; ++u) {
                                asm volatile("" : "+v"(tz[u]));                      // (not before the wait)
                                acc[0] += tz[u][0]; acc[1] += tz[u][1]; acc[2] += tz[u][2]; acc[3] += tz[u][3];
                            }
                        };
                        auto add_blocks4 = [&](const float *Pp) __attribute__((always_inline)) -> f32x4 {
                            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                            int z0 = 0;
                            for (; z0 + 8 <= a.splits; z0 += 8) add_batch(Pp, z0, std::integral_constant<int, 8>{}, acc);
                            switch (a.splits - z0) {
                            case 7: add_batch(Pp, z0, std::integral_constant<int, 7>{}, acc); break;
                            case 6: add_batch(Pp, z0, std::integral_constant<int, 6>{}, acc); break;
                            case 5: add_batch(Pp, z0, std::integral_constant<int, 5>{}, acc); break;
                            case 4: add_batch(Pp, z0, std::integral_constant<int, 4>{}, acc); break;
                            case 3: add_batch(Pp, z0, std::integral_constant<int, 3>{}, acc); break;
                            case 2: add_batch(Pp, z0, std::integral_constant<int, 2>{}, acc); break;
                            case 1: add_batch(Pp, z0, std::integral_constant<int, 1>{}, acc); break;
                            default: break;
                            }
                            return acc;
                        };
                        f32x4 sv = add_blocks4(Pg);
                        if (pair) {
                            const f32x4 up = add_blocks4(Pu);
#pragma unroll
                            for (int e4 = 0; e4 < 4; ++e4) sv[e4] = sv[e4] / (1.0f + __expf(-sv[e4])) * up[e4];
                        }
                        if (a.y_f32) {
                            *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(Yout) + (size_t)m * N + n) = sv;
                        } else {
                            typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
                            u32x2 o;
                            o[0] = (uint32_t)bf16_bits(sv[0]) | ((uint32_t)bf16_bits(sv[1]) << 16);
                            o[1] = (uint32_t)bf16_bits(sv[2]) | ((uint32_t)bf16_bits(sv[3]) << 16);
                            *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(Yout) + (size_t)m * N + n) = o;
                        }
                        return;
                    }
                    const int m = q / rows, n = row0 + (q - m * rows);
                    if (n >= N) return;
                    auto add_blocks = [&](const float *Pp) __attribute__((always_inline)) -> float {
                        float acc = 0.f;
                        for (int z0 = 0; z0 < a.splits; z0 += 8) {
                            float t8[8];
#pragma unroll
                            for (int u = 0; u < 8; ++u) {
                                const int z = min(z0 + u, a.splits - 1);
                                t8[u] = __hip_atomic_load(&Pp[((size_t)z * M + m) * N + n], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            }
#pragma unroll
                            for (int u = 0; u < 8; ++u)
                                if (z0 + u < a.splits) acc += t8[u];
                        }
                        return acc;
                    };
                    float sc = add_blocks(Pg);
                    if (pair) {
                        // SwiGLU gate: silu(gate) * up on the fp32 sums, one rounding at the store
                        const float up = add_blocks(Pu);
                        sc = sc / (1.0f + __expf(-sc)) * up;
                    }
                    if (a.y_f32) reinterpret_cast<float *>(Yout)[(size_t)m * N + n] = sc;
                    else reinterpret_cast<uint16_t *>(Yout)[(size_t)m * N + n] = bf16_bits(sc);
                };
                if (P == 1) {
                    for (int t = 0; t < nt; ++t) {
                        const i32x4 d = ent[t];
                        if (!d[0]) continue;
                        for (int q = tid; q < T; q += kMxThreads) reduce_item(q, d[3]);
                    }
                } else {
                    // all shares won in this batch at once: item j = (ticket of the batch, output of its share)
                    for (int j = tid; j < nt * ipp; j += kMxThreads) {
                        const int e = (int)((unsigned)j / (unsigned)ipp);
                        const i32x4 d = ent[e];
                        const int q = d[1] + (j - e * ipp);
                        if (d[0] && q < d[2]) reduce_item(q, d[3]);
                    }
                }
                __syncthreads();                               // the flags are rewritten by the next batch
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct MxPlan {
    int ss, G, WK, splits, ns, nchunks, gx, parts;
};

// Read-back shares per chunk: one per workgroup that meets in a chunk, at most 32, and no more than the ticket
// array holds.  Taking the tickets in two rounds costs a round trip (measured 1.5 us at 4 tokens on 14336 x 4096,
// where a last arriver reads 14 KB back, 0.4 us at 16 tokens, 57 KB) and pays from about 200 KB per last arriver
// (16 tokens: 14336 x 4096 at rank 48 22.4 -> 20.3 us, 4096 x 14336 at rank 32 20.3 -> 18.3): one share, i.e. the
// last arriver alone, below 128 KB.  `splits * splits * M * N / 64` bytes: splits * M * N * 4 in all, read by
// 256 / splits workgroups.
static int mx_parts(int arrivals, size_t chunks, int splits, int M, int N)
{
    if ((size_t)splits * splits * M * N / 64 < ((size_t)128 << 10)) return 1;
    int parts = arrivals < 32 ? arrivals : 32;
    while (parts > 1 && chunks * (size_t)parts * sizeof(unsigned) > kTicketBytes) parts /= 2;
    return parts < 1 ? 1 : parts;
}

static int mx_ss(const MatmulProblem &p)
{
    if (p.f32fact) return 0;
    const int rp = (p.r + 31) / 32;
    return rp <= 1 ? 1 : rp <= 2 ? 2 : 0;
}

// Slabs per wave and chunk when `nslabs` slabs are shared by `lanes` waves (all workgroups of a
// column range): a wave's share is cut into the fewest passes of at most kNS slabs, all equally long.
static int mx_slabs_per_chunk(long nslabs, long lanes)
{
    long share = (nslabs + lanes - 1) / lanes;
    if (share < 1) share = 1;
    const long passes = (share + kNS - 1) / kNS;
    return (int)((share + passes - 1) / passes);
}

static MxPlan mx_plan(const MatmulProblem &p)
{
    MxPlan d;
    d.ss = mx_ss(p);
    d.G = d.ss == 1 ? 2 : 1;
    d.WK = 4 * 128 * d.G;
    d.splits = (p.K + d.WK - 1) / d.WK;
    const int nslabs = (p.N + 15) / 16;
    int gx = 256 / d.splits;                           // one resident workgroup per CU
    if (gx < 1) gx = 1;
    d.ns = mx_slabs_per_chunk(nslabs, 2 * gx);
    d.nchunks = (nslabs + 2 * d.ns - 1) / (2 * d.ns);
    d.gx = gx < d.nchunks ? gx : d.nchunks;
    d.parts = mx_parts(d.splits, (size_t)d.nchunks, d.splits, p.M < 16 ? p.M : 16, p.N);
    return d;
}

bool decode_mx_supported(const MatmulProblem &p)
{
    if (p.M < 1 || mx_ss(p) == 0) return false;
    const MxPlan d = mx_plan(p);
    return (size_t)d.nchunks * sizeof(unsigned) <= kTicketBytes && d.splits <= 65535;
}

size_t decode_mx_workspace_bytes(const MatmulProblem &p)
{
    const MxPlan d = mx_plan(p);
    if (d.splits <= 1) return 0;
    const int mchunk = p.M < 16 ? p.M : 16;
    return kTicketBytes + (size_t)d.splits * mchunk * p.N * sizeof(float);
}

template <int BITS, int SS, int G, bool BVEC, bool MULTI>
static hipError_t launch_mx_t(const MxArgsT<MULTI ? kMaxBatch : 1> &a, dim3 grid, hipStream_t st)
{
    constexpr int WK = 4 * 128 * G, AST = WK + 8;
    const size_t smem = (size_t)(BITS == 2 ? 256 : 1 << (2 * BITS)) * 256 + (size_t)SS * 32 * AST * 2 + kMxTickets * sizeof(int);   // (2 bits: entries of four codes)
    static LdsOptIn lds_opt_in;
    if (smem > 48 * 1024) {
        const hipError_t e = allow_dynamic_lds(lds_opt_in, reinterpret_cast<const void *>(&decode_mx_kernel<BITS, SS, G, BVEC, MULTI>), smem);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((decode_mx_kernel<BITS, SS, G, BVEC, MULTI>), grid, dim3(kMxThreads), smem, st, a);
    return hipGetLastError();
}

// `workspace` must be zero-filled when first handed over (tickets) and hold
// decode_mx_workspace_bytes(p) bytes; the kernel leaves the tickets at zero again.
hipError_t launch_decode_mx(const MatmulProblem &p, void *workspace, hipStream_t st)
{
    const MxPlan d = mx_plan(p);
    for (int m0 = 0; m0 < p.M; m0 += 16) {
        MxArgs a;
        a.M = (p.M - m0) < 16 ? (p.M - m0) : 16;
        a.X = (const uint16_t *)p.X + (size_t)m0 * p.K;
        a.codebook = p.codebook;
        a.K = p.K; a.r = p.r;
        a.y_f32 = p.f32out ? 1 : 0;
        a.row_bytes = p.K / 8 * p.bits;
        a.splits = d.splits;
        a.parts = d.parts;
        a.L = 1;
        a.act = 0;
        a.tiled = p.tiled ? 1 : 0;
        a.nct = (p.K + 127) / 128;
        MxLayer &ly = a.layer[0];
        ly.Y = p.f32out ? (void *)((float *)p.Y + (size_t)m0 * p.N) : (void *)((uint16_t *)p.Y + (size_t)m0 * p.N);
        ly.codes = (const uint8_t *)p.codes;
        ly.A = (const uint16_t *)p.A;
        ly.B = (const uint16_t *)p.B;
        ly.counters = (unsigned *)workspace;
        ly.partial = workspace ? (float *)((unsigned char *)workspace + kTicketBytes) : nullptr;
        ly.N = p.N;
        ly.nslabs = (p.N + 15) / 16;
        ly.ns = d.ns;
        ly.nchunks = d.nchunks;
        ly.gx0 = 0;
        ly.gxn = d.gx;
        const bool bvec = (p.r % 8) == 0;
        const dim3 grid(d.gx, 1, d.splits);
        hipError_t e = hipErrorInvalidValue;
#define LORDS_MXCASE(B_, S_, G_) \
    if (p.bits == B_ && d.ss == S_) e = bvec ? launch_mx_t<B_, S_, G_, true, false>(a, grid, st) : launch_mx_t<B_, S_, G_, false, false>(a, grid, st);
        LORDS_MXCASE(2, 1, 2) LORDS_MXCASE(2, 2, 1)
        LORDS_MXCASE(3, 1, 2) LORDS_MXCASE(3, 2, 1)
        LORDS_MXCASE(4, 1, 2) LORDS_MXCASE(4, 2, 1)
#undef LORDS_MXCASE
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---------------------------------------------------------------------------------------------
// batched launch: several matrices, the same (up to 16) tokens
// ---------------------------------------------------------------------------------------------
struct MxBatchPlan {
    int ss, G, splits, total_gx, parts;
    int ns[kMaxBatch], nchunks[kMaxBatch], gx0[kMaxBatch], gxn[kMaxBatch];
    size_t ticket0[kMaxBatch], partial0[kMaxBatch];           // offsets in tickets / floats
    size_t tickets, partial_floats;
};

static bool mx_batch_plan(const BatchedProblem &p, MxBatchPlan &d)
{
    if (p.M < 2 || p.M > 16 || p.f32fact || p.L < 1 || p.L > kMaxBatch) return false;
    if (p.act && (p.L != 2 || p.N[0] != p.N[1])) return false;
    const int rp = (p.r + 31) / 32;
    d.ss = rp <= 1 ? 1 : rp <= 2 ? 2 : 0;
    if (d.ss == 0) return false;
    d.G = d.ss == 1 ? 2 : 1;
    const int wk = 4 * 128 * d.G;
    d.splits = (p.K + wk - 1) / wk;
    if (d.splits > 65535) return false;
    // workgroups per matrix: one resident workgroup per CU in total, shared out by row count
    int budget = 256 / d.splits;
    if (budget < p.L) budget = p.L;
    long nslabs[kMaxBatch], sum = 0;
    for (int l = 0; l < p.L; ++l) { nslabs[l] = (p.N[l] + 15) / 16; sum += nslabs[l]; }
    int gx[kMaxBatch], used = 0;
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
        d.ns[l] = mx_slabs_per_chunk(nslabs[l], 2L * gx[l]);
        d.nchunks[l] = (int)((nslabs[l] + 2 * d.ns[l] - 1) / (2 * d.ns[l]));
        d.gxn[l] = gx[l] < d.nchunks[l] ? gx[l] : d.nchunks[l];
        d.gx0[l] = x0;
        x0 += d.gxn[l];
        d.ticket0[l] = (p.act && l == 1) ? d.ticket0[0] : d.tickets;
        if (!(p.act && l == 1)) d.tickets += (size_t)d.nchunks[l];
        d.partial0[l] = d.partial_floats;
        d.partial_floats += (size_t)d.splits * p.M * p.N[l];
    }
    d.total_gx = x0;
    int nmax = 0;
    for (int l = 0; l < p.L; ++l) nmax = p.N[l] > nmax ? p.N[l] : nmax;
    // (a gate/up pair: twice the workgroups meet in a chunk, and its last arriver reads both matrices' sums;
    //  measured at 14336 x 4096: 3-bit rank 48 at 4 tokens 39.7 -> 32.1 us, 2-bit rank 32 at 16 tokens 28.7 -> 26.4)
    const int arrivals = p.act ? 2 * d.splits : d.splits;
    d.parts = mx_parts(arrivals, d.tickets, arrivals, p.M, nmax);
    return d.tickets * sizeof(unsigned) <= kTicketBytes;
}

bool decode_mx_batched_supported(const BatchedProblem &p)
{
    MxBatchPlan d;
    return mx_batch_plan(p, d);
}

size_t decode_mx_batched_workspace_bytes(const BatchedProblem &p)
{
    MxBatchPlan d;
    if (!mx_batch_plan(p, d)) return 0;
    return kTicketBytes + d.partial_floats * sizeof(float);
}

hipError_t launch_decode_mx_batched(const BatchedProblem &p, void *workspace, hipStream_t st)
{
    MxBatchPlan d;
    if (!mx_batch_plan(p, d) || !workspace) return hipErrorInvalidValue;
    MxMultiArgs a;
    a.X = (const uint16_t *)p.X;
    a.codebook = p.codebook;
    a.M = p.M; a.K = p.K; a.r = p.r;
    a.y_f32 = p.f32out ? 1 : 0;
    a.row_bytes = p.K / 8 * p.bits;
    a.splits = d.splits;
    a.parts = d.parts;
    a.L = p.L;
    a.act = p.act ? 1 : 0;
    a.tiled = p.tiled ? 1 : 0;
    a.nct = (p.K + 127) / 128;
    for (int l = 0; l < kMaxBatch; ++l) {
        const int s = l < p.L ? l : 0;                      // unused entries: copies of the first
        MxLayer &ly = a.layer[l];
        ly.codes = (const uint8_t *)p.codes[s];
        ly.A = (const uint16_t *)p.A[s];
        ly.B = (const uint16_t *)p.B[s];
        ly.Y = p.Y[s];
        ly.counters = (unsigned *)workspace + d.ticket0[s] * d.parts;
        ly.partial = (float *)((unsigned char *)workspace + kTicketBytes) + d.partial0[s];
        ly.N = p.N[s];
        ly.nslabs = (p.N[s] + 15) / 16;
        ly.ns = d.ns[s];
        ly.nchunks = d.nchunks[s];
        ly.gx0 = d.gx0[s];
        ly.gxn = d.gxn[s];
    }
    const bool bvec = (p.r % 8) == 0;
    const dim3 grid(d.total_gx, 1, d.splits);
    hipError_t e = hipErrorInvalidValue;
#define LORDS_MXCASE(B_, S_, G_)                                                                  \
    if (p.bits == B_ && d.ss == S_)                                                                \
        e = bvec ? launch_mx_t<B_, S_, G_, true, true>(a, grid, st) : launch_mx_t<B_, S_, G_, false, true>(a, grid, st);
    LORDS_MXCASE(2, 1, 2) LORDS_MXCASE(2, 2, 1)
    LORDS_MXCASE(3, 1, 2) LORDS_MXCASE(3, 2, 1)
    LORDS_MXCASE(4, 1, 2) LORDS_MXCASE(4, 2, 1)
#undef LORDS_MXCASE
    return e;
}

}  // namespace lords

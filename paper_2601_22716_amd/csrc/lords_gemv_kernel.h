// One- and two-token decode kernel of  y = (C[Q] (.) (B A)) x  on gfx950: the GEMV.
//
// Arithmetic.  With few activation vectors the scale never has to be formed per element:
//      y[m][n] = sum_k C[q[n][k]] * (sum_j B[n][j] A[j][k]) * x[m][k]
//              = sum_j B[n][j] * T_m[n][j],      T_m = C[Q] (A (.) x_m)^T      (Sec. 3.3, regrouped)
// T is a dense N x K by K x r contraction, so it runs on the matrix cores: the b-operand is the
// looked-up level of each code (bf16), the a-operand the A tile with the activation folded in
// (A[j][k] * x[m][k], rounded to bf16).  The only per-element vector work left is the table
// look-up itself; the B factor enters once per row and rank entry, in fp32, on the accumulator.
//
// Work split.  A workgroup of eight waves owns a range of 16-row slabs and WK = 8 * 128 * G
// consecutive columns: wave w owns the 128*G columns from kw + w*128*G on and walks down ALL slabs
// of the workgroup.  The folded a-operands of a wave's columns (16*G*JT*MT registers) are made
// once and stay in registers for the whole row stream: the wave fetches its part of the A tile
// with loads that take whole rows (the load unit of a CU pays per cache line touched, see below),
// passes it through a staging buffer of its own in LDS to reach the layout the MFMA wants (eight
// consecutive columns of one rank entry per lane), and folds the activation in on the way.  The
// rows of B of all slabs are staged in LDS by the waves together, the level table is built by the
// first four waves (one per SIMD); both are handed over through flags in LDS (release / acquire at
// workgroup scope), so that the only barrier before the stream is the one that clears those flags,
// taken when every wave is still at the start.  The planner (lords_gemv.hip) takes G = 1 wherever
// that gives every CU one workgroup: 1024-column blocks, four of them on a 4096-column layer.
// Where K is wider than WK, the column blocks (gridDim.z of them) meet pairwise up a fixed
// binary tree through one atomic exchange per row and tree node: the first of a pair to arrive
// leaves its sum in the slot and is done, the second takes it, adds, empties the slot and climbs.
// The exchange carries the data itself, so no other memory has to be ordered around it (relaxed
// device-scope atomics suffice), a hand-over costs one round trip, and because a + b = b + a the
// result does not depend on who came first: results are run-to-run identical.
//
// Every load of the stream (the codes of the first D slabs) is requested before the set-up
// starts, so the set-up (level table, folded operands, rows of B) runs under the first memory
// round trip; later slabs are requested as registers come free.  The table look-ups run kGvAhead
// steps ahead of the MFMAs that consume them, across slab boundaries.
//
// Lane mapping (v_mfma_f32_16x16x32_bf16; lane l = (c = l%16, g = l/16)): the lane holds the codes
// of row n0+c at columns col(v, g) = kb + 32*LG*(4*(v/LG) + g) + 32*(v%LG), v = 0..G-1 (LG groups
// of 32 codes per load, so that a wave-level load fetches 128*LG consecutive columns of 16 rows);
// MFMA (v, u) contracts codes 8u..8u+7 of group v of all four lane groups against the a-operand
// rows j = QW*(i/4) + 4t + i%4 (tile t, tile row i; QW = 4*JT rank entries per lane group), which
// leaves accumulator lane (c, g) with T[n0+c][j] for the contiguous run j = QW*g .. QW*g+QW-1: its
// share of B[n0+c][.] is one or two 16-byte loads.  Table entry (code_hi << BITS) | code_lo holds
// the two levels as a bf16 pair, replicated once per lane (address = entry*256 + lane*4: no bank
// conflicts).
#pragma once
#include "lords_decode_common.h"

namespace lords {

// Builds with -DLORDS_GV_STAMPS (liblords_stamps.so, see build.py and decode_timeline.py) record device
// time stamps at the phase boundaries of the kernel: kept in registers and written when the kernel ends
// (a store would queue behind the loads); wave 0 and the last wave of every workgroup report, into
// GvArgs::stamps[workgroup][16].  Ordinary builds contain none of it.
#ifdef LORDS_GV_STAMPS
#define GV_STAMP(i) do { gv_t[i] = __builtin_amdgcn_s_memrealtime(); } while (0)
#define GV_STAMP_DECL unsigned long long gv_t[8] = {}
#define GV_STAMP_FLUSH(nw) do { if (a.stamps && (threadIdx.x & 63) == 0 && ((threadIdx.x >> 6) == 0 || (threadIdx.x >> 6) == (nw) - 1)) \
    for (int i_ = 0; i_ < 8; ++i_) a.stamps[((size_t)blockIdx.z * gridDim.x + blockIdx.x) * 16 + ((threadIdx.x >> 6) ? 8 : 0) + i_] = gv_t[i_]; } while (0)
#else
#define GV_STAMP(i) do { } while (0)
#define GV_STAMP_DECL do { } while (0)
#define GV_STAMP_FLUSH(nw) do { } while (0)
#endif

constexpr int kGvMaxSlabs = 32;           // slabs of 16 rows per workgroup
constexpr int kGvWaves = 8;
constexpr int kGvThreads = 64 * kGvWaves;
constexpr int kGvAhead = 3;               // steps (of four table reads) the look-ups run ahead of their MFMAs
constexpr int kGvBuilders = 4;            // waves that build the level table
constexpr int kGvFlags = 2 * kGvWaves + kGvBuilders;   // LDS flags: B rows staged [round][wave], table part built [builder]
constexpr int kGvBRounds = 2;             // 16-byte chunks of B a thread holds in registers until they are staged
constexpr int kGvMaxG = 4;                // widest column range of a wave: 128*G columns
// rows of a staging unit of the A tile: two tiles, or one where the units are many or wide (LDS room)
constexpr int gv_unit_rows(int lg, int jt) { return (lg == 2 || (jt & 1)) ? 16 : 32; }   // (three tiles: one at a time)

// most ring slots (slabs in flight) of an instantiation: eight where 64 registers hold the operands,
// with 128 what the remaining registers take (G*bits per slab)
constexpr int gv_dmax(int G, int JT, int MT, int bits)
{
    return 16 * G * JT * MT <= 64 ? 8 : (72 / (G * bits) < 8 ? 72 / (G * bits) : 8);
}
#ifndef LORDS_GV_FIRST
#define LORDS_GV_FIRST 1                  // slabs requested ahead of the A tile
#endif

// One quantised matrix of a launch.  A launch serves up to kGvMaxLayers matrices that read the same
// activations (same K, rank and code width): matrix l gets the workgroups bx0[l] .. bx0[l] + gx - 1
// of gridDim.x, each an even share of its slabs.
constexpr int kGvMaxLayers = 8;
struct GvLayer {
    const uint8_t *codes;
    const uint16_t *A;     // r x K bf16
    const uint16_t *B;     // N x r bf16
    void *Y;               // M x N
    uint32_t *slots;       // [tree nodes][M][N] exchange slots of this matrix, zero between calls
    int N;
    int share, extra;      // slabs per workgroup: ceil(N / 16) = gx * share + extra, the first `extra` workgroups take one more
};
struct GvArgs {
    // (what every launch reads comes first, within the first cache lines of the argument block; the other
    //  matrices of a shared launch follow)
    const uint16_t *X;     // M x K bf16
    const float *codebook;
    uint32_t *pair_slots;  // act: [M][N] slots where the two matrices of a gate/up pair meet
    int L;                 // matrices
    int act;               // L == 2, equal shapes: Y = silu(matrix 0) * matrix 1, written to layer[0].Y
    int M, K, r;
    int y_f32;
    int row_bytes;
    int kblocks;           // gridDim.z
    int tiled;             // codes in the slab-tile layout (16 rows x 128 columns per tile, lane-ordered): LG = 1 only
    int nct;               // column tiles per slab, ceil(K / 128)
#ifdef LORDS_GV_STAMPS
    unsigned long long *stamps;
#endif
    GvLayer layer[kGvMaxLayers];
    int bx0[kGvMaxLayers]; // first workgroup of each matrix (increasing)
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// BITS: code width.  JT: 16-row a-operand tiles (one per 16 rank entries: 2, 3 or 4).  G: 32-code
// groups per lane.  LG: groups per load.  MT: tokens.  D: slabs whose loads are in flight.
// RING: a workgroup may hold more than D slabs (slots are refilled).  BVEC: rows of B can be read with
// 16-byte loads.  MULTI: the launch serves several matrices.  QT: 2-bit codes looked up four at a time.
template <int BITS, int JT, int G, int LG, int MT, int D, bool RING, bool BVEC, bool MULTI, bool QT = false>
__global__ __launch_bounds__(kGvThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemv_kernel(GvArgs a)
{
    // A load unit is LG groups of 32 codes per lane.  HL: the unit is fetched as TWO loads of eight
    // rows each, every row as one run of 8 chunks (a whole 128-byte line at 4 bits), and the two
    // halves of the slab are exchanged across lanes afterwards: the load unit of the CU takes about
    // four cycles per cache line an instruction touches, so 16 rows x 64 bytes cost twice as much per
    // byte as 8 rows x 128 bytes.
    constexpr bool HL = BITS != 2 && LG == 2;
    constexpr int NV = G / LG, NH = HL ? 2 : 1, DW = HL ? BITS : LG * BITS;    // units per slab; loads per unit; dwords per load
    constexpr int KTW = 128 * G, WK = kGvWaves * KTW;
    // QUAD (2-bit codes): the table is indexed by a byte of four codes and holds four bf16 levels per entry, 32
    // copies of 8 bytes (lanes l and l + 32 share a copy; an 8-byte read serves them in different cycles): half
    // the address operations and half the LDS reads per weight of the pair table, which at 2 bits would be as
    // many per weight as at 4 bits, so that a 2-bit layer would take as long as a 4-bit one.
    constexpr bool QUAD = QT;
    static_assert(!QT || BITS == 2, "the table of code quadruples is for 2-bit codes");
    constexpr int NL = 1 << BITS, NE = QUAD ? 256 : 1 << (2 * BITS);
    constexpr int QW = 4 * JT, BW = QW / 2;                 // rank entries / dwords of B per lane and slab
    constexpr int RP = 16 * JT, BCH = RP / 8;               // padded rank; 16-byte chunks of a staged B row
    // staging of the A tile: units of UR tile rows x PCOL columns, one buffer per wave
    constexpr int UR = gv_unit_rows(LG, JT), TPU = UR / 16; // rows and tiles of a unit
    constexpr int PCOL = 128 * LG, NUC = G / LG, NUR = JT / TPU;
    constexpr int CPRW = PCOL / 8, RPI = 64 / CPRW, NLD = UR / RPI;    // 16-byte chunks per row, rows per load, loads per unit
    constexpr int SST = PCOL + 8;                           // staged row stride in bf16
    constexpr int LUT_BYTES = NE * 256, STG_BYTES = UR * SST * 2;
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    uint16_t *stage = reinterpret_cast<uint16_t *>(smem + LUT_BYTES + wave * STG_BYTES);   // [UR][SST], this wave's
    float *red = reinterpret_cast<float *>(stage);                                         // later: [MT][slabs][64] lane sums
    int *bflag = reinterpret_cast<int *>(smem + LUT_BYTES + kGvWaves * STG_BYTES);         // [rounds][waves]: that wave's rows of B are staged
    uint16_t *Bs = reinterpret_cast<uint16_t *>(smem + LUT_BYTES + kGvWaves * STG_BYTES + 256);  // [slabs*16][RP] rows of B
    const int kw = blockIdx.z * WK;                            // first column of the workgroup
    const int kb = kw + wave * KTW;                            // first column of this wave
    // The matrix this workgroup belongs to (wave-uniform: scalar registers).  A launch of one matrix (MULTI
    // false) finds everything at fixed places among the kernel arguments, with the first fetch; only a launch
    // of several matrices pays a second, dependent fetch (for one matrix that chain cost 0.2 to 0.4 us).
    int li = 0, bx_first = 0;
    GvLayer ly = a.layer[0];
    if constexpr (MULTI) {
        for (int l = 1; l < a.L; ++l) li = (int)blockIdx.x >= a.bx0[l] ? l : li;
        ly = a.layer[li];
        bx_first = a.bx0[li];
    }
    const int bx = (int)blockIdx.x - bx_first;
    const int N = ly.N, K = a.K, r = a.r;
    const uint32_t laneoff = QUAD ? (uint32_t)(lane & 31) * 8u : (uint32_t)lane * 4u;
    // (the mask of a bf16 pair's upper half, kept in a vector register: a logic operation whose operands are all
    //  vector registers issues every 2.3 clocks per SIMD, with a literal or scalar operand every 4)
    uint32_t himask = 0xFFFF0000u;
    asm volatile("" : "+v"(himask));
    const int ngroups = K >> 5;
    // this workgroup's slabs: an even share of the matrix (the host keeps it within the LDS budget), from
    // a quotient and remainder the host worked out (a division here is a hundred dependent scalar instructions)
    const int s0 = bx * ly.share + min(bx, ly.extra);
    const int nsw = ly.share + (bx < ly.extra ? 1 : 0);
    const int last = s0 + max(nsw, 1) - 1;

    // Code loads of one slab into ring slot `slot`, branch-free (addresses clamped into the array):
    // codes of columns >= K meet zero a-operands, rows >= N are dropped at the store.
    // One form of address serves both layouts, so that a load of the stream costs a scalar multiply and three
    // vector operations: byte offset = min(slab * cstep + cbase, cmax) + ccol (32 bits: the host keeps the code
    // array below 4 GB), with the lane's share worked out once, here.
    //   rows of K codes: cstep = 16 rows, cbase = the lane's row within the slab (HL: lane (c, g) fetches chunk
    //     2g + c/8 of row 8h + c%8; otherwise its own LG groups of row c), cmax = row N - 1, ccol = the group;
    //   slab tiles (LG = 1): the wave's load is one contiguous piece, chunk = lane; cstep = a slab of tiles,
    //     cbase = tile and lane, no clamp (rows >= N and column tiles beyond K are zero padding there).
    const uint32_t cstep = a.tiled ? (uint32_t)a.nct * (256u * BITS) : 16u * (uint32_t)a.row_bytes;
    const uint32_t cmax = a.tiled ? 0xFFFFFFFFu : (uint32_t)(N - 1) * (uint32_t)a.row_bytes;
    uint32_t cbase[NV][NH], ccol[NV][NH];
#pragma unroll
    for (int vv = 0; vv < NV; ++vv)
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            const int grp = HL ? min((kb >> 5) + 8 * vv + 2 * g + (c >> 3), ngroups - 1) : min((kb >> 5) + LG * (4 * vv + g), ngroups - LG);
            cbase[vv][h] = (uint32_t)(HL ? 8 * h + (c & 7) : c) * (uint32_t)a.row_bytes;
            ccol[vv][h] = (uint32_t)grp * (4u * BITS);
            if constexpr (LG == 1) {                       // (the planner gives the slab-tile layout to LG = 1 kernels only)
                if (a.tiled) {
                    cbase[vv][h] = ((uint32_t)min((kb >> 7) + vv, a.nct - 1) * 64u + (uint32_t)lane) * (4u * BITS);
                    ccol[vv][h] = 0u;
                }
            }
        }
    uint32_t cw[D][NV][NH][DW];
    auto issue = [&](int slot, int slab) __attribute__((always_inline)) {
        const uint32_t sbase = (uint32_t)slab * cstep;
#pragma unroll
        for (int vv = 0; vv < NV; ++vv)
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                const uint32_t off = min(sbase + cbase[vv][h], cmax) + ccol[vv][h];
                const uint32_t *q = reinterpret_cast<const uint32_t *>(ly.codes + off);
                if (DW == 4) {
                    const u32x4 t = *reinterpret_cast<const u32x4 *>(q);
#pragma unroll
                    for (int e = 0; e < 4; ++e) cw[slot][vv][h][e] = t[e];
                } else if (DW == 3) {
                    // (one 12-byte load into a vector value: three separate dword loads made the compiler
                    //  keep the whole ring of codes in scratch memory in some instantiations)
                    typedef uint32_t u32x3 __attribute__((ext_vector_type(3), aligned(4)));
                    const u32x3 t = *reinterpret_cast<const u32x3 *>(q);
#pragma unroll
                    for (int e = 0; e < 3; ++e) cw[slot][vv][h][e] = t[e];
                } else {
#pragma unroll
                    for (int e = 0; e < DW; ++e) cw[slot][vv][h][e] = q[e];
                }
            }
    };
    // the BITS dwords of group v of the lane's row in slot `slot`
    auto group_words = [&](int slot, int v, uint32_t (&gw)[BITS]) __attribute__((always_inline)) {
#pragma unroll
        for (int e = 0; e < BITS; ++e) {
            if (HL) {
                // rows 0..7 came with load 0, rows 8..15 with load 1, each lane holding the chunk 2g + c/8:
                // chunk 2g (v even) sits in lanes c < 8 of load 0 and of load 1, chunk 2g+1 in lanes c >= 8
                const int lo = (int)cw[slot][v / 2][0][e], hi = (int)cw[slot][v / 2][1][e];
                gw[e] = (v & 1) ? (uint32_t)__builtin_amdgcn_update_dpp(hi, lo, 0x128, 0xF, 0x3, false)     // lanes c < 8 take load 0 of lane c + 8
                                : (uint32_t)__builtin_amdgcn_update_dpp(lo, hi, 0x128, 0xF, 0xC, false);    // lanes c >= 8 take load 1 of lane c - 8
            } else {
                gw[e] = cw[slot][v / LG][0][(v % LG) * BITS + e];
            }
        }
    };
    // 16-byte chunk q of the workgroup's rows of B (row q / BCH, rank entries 8*(q % BCH) ..), zero beyond the rank
    auto load_B = [&](int q) __attribute__((always_inline)) -> u32x4 {
        const int n = min(s0 * 16 + q / BCH, N - 1), j0 = 8 * (q % BCH);
        u32x4 t = u32x4{0u, 0u, 0u, 0u};
        if (BVEC) {
            const u32x4 w = *reinterpret_cast<const u32x4 *>(ly.B + (size_t)n * r + (j0 < r ? j0 : 0));
            if (j0 < r) t = w;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = j0 + e;
                const uint32_t w = ly.B[(size_t)n * r + (j < r ? j : 0)];
                if (j < r) t[e >> 1] |= w << (16 * (e & 1));
            }
        }
        return t;
    };

    GV_STAMP_DECL;
    GV_STAMP(0);
    // ---- 1. flags cleared (one barrier, at once, when every wave is still at the start).  Then the
    //         rows of B this wave will stage (16-byte chunks tid, tid + threads: whole rows, in row
    //         order) are requested; with many slabs per workgroup the chunks beyond those are staged
    //         here and now, before anything else is in flight.  The first four waves (one per SIMD)
    //         build the level table, from scalar loads of the levels, while the other waves already
    //         keep the load unit busy; everybody meets the table through flags, not a barrier, so
    //         that a wave that is late with its loads holds up nobody -----------------------------------
    if (tid < kGvFlags) bflag[tid] = 0;
    __syncthreads();
    const int nbch = nsw * 16 * BCH;                          // chunks of B to stage
    u32x4 Braw[kGvBRounds];
#pragma unroll
    for (int qq = 0; qq < kGvBRounds; ++qq) Braw[qq] = load_B(min(tid + kGvThreads * qq, nbch - 1));
    for (int q = tid + kGvThreads * kGvBRounds; q < nbch; q += kGvThreads) *reinterpret_cast<u32x4 *>(Bs + 8 * q) = load_B(q);
    __builtin_amdgcn_sched_barrier(0);
    if (wave < kGvBuilders) {
        uint32_t *lut32 = reinterpret_cast<uint32_t *>(smem);
        float cb[NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) cb[i] = a.codebook[i];                  // uniform addresses: scalar loads
        if constexpr (QUAD) {
            // entry idx = (t >> 4) + 16 * it, a byte of four codes: dword 0 = levels of codes 0, 1 (idx & 15, the
            // same in every pass), dword 1 = levels of codes 2, 3 (idx >> 4 = it); thread t writes copies
            // 2 (t & 15) and 2 (t & 15) + 1
            const int x = (tid >> 4) & 15;
            float l0 = cb[0], l1 = cb[0];
#pragma unroll
            for (int i = 1; i < NL; ++i) {
                l0 = (x & 3) == i ? cb[i] : l0;
                l1 = (x >> 2) == i ? cb[i] : l1;
            }
            const uint32_t pv0 = bf16_bits(l0) | ((uint32_t)bf16_bits(l1) << 16);
#pragma unroll
            for (int it = 0; it < 16; ++it) {
                const uint32_t pv1 = bf16_bits(cb[it & 3]) | ((uint32_t)bf16_bits(cb[it >> 2]) << 16);
                *reinterpret_cast<u32x4 *>(lut32 + ((tid >> 4) + 16 * it) * 64 + 4 * (tid & 15)) = u32x4{pv0, pv1, pv0, pv1};
            }
        } else {
        // entry (hi << BITS) | lo as a bf16 pair, once per lane.  Builder thread t writes four lanes'
        // copies of entry (t >> 4) + 16 * it: its low code is the same in every pass, its high code
        // the same for the whole wave
        float lov = cb[0];
#pragma unroll
        for (int i = 1; i < NL; ++i) lov = ((tid >> 4) & (NL - 1)) == i ? cb[i] : lov;
        const uint32_t lo = bf16_bits(lov);
        const int hi0 = __builtin_amdgcn_readfirstlane((tid >> 4) >> BITS);
        constexpr int NIT = NE / 16 > 0 ? NE / 16 : 1;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int idx = (tid >> 4) + 16 * it;
            const int hidx = (hi0 + (16 >> BITS) * it) & (NL - 1);          // wave-uniform
            float hi = cb[0];
#pragma unroll
            for (int i = 1; i < NL; ++i) hi = hidx == i ? cb[i] : hi;
            if (idx < NE) {
                const uint32_t pv = lo | ((uint32_t)bf16_bits(hi) << 16);
                *reinterpret_cast<u32x4 *>(lut32 + idx * 64 + 4 * (tid & 15)) = u32x4{pv, pv, pv, pv};
            }
        }
        }
        if (lane == 0) __hip_atomic_store(&bflag[kGvBRounds * kGvWaves + wave], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    GV_STAMP(1);

    // ---- 2. every other load goes out now: the first slab(s) of the stream (so that the memory
    //         starts on them at once), the A tile with the activations, then the rest of the stream.
    //         A wave's loads return in order: what its set-up needs goes early.
    //         A tile: unit (uc, ur) = tile rows UR*ur .. x columns kb + PCOL*uc ..; load q of a unit
    //         fetches RPI whole rows of it (CPRW lanes x 16 bytes each) ---------------------------------
    constexpr int DF = D < LORDS_GV_FIRST ? D : LORDS_GV_FIRST;
#pragma unroll
    for (int d = 0; d < DF; ++d) issue(d, min(s0 + d, last));
    __builtin_amdgcn_sched_barrier(0);
    const int ch = lane % CPRW, rsub = lane / CPRW;
    // Every workgroup of a column block reads the same A tile at the same time.  Workgroups i, i+8, ..
    // share an L2 (one XCD): they and their waves walk the rows of a unit from different starting
    // points, so that at any moment the requests spread over all rows (and L2 channels) instead of
    // all asking for the same few lines.
    const int rot = (int)(((blockIdx.z * gridDim.x + blockIdx.x) >> 3) + wave) % NLD;
    u32x4 xr[NUC][MT];
    u32x4 Araw[NUC][NUR][NLD];
#pragma unroll
    for (int uc = 0; uc < NUC; ++uc) {
        const int col = kb + PCOL * uc + 8 * ch;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const bool ok = m < a.M && col < K;
            const u32x4 t = *reinterpret_cast<const u32x4 *>(a.X + (ok ? (size_t)m * K + col : 0));
            xr[uc][m] = ok ? t : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int ur = 0; ur < NUR; ++ur)
#pragma unroll
            for (int q = 0; q < NLD; ++q) {
                const int rho = ((q + rot) % NLD) * RPI + rsub, t = TPU * ur + (rho >> 4), i = rho & 15;
                const int j = QW * (i >> 2) + 4 * t + (i & 3);
                // (rank entries >= r read row 0 and meet zeros in the staged rows of B; columns >= K
                //  read column 0 and meet zero activations)
                Araw[uc][ur][q] = *reinterpret_cast<const u32x4 *>(ly.A + ((j < r && col < K) ? (size_t)j * K + col : 0));
            }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int d = DF; d < D; ++d) issue(d, min(s0 + d, last));
    __builtin_amdgcn_sched_barrier(0);

    // the rows of B this wave asked for (its oldest loads) go to LDS; a flag per wave and round tells
    // the others (release: the flag follows the data)
#pragma unroll
    for (int qq = 0; qq < kGvBRounds; ++qq) {
        if (kGvThreads * qq < nbch) {
            if (tid + kGvThreads * qq < nbch) *reinterpret_cast<u32x4 *>(Bs + 8 * (tid + kGvThreads * qq)) = Braw[qq];
            if (lane == 0) __hip_atomic_store(&bflag[qq * kGvWaves + wave], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
    GV_STAMP(2);

    // ---- 3. a-operands (from here on a wave depends on no other wave until the row sums meet): A[j][k] * x[m][k] rounded to bf16, through this wave's staging buffer (the
    //         loads above fetch whole rows; the MFMA wants eight columns of one tile row per lane) ------
    bf16x8 Aop[G][4][JT][MT];
#pragma unroll
    for (int uc = 0; uc < NUC; ++uc)
#pragma unroll
        for (int ur = 0; ur < NUR; ++ur)
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                float xl[4], xh[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    xl[e] = __builtin_bit_cast(float, xr[uc][m][e] << 16);
                    xh[e] = __builtin_bit_cast(float, xr[uc][m][e] & himask);
                }
#pragma unroll
                for (int q = 0; q < NLD; ++q) {
                    u32x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const f32x2 pr = {__builtin_bit_cast(float, Araw[uc][ur][q][e] << 16) * xl[e],
                                          __builtin_bit_cast(float, Araw[uc][ur][q][e] & himask) * xh[e]};
                        o[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));   // one v_cvt_pk_bf16_f32
                    }
                    *reinterpret_cast<u32x4 *>(stage + (((q + rot) % NLD) * RPI + rsub) * SST + 8 * ch) = o;
                }
#pragma unroll
                for (int l = 0; l < LG; ++l)
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int tt = 0; tt < TPU; ++tt)
                            Aop[uc * LG + l][u][TPU * ur + tt][m] =
                                *reinterpret_cast<const bf16x8 *>(stage + (16 * tt + c) * SST + 32 * LG * g + 32 * l + 8 * u);
            }
    // The level table was built by the first waves, the rows of B were staged by the waves that own
    // their chunks (chunks beyond the flagged rounds before anything else): wait for all of them here,
    // once, so that the stream below is straight-line code.  Every wave sets its flags without
    // waiting for anybody, so these waits end.
    // One lane per flag, so that a poll is ONE LDS round trip (polled one after the other the twenty
    // flags cost twenty dependent round trips, 1.2 us, even when all were set long ago).
    {
        static_assert(kGvFlags <= 64, "one lane per flag");
        const bool mine = lane < kGvBRounds * kGvWaves ? (lane / kGvWaves) * kGvThreads < nbch : lane < kGvFlags;
        while (true) {
            const int v = mine ? __hip_atomic_load(&bflag[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) : 1;
            if (__builtin_amdgcn_ballot_w64(v == 0) == 0) break;
            __builtin_amdgcn_s_sleep(1);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    }
    GV_STAMP(3);
    // ---- 4. the row stream.  A step = the four table reads of (slab, u, v) and its JT*MT MFMAs; the
    //         reads run kGvAhead steps ahead of the MFMAs that use them, across slab boundaries (every
    //         slot of the ring is computed, slots beyond the workgroup's last slab on stale codes, only
    //         their sums are dropped: the code is one straight line and the waits are on the oldest reads only) --
    constexpr int STEPS = 4 * G, TOT = D * STEPS;
    for (int i0 = 0; i0 < (RING ? nsw : 1); i0 += D) {
        u32x4 wq[kGvAhead + 1];
        f32x4 acc[JT][MT];
        // (unrolled in full whatever its size: the ring slots and the look-up queue are register arrays, and
        //  an index left to run time sends them to scratch memory)
#pragma clang loop unroll(full)
        for (int gs = 0; gs < TOT + kGvAhead; ++gs) {
            if (gs < TOT) {
                const int d = gs / STEPS, u = (gs % STEPS) / G, v = gs % G;
                uint32_t gw[BITS];
                group_words(d, v, gw);
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    if constexpr (QUAD) {
                        if (p < 2) {                   // bytes 2u, 2u + 1 of the group's eight: codes 8u .. 8u + 7
                            const int b = 2 * u + p;
                            const uint32_t ad = __builtin_amdgcn_perm(gw[b >> 2], laneoff, 0x0C0C0000u | ((4u + (b & 3)) << 8));
                            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                            const u32x2 t = *reinterpret_cast<const __attribute__((address_space(3))) u32x2 *>((uintptr_t)ad);
                            wq[gs % (kGvAhead + 1)][2 * p] = t[0];
                            wq[gs % (kGvAhead + 1)][2 * p + 1] = t[1];
                        }
                    } else {
                        wq[gs % (kGvAhead + 1)][p] = lds_load_u32(pair_addr<BITS>(gw, 4 * u + p, laneoff));
                    }
                }
            }
            if (gs >= kGvAhead) {
                const int cs = gs - kGvAhead, d = cs / STEPS, u = (cs % STEPS) / G, v = cs % G;
                const int i = i0 + d;
                const bf16x8 Wop = __builtin_bit_cast(bf16x8, wq[cs % (kGvAhead + 1)]);
#pragma unroll
                for (int t = 0; t < JT; ++t)
#pragma unroll
                    for (int m = 0; m < MT; ++m)
                        acc[t][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aop[v][u][t][m], Wop,
                                                                            (u == 0 && v == 0) ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[t][m], 0, 0, 0);
                if (cs % STEPS == STEPS - 1) {
                    // the slab is complete: accumulator element e of tile t is T[n][QW*g + 4t + e]; weigh with the lane's run of B
                    uint32_t Bq[BW];
                    if constexpr (BW % 4 == 0) {
#pragma unroll
                        for (int h = 0; h < BW / 4; ++h) {
                            const u32x4 t = *reinterpret_cast<const u32x4 *>(Bs + (min(i, nsw - 1) * 16 + c) * RP + QW * g + 8 * h);
#pragma unroll
                            for (int e = 0; e < 4; ++e) Bq[4 * h + e] = t[e];
                        }
                    } else {                               // (three tiles: runs of 24 bytes, 8-byte aligned)
                        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
                        for (int h = 0; h < BW / 2; ++h) {
                            const u32x2 t = *reinterpret_cast<const u32x2 *>(Bs + (min(i, nsw - 1) * 16 + c) * RP + QW * g + 4 * h);
                            Bq[2 * h] = t[0];
                            Bq[2 * h + 1] = t[1];
                        }
                    }
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        float y0 = 0.f, y1 = 0.f;
#pragma unroll
                        for (int t = 0; t < JT; ++t)
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float sv = acc[t][m][e];
                                const int q = 4 * t + e;                       // position in the lane's run
                                const uint32_t raw = (q & 1) ? (Bq[q >> 1] & himask) : (Bq[q >> 1] << 16);
                                const float bv = __builtin_bit_cast(float, raw);
                                if (e & 1) y1 = __builtin_fmaf(sv, bv, y1);
                                else y0 = __builtin_fmaf(sv, bv, y0);
                            }
                        if (i < nsw) red[(m * nsw + i) * 64 + lane] = y0 + y1;
                    }
                    if (RING) {
                        __builtin_amdgcn_sched_barrier(0);
                        if (i + D < nsw) issue(d, s0 + i + D);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        }
    }
    GV_STAMP(4);
    __syncthreads();
    GV_STAMP(5);

    // ---- 5. the four lane groups and the eight column ranges of the workgroup, added in a fixed order;
    //         then the other column blocks through the exchange slots
    for (int q = tid; q < MT * nsw * 16; q += kGvThreads) {
        const int m = q / (nsw * 16), rem = q - m * (nsw * 16);
        const int n = s0 * 16 + rem;
        if (m >= a.M || n >= N) continue;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < kGvWaves; ++w) {
            const float *rw = reinterpret_cast<const float *>(smem + LUT_BYTES + w * STG_BYTES) + (m * nsw + (rem >> 4)) * 64 + (rem & 15);
            v += (rw[0] + rw[16]) + (rw[32] + rw[48]);
        }
        bool mine = true;                                   // this thread still carries the row's sum
        int z = blockIdx.z, nodes0 = 0;
        for (int width = a.kblocks; width > 1 && mine; width = (width + 1) >> 1) {
            // at this level `width` subtrees are left; subtree z meets subtree z^1 in node z>>1
            if ((z ^ 1) < width) {
                uint32_t *slot = ly.slots + ((size_t)(nodes0 + (z >> 1)) * a.M + m) * N + n;
                uint32_t bits = __builtin_bit_cast(uint32_t, v);
                if (bits == 0u) bits = 0x80000000u;       // an empty slot reads 0: +0 travels as -0
                const uint32_t old = __hip_atomic_exchange(slot, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (old == 0u) mine = false;               // first of the pair: the other one carries on
                else {
                    __hip_atomic_store(slot, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    v += __builtin_bit_cast(float, old);
                }
            }
            nodes0 += width >> 1;
            z >>= 1;
        }
        if (!mine) continue;
        void *Yout = ly.Y;
        if (MULTI && a.act) {
            // gate/up pair: the two finished sums of a row meet in one more slot; the second to arrive
            // knows which of the two it holds itself and writes silu(gate) * up
            uint32_t *slot = a.pair_slots + (size_t)m * N + n;
            uint32_t bits = __builtin_bit_cast(uint32_t, v);
            if (bits == 0u) bits = 0x80000000u;
            const uint32_t old = __hip_atomic_exchange(slot, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (old == 0u) continue;
            __hip_atomic_store(slot, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float other = __builtin_bit_cast(float, old);
            const float gate = li == 0 ? v : other, up = li == 0 ? other : v;
            v = gate / (1.0f + __expf(-gate)) * up;
            Yout = a.layer[0].Y;
        }
        if (a.y_f32) reinterpret_cast<float *>(Yout)[(size_t)m * N + n] = v;
        else reinterpret_cast<uint16_t *>(Yout)[(size_t)m * N + n] = bf16_bits(v);
    }
    GV_STAMP(6);
    GV_STAMP_FLUSH(kGvWaves);
}

// ---------------------------------------------------------------------------------------------
// launch side (one translation unit per code width instantiates its kernels)
// ---------------------------------------------------------------------------------------------
constexpr size_t kGvLdsLimit = 160 * 1024;

struct GvPlan {
    int jt, G, LG, MT, kblocks, gx;
    int per;           // most slabs of one workgroup
    int depth;         // ring slots (template D)
    bool ring;         // a workgroup has more slabs than ring slots: slots are refilled
    bool quad;         // 2-bit codes: the 64 KB table of code quadruples (where the slabs still fit beside it)
    size_t smem;       // dynamic LDS bytes
    size_t nodes;      // exchange-tree nodes
};

template <int BITS, int JT, int G, int LG, int MT, int D, bool RING, bool BVEC, bool QT = false>
static hipError_t launch_gv_t(const GvArgs &a, dim3 grid, size_t smem, hipStream_t st)
{
    static LdsOptIn lds_opt_in;
    if (a.L > 1) {
        static LdsOptIn lds_opt_in_multi;
        const hipError_t e = allow_dynamic_lds(lds_opt_in_multi, reinterpret_cast<const void *>(&gemv_kernel<BITS, JT, G, LG, MT, D, RING, BVEC, true, QT>), kGvLdsLimit);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((gemv_kernel<BITS, JT, G, LG, MT, D, RING, BVEC, true, QT>), grid, dim3(kGvThreads), smem, st, a);
        return hipGetLastError();
    }
    const hipError_t e = allow_dynamic_lds(lds_opt_in, reinterpret_cast<const void *>(&gemv_kernel<BITS, JT, G, LG, MT, D, RING, BVEC, false, QT>), kGvLdsLimit);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((gemv_kernel<BITS, JT, G, LG, MT, D, RING, BVEC, false, QT>), grid, dim3(kGvThreads), smem, st, a);
    return hipGetLastError();
}

// Ring depths built without refill: 1 .. 8 (a workgroup with fewer slabs than slots repeats its last one).
// With refill every pass computes all slots of the ring, also those beyond the workgroup's last slab, and the
// row stream is bound by instruction issue, not by the arrival of the codes: of the three deepest rings the
// registers allow, the one whose last pass idles the fewest slots is taken (14 slabs: two passes of 7, not
// 8 + 6 of 8), the deeper on ties.  Ranks that are not a multiple of 8 (element-wise B loads) only get depth 2.
constexpr int gv_round_depth(int per) { return per <= 8 ? per : 8; }
constexpr int gv_ring_depth(int per, int dmax)
{
    int best = dmax, waste = (dmax - per % dmax) % dmax;
    for (int D = dmax - 1; D >= dmax - 2 && D >= 2; --D) {
        const int w = (D - per % D) % D;
        if (w < waste) { best = D; waste = w; }
    }
    return best;
}

template <int BITS, int JT, int G, int LG, int MT, bool QT = false>
static hipError_t launch_gv_d(const GvArgs &a, dim3 grid, const GvPlan &d, bool bvec, hipStream_t st)
{
    constexpr int DM = gv_dmax(G, JT, MT, BITS);
    if (!bvec) {
        if (d.ring) return launch_gv_t<BITS, JT, G, LG, MT, 2, true, false, QT>(a, grid, d.smem, st);
        return launch_gv_t<BITS, JT, G, LG, MT, 2, false, false, QT>(a, grid, d.smem, st);
    }
    if (d.ring) {
        if constexpr (DM >= 4) if (d.depth == DM - 2) return launch_gv_t<BITS, JT, G, LG, MT, DM - 2, true, true, QT>(a, grid, d.smem, st);
        if constexpr (DM >= 3) if (d.depth == DM - 1) return launch_gv_t<BITS, JT, G, LG, MT, DM - 1, true, true, QT>(a, grid, d.smem, st);
        if (d.depth == DM) return launch_gv_t<BITS, JT, G, LG, MT, DM, true, true, QT>(a, grid, d.smem, st);
        return hipErrorInvalidValue;
    }
#define LORDS_GVD(D_) \
    if constexpr (D_ <= DM) if (d.depth == D_) return launch_gv_t<BITS, JT, G, LG, MT, D_, false, true, QT>(a, grid, d.smem, st);
    LORDS_GVD(1) LORDS_GVD(2) LORDS_GVD(3) LORDS_GVD(4) LORDS_GVD(5) LORDS_GVD(6) LORDS_GVD(7) LORDS_GVD(8)
#undef LORDS_GVD
    return hipErrorInvalidValue;
}

template <int BITS, bool QT = false>
static hipError_t launch_gv_bits(const GvArgs &a, const GvPlan &d, bool bvec, dim3 grid, hipStream_t st)
{
#define LORDS_GVCASE(J_, G_, L_, M_) \
    if (d.jt == J_ && d.G == G_ && d.LG == L_ && d.MT == M_) return launch_gv_d<BITS, J_, G_, L_, M_, QT>(a, grid, d, bvec, st);
    LORDS_GVCASE(2, 1, 1, 1) LORDS_GVCASE(2, 2, 2, 1) LORDS_GVCASE(2, 2, 1, 1)
    LORDS_GVCASE(4, 1, 1, 1) LORDS_GVCASE(4, 2, 2, 1) LORDS_GVCASE(4, 2, 1, 1)
    LORDS_GVCASE(2, 1, 1, 2) LORDS_GVCASE(2, 2, 2, 2) LORDS_GVCASE(2, 2, 1, 2) LORDS_GVCASE(4, 1, 1, 2)
    LORDS_GVCASE(3, 1, 1, 1) LORDS_GVCASE(3, 2, 2, 1) LORDS_GVCASE(3, 2, 1, 1)
#undef LORDS_GVCASE
    return hipErrorInvalidValue;
}

// defined in lords_gemv_b2.hip, lords_gemv_b2q.hip, lords_gemv_b3.hip, lords_gemv_b4.hip
hipError_t launch_gemv_2bit_quads(const GvArgs &a, const GvPlan &d, bool bvec, dim3 grid, hipStream_t st);
hipError_t launch_gemv_2bit(const GvArgs &a, const GvPlan &d, bool bvec, dim3 grid, hipStream_t st);
hipError_t launch_gemv_3bit(const GvArgs &a, const GvPlan &d, bool bvec, dim3 grid, hipStream_t st);
hipError_t launch_gemv_4bit(const GvArgs &a, const GvPlan &d, bool bvec, dim3 grid, hipStream_t st);

}  // namespace lords

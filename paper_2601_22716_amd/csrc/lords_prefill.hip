// Large-M (prefill) kernel of  Y = X (C[Q] (.) (B A))^T  on gfx950: a bf16 MFMA GEMM whose weight
// operand is dequantised on the fly and never leaves the registers.
//
// Tiling.  A workgroup owns a (16*R*WN)-row x (16*MB*WM)-token tile of Y and walks K in tiles of
// 128 columns.  It has WN*WM waves: wave (wn, wm) owns rows 16R wn .. (R slabs of 16 rows) and
// tokens 16MB wm .., so each dequantised weight is reused for 16*MB tokens from registers; the
// accumulators (R slabs x MB token blocks x 4 registers, 128 in the large tiles) stay in
// registers over the whole K range.  The main shape is 256 x 256 with eight waves side by side
// along the rows (WN = 8, WM = 1, R = 2, MB = 16): every weight of the tile is dequantised by
// exactly one wave and meets all 256 tokens there.  (Waves of 64 rows x 128 tokens, two of
// which dequantise the same rows, were 9 % slower on the same tile although they read X from
// LDS half as often: the vector work and the scale MFMAs weigh more than the LDS reads.)  Two
// waves per SIMD, at most 256 registers each, so that every MFMA writes plain VGPRs (results of
// the scale MFMAs are read by vector ALU instructions, which cannot read the accumulation
// registers).  Smaller shapes for small problems and ranks above 32: see the launcher.
//
// Work division.  The launcher either gives every workgroup one whole output tile, or deals the
// K tiles of all output tiles, numbered tile by tile, to the workgroups in equal contiguous runs,
// so that every CU gets the same amount of work whatever the tile count.  A tile that a run
// boundary cuts is summed from its parts in column order: the parts that do not start at the
// tile's first column are written out as fp32 and counted in; the part that does adds them up
// in order and writes Y (see the epilogue).  The result does not depend on timing.
//
// Per K tile the X tile (BM x 128 bf16) and the A tile (padded rank x 128 bf16) are brought from
// global memory straight into LDS (global_load_lds_dwordx4, no registers), double-buffered, one
// barrier per tile.  16-byte chunks are XOR-swizzled by row so that the b-operand reads of X
// (ds_read_b128) and the transposing reads of A (ds_read_b64_tr_b16) are free of bank conflicts;
// the layouts are described where the tiles are staged.
//
// Lane mapping as in the decode kernels (v_mfma_f32_16x16x32_bf16, lane l = (c = l%16, g = l/16)):
// the lane holds the 32 codes of row n0+c at columns kb + 32g ..; scale MFMA t gives it the scales
// of codes 4t..4t+3; product MFMA u contracts columns 32g + 8u .. +8 with
// a-operand = the lane's 8 dequantised weights and b-operand = X[token c][same 8 columns].
// A K tile is processed in four stages u = 0..3 (scale MFMAs 2u, 2u+1 -> dequantise 8 weights per
// slab -> BM/16 x 4 product MFMAs); for ranks up to 32 the stages overlap as a software pipeline
// (stage u+1's dequantisation is spread over stage u's product MFMAs, see the K loop).
//
// Level look-up: two codes index an LDS table of fp16 pairs, 8 copies (address =
// index*32 + (lane%8)*4); v_fma_mix_f32 multiplies fp16 level by fp32 scale; one rounding to bf16.
#include "lords_decode_common.h"

namespace lords {

struct PrefillArgs {
    const uint16_t *X;
    const uint8_t *codes;
    const float *codebook;
    const uint16_t *B;     // N x r bf16
    const uint16_t *A;     // r x K bf16
    void *Y;
    int M, N, K, r;
    int y_f32;
    int row_bytes;
    int nt, mt;            // tiles along N and M
    int ntiles_k;          // ceil(K / 128)
    int tiled;             // codes in the slab-tile layout: tile (slab, K tile) contiguous, chunk = 16 g + c
    int per;               // work units (one K tile of one output tile) per workgroup; units are numbered tile by tile
    uint32_t *arrived;     // per output tile: parts handed over so far (zero before and after a launch)
    float *part;           // per workgroup: the accumulators of a part that does not start at the tile's first column
};

constexpr int kPfCopies = 8;

__device__ __forceinline__ void lds_direct_16(const void *gbase, uint32_t goff, uint32_t lds_wave_base)
{
    // Every active lane fetches 16 bytes from gbase + goff (gbase and lds_wave_base are the same
    // in all lanes and travel in scalar registers, goff is the lane's own byte offset); they land
    // at lds_wave_base + 16*lane (M0 holds the wave's LDS base).  With the row offsets of a tile
    // computed once, a tile load costs no vector instruction besides the load itself.
    // Written as assembly on purpose: when the compiler knows of an outstanding load into LDS it
    // makes the next LDS read wait for ALL outstanding memory loads, i.e. for the tile that was
    // just requested, which exposes the whole memory latency once per K tile.  The kernel orders
    // these loads itself: s_waitcnt vmcnt(0) and a barrier before a buffer is read.
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_wave_base), "v"(goff), "s"(gbase) : "memory", "m0");
}

template <int BITS>
__device__ __forceinline__ uint32_t pair_index(const uint32_t (&w)[BITS], int p)
{
    const int o = 2 * BITS * p, d = o >> 5, s = o & 31;
    uint32_t v = w[d] >> s;
    if (s + 2 * BITS > 32) v |= w[(d + 1) < BITS ? d + 1 : d] << (32 - s);
    return v & ((1u << (2 * BITS)) - 1u);
}

template <int BITS, int SS, int WM, int R, int WN = 4, int MB = 8>
__global__ __launch_bounds__(64 * WN * WM) __attribute__((amdgpu_waves_per_eu(WN * WM / 4, WN * WM / 4))) void prefill_kernel(PrefillArgs a)
{
    constexpr int BN = 16 * R * WN, BM = 16 * MB * WM, NT = 64 * WN * WM, RP = 32 * SS, NL = 1 << BITS, NE = 1 << (2 * BITS);
    constexpr int RPP = 4 * WN * WM;                           // A tile rows one staging pass of the workgroup covers
    constexpr int XBUF = BM * 256, ABUF = RP * 256;            // bytes per buffer
    constexpr bool kPipe = (R == 2 && SS <= 2 && (MB == 8 || MB == 16));   // ranks up to 64: pipelined K loop
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *Xs = smem;                                   // [2][BM / 4 token groups][1 KB]
    unsigned char *As = smem + 2 * XBUF;                        // [2][RP][256 B]
    uint32_t *lut = reinterpret_cast<uint32_t *>(smem + 2 * XBUF + 2 * ABUF);   // [NE][8]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int M = a.M, N = a.N, K = a.K;

    // ---- work of this workgroup.  The work is cut into units, one K tile of one output tile each, numbered
    //      tile by tile (n fastest); workgroup w takes units w per .. w per + per - 1, so a workgroup walks a
    //      tail of one output tile, whole tiles, and a head of another.  Workgroups are dealt round-robin to
    //      the 8 XCDs, so each XCD gets a contiguous run of ranges: its workgroups then share X panels in its L2.
    const int total_units = a.nt * a.mt * a.ntiles_k;
    const int wg = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    int unit = wg * a.per;
    const int unit_end = min(unit + a.per, total_units);
    if (unit >= unit_end) return;
    const int wn = wave % WN, wm = wave / WN;

    // ---- level table --------------------------------------------------------------------------------
    for (int id = tid; id < NE * kPfCopies; id += NT) {
        const int idx = id / kPfCopies;
        f16x2 h;
        h[0] = (_Float16)a.codebook[idx & (NL - 1)];
        h[1] = (_Float16)a.codebook[idx >> BITS];
        lut[id] = __builtin_bit_cast(uint32_t, h);
    }
    // ---- zero the A buffers once: rank rows >= r are never loaded and must read as zero --------------
    for (int id = tid; id < 2 * ABUF / 16; id += NT) reinterpret_cast<u32x4 *>(As)[id] = u32x4{0u, 0u, 0u, 0u};
    if (K & 127)                                               // ragged last K tile: stale X must at least be finite
        for (int id = tid; id < 2 * XBUF / 16; id += NT) reinterpret_cast<u32x4 *>(Xs)[id] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();

    while (unit < unit_end) {
    // ---- this part: K tiles kt0 .. kt1 - 1 of output tile T ------------------------------------------------
    const int T = unit / a.ntiles_k;
    const int kt0 = unit - T * a.ntiles_k, kt1 = min(a.ntiles_k, kt0 + (unit_end - unit));
    unit += kt1 - kt0;
    const int m_blk = (T / a.nt) * BM, n_blk = (T % a.nt) * BN;
    const int n_wave = n_blk + 16 * R * wn;
    const int m_wave = m_blk + 16 * MB * wm;

    // ---- B operands of the scale MFMAs: rows n_wave + 16 rho + c, rank entries 32 s + 8 g .. ----------
    bf16x8 Bop[R][SS];
#pragma unroll
    for (int rho = 0; rho < R; ++rho) {
        const int n = n_wave + 16 * rho + c;
#pragma unroll
        for (int s = 0; s < SS; ++s) {
            const int jj0 = 32 * s + 8 * g;
            typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
            s16x8 t;
#pragma unroll
            for (int e = 0; e < 8; ++e) t[e] = 0;
            if (n < N) {
                if ((a.r & 7) == 0) {
                    if (jj0 + 8 <= a.r) t = *reinterpret_cast<const s16x8 *>(a.B + (size_t)n * a.r + jj0);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (jj0 + e < a.r) t[e] = (short)a.B[(size_t)n * a.r + jj0 + e];
                }
            }
            Bop[rho][s] = __builtin_bit_cast(bf16x8, t);
        }
    }

    // ---- staging of one K tile into buffer p (direct to LDS) and of its codes into registers ---------
    // X tile in LDS: groups of four tokens, 1 KB each = [2 halves of 64 columns][4 tokens][128 B]; a
    // wave load fills one group, lane l landing in half l / 32, token (l / 8) % 4, slot l % 8, and
    // fetches whole 256-byte token rows from global memory (8 full cache lines per wave load).
    // Slot s of token t of half h holds the 8 columns 32 gg + 8 uu + 16 h with 4 uu + gg = s ^ (t & 7):
    // the four 16-byte chunks that the four lane groups g of an MFMA b-operand want at stage
    // u = 2 h + uu then sit in one 64-byte quarter-row, XOR-swizzled by token, and a wave's operand
    // read (16 tokens x 4 chunks) is free of bank conflicts (5.0 cycles per wave instruction; rows
    // of 256 bytes, one per token, cost 8.2 however they were swizzled).
    // A tile: row-major, 256 B per rank row, lane (wave, l) fetches chunk (l & 15) ^ (row & 15) of
    // row 4 wave + l / 16 (+ RPP per pass).  The byte offsets of a lane's chunks from the tile's
    // first element do not change along K and are kept in registers.
    constexpr int AQ = (RP + RPP - 1) / RPP;
    constexpr int TPP = 4 * WN * WM, XJ = BM / TPP;             // tokens per staging pass, passes
    static_assert(BM % TPP == 0, "a staging pass covers whole token groups");
    const int xm0 = 4 * wave + (lane >> 4);
    const int xkc = (lane & 15) ^ (xm0 & 15);
    const int xt0 = 4 * wave + ((lane >> 3) & 3);             // the lane's token in pass 0 (then + TPP per pass)
    const int xv = (lane & 7) ^ (xt0 & 7);                    // (TPP is a multiple of 8: the same in every pass)
    const int xkcol = 32 * (xv & 3) + 8 * (xv >> 2) + 16 * (lane >> 5);
    uint32_t xo[XJ], ao[AQ];
#pragma unroll
    for (int j = 0; j < XJ; ++j) {
        const int m = min(m_blk + xt0 + TPP * j, M - 1);       // rows >= M: a copy of the last row, never stored
        xo[j] = ((uint32_t)(m - m_blk) * (uint32_t)K + (uint32_t)xkcol) * 2u;
    }
#pragma unroll
    for (int q = 0; q < AQ; ++q) ao[q] = ((uint32_t)min(xm0 + RPP * q, max(a.r - 1, 0)) * (uint32_t)K + 8u * xkc) * 2u;
    const uint32_t xl0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(Xs + wave * 1024));
    const uint32_t al0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(As + wave * 1024));
    const uint16_t *Xtile = a.X + (size_t)m_blk * K;
    auto stage = [&](int kt, int p) {
        const int kb = kt * 128;
        if (kb + 128 <= K) {
#pragma unroll
            for (int j = 0; j < XJ; ++j) lds_direct_16(Xtile + kb, xo[j], xl0 + p * XBUF + j * (TPP * 256));
#pragma unroll
            for (int q = 0; q < AQ; ++q)
                if (xm0 + RPP * q < a.r) lds_direct_16(a.A + kb, ao[q], al0 + p * ABUF + q * (RPP * 256));
        } else {
            // ragged last tile: X chunks beyond K are fetched from further left (any finite data will
            // do: their weights are zero), A columns beyond K of a live rank row must read as zero
            {
                const int over = kb + xkcol - (K - 8);
                const uint32_t back = over > 0 ? 2u * over : 0u;
#pragma unroll
                for (int j = 0; j < XJ; ++j) lds_direct_16(Xtile + kb, xo[j] - back, xl0 + p * XBUF + j * (TPP * 256));
            }
#pragma unroll
            for (int q = 0; q < AQ; ++q) {
                if (xm0 + RPP * q >= a.r) continue;
                if (kb + 8 * xkc < K) lds_direct_16(a.A + kb, ao[q], al0 + p * ABUF + q * (RPP * 256));
                else *reinterpret_cast<u32x4 *>(As + p * ABUF + wave * 1024 + q * (RPP * 256) + 16 * lane) = u32x4{0u, 0u, 0u, 0u};
            }
        }
    };
    // Codes of K tile kt, row n, lane group g: canonical rows: n * row_bytes + (4 kt + g) * 4 BITS (clamped
    // into the row for a ragged last tile); slab-tile layout: the tile (n / 16, kt) is contiguous and the
    // lane's chunk is 16 g + n % 16.  Either way: a per-row base, a step per K tile, an offset per lane.
    const int ngroups = K >> 5;
    const uint8_t *crow[R];
#pragma unroll
    for (int rho = 0; rho < R; ++rho) {
        const int n = min(n_wave + 16 * rho + c, N - 1);
        crow[rho] = a.tiled ? a.codes + ((size_t)(n >> 4) * a.ntiles_k * 64 + (n & 15)) * (4 * BITS)
                            : a.codes + (size_t)n * a.row_bytes;
    }
    const uint32_t cstep = a.tiled ? 64u * 4 * BITS : 4u * 4 * BITS;
    const uint32_t cgoff = a.tiled ? (uint32_t)g * 16 * 4 * BITS : (uint32_t)g * 4 * BITS;
    const uint32_t cmax = a.tiled ? 0xffffffffu : (uint32_t)(ngroups - 1) * 4 * BITS;
    auto load_codes = [&](int kt, uint32_t (&cw)[R][BITS]) {
        const uint32_t off = min((uint32_t)kt * cstep + cgoff, cmax);
#pragma unroll
        for (int rho = 0; rho < R; ++rho) load_group<BITS>(crow[rho] + off, cw[rho]);
    };

    f32x4 acc[R][MB];
#pragma unroll
    for (int rho = 0; rho < R; ++rho)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[rho][mb] = f32x4{0.f, 0.f, 0.f, 0.f};

    uint32_t cw[R][BITS], cwn[R][BITS];
    stage(kt0, 0);
    load_codes(kt0, cw);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // per-lane LDS offsets
    uint32_t xoff[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
        xoff[u] = (uint32_t)((u >> 1) * 512 + (c >> 2) * 1024 + (c & 3) * 128 + (((4 * (u & 1) + g) ^ (c & 7)) * 16));

    const uint32_t lutoff = (uint32_t)(2 * XBUF + 2 * ABUF) + (uint32_t)(lane & 7) * 4u;

    for (int kt = kt0; kt < kt1; ++kt) {
        const int p = (kt - kt0) & 1;
        if (kt + 1 < kt1) {
            // (the main shape issues the loads of a whole next tile one by one from its pipeline steps)
            if (!kPipe || (kt + 2) * 128 > K) stage(kt + 1, p ^ 1);
            load_codes(kt + 1, cwn);
        }
        const unsigned char *Xp = Xs + p * XBUF + wm * (16 * MB * 256);
        const unsigned char *Ap = As + p * ABUF;

        // a-operand of scale MFMA t: 8 rank entries of 16 A columns, transposed out of LDS
        auto read_Aop = [&](int s, int t) -> bf16x8 {
            typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
            const int row0 = 32 * s + 8 * g + (c >> 2);                 // +4 for the second half
            const int kc = 4 * (c & 3) + (t >> 1);
            const unsigned char *p0 = Ap + row0 * 256 + ((kc ^ (row0 & 15)) * 16) + (t & 1) * 8;
            const unsigned char *p1 = Ap + (row0 + 4) * 256 + ((kc ^ ((row0 + 4) & 15)) * 16) + (t & 1) * 8;
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)p0);
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)p1);
            return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        };

        // Stage u of the dequantisation, two slabs at a time.  The LDS reads of a pair of slabs
        // (table entries, transposed A columns) are all issued before the first use, so that the
        // wave pays two LDS round trips per pair rather than one per table entry.
        auto dequant_stage = [&](int u, bf16x8 (&W)[R]) {
            bf16x8 Aop0[SS], Aop1[SS];
#pragma unroll
            for (int s = 0; s < SS; ++s) { Aop0[s] = read_Aop(s, 2 * u); Aop1[s] = read_Aop(s, 2 * u + 1); }
#pragma unroll
            for (int hp = 0; hp < R / 2; ++hp) {
                uint32_t lv[2][4];
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int pp = 0; pp < 4; ++pp) {
                        uint32_t idx = pair_index<BITS>(cw[2 * hp + q], 4 * u + pp);
                        lv[q][pp] = lds_load_u32((idx << 5) + lutoff);
                    }
                f32x4 S0[2], S1[2];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    S0[q] = f32x4{0.f, 0.f, 0.f, 0.f};
                    S1[q] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < SS; ++s) {
                        S0[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aop0[s], Bop[2 * hp + q][s], S0[q], 0, 0, 0);
                        S1[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aop1[s], Bop[2 * hp + q][s], S1[q], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int pp = 0; pp < 4; ++pp) {
                        const f16x2 h = __builtin_bit_cast(f16x2, lv[q][pp]);
                        const float s0 = pp < 2 ? S0[q][2 * pp] : S1[q][2 * pp - 4];
                        const float s1 = pp < 2 ? S0[q][2 * pp + 1] : S1[q][2 * pp - 3];
                        W[2 * hp + q][2 * pp] = (__bf16)__builtin_fmaf((float)h[0], s0, 0.0f);
                        W[2 * hp + q][2 * pp + 1] = (__bf16)__builtin_fmaf((float)h[1], s1, 0.0f);
                    }
            }
        };

        if constexpr (kPipe) {
            // Ranks up to 64: the K tile as one software pipeline of 4 MB steps (4 stages x MB token
            // blocks), pinned step by step with scheduling barriers.  A step is the two product MFMAs
            // of one token block; riding on it are the X operand read of the block kAhead steps later
            // and a slice of the NEXT stage's dequantisation (with 16 token blocks: A columns and
            // table addresses in steps 0-3 of a stage, table reads in steps 1-4, scale MFMAs in step
            // 3, one pair of weights converted in each of steps 5-12; with 8 blocks the same slices at
            // twice the density), so that vector and LDS instructions issue in the shadow of MFMAs of
            // the same wave and every result is asked for several MFMAs before it is needed.  Only
            // stage 0 of a tile is dequantised in the open (its A tile arrives with the barrier).
            // The tile loads for the next K tile also ride on the steps, one each: issued in one
            // burst at the head of the tile they cost 3-4 % more.
            constexpr int H = MB / 8;                           // 1 or 2
            constexpr int NPS = 4 / H;                          // table addresses (and table reads) per step
            constexpr int kScaleStep = H == 2 ? 3 : 2;
            constexpr int kConv0 = H == 2 ? 5 : 4, CPS = 2 / H; // first converting step, weight pairs per step
            constexpr int kAhead = 3;
            constexpr int kLoad0 = 6, kLoads = XJ + AQ;      // steps kLoad0 .. of the tile carry its loads
            static_assert(kLoad0 + kLoads <= 4 * MB, "more tile loads than steps");
            const bool spread = kt + 1 < kt1 && (kt + 2) * 128 <= K;
            bf16x8 Wc[2], Wn[2];
            bf16x8 Xq[kAhead];
#pragma unroll
            for (int i = 0; i < kAhead; ++i) Xq[i] = *reinterpret_cast<const bf16x8 *>(Xp + i * 4096 + xoff[0]);
            __builtin_amdgcn_sched_barrier(0);
            dequant_stage(0, Wc);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                bf16x8 Aop0[SS], Aop1[SS];
                uint32_t ad[2][4], lv[2][4];
                f32x4 S0[2], S1[2];
                const int un = u < 3 ? u + 1 : 3;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const int t = MB * u + mb;
                    const bf16x8 Xop = Xq[t % kAhead];
                    acc[0][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Wc[0], Xop, acc[0][mb], 0, 0, 0);
                    acc[1][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Wc[1], Xop, acc[1][mb], 0, 0, 0);
                    if (t >= kLoad0 && t < kLoad0 + kLoads && spread) {
                        const int i = t - kLoad0, kbn = (kt + 1) * 128;
                        if (i < XJ) {
                            lds_direct_16(Xtile + kbn, xo[i], xl0 + (p ^ 1) * XBUF + i * (TPP * 256));
                        } else if (xm0 + RPP * (i - XJ) < a.r) {
                            lds_direct_16(a.A + kbn, ao[i - XJ], al0 + (p ^ 1) * ABUF + (i - XJ) * (RPP * 256));
                        }
                    }
                    if (t + kAhead < 4 * MB) {
                        const int tn = t + kAhead;
                        Xq[t % kAhead] = *reinterpret_cast<const bf16x8 *>(Xp + (tn % MB) * 4096 + xoff[tn / MB]);
                    }
                    if (u < 3) {
                        if (mb == 0) {
#pragma unroll
                            for (int ss = 0; ss < SS; ++ss) { Aop0[ss] = read_Aop(ss, 2 * un); Aop1[ss] = read_Aop(ss, 2 * un + 1); }
                        }
                        if (mb < 2 * H) {
#pragma unroll
                            for (int e = 0; e < NPS; ++e) {
                                const int lin = mb * NPS + e, q = lin >> 2, pp = lin & 3;
                                ad[q][pp] = (pair_index<BITS>(cw[q], 4 * un + pp) << 5) + lutoff;
                            }
                        }
                        if (mb >= 1 && mb < 1 + 2 * H) {
#pragma unroll
                            for (int e = 0; e < NPS; ++e) {
                                const int lin = (mb - 1) * NPS + e, q = lin >> 2, pp = lin & 3;
                                lv[q][pp] = lds_load_u32(ad[q][pp]);
                            }
                        }
                        if (mb == kScaleStep) {
#pragma unroll
                            for (int q = 0; q < 2; ++q) {
                                S0[q] = f32x4{0.f, 0.f, 0.f, 0.f};
                                S1[q] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                                for (int ss = 0; ss < SS; ++ss) {
                                    S0[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aop0[ss], Bop[q][ss], S0[q], 0, 0, 0);
                                    S1[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aop1[ss], Bop[q][ss], S1[q], 0, 0, 0);
                                }
                            }
                        }
                        if (mb >= kConv0 && mb < kConv0 + 8 / CPS) {
#pragma unroll
                            for (int e = 0; e < CPS; ++e) {
                                const int j = (mb - kConv0) * CPS + e, q = j >> 2, pp = j & 3;
                                const f16x2 h = __builtin_bit_cast(f16x2, lv[q][pp]);
                                const float s0 = pp < 2 ? S0[q][2 * pp] : S1[q][2 * pp - 4];
                                const float s1 = pp < 2 ? S0[q][2 * pp + 1] : S1[q][2 * pp - 3];
                                Wn[q][2 * pp] = (__bf16)__builtin_fmaf((float)h[0], s0, 0.0f);
                                Wn[q][2 * pp + 1] = (__bf16)__builtin_fmaf((float)h[1], s1, 0.0f);
                            }
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                Wc[0] = Wn[0];
                Wc[1] = Wn[1];
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                // X operands run kXAhead token blocks ahead of their MFMAs: the first ones of a stage
                // are requested before its dequantisation, each later one as the block kXAhead before
                // it is issued
                constexpr int kXAhead = 2;
                bf16x8 W[R];
                bf16x8 Xq[kXAhead];
#pragma unroll
                for (int i = 0; i < kXAhead; ++i)
                    Xq[i] = *reinterpret_cast<const bf16x8 *>(Xp + i * 4096 + xoff[u]);
                __builtin_amdgcn_sched_barrier(0);
                dequant_stage(u, W);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const bf16x8 Xop = Xq[mb % kXAhead];
#pragma unroll
                    for (int rho = 0; rho < R; ++rho)
                        acc[rho][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(W[rho], Xop, acc[rho][mb], 0, 0, 0);
                    if (mb + kXAhead < MB) {
                        Xq[mb % kXAhead] =
                            *reinterpret_cast<const bf16x8 *>(Xp + (mb + kXAhead) * 4096 + xoff[u]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0);          // the next tile has landed in LDS, the next codes in registers
        __syncthreads();
#pragma unroll
        for (int rho = 0; rho < R; ++rho)
#pragma unroll
            for (int q = 0; q < BITS; ++q) cw[rho][q] = cwn[rho][q];
    }

    // ---- epilogue: lane (c,g) holds token 16 mb + c, rows 16 rho + 4 g + {0..3} ------------------------
    // A part that does not start at the tile's first column hands its accumulators over in memory (it is
    // always the first part of its workgroup, so it waits for nothing); the part that does start there
    // is the last one of its workgroup, collects the others in column order and writes Y.  The sum of a
    // tile is therefore taken in a fixed order whatever the timing.
    constexpr int kPartFloats = R * MB * NT * 4;
    if (kt0 != 0) {
        float *dst = a.part + (size_t)wg * kPartFloats + tid * 4;
        asm volatile("" : "+v"(dst));        // (addresses are made here, not kept in registers over the K loop)
#pragma unroll
        for (int rho = 0; rho < R; ++rho)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) store16_agent(dst + (rho * MB + mb) * (NT * 4), acc[rho][mb]);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) __hip_atomic_fetch_add(a.arrived + T, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        continue;
    }
    if (kt1 != a.ntiles_k) {
        const int others = (a.ntiles_k - kt1 + a.per - 1) / a.per;       // the workgroups after this one, up to the tile's end
        if (tid == 0) {
            // (bounded: the parts waited for are first parts of their workgroups and never wait themselves)
            int spins = 0;
            while ((int)__hip_atomic_load(a.arrived + T, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < others && ++spins < (1 << 21))
                __builtin_amdgcn_s_sleep(8);
            __hip_atomic_store(a.arrived + T, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }
        __syncthreads();
        for (int j = 1; j <= others; ++j) {
            const float *src = a.part + (size_t)(wg + j) * kPartFloats + tid * 4;
            asm volatile("" : "+v"(src));
            // (sixteen loads in flight: what the registers beside the accumulators hold; each wait is a
            // round trip to memory)
            constexpr int kBatch = (R * MB) % 16 == 0 ? 16 : 8;
            static_assert((R * MB) % kBatch == 0, "whole batches");
#pragma unroll
            for (int b0 = 0; b0 < R * MB; b0 += kBatch) {
                f32x4 t[kBatch];
#pragma unroll
                for (int i = 0; i < kBatch; ++i) t[i] = load16_agent(src + (b0 + i) * (NT * 4));
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
                for (int i = 0; i < kBatch; ++i) {
                    asm volatile("" : "+v"(t[i]));               // (not before the wait)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[(b0 + i) / MB][(b0 + i) % MB][e] += t[i][e];
                }
            }
        }
    }
    void *Yp = a.Y;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = m_wave + 16 * mb + c;
        if (m >= M) continue;
#pragma unroll
        for (int rho = 0; rho < R; ++rho) {
            const int n = n_wave + 16 * rho + 4 * g;
            if (n + 3 < N && (N & 3) == 0) {
                if (a.y_f32) {
                    *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(Yp) + (size_t)m * N + n) = acc[rho][mb];
                } else {
                    typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
                    u32x2 o;
                    o[0] = (uint32_t)bf16_bits(acc[rho][mb][0]) | ((uint32_t)bf16_bits(acc[rho][mb][1]) << 16);
                    o[1] = (uint32_t)bf16_bits(acc[rho][mb][2]) | ((uint32_t)bf16_bits(acc[rho][mb][3]) << 16);
                    *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(Yp) + (size_t)m * N + n) = o;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (n + e >= N) continue;
                    if (a.y_f32) reinterpret_cast<float *>(Yp)[(size_t)m * N + n + e] = acc[rho][mb][e];
                    else reinterpret_cast<uint16_t *>(Yp)[(size_t)m * N + n + e] = bf16_bits(acc[rho][mb][e]);
                }
            }
        }
    }
    }   // parts of this workgroup
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
static int pf_ss(int r)
{
    const int rp = (r + 31) / 32;
    return rp <= 1 ? 1 : rp <= 2 ? 2 : rp <= 4 ? 4 : 0;
}

bool prefill_fast_supported(const MatmulProblem &p) { return !p.f32fact && pf_ss(p.r) != 0; }

// Tile shape and the cut of the work.  Tile shapes: 256 tokens x 256 rows (8 waves of 32 rows x 256
// tokens), 256 x 128 (8 waves), and for at most 128 tokens 128 x 256 (8 waves side by side) and
// 128 x 128 (4 waves).  Padded ranks above 32 take 128-token tiles only (their B operands need the
// registers, their A tile the LDS): 256 rows when that still gives every CU a tile, else 128.
//
// The work (output tiles x K tiles) is dealt to the CUs in equal contiguous runs of units, so that
// a tile count that is no multiple of the CU count costs no half-empty last round (448 tiles of the
// headline layer at 2048 tokens on 256 CUs: 56 K tiles per CU instead of 64).  A tile cut by a run
// boundary is summed from its parts in column order (see the kernel's epilogue); the parts travel as
// fp32 through `part`, one tile-sized buffer per workgroup.  Without that buffer (callers whose
// workspace is too small for it) every workgroup takes one whole tile.
struct PfPlan {
    int ss, wm, R, wn, mb, nt, mt;
    int per, wgs;          // units per workgroup, workgroups that get any
    size_t part_bytes;     // 0: whole tiles
};

constexpr int kPfCUs = 256;

static PfPlan pf_plan(const MatmulProblem &p, size_t avail)
{
    PfPlan d;
    d.ss = pf_ss(p.r);
    const int ntiles_k = (p.K + 127) / 128;
    // Candidates (tokens x rows of a tile) with the measured time of one K tile of one workgroup at
    // 4 bits and rank 32, all CUs busy, clocks settled:
    //   256 x 256, eight waves of 32 rows x 256 tokens each    3.45 us   (no weight is dequantised twice in a workgroup)
    //   256 x 128, eight waves of 32 rows x 128 tokens         2.4 us
    //   128 x 256, eight waves; 128 x 128, four waves          2.15 us, 1.75 us   (up to 128 tokens)
    // Padded ranks of 64 and 128 take the last two shapes at 1.4 and 2 times the cost.
    struct Cand { int wm, R, wn, mb; double t; };
    const double rank_cost = d.ss == 1 ? 1.0 : d.ss == 2 ? 1.4 : 2.0;
    const Cand small_rank[4] = {{1, 2, 8, 16, 3.45}, {2, 2, 4, 8, 2.4}, {1, 2, 8, 8, 2.15}, {1, 2, 4, 8, 1.75}};
    const Cand large_rank[2] = {{1, 2, 8, 8, 2.15 * rank_cost}, {1, 2, 4, 8, 1.75 * rank_cost}};
    const Cand *cands = d.ss == 1 ? small_rank : large_rank;
    const int ncands = d.ss == 1 ? 4 : 2;
    double best = 1e30;
    d.wm = 1; d.R = 2; d.wn = 4; d.mb = 8; d.per = ntiles_k; d.part_bytes = 0;
    for (int i = 0; i < ncands; ++i) {
        const Cand &c = cands[i];
        const int tokens = 16 * c.mb * c.wm, rows = 16 * c.R * c.wn;
        if (d.ss == 1 && (tokens == 128) != (p.M <= 128)) continue;
        const long tiles = (long)((p.N + rows - 1) / rows) * ((p.M + tokens - 1) / tokens);
        const long units = tiles * ntiles_k;
        const size_t tile_bytes = (size_t)tokens * rows * sizeof(float);
        // whole tiles, dealt by the hardware in rounds
        {
            const double cost = (double)((tiles + kPfCUs - 1) / kPfCUs) * ntiles_k * c.t;
            if (cost < best) { best = cost; d.wm = c.wm; d.R = c.R; d.wn = c.wn; d.mb = c.mb; d.per = ntiles_k; d.part_bytes = 0; }
        }
        // equal runs of units over `wgs` workgroups.  Its price is the hand-over of the parts: measured
        // 4 us + 1 us per 1.2 MB of parts written when the runs are shorter than a tile (every part is
        // written and read at about the same time), half of that per MB when they are longer; and runs
        // that are out of step with each other walk their K tiles about 8 % slower than whole tiles
        // dealt in rounds do.
        if (tiles * sizeof(uint32_t) > kZeroBytes || units > (1L << 30)) continue;
        static const int kWgs[] = {256, 224, 192, 160, 128, 112, 96, 80, 64, 48, 32, 16, 8};
        for (int wgs : kWgs) {
            const int per = (int)((units + wgs - 1) / wgs);
            if (per < 2 || (per % ntiles_k) == 0) continue;                      // (the second: whole tiles again)
            const size_t bytes = (size_t)wgs * tile_bytes;
            if (bytes > avail) continue;
            long written = 0;                                                    // parts that start inside a tile
            for (long b = per; b < units; b += per) written += (b % ntiles_k) != 0;
            const double mb_written = (double)written * tile_bytes / 1048576.0;
            const double cost = per >= ntiles_k ? per * c.t * 1.08 + 4.0 + mb_written / 2.4
                                                : per * c.t + 4.0 + mb_written / 1.2;
            if (cost < best) { best = cost; d.wm = c.wm; d.R = c.R; d.wn = c.wn; d.mb = c.mb; d.per = per; d.part_bytes = bytes; }
        }
    }
    const int tokens = 16 * d.mb * d.wm, rows = 16 * d.R * d.wn;
    d.nt = (p.N + rows - 1) / rows;
    d.mt = (p.M + tokens - 1) / tokens;
    const long units = (long)d.nt * d.mt * ntiles_k;
    d.wgs = (int)((units + d.per - 1) / d.per);
    return d;
}

size_t prefill_fast_workspace_bytes(const MatmulProblem &p, size_t limit)
{
    return pf_plan(p, limit).part_bytes;
}

template <int BITS, int SS, int WM, int R, int WN = 4, int MB = 8>
static hipError_t launch_pf_t(const PrefillArgs &a, dim3 grid, hipStream_t st)
{
    const size_t smem = (size_t)2 * (16 * MB * WM) * 256 + (size_t)2 * (32 * SS) * 256 + (size_t)(1 << (2 * BITS)) * kPfCopies * 4;
    static LdsOptIn lds_opt_in;
    {
        const hipError_t e = allow_dynamic_lds(lds_opt_in, reinterpret_cast<const void *>(&prefill_kernel<BITS, SS, WM, R, WN, MB>), smem);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((prefill_kernel<BITS, SS, WM, R, WN, MB>), grid, dim3(64 * WN * WM), smem, st, a);
    return hipGetLastError();
}

// `part`: part_bytes bytes of scratch (what prefill_fast_workspace_bytes returned for a limit of at most
// part_bytes), `zeroed`: kZeroBytes of device memory, zero when handed over and left at zero.
hipError_t launch_prefill_fast(const MatmulProblem &p, void *part, size_t part_bytes, void *zeroed, hipStream_t st)
{
    const PfPlan d = pf_plan(p, (part && zeroed) ? part_bytes : 0);
    const int ss = d.ss, wm = d.wm, wn = d.wn;
    PrefillArgs a;
    a.X = (const uint16_t *)p.X;
    a.codes = (const uint8_t *)p.codes;
    a.codebook = p.codebook;
    a.B = (const uint16_t *)p.B;
    a.A = (const uint16_t *)p.A;
    a.Y = p.Y;
    a.M = p.M; a.N = p.N; a.K = p.K; a.r = p.r;
    a.y_f32 = p.f32out ? 1 : 0;
    a.row_bytes = p.K / 8 * p.bits;
    a.nt = d.nt;
    a.mt = d.mt;
    a.ntiles_k = (p.K + 127) / 128;
    a.tiled = p.tiled ? 1 : 0;
    a.per = d.per;
    a.arrived = (uint32_t *)zeroed;
    a.part = (float *)part;
    const dim3 grid(((d.wgs + 7) / 8) * 8);
    hipError_t e = hipErrorInvalidValue;
#define LORDS_PCASE(B_, S_)                                                                     \
    if (p.bits == B_ && ss == S_) {                                                              \
        if (S_ == 1 && d.mb == 16) e = launch_pf_t<B_, 1, 1, 2, 8, 16>(a, grid, st);               \
        else if (S_ == 1 && wm == 2) e = launch_pf_t<B_, 1, 2, 2>(a, grid, st);                   \
        else if (wn == 8) e = launch_pf_t<B_, S_, 1, 2, 8>(a, grid, st);                         \
        else e = launch_pf_t<B_, S_, 1, 2>(a, grid, st);                                         \
    }
    LORDS_PCASE(2, 1) LORDS_PCASE(2, 2) LORDS_PCASE(2, 4)
    LORDS_PCASE(3, 1) LORDS_PCASE(3, 2) LORDS_PCASE(3, 4)
    LORDS_PCASE(4, 1) LORDS_PCASE(4, 2) LORDS_PCASE(4, 4)
#undef LORDS_PCASE
    return e;
}

}  // namespace lords

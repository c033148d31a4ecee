// Host side of the one-/two-token decode path (kernel: lords_gemv_kernel.h): shape of the launch.
#include "lords_gemv_kernel.h"

namespace lords {

#ifdef LORDS_GV_STAMPS
static unsigned long long *g_gv_stamps = nullptr;     // where the next launches report (see lords_debug_gemv_stamps)
#endif

static size_t gv_tree_nodes(int kblocks)
{
    size_t n = 0;
    for (int w = kblocks; w > 1; w = (w + 1) >> 1) n += (size_t)(w >> 1);
    return n;
}

// Shape of the launch for L matrices of N[l] rows that share K, rank, code width and activations.
// Returns false if no instantiation takes the case.
//
// A workgroup spans 1024*G columns.  Every CU has to pull the A tile of its columns (64 bytes per
// column) through its load unit, which takes about four cycles per 128-byte line, and to fold the
// activations into it on the vector ALUs: narrow column blocks keep that small, and the column blocks
// (K / (1024 G) of them) then meet through one exchange per tree level, about a microsecond each.  Measured on
// the Llama-3-8B/70B layer shapes, the narrowest block that still gives every CU one workgroup is
// the fastest: G = 1 unless the workgroups would then hold more slabs than their LDS takes.
// Matrix l gets gxl[l] row ranges of at most d.per slabs each; d.gx is their sum.
static bool gv_plan_table(int M, const int *N, int L, int K, int r, int bits, bool f32fact, bool tiled, bool quad, GvPlan &d, int *gxl, bool *fits_out)
{
    d.quad = quad;
    if (f32fact || M < 1 || M > 2 || L < 1 || L > kGvMaxLayers) return false;
    const int tiles = (r + 15) / 16;
    d.jt = tiles <= 2 ? 2 : (tiles == 3 && M == 1) ? 3 : tiles <= 4 ? 4 : 0;    // (three tiles at one token: the smaller staging unit leaves two tokens too little room for their lane sums)
    d.MT = M;
    if (d.jt == 0 || d.jt * d.MT > 8) return false;
    const int gmax = 8 / (d.jt * d.MT) < 2 ? 8 / (d.jt * d.MT) : 2;       // operands within 128 registers
    int nslabs[kGvMaxLayers];
    long total = 0;
    for (int l = 0; l < L; ++l) { nslabs[l] = (N[l] + 15) / 16; total += nslabs[l]; }
    // (the kernel addresses the codes of a matrix with 32-bit byte offsets, in either layout)
    for (int l = 0; l < L; ++l)
        if ((size_t)nslabs[l] * 16 * (size_t)((K + 127) / 128) * 16 * (size_t)bits >= ((size_t)1 << 32) - 64) return false;
    // (2-bit codes: a lane's two groups of a 2048-column block come with one 16-byte load and no lane swap, and on
    //  layers of 32 M weights and more the wider block measured 3-4 % faster at one token: 14336 x 4096 11.8 -> 11.3 us,
    //  4096 x 14336 13.6 -> 13.1; smaller layers lose, 4096 x 4096 6.9 -> 7.5)
    const int g_first = (bits == 2 && M == 1 && L == 1 && gmax >= 2 && total * 16 * (long)K >= (32L << 20)) ? 2 : 1;
    for (int G = g_first; G <= gmax; G *= 2) {
        d.G = G;
        d.LG = (G >= 2 && (K % 64) == 0 && !tiled) ? 2 : 1;               // (the slab-tile layout is read one 128-column tile at a time)
        const int wk = kGvWaves * 128 * G;
        d.kblocks = (K + wk - 1) / wk;
        // slabs a workgroup can take: its rows of B and its lane sums must fit LDS
        const size_t lut = (size_t)(quad ? 256 : 1 << (2 * bits)) * 256,           // (quad: entries of four 2-bit codes)
                      stg = (size_t)gv_unit_rows(d.LG, d.jt) * (128 * d.LG + 8) * 2;
        const size_t b_slab = (size_t)16 * 16 * d.jt * 2;
        long cap = (long)((kGvLdsLimit - 256 - lut - kGvWaves * stg) / b_slab);
        if (cap > (long)(stg / ((size_t)d.MT * 256))) cap = (long)(stg / ((size_t)d.MT * 256));
        if (cap > kGvMaxSlabs) cap = kGvMaxSlabs;
        if (cap < 1 || d.kblocks > 256) continue;
        int want = 256 / d.kblocks;                                      // one workgroup per CU
        if (want < L) want = L;
        // the smallest share per workgroup with which the matrices together need at most `want` row ranges
        long per = (total + want - 1) / want;
        if (per < 1) per = 1;
        int sum = 0;
        for (;; ++per) {
            sum = 0;
            for (int l = 0; l < L; ++l) sum += (int)((nslabs[l] + per - 1) / per);
            if (sum <= want || per >= total) break;
        }
        const bool fits = per <= cap;
        if (!fits) {
            per = cap;
            sum = 0;
            for (int l = 0; l < L; ++l) sum += (int)((nslabs[l] + per - 1) / per);
        }
        d.gx = sum;
        d.per = 0;
        for (int l = 0; l < L; ++l) {
            gxl[l] = (int)((nslabs[l] + per - 1) / per);
            const int most = (nslabs[l] + gxl[l] - 1) / gxl[l];           // even shares: the largest one
            if (most > d.per) d.per = most;
        }
        const int dmax = gv_dmax(d.G, d.jt, d.MT, bits);
        d.ring = d.per > dmax;
        d.depth = d.ring ? gv_ring_depth(d.per, dmax) : gv_round_depth(d.per);
        d.smem = lut + kGvWaves * stg + 256 + (size_t)d.per * b_slab;
        d.nodes = gv_tree_nodes(d.kblocks);
        if (fits || G == gmax) { *fits_out = fits; return true; }
    }
    return false;
}

// 2-bit codes are looked up four at a time (a 64 KB table instead of 4 KB) where every workgroup's slabs still fit
// beside the larger table; otherwise, and at 3 and 4 bits, two at a time.
static bool gv_plan(int M, const int *N, int L, int K, int r, int bits, bool f32fact, bool tiled, GvPlan &d, int *gxl)
{
    bool fits = false;
    if (bits == 2 && gv_plan_table(M, N, L, K, r, bits, f32fact, tiled, true, d, gxl, &fits) && fits) return true;
    return gv_plan_table(M, N, L, K, r, bits, f32fact, tiled, false, d, gxl, &fits);
}

// bytes of exchange slots: the trees of all matrices, plus the slots where a gate/up pair meets
static size_t gv_slot_bytes(const GvPlan &d, int M, const int *N, int L, bool act)
{
    size_t rows = 0;
    for (int l = 0; l < L; ++l) rows += (size_t)N[l];
    return (d.nodes * rows + (act ? (size_t)N[0] : 0)) * (size_t)M * sizeof(uint32_t);
}

bool decode_gemv_supported(const MatmulProblem &p)
{
    GvPlan d;
    int gxl[kGvMaxLayers];
    if (!gv_plan(p.M, &p.N, 1, p.K, p.r, p.bits, p.f32fact, p.tiled, d, gxl)) return false;
    return gv_slot_bytes(d, p.M, &p.N, 1, false) <= kZeroBytes;
}

bool decode_gemv_batched_supported(const BatchedProblem &bp)
{
    GvPlan d;
    int gxl[kGvMaxLayers];
    if (bp.L > kGvMaxLayers || (bp.act && (bp.L != 2 || bp.N[0] != bp.N[1]))) return false;
    if (!gv_plan(bp.M, bp.N, bp.L, bp.K, bp.r, bp.bits, bp.f32fact, bp.tiled, d, gxl)) return false;
    return gv_slot_bytes(d, bp.M, bp.N, bp.L, bp.act) <= kZeroBytes;
}

hipError_t launch_decode_gemv_batched(const BatchedProblem &bp, void *zeroed, hipStream_t st)
{
    GvPlan d;
    int gxl[kGvMaxLayers];
    if (bp.L > kGvMaxLayers || !gv_plan(bp.M, bp.N, bp.L, bp.K, bp.r, bp.bits, bp.f32fact, bp.tiled, d, gxl)) return hipErrorInvalidValue;
    if ((d.kblocks > 1 || bp.act) && !zeroed) return hipErrorInvalidValue;
    GvArgs a;
    a.X = (const uint16_t *)bp.X;
    a.codebook = bp.codebook;
    uint32_t *slots = (uint32_t *)zeroed;
    int bx0 = 0;
    for (int l = 0; l < kGvMaxLayers; ++l) {
        const int s = l < bp.L ? l : 0;
        GvLayer &ly = a.layer[l];
        ly.codes = (const uint8_t *)bp.codes[s];
        ly.A = (const uint16_t *)bp.A[s];
        ly.B = (const uint16_t *)bp.B[s];
        ly.Y = bp.Y[s];
        ly.N = bp.N[s];
        ly.share = (bp.N[s] + 15) / 16 / gxl[s];
        ly.extra = (bp.N[s] + 15) / 16 % gxl[s];
        ly.slots = slots;
        a.bx0[l] = l < bp.L ? bx0 : 0x7fffffff;
        if (l < bp.L) {
            bx0 += gxl[l];
            if (slots) slots += d.nodes * (size_t)bp.M * bp.N[l];
        }
    }
    a.pair_slots = slots;
    a.L = bp.L;
    a.act = bp.act ? 1 : 0;
    a.M = bp.M; a.K = bp.K; a.r = bp.r;
    a.y_f32 = bp.f32out ? 1 : 0;
    a.row_bytes = bp.K / 8 * bp.bits;
    a.kblocks = d.kblocks;
    a.tiled = bp.tiled ? 1 : 0;
    a.nct = (bp.K + 127) / 128;
#ifdef LORDS_GV_STAMPS
    a.stamps = g_gv_stamps;
#endif
    const bool bvec = (bp.r % 8) == 0;
    const dim3 grid(d.gx, 1, d.kblocks);
    switch (bp.bits) {
        case 2: return d.quad ? launch_gemv_2bit_quads(a, d, bvec, grid, st) : launch_gemv_2bit(a, d, bvec, grid, st);
        case 3: return launch_gemv_3bit(a, d, bvec, grid, st);
        case 4: return launch_gemv_4bit(a, d, bvec, grid, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_decode_gemv(const MatmulProblem &p, void *zeroed, hipStream_t st)
{
    BatchedProblem bp;
    bp.X = p.X; bp.codebook = p.codebook;
    for (int l = 0; l < kMaxBatch; ++l) { bp.codes[l] = p.codes; bp.B[l] = p.B; bp.A[l] = p.A; bp.Y[l] = p.Y; bp.N[l] = p.N; }
    bp.L = 1; bp.M = p.M; bp.K = p.K; bp.r = p.r; bp.bits = p.bits;
    bp.f32fact = p.f32fact; bp.f32out = p.f32out; bp.act = false;
    bp.tiled = p.tiled;
    return launch_decode_gemv_batched(bp, zeroed, st);
}

}  // namespace lords

#ifdef LORDS_GV_STAMPS
// Timing builds only: the next launches of the one-/two-token kernel write their time stamps
// (100 MHz ticks; 16 per workgroup: phases 0..6 of wave 0, then of the last wave) to `buffer`
// (device memory, 128 bytes per workgroup, at least 2048 workgroups; NULL: stop).  *workgroups
// receives the grid size of the plan for that problem.
extern "C" int lords_debug_gemv_stamps(void *buffer, int M, int N, int K, int r, int bits, int *workgroups)
{
    lords::g_gv_stamps = (unsigned long long *)buffer;
    lords::GvPlan d;
    int gxl[lords::kGvMaxLayers];
    if (workgroups) *workgroups = lords::gv_plan(M, &N, 1, K, r, bits, false, false, d, gxl) ? d.gx * d.kblocks : 0;
    return 0;
}
#endif

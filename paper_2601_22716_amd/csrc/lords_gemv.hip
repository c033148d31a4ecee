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

// Shape of the launch.  Returns false if no instantiation takes the case.
//
// A workgroup spans 1024*G columns.  Every CU has to pull the A tile of its columns (64 bytes per
// column) through its load unit, which takes about four cycles per 128-byte line, and to fold the
// activations into it on the vector ALUs: narrow column blocks keep that small, and the column blocks
// (K / (1024 G) of them) then meet through one exchange per tree level, about a microsecond each.  Measured on
// the Llama-3-8B/70B layer shapes, the narrowest block that still gives every CU one workgroup is
// the fastest: G = 1 unless the workgroups would then hold more slabs than their LDS takes.
static bool gv_plan(int M, int N, int K, int r, int bits, bool f32fact, GvPlan &d)
{
    if (f32fact || M < 1 || M > 2) return false;
    const int tiles = (r + 15) / 16;
    d.jt = tiles <= 2 ? 2 : tiles <= 4 ? 4 : 0;
    d.MT = M;
    if (d.jt == 0 || d.jt * d.MT > 8) return false;
    const int gmax = 8 / (d.jt * d.MT) < 2 ? 8 / (d.jt * d.MT) : 2;       // operands within 128 registers
    const int nslabs = (N + 15) / 16;
    for (int G = 1; G <= gmax; G *= 2) {
        d.G = G;
        d.LG = (G >= 2 && (K % 64) == 0) ? 2 : 1;
        const int wk = kGvWaves * 128 * G;
        d.kblocks = (K + wk - 1) / wk;
        // slabs a workgroup can take: its rows of B and its lane sums must fit LDS
        const size_t lut = (size_t)(1 << (2 * bits)) * 256, stg = (size_t)gv_unit_rows(d.LG) * (128 * d.LG + 8) * 2;
        const size_t b_slab = (size_t)16 * 16 * d.jt * 2;
        long cap = (long)((kGvLdsLimit - 256 - lut - kGvWaves * stg) / b_slab);
        if (cap > (long)(stg / ((size_t)d.MT * 256))) cap = (long)(stg / ((size_t)d.MT * 256));
        if (cap > kGvMaxSlabs) cap = kGvMaxSlabs;
        if (cap < 1 || d.kblocks > 256) continue;
        int gx = 256 / d.kblocks;                                        // one workgroup per CU
        if (gx < 1) gx = 1;
        if (gx > nslabs) gx = nslabs;
        const int need = (int)((nslabs + cap - 1) / cap);
        const bool fits = gx >= need;
        if (!fits) gx = need;
        d.gx = gx;
        d.per = (nslabs + gx - 1) / gx;
        const int dmax = gv_dmax(d.G, d.jt, d.MT, bits);
        d.ring = d.per > dmax;
        d.depth = d.ring ? dmax : gv_round_depth(d.per);
        if (d.depth > dmax) { d.depth = dmax; d.ring = d.per > dmax; }
        d.smem = lut + kGvWaves * stg + 256 + (size_t)d.per * b_slab;
        d.nodes = gv_tree_nodes(d.kblocks);
        if (fits || G == gmax) return true;
    }
    return false;
}

bool decode_gemv_supported(const MatmulProblem &p)
{
    GvPlan d;
    if (!gv_plan(p.M, p.N, p.K, p.r, p.bits, p.f32fact, d)) return false;
    return d.nodes * (size_t)p.M * p.N * sizeof(uint32_t) <= kZeroBytes;
}

hipError_t launch_decode_gemv(const MatmulProblem &p, void *zeroed, hipStream_t st)
{
    GvPlan d;
    if (!gv_plan(p.M, p.N, p.K, p.r, p.bits, p.f32fact, d)) return hipErrorInvalidValue;
    if (d.kblocks > 1 && !zeroed) return hipErrorInvalidValue;
    GvArgs a;
    a.X = (const uint16_t *)p.X;
    a.codebook = p.codebook;
    a.codes = (const uint8_t *)p.codes;
    a.A = (const uint16_t *)p.A;
    a.B = (const uint16_t *)p.B;
    a.Y = p.Y;
    a.slots = (uint32_t *)zeroed;
    a.M = p.M; a.N = p.N; a.K = p.K; a.r = p.r;
    a.nslabs = (p.N + 15) / 16;
    a.y_f32 = p.f32out ? 1 : 0;
    a.row_bytes = p.K / 8 * p.bits;
    a.kblocks = d.kblocks;
#ifdef LORDS_GV_STAMPS
    a.stamps = g_gv_stamps;
#endif
    const bool bvec = (p.r % 8) == 0;
    const dim3 grid(d.gx, 1, d.kblocks);
    switch (p.bits) {
        case 2: return launch_gemv_2bit(a, d, bvec, grid, st);
        case 3: return launch_gemv_3bit(a, d, bvec, grid, st);
        case 4: return launch_gemv_4bit(a, d, bvec, grid, st);
        default: return hipErrorInvalidValue;
    }
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
    if (workgroups) *workgroups = lords::gv_plan(M, N, K, r, bits, false, d) ? d.gx * d.kblocks : 0;
    return 0;
}
#endif

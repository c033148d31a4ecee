// Backward of the LoRDS linear layer for fine-tuning the scale factors (Sec. 3.4: B and A are the
// trainable parameters, the codes stay fixed).  With Y = X W_hat^T, W_hat = C[Q] (.) (B A):
//
//   dX = dY W_hat                      gradient with respect to the activations
//   G  = dY^T X,  P = C[Q] (.) G       gradient with respect to W_hat and to the scale S = B A
//   dB = P A^T,   dA = B^T P           gradients with respect to the factors
//
// dX.  The codes of a row run along K, but dX contracts over N.  Since Q is frozen during this kind
// of fine-tuning, a second packed copy of it with the codes running along N (transpose_codes_kernel,
// made once per layer, bits/8 bytes per weight) turns dX = dY W_hat into the forward product of the
// transposed layer: W_hat^T = C[Q^T] (.) (A^T B^T), i.e. the ordinary kernels with (codes^T, A^T, B^T)
// in the places of (codes, B, A).  Only the small factor transposes are done per call.
//
// dB, dA.  factor_grad_kernel: a workgroup of eight waves owns a 256-row x 256-column tile of G.
// It walks M in chunks of 32 tokens; the dY tile (32 x 256) and the X tile (32 x 256) go from
// global memory straight into LDS (global_load_lds_dwordx4), three buffers with two chunks in
// flight (two buffers for ranks above 32), 16-byte chunks XOR-swizzled by the row number
// (slot = chunk ^ 2(row & 7)).  Both are row-major along the token axis, which is the
// contraction axis here, so both MFMA operands come out of LDS through the transposing read
// (ds_read_b64_tr_b16).  Wave (wn, wk) owns rows 64wn .. 64wn+63 and columns 128wk .. 128wk+127:
// accumulator block (kb, nb) holds G[k = 128wk + 16kb + 4g + e][n = 64wn + 16nb + c] in lane (c, g), element e -- four
// consecutive columns of one row, which is (i) how the packed codes of that row are laid out, and
// (ii) after the multiplication by the level, exactly the a-operand layout of
// v_mfma_f32_16x16x16_bf16 for the contraction over k: dB needs no data movement at all.
// For dA (contraction over n) the same P values go to LDS as a row-major bf16 tile and come back
// through the transposing read, with the B tile as the other operand.
// G and P never reach HBM.  The sums over the other tiles (column tiles for dB, row tiles for dA)
// are written as fp32 partial results and added in a fixed order by reduce_partials_kernel:
// results are run-to-run identical.
#include "lords_decode_common.h"

namespace lords {

// ---------------------------------------------------------------------------------------------
// packed codes, transposed: codes_t row k holds the codes of column k, code n at bits [bits*n, ..)
// ---------------------------------------------------------------------------------------------
// One thread per (column k, group of 32 rows): gathers 32 codes, one from each of 32 rows, and
// writes the BITS dwords of the group.  A workgroup takes 32 consecutive columns of the same 32 rows
// so that the 32 row segments it reads are contiguous.
template <int BITS>
__global__ __launch_bounds__(256) void transpose_codes_kernel(const uint8_t *__restrict__ codes, uint8_t *__restrict__ codes_t,
                                                              int N, int K)
{
    __shared__ uint32_t tile[32][BITS * 8 + 1];             // 32 rows x 256 columns of codes
    const int n0 = blockIdx.y * 32, k0 = blockIdx.x * 256;
    const int row_bytes = K / 8 * BITS, rowt_bytes = N / 8 * BITS;
    // the 32 x (256 codes = BITS*8 dwords) source block, coalesced
    for (int id = threadIdx.x; id < 32 * BITS * 8; id += 256) {
        const int rr = id / (BITS * 8), d = id % (BITS * 8);
        const int kd = (k0 >> 5) * BITS + d;                 // dword within the row
        uint32_t v = 0;
        if (n0 + rr < N && kd < row_bytes / 4)
            v = reinterpret_cast<const uint32_t *>(codes + (size_t)(n0 + rr) * row_bytes)[kd];
        tile[rr][d] = v;
    }
    __syncthreads();
    const int kk = threadIdx.x;                              // column within the block
    if (k0 + kk >= K) return;
    const int grp = kk >> 5, e = kk & 31;                    // its 32-code group and place in it
    uint32_t out[BITS];
#pragma unroll
    for (int i = 0; i < BITS; ++i) out[i] = 0;
#pragma unroll
    for (int rr = 0; rr < 32; ++rr) {
        // code e of group grp of source row rr
        const int o = BITS * e, d = o >> 5, s = o & 31;
        uint32_t v = tile[rr][grp * BITS + d] >> s;
        if (s + BITS > 32) v |= tile[rr][grp * BITS + d + 1] << (32 - s);
        v &= (1u << BITS) - 1u;
        // becomes code rr of the destination group
        const int o2 = BITS * rr, d2 = o2 >> 5, s2 = o2 & 31;
        out[d2] |= v << s2;
        if (s2 + BITS > 32) out[d2 + 1 < BITS ? d2 + 1 : d2] |= v >> (32 - s2);
    }
    uint32_t *dst = reinterpret_cast<uint32_t *>(codes_t + (size_t)(k0 + kk) * rowt_bytes) + (n0 >> 5) * BITS;
#pragma unroll
    for (int i = 0; i < BITS; ++i) dst[i] = out[i];
}

hipError_t launch_transpose_codes(const void *codes, void *codes_t, int N, int K, int bits, hipStream_t st)
{
    const dim3 grid((unsigned)((K + 255) / 256), (unsigned)(N / 32)), block(256);
    switch (bits) {
        case 2: hipLaunchKernelGGL(transpose_codes_kernel<2>, grid, block, 0, st, (const uint8_t *)codes, (uint8_t *)codes_t, N, K); break;
        case 3: hipLaunchKernelGGL(transpose_codes_kernel<3>, grid, block, 0, st, (const uint8_t *)codes, (uint8_t *)codes_t, N, K); break;
        default: hipLaunchKernelGGL(transpose_codes_kernel<4>, grid, block, 0, st, (const uint8_t *)codes, (uint8_t *)codes_t, N, K); break;
    }
    return hipGetLastError();
}

// out[c][r] = in[r][c] for a small rows x cols factor (bf16 or fp32 elements), through a 32 x 32 tile
template <typename T>
__global__ __launch_bounds__(256) void transpose_factor_kernel(const T *__restrict__ in, T *__restrict__ out, int rows, int cols)
{
    __shared__ T tile[32][33];
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    for (int id = threadIdx.x; id < 1024; id += 256) {
        const int rr = id >> 5, cc = id & 31;
        if (r0 + rr < rows && c0 + cc < cols) tile[rr][cc] = in[(size_t)(r0 + rr) * cols + c0 + cc];
    }
    __syncthreads();
    for (int id = threadIdx.x; id < 1024; id += 256) {
        const int cc = id >> 5, rr = id & 31;
        if (r0 + rr < rows && c0 + cc < cols) out[(size_t)(c0 + cc) * rows + r0 + rr] = tile[rr][cc];
    }
}

hipError_t launch_transpose_factor(const void *in, void *out, int rows, int cols, bool f32, hipStream_t st)
{
    const dim3 grid((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32)), block(256);
    if (f32) hipLaunchKernelGGL(transpose_factor_kernel<float>, grid, block, 0, st, (const float *)in, (float *)out, rows, cols);
    else hipLaunchKernelGGL(transpose_factor_kernel<uint16_t>, grid, block, 0, st, (const uint16_t *)in, (uint16_t *)out, rows, cols);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// factor gradients
// ---------------------------------------------------------------------------------------------
struct FgArgs {
    const uint16_t *dY;    // M x N bf16
    const uint16_t *X;     // M x K bf16
    const uint8_t *codes;
    const float *codebook;
    const void *B;         // N x r
    const void *A;         // r x K
    float *partB;          // [2*ktiles][N][r]: one part per half tile (128 columns)
    float *partA;          // [ntiles][r][K]
    int M, N, K, r;
    int f32fact;
    int row_bytes;
    int ntiles, ktiles;
};

constexpr int kFgThreads = 512;
constexpr int kFgBN = 256, kFgBK = 256, kFgMC = 32;
constexpr int kFgTile = kFgMC * 512;                                      // bytes of one dY or X tile (32 tokens x 256 columns)
constexpr int kFgLoads = 4;                                               // direct-to-LDS loads per wave and chunk
constexpr int kFgAST = 520;                                               // bytes per row of the A tile (256 columns + pad)

__device__ __forceinline__ void fg_lds_direct_16(const void *gbase, uint32_t goff, uint32_t lds_wave_base)
{
    // Every active lane fetches 16 bytes from gbase + goff (gbase and lds_wave_base are the same in all
    // lanes and travel in scalar registers, goff is the lane's own byte offset); they land at
    // lds_wave_base + 16*lane (M0 holds the wave's LDS base).  Written as assembly so that the compiler
    // does not make later LDS reads wait for these loads; the kernel waits for them itself before a
    // buffer is read.
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_wave_base), "v"(goff), "s"(gbase) : "memory", "m0");
}

// Transposing read of 8 consecutive rows of one column block out of a row-major, chunk-swizzled
// tile (rows of ROWB bytes; the 16-byte chunk ch of row m sits in slot ch ^ 2(m & 7), so that the four
// rows a group of 16 lanes reads, 32 bytes each, fall into different banks): lane (c, g)
// passes row0 = first row + 8g and col0 = first column of the 16-column block and receives
// tile[row0 + e][col0 + c], e = 0..7.
// XOR mask for the 16-byte chunk index of tile row `row`.  A transposing read takes rows 8 g + (c >> 2)
// (+ 4 for its second half) and 32 bytes of each; the hardware serves lane groups g = 0, 1 together and
// g = 2, 3 together, so rows that differ in bits 0-1 or in bit 3 must fall into different 32-byte
// segments of the 256-byte bank window (2.8 cycles per wave instruction; with (row & 7) << 1, which
// separates rows 0-7 only, the two groups collide: 4.8).
__device__ __forceinline__ int fg_swz(int row) { return ((row & 3) << 1) | (((row >> 3) & 1) << 3); }

template <int ROWB>
__device__ __forceinline__ bf16x8 fg_tr_read(const unsigned char *tile, int row0, int col0, int c)
{
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
    const int col = col0 + 4 * (c & 3);
    const int ra = row0 + (c >> 2), rb = ra + 4;
    const unsigned char *p0 = tile + ra * ROWB + (((col >> 3) ^ fg_swz(ra)) << 4) + ((col & 7) << 1);
    const unsigned char *p1 = tile + rb * ROWB + (((col >> 3) ^ fg_swz(rb)) << 4) + ((col & 7) << 1);
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)p0);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)p1);
    return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// BITS: code width.  SS: the rank padded to 32*SS (1 or 2).
template <int BITS, int SS>
__global__ __launch_bounds__(kFgThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void factor_grad_kernel(FgArgs a)
{
    constexpr int RP = 32 * SS, JB = 2 * SS;                  // padded rank, 16-entry rank blocks
    constexpr int BST = (RP + 4) * 2;                         // bytes per row of the B tile
    constexpr int NB = SS == 1 ? 3 : 2;                       // staging buffers (what LDS leaves room for)
    constexpr int STAGE = NB * 2 * kFgTile;
    constexpr int CW = 4 * BITS, CST = CW + 1;                // dwords of 128 codes of a row; padded LDS row
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *As = smem + STAGE;                         // [RP][kFgAST]  bf16
    unsigned char *Bs = As + RP * kFgAST;                     // [256][BST]    bf16
    float *cb = reinterpret_cast<float *>(Bs + kFgBN * BST);  // [2^BITS]
    // codes of one half of the tile (256 rows x 128 columns): behind the P tile where the staging
    // region is large enough, else in a region of its own
    uint32_t *ct = SS == 1 ? reinterpret_cast<uint32_t *>(smem + 65536) : reinterpret_cast<uint32_t *>(cb + (1 << BITS));

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int wn = wave & 3, wk = wave >> 2;                  // this wave's 64 rows and 128 columns of the tile
    const int M = a.M, N = a.N, K = a.K, r = a.r;
    const int nt = blockIdx.x / a.ktiles, kt = blockIdx.x % a.ktiles;
    const int n0 = nt * kFgBN, k0 = kt * kFgBK;

    // ---- staging of one chunk of 32 tokens into buffer p: always kFgLoads loads per wave, so that the
    //      loop can wait for "all but the loads of the chunk behind this one" ------------------------------
    // A wave-level load covers two rows of 512 bytes: lane l brings row 2 wave + l / 32 (+ 16 for the
    // wave's second load) and the 16-byte chunk that belongs into slot l % 32 of that row.  The lane's
    // byte offsets from the chunk's first token do not change along M and are kept in registers.
    const int srow = 2 * wave + (lane >> 5);
    const int sch = (lane & 31) ^ fg_swz(srow);              // (rows 16 apart share their swizzle)
    const int scoln = min(n0 + 8 * sch, N - 8);              // (columns >= N or K: finite filler, masked later)
    const int scolk = min(k0 + 8 * sch, K - 8);
    uint32_t offY[2], offX[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        offY[q] = ((uint32_t)(srow + 16 * q) * (uint32_t)N + (uint32_t)scoln) * 2u;
        offX[q] = ((uint32_t)(srow + 16 * q) * (uint32_t)K + (uint32_t)scolk) * 2u;
    }
    const uint32_t sl0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(smem + 2 * wave * 512));
    // load i (0..3) of chunk ch into buffer p: i / 2 picks the wave's rows, i % 2 dY or X
    auto stage_one = [&](int ch, int p, int i) {
        const int q = i >> 1;
        const uint32_t l = sl0 + p * (2 * kFgTile) + (i & 1) * kFgTile + q * (16 * 512);
        const uint16_t *b = (i & 1) ? a.X + (size_t)ch * kFgMC * K : a.dY + (size_t)ch * kFgMC * N;
        if ((ch + 1) * kFgMC <= M) {
            fg_lds_direct_16(b, (i & 1) ? offX[q] : offY[q], l);
        } else {
            // tokens >= M: a copy of the last token; its X row is zeroed before use
            const uint32_t m = (uint32_t)(min(ch * kFgMC + srow + 16 * q, M - 1) - ch * kFgMC);
            fg_lds_direct_16(b, (i & 1) ? (m * (uint32_t)K + (uint32_t)scolk) * 2u : (m * (uint32_t)N + (uint32_t)scoln) * 2u, l);
        }
    };
    auto stage = [&](int ch, int p) {
#pragma unroll
        for (int i = 0; i < kFgLoads; ++i) stage_one(ch, p, i);
    };
    // ---- the packed codes of the tile (256 rows x 8*BITS dwords), requested now with coalesced loads and
    //      parked in registers over the token loop; they go to LDS, half a tile at a time, afterwards ------
    const int row_dwords = a.row_bytes >> 2;
    uint32_t ctile[4 * BITS];
#pragma unroll
    for (int q = 0; q < 4 * BITS; ++q) {
        const int id = tid + kFgThreads * q, row = id / (2 * CW), dd = id % (2 * CW);
        const int gd = (k0 >> 5) * BITS + dd;
        ctile[q] = 0;
        if (n0 + row < N && gd < row_dwords)
            ctile[q] = reinterpret_cast<const uint32_t *>(a.codes + (size_t)(n0 + row) * a.row_bytes)[gd];
    }
    const int nchunks = (M + kFgMC - 1) / kFgMC;
#pragma unroll
    for (int d = 0; d < NB - 1; ++d)
        if (d < nchunks) stage(d, d);

    // ---- A tile (rank x 256 columns), B tile (256 rows x rank), level table: once per workgroup ------
    typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
    if (!a.f32fact && (r & 7) == 0) {
        // 16-byte pieces, all loads of a thread in flight together (rows of the LDS tiles are only
        // 8-byte aligned: two stores per piece)
        u32x4 va[RP * 32 / kFgThreads], vb[kFgBN * (RP / 8) / kFgThreads];
#pragma unroll
        for (int q = 0; q < RP * 32 / kFgThreads; ++q) {
            const int id = tid + kFgThreads * q, j = id >> 5, kk = 8 * (id & 31);
            va[q] = u32x4{0u, 0u, 0u, 0u};
            if (j < r && k0 + kk < K) va[q] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(a.A) + (size_t)j * K + k0 + kk);
        }
#pragma unroll
        for (int q = 0; q < kFgBN * (RP / 8) / kFgThreads; ++q) {
            const int id = tid + kFgThreads * q, nn = id / (RP / 8), j = 8 * (id % (RP / 8));
            vb[q] = u32x4{0u, 0u, 0u, 0u};
            if (j < r && n0 + nn < N) vb[q] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(a.B) + (size_t)(n0 + nn) * r + j);
        }
#pragma unroll
        for (int q = 0; q < RP * 32 / kFgThreads; ++q) {
            const int id = tid + kFgThreads * q, j = id >> 5, kk = 8 * (id & 31);
            u32x2 *dst = reinterpret_cast<u32x2 *>(As + j * kFgAST + kk * 2);
            dst[0] = u32x2{va[q][0], va[q][1]};
            dst[1] = u32x2{va[q][2], va[q][3]};
        }
#pragma unroll
        for (int q = 0; q < kFgBN * (RP / 8) / kFgThreads; ++q) {
            const int id = tid + kFgThreads * q, nn = id / (RP / 8), j = 8 * (id % (RP / 8));
            u32x2 *dst = reinterpret_cast<u32x2 *>(Bs + nn * BST + j * 2);
            dst[0] = u32x2{vb[q][0], vb[q][1]};
            dst[1] = u32x2{vb[q][2], vb[q][3]};
        }
    } else {
        // fp32 factors (rounded to bf16 here) or a rank that is not a multiple of 8: entry by entry
#pragma unroll 8
        for (int id = tid; id < RP * kFgBK; id += kFgThreads) {
            const int j = id / kFgBK, kk = id % kFgBK;
            uint16_t v = 0;
            if (j < r && k0 + kk < K)
                v = a.f32fact ? bf16_bits(reinterpret_cast<const float *>(a.A)[(size_t)j * K + k0 + kk])
                              : reinterpret_cast<const uint16_t *>(a.A)[(size_t)j * K + k0 + kk];
            *reinterpret_cast<uint16_t *>(As + j * kFgAST + kk * 2) = v;
        }
#pragma unroll 8
        for (int id = tid; id < kFgBN * RP; id += kFgThreads) {
            const int nn = id / RP, j = id % RP;
            uint16_t v = 0;
            if (j < r && n0 + nn < N)
                v = a.f32fact ? bf16_bits(reinterpret_cast<const float *>(a.B)[(size_t)(n0 + nn) * r + j])
                              : reinterpret_cast<const uint16_t *>(a.B)[(size_t)(n0 + nn) * r + j];
            *reinterpret_cast<uint16_t *>(Bs + nn * BST + j * 2) = v;
        }
    }
    if (tid < (1 << BITS)) cb[tid] = a.codebook[tid];

    // ---- G = dY^T X over the tokens -----------------------------------------------------------------
    f32x4 acc[8][4];
#pragma unroll
    for (int kb = 0; kb < 8; ++kb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) acc[kb][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

    __syncthreads();                                       // A and B tiles, level table
    int p = 0;                                             // buffer of chunk ch
    for (int ch = 0; ch < nchunks; ++ch) {
        // chunk ch has landed once at most the loads of the chunk requested after it are outstanding
        if (NB == 3 && ch + 1 < nchunks) __builtin_amdgcn_s_waitcnt(0x0070 | kFgLoads);
        else __builtin_amdgcn_s_waitcnt(0x0070);
        __builtin_amdgcn_s_barrier();                      // ... for every wave; and every wave has left chunk ch-1
        asm volatile("" ::: "memory");
        unsigned char *dYs = smem + p * (2 * kFgTile), *Xs = dYs + kFgTile;
        if ((ch + 1) * kFgMC > M) {
            // ragged last chunk: tokens >= M must add nothing: their X rows become zero
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int id = tid + kFgThreads * q, row = id >> 5;
                if (ch * kFgMC + row >= M) *reinterpret_cast<u32x4 *>(Xs + row * 512 + 16 * (id & 31)) = u32x4{0u, 0u, 0u, 0u};
            }
            __syncthreads();
        }
        const int pprev = p == 0 ? NB - 1 : p - 1;         // the buffer of chunk ch-1, free now
        if (ch + NB - 1 < nchunks) stage(ch + NB - 1, pprev);
        bf16x8 Yop[4], Xop[8];
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) Yop[nb] = fg_tr_read<512>(dYs, 8 * g, 64 * wn + 16 * nb, c);
#pragma unroll
        for (int kb = 0; kb < 8; ++kb) Xop[kb] = fg_tr_read<512>(Xs, 8 * g, 128 * wk + 16 * kb, c);
#pragma unroll
        for (int kb = 0; kb < 8; ++kb)
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
                acc[kb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Xop[kb], Yop[nb], acc[kb][nb], 0, 0, 0);
        p = p + 1 == NB ? 0 : p + 1;
    }
    __syncthreads();                                       // every wave has left the last chunk: the buffers are free

    // ---- per half of the tile's columns (h = 0: the waves with wk = 0 hold it, then h = 1):
    //      P = level (.) G; dB = P A^T straight from the registers; P to LDS; dA = B^T P from there ------
    unsigned char *Ps = smem;                                 // [256][256 bytes], chunk-swizzled
    typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4v;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int q = 0; q < 4 * BITS; ++q) {
            const int id = tid + kFgThreads * q, row = id / (2 * CW), dd = id % (2 * CW);
            if (dd / CW == h) ct[row * CST + dd % CW] = ctile[q];
        }
        __syncthreads();
        if (wk == h) {
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const int nl = 64 * wn + 16 * nb + c, n = n0 + nl;    // the row whose four values this lane holds
                // all LDS reads of a pass are issued before any is used: code words, then levels
                uint32_t cv[8];
#pragma unroll
                for (int kb = 0; kb < 8; ++kb) {
                    const int off = BITS * (16 * kb + 4 * g), d = off >> 5, sh = off & 31;   // within the row's 128 codes of this half
                    const uint64_t w = (uint64_t)ct[nl * CST + d] | ((uint64_t)ct[nl * CST + min(d + 1, CW - 1)] << 32);
                    cv[kb] = (uint32_t)(w >> sh);
                }
                float lv[8][4];
#pragma unroll
                for (int kb = 0; kb < 8; ++kb)
#pragma unroll
                    for (int e = 0; e < 4; ++e) lv[kb][e] = cb[(cv[kb] >> (BITS * e)) & ((1u << BITS) - 1u)];
                f32x4 dBacc[JB];
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) dBacc[jb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kb = 0; kb < 8; ++kb) {
                    const int kl = 16 * kb + 4 * g, kk = k0 + 128 * h + kl;      // its four columns kk .. kk+3
                    const bool ok = n < N && kk < K;
                    s16x4v pb;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float pv = ok ? lv[kb][e] * acc[kb][nb][e] : 0.f;
                        pb[e] = (short)bf16_bits(pv);
                    }
                    // dB[n][j] += sum over these four columns of P[n][k] A[j][k]
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb) {
                        const s16x4v aop = *reinterpret_cast<const s16x4v *>(As + (16 * jb + c) * kFgAST + (128 * h + kl) * 2);
                        dBacc[jb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pb, aop, dBacc[jb], 0, 0, 0);
                    }
                    *reinterpret_cast<s16x4v *>(Ps + nl * 256 + (((kl >> 3) ^ fg_swz(nl)) << 4) + ((kl & 7) << 1)) = pb;
                }
                // dB partial of this half tile: lane (c, g) holds rows 4g+e of rank entry 16 jb + c
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) {
                    const int j = 16 * jb + c;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int nn = n0 + 64 * wn + 16 * nb + 4 * g + e;
                        if (nn < N && j < r) a.partB[((size_t)(2 * kt + h) * N + nn) * r + j] = dBacc[jb][e];
                    }
                }
            }
        }
        __syncthreads();

        // dA = B^T P over the 256 rows: wave w takes columns 16w .. 16w+15 of the half, all rank blocks
        f32x4 dAacc[JB];
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) dAacc[jb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ns = 0; ns < 8; ++ns) {
            const bf16x8 Pop = fg_tr_read<256>(Ps, 32 * ns + 8 * g, 16 * wave, c);
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) {
                typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
                const int ra = 32 * ns + 8 * g + (c >> 2), col = 16 * jb + 4 * (c & 3);
                s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(Bs + ra * BST + col * 2));
                s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(Bs + (ra + 4) * BST + col * 2));
                const bf16x8 Bop = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                dAacc[jb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Bop, Pop, dAacc[jb], 0, 0, 0);
            }
        }
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) {
            const int k = k0 + 128 * h + 16 * wave + c;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = 16 * jb + 4 * g + e;
                if (j < r && k < K) a.partA[((size_t)nt * r + j) * K + k] = dAacc[jb][e];
            }
        }
        if (h == 0) __syncthreads();                       // the P tile and the codes are rewritten by the other half
    }
}

// out[i] = sum over p of part[p][i], p increasing
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ part, float *__restrict__ out,
                                                              long count, int nparts)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float s = 0.f;
    for (int p = 0; p < nparts; ++p) s += part[(size_t)p * count + i];
    out[i] = s;
}

bool factor_grad_supported(int N, int K, int r) { return r >= 1 && r <= 64 && (N % 8) == 0 && N >= 8 && K >= 32; }

size_t factor_grad_workspace_bytes(int N, int K, int r)
{
    const size_t ntiles = (N + kFgBN - 1) / kFgBN, ktiles = (K + kFgBK - 1) / kFgBK;
    return (2 * ktiles * (size_t)N * r + ntiles * (size_t)r * K) * sizeof(float);    // dB: one part per half tile of columns
}

template <int BITS, int SS>
static hipError_t launch_fg_t(const FgArgs &a, hipStream_t st)
{
    constexpr int RP = 32 * SS;
    const size_t smem = (size_t)(SS == 1 ? 3 : 2) * 2 * kFgTile + (size_t)RP * kFgAST + (size_t)kFgBN * (RP + 4) * 2 +
                        (size_t)(1 << BITS) * 4 + (SS == 1 ? 0 : (size_t)kFgBN * (4 * BITS + 1) * 4);
    static LdsOptIn lds_opt_in;
    {
        const hipError_t e = allow_dynamic_lds(lds_opt_in, reinterpret_cast<const void *>(&factor_grad_kernel<BITS, SS>), smem);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((factor_grad_kernel<BITS, SS>), dim3(a.ntiles * a.ktiles), dim3(kFgThreads), smem, st, a);
    return hipGetLastError();
}

hipError_t launch_factor_grad(const void *dY, const void *X, const void *codes, const float *codebook, const void *B,
                              const void *A, float *dB, float *dA, int M, int N, int K, int r, int bits, bool f32fact,
                              void *workspace, hipStream_t st)
{
    FgArgs a;
    a.dY = (const uint16_t *)dY;
    a.X = (const uint16_t *)X;
    a.codes = (const uint8_t *)codes;
    a.codebook = codebook;
    a.B = B;
    a.A = A;
    a.M = M; a.N = N; a.K = K; a.r = r;
    a.f32fact = f32fact ? 1 : 0;
    a.row_bytes = K / 8 * bits;
    a.ntiles = (N + kFgBN - 1) / kFgBN;
    a.ktiles = (K + kFgBK - 1) / kFgBK;
    a.partB = (float *)workspace;
    a.partA = a.partB + (size_t)2 * a.ktiles * N * r;
    const int ss = r <= 32 ? 1 : 2;
    hipError_t e = hipErrorInvalidValue;
#define LORDS_FGCASE(B_, S_) if (bits == B_ && ss == S_) e = launch_fg_t<B_, S_>(a, st);
    LORDS_FGCASE(2, 1) LORDS_FGCASE(2, 2) LORDS_FGCASE(3, 1) LORDS_FGCASE(3, 2) LORDS_FGCASE(4, 1) LORDS_FGCASE(4, 2)
#undef LORDS_FGCASE
    if (e != hipSuccess) return e;
    const long cb = (long)N * r, ca = (long)r * K;
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((cb + 255) / 256)), dim3(256), 0, st, a.partB, dB, cb, 2 * a.ktiles);
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((ca + 255) / 256)), dim3(256), 0, st, a.partA, dA, ca, a.ntiles);
    return hipGetLastError();
}

}  // namespace lords

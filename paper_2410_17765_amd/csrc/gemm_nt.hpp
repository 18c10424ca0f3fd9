// bf16 "NT" matrix-core GEMM main loop for gfx950 with pluggable epilogues.
//
//   acc[m, n] = sum_k A[m, k] * B[n, k]        A[M, lda], B[N, ldb] bf16, both K-contiguous
//
// Every large contraction of the CP head (y = W h, z = U y, and the five products of the
// backward pass) is brought into this one form, if necessary by transposing an operand first,
// so that a single tuned main loop serves them all; what differs is the epilogue that consumes
// the fp32 accumulators (plain store, running log-sum-exp statistics, softmax gradient, ...).
//
// Tiling: a workgroup owns a BM x BN tile of the output and walks K in steps of BK = 64.
// WM x WN wavefronts split the tile; each wavefront issues 32x32x16 bf16 MFMAs on a
// (BM/WM) x (BN/WN) sub-tile whose fp32 accumulators stay in registers for the whole K loop.
// Operand tiles are fetched with 16-byte buffer loads (rows beyond M or N read as zero through
// the buffer descriptor's range check), staged through double-buffered LDS in an XOR-swizzled
// layout so that the 16-byte fragment reads of a wavefront are free of bank conflicts.
//
// K must be a multiple of 64; M and N are arbitrary.
#pragma once

#include "cp_internal.hpp"

namespace cph {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

struct GemmOperands {
    const bf16_t *A;   // [M, lda]
    const bf16_t *B;   // [N, ldb]
    long lda, ldb;     // elements
    int M, N, K;       // K % 64 == 0
    int tiles_m, tiles_n;
};

template <int BM_, int BN_, int WM_, int WN_>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, BK = 64;
    static constexpr int THREADS = WM * WN * kWave;
    static constexpr int WTM = BM / WM, WTN = BN / WN;       // wavefront sub-tile
    static constexpr int TM = WTM / 32, TN = WTN / 32;       // 32x32 MFMA blocks per wavefront
    static constexpr int ROWS_PER_PASS = THREADS / 8;        // a pass moves one 16-byte chunk per thread
    static constexpr int A_PASSES = BM / ROWS_PER_PASS, B_PASSES = BN / ROWS_PER_PASS;
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "wave tile must be a multiple of 32x32");
    static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile rows must divide into load passes");
};

// Raw buffer descriptor for `bytes` bytes at `base` (no stride, range-checked).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// Workgroup id -> output tile.  Consecutive workgroup ids go round-robin over the 8 XCDs, so the
// id is first unrolled into a per-XCD contiguous range; inside it tiles are walked in groups of 8
// rows of tiles so that the tiles in flight on one XCD share operand panels in its L2.
__device__ __forceinline__ bool tile_of_block(int bid, int nblocks, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int per_xcd = nblocks >> 3;
    const int lid = (bid & 7) * per_xcd + (bid >> 3);
    if (lid >= tiles_m * tiles_n) return false;
    constexpr int GM = 8;     // 4, 16 and 32 tile rows per group were measured slower
    const int per_group = GM * tiles_n;
    const int group = lid / per_group;
    const int first_m = group * GM;
    const int gsize = min(tiles_m - first_m, GM);
    const int in = lid - group * per_group;
    tm = first_m + in % gsize;
    tn = in / gsize;
    return true;
}
inline int gemm_grid(int tiles_m, int tiles_n) { return (tiles_m * tiles_n + 7) / 8 * 8; }

// The main loop.  On return acc[i][j] holds the 32x32 block (i, j) of this wavefront's sub-tile:
// element v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32 of that block.
template <class Cfg>
__device__ __forceinline__ void gemm_nt_mainloop(const GemmOperands &g, int tm, int tn, char *smem,
                                                 f32x16_t (&acc)[Cfg::TM][Cfg::TN])
{
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / Cfg::WN) * Cfg::WTM;
    const int wn0 = (wave % Cfg::WN) * Cfg::WTN;

    // operand descriptors restricted to this tile's rows: rows past the matrix read as zeros
    const int m0 = tm * BM, n0 = tn * BN;
    const int rows_a = min(BM, g.M - m0), rows_b = min(BN, g.N - n0);
    const __amdgpu_buffer_rsrc_t ra = make_rsrc(g.A + (size_t)m0 * g.lda, (unsigned)((size_t)rows_a * g.lda * 2));
    const __amdgpu_buffer_rsrc_t rb = make_rsrc(g.B + (size_t)n0 * g.ldb, (unsigned)((size_t)rows_b * g.ldb * 2));

    // this thread's 16-byte chunk in each load pass: row = pass*ROWS_PER_PASS + tid/8, chunk = tid%8
    const int lrow = tid >> 3, lchunk = tid & 7;
    const unsigned voff_a = (unsigned)lrow * (unsigned)g.lda * 2u + lchunk * 16u;
    const unsigned voff_b = (unsigned)lrow * (unsigned)g.ldb * 2u + lchunk * 16u;
    const unsigned pass_a = (unsigned)Cfg::ROWS_PER_PASS * (unsigned)g.lda * 2u;
    const unsigned pass_b = (unsigned)Cfg::ROWS_PER_PASS * (unsigned)g.ldb * 2u;
    // LDS position of that chunk: rows are 128 bytes, the 16-byte chunk index is XORed with (row/2)%8,
    // which spreads the 16 rows that one quarter-wavefront reads over all 64 banks
    const int lds_w = lrow * 128 + ((lchunk ^ ((lrow >> 1) & 7)) << 4);

    // fragment reads: lane l reads row l%32 of a 32-row block, k-chunk 2*kk + l/32
    const int frag_row = lane & 31, frag_half = lane >> 5, frag_sw = (lane >> 1) & 7;
    const int lds_ra = (wm0 + frag_row) * 128;
    const int lds_rb = Cfg::A_BYTES + (wn0 + frag_row) * 128;

    u32x4_t sa[Cfg::A_PASSES], sb[Cfg::B_PASSES];

    auto load_global = [&](int kt) {
        const int soff = kt * BK * 2;
#pragma unroll
        for (int p = 0; p < Cfg::A_PASSES; ++p)
            sa[p] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)(voff_a + p * pass_a), soff, 0);
#pragma unroll
        for (int p = 0; p < Cfg::B_PASSES; ++p)
            sb[p] = __builtin_amdgcn_raw_buffer_load_b128(rb, (int)(voff_b + p * pass_b), soff, 0);
    };
    auto store_lds = [&](int stage) {
        char *base = smem + stage * Cfg::STAGE_BYTES + lds_w;
#pragma unroll
        for (int p = 0; p < Cfg::A_PASSES; ++p)
            *reinterpret_cast<u32x4_t *>(base + p * Cfg::ROWS_PER_PASS * 128) = sa[p];
#pragma unroll
        for (int p = 0; p < Cfg::B_PASSES; ++p)
            *reinterpret_cast<u32x4_t *>(base + Cfg::A_BYTES + p * Cfg::ROWS_PER_PASS * 128) = sb[p];
    };

#pragma unroll
    for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int KT = g.K / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    if (KT > 1) load_global(1);

    for (int kt = 0; kt < KT; ++kt) {
        const char *st = smem + (kt & 1) * Cfg::STAGE_BYTES;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int coff = ((kk * 2 + frag_half) ^ frag_sw) << 4;
            bf16x8_t af[Cfg::TM], bfr[Cfg::TN];
#pragma unroll
            for (int i = 0; i < Cfg::TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8_t *>(st + lds_ra + i * 32 * 128 + coff);
#pragma unroll
            for (int j = 0; j < Cfg::TN; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8_t *>(st + lds_rb + j * 32 * 128 + coff);
#pragma unroll
            for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
                for (int j = 0; j < Cfg::TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds((kt + 1) & 1);
        __syncthreads();
        if (kt + 2 < KT) load_global(kt + 2);
    }
}

// Main loop with direct global->LDS loads (no staging registers, no LDS write instructions).
// Each wavefront load instruction moves 64 x 16 bytes = 8 operand rows of 128 bytes into 1 KB of
// consecutive LDS; the XOR swizzle is realised by permuting which 16-byte chunk of its row each
// lane fetches.
//
// Schedule of one K-step of 64 (stage s = kt & 1), four phases of 16 MFMAs per wavefront:
//   phase 0   MFMAs k 0..15    + LDS reads of the k 16..31 fragments + 2nd half of the loads of tile kt+1
//   phase 1   MFMAs k 16..31   + LDS reads of the k 32..47 fragments
//   phase 2   MFMAs k 32..47   + LDS reads of the k 48..63 fragments
//   wait for tile kt+1, workgroup barrier (stage s is dead from here on)
//   phase 3   MFMAs k 48..63   + LDS reads of the first fragments of tile kt+1 + 1st half of the loads of tile kt+2
// Memory instructions are issued one at a time between MFMAs (the order is pinned with scheduling
// barriers): a wavefront issues in order, so a cluster of loads would hold back its MFMAs.
template <class Cfg>
__device__ __forceinline__ void gemm_nt_mainloop_direct(const GemmOperands &g, int tm, int tn, char *smem,
                                                        f32x16_t (&acc)[Cfg::TM][Cfg::TN])
{
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, TM = Cfg::TM, TN = Cfg::TN;
    constexpr int NLOAD = Cfg::A_PASSES + Cfg::B_PASSES;     // direct loads per wavefront and K-step
    constexpr int NFRAG = TM + TN, NMFMA = TM * TN;
    static_assert(BK == 64, "four phases of k = 16");
    constexpr int NEARLY = NLOAD / 2;                        // loads of tile kt+2 issued right after the barrier
    static_assert(NEARLY >= 0 && NEARLY <= NLOAD && NFRAG <= NMFMA, "schedule slots");
    typedef __attribute__((address_space(3))) void lds_void;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave / Cfg::WN) * Cfg::WTM;
    const int wn0 = (wave % Cfg::WN) * Cfg::WTN;

    const int m0 = tm * BM, n0 = tn * BN;
    const int rows_a = min(BM, g.M - m0), rows_b = min(BN, g.N - n0);
    const __amdgpu_buffer_rsrc_t ra = make_rsrc(g.A + (size_t)m0 * g.lda, (unsigned)((size_t)rows_a * g.lda * 2));
    const __amdgpu_buffer_rsrc_t rb = make_rsrc(g.B + (size_t)n0 * g.ldb, (unsigned)((size_t)rows_b * g.ldb * 2));

    // lane -> (row, physical chunk) inside a pass; the lane fetches the global chunk that belongs there
    const int lrow = tid >> 3, pchunk = tid & 7;
    const int gchunk = pchunk ^ ((lrow >> 1) & 7);
    const unsigned voff_a = (unsigned)lrow * (unsigned)g.lda * 2u + gchunk * 16u;
    const unsigned voff_b = (unsigned)lrow * (unsigned)g.ldb * 2u + gchunk * 16u;
    const unsigned pass_a = (unsigned)Cfg::ROWS_PER_PASS * (unsigned)g.lda * 2u;
    const unsigned pass_b = (unsigned)Cfg::ROWS_PER_PASS * (unsigned)g.ldb * 2u;
    const int lds_wave = wave * 8 * 128;     // this wavefront's 1 KB slot inside a pass of 32 rows

    const int frag_row = lane & 31, frag_half = lane >> 5, frag_sw = (lane >> 1) & 7;
    const int lds_ra = (wm0 + frag_row) * 128;
    const int lds_rb = Cfg::A_BYTES + (wn0 + frag_row) * 128;
    int coff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) coff[kk] = ((kk * 2 + frag_half) ^ frag_sw) << 4;

    bf16x8_t fa[2][TM], fb[2][TN];

    // load number q of a K-step: q < A_PASSES moves 32 rows of A, the rest 32 rows of B
    auto load_one = [&](int kt, int stage, int q) {
        const int soff = kt * BK * 2;
        char *base = smem + stage * Cfg::STAGE_BYTES + lds_wave;
        if (q < Cfg::A_PASSES)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void *)(base + q * Cfg::ROWS_PER_PASS * 128), 16,
                                                     (int)(voff_a + q * pass_a), soff, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rb, (lds_void *)(base + Cfg::A_BYTES + (q - Cfg::A_PASSES) * Cfg::ROWS_PER_PASS * 128), 16,
                (int)(voff_b + (q - Cfg::A_PASSES) * pass_b), soff, 0, 0);
    };
    // fragment number q of a phase, in the order the MFMAs need them: A0, B0..B(TN-1), A1..A(TM-1)
    auto frag_one = [&](const char *st, int kk, int buf, int q) {
        if (q == 0) fa[buf][0] = *reinterpret_cast<const bf16x8_t *>(st + lds_ra + coff[kk]);
        else if (q <= TN) fb[buf][q - 1] = *reinterpret_cast<const bf16x8_t *>(st + lds_rb + (q - 1) * 32 * 128 + coff[kk]);
        else fa[buf][q - TN] = *reinterpret_cast<const bf16x8_t *>(st + lds_ra + (q - TN) * 32 * 128 + coff[kk]);
    };
    auto mfma_one = [&](int buf, int idx) {
        const int i = idx / TN, j = idx % TN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
    };
#define CPH_PIN() __builtin_amdgcn_sched_barrier(0)
    // one phase: MFMAs on fragment buffer BUF, fragments of (ST, KK) into the other buffer and,
    // if LOAD_KT >= 0, the loads LOAD_Q0 .. LOAD_Q0 + NLOAD/2 - 1 of tile LOAD_KT into LOAD_STAGE
#define CPH_PHASE(BUF, ST, KK, DO_LOAD, LOAD_KT, LOAD_STAGE, LOAD_Q0, LOAD_CNT)                    \
    _Pragma("unroll") for (int m = 0; m < NMFMA; ++m) {                                            \
        mfma_one(BUF, m);                                                                          \
        CPH_PIN();                                                                                 \
        if ((DO_LOAD) && (LOAD_CNT) > 0) {                                                         \
            _Pragma("unroll") for (int q = 0; q < (LOAD_CNT); ++q)                                 \
                if ((q * NMFMA) / ((LOAD_CNT) > 0 ? (LOAD_CNT) : 1) == m) { load_one(LOAD_KT, LOAD_STAGE, (LOAD_Q0) + q); CPH_PIN(); } \
        }                                                                                          \
        _Pragma("unroll") for (int q = 0; q < NFRAG; ++q)                                          \
            if (((q + 1) * NMFMA) / NFRAG - 1 == m) { frag_one(ST, KK, (BUF) ^ 1, q); CPH_PIN(); } \
    }

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // No load is ever issued for a tile past the end of K: a late arrival would land in LDS while the
    // epilogue is using it.  The last two K-steps are therefore peeled off with their loads removed.
    const int KT = g.K / BK;
#pragma unroll
    for (int q = 0; q < NLOAD; ++q) load_one(0, 0, q);
    if (KT > 1) {
#pragma unroll
        for (int q = 0; q < NEARLY; ++q) load_one(1, 1, q);
        __builtin_amdgcn_s_waitcnt(0x0F70 | (NEARLY & 15) | ((NEARLY >> 4) << 14));   // vmcnt(NEARLY): tile 0 has landed
    } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NFRAG; ++q) frag_one(smem, 0, 0, q);

#define CPH_K_STEP_DIRECT(KT_, LOAD_NEXT, LOAD_AFTER)                                              \
    {                                                                                              \
        const int cur = (KT_) & 1;                                                                 \
        const char *st = smem + cur * Cfg::STAGE_BYTES;                                            \
        const char *nx = smem + (cur ^ 1) * Cfg::STAGE_BYTES;                                      \
        CPH_PHASE(0, st, 1, LOAD_NEXT, (KT_) + 1, cur ^ 1, NEARLY, NLOAD - NEARLY)                 \
        CPH_PHASE(1, st, 2, false, 0, 0, 0, 0)                                                     \
        CPH_PHASE(0, st, 3, false, 0, 0, 0, 0)                                                     \
        __builtin_amdgcn_s_waitcnt(0x0F70); /* vmcnt(0): tile kt+1 is complete in the other stage */ \
        __syncthreads();                                                                           \
        CPH_PHASE(1, nx, 0, LOAD_AFTER, (KT_) + 2, cur, 0, NEARLY)                                 \
    }
    int kt = 0;
    for (; kt < KT - 2; ++kt) CPH_K_STEP_DIRECT(kt, true, true)
    if (kt == KT - 2) {
        CPH_K_STEP_DIRECT(kt, true, false)
        ++kt;
    }
    CPH_K_STEP_DIRECT(kt, false, false)
#undef CPH_K_STEP_DIRECT
#undef CPH_PHASE
#undef CPH_PIN
}

// Generic kernel: main loop + epilogue functor.  Epi::operator() receives the accumulators of one
// wavefront together with the global row/column of its sub-tile's origin.
// One workgroup per output tile.  (A persistent variant that walks several tiles per workgroup was
// measured: the extra live state made the compiler spill accumulators and it ran slower.)
template <class Cfg, class Epi>
__global__ void __launch_bounds__(Cfg::THREADS) k_gemm_nt(GemmOperands g, Epi epi)
{
    __shared__ __attribute__((aligned(16))) char smem[Cfg::LDS_BYTES];
    int tm, tn;
    if (!tile_of_block(blockIdx.x, gridDim.x, g.tiles_m, g.tiles_n, tm, tn)) return;
    f32x16_t acc[Cfg::TM][Cfg::TN];
#if defined(CPH_MAINLOOP_SIMPLE)
    gemm_nt_mainloop<Cfg>(g, tm, tn, smem, acc);          // plain reference loop, for debugging builds only
#else
    gemm_nt_mainloop_direct<Cfg>(g, tm, tn, smem, acc);
#endif
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row0 = tm * Cfg::BM + (wave / Cfg::WN) * Cfg::WTM;
    const int col0 = tn * Cfg::BN + (wave % Cfg::WN) * Cfg::WTN;
    epi.template run<Cfg>(acc, row0, col0, lane, wave, tn, smem);
}

template <class Cfg, class Epi>
inline void launch_gemm_nt(const char *name, const bf16_t *A, long lda, int M, const bf16_t *B, long ldb, int N, int K,
                           const Epi &epi, hipStream_t st)
{
    ProfileScope prof(name, 2.0 * (double)M * (double)N * (double)K, st);
    GemmOperands g;
    g.A = A; g.B = B; g.lda = lda; g.ldb = ldb; g.M = M; g.N = N; g.K = K;
    g.tiles_m = (M + Cfg::BM - 1) / Cfg::BM;
    g.tiles_n = (N + Cfg::BN - 1) / Cfg::BN;
    k_gemm_nt<Cfg, Epi><<<gemm_grid(g.tiles_m, g.tiles_n), Cfg::THREADS, 0, st>>>(g, epi);
}

// Cross-lane steps of the row statistics, as data-parallel-primitive moves (no LDS traffic):
// quad swaps, mirror inside 8 and inside 16 lanes give every lane of a 16-lane row the row's value;
// the last lane of rows 0 and 2 is then broadcast into rows 1 and 3.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_move(float old, float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float row16_max(float v)
{
    v = fmaxf(v, dpp_move<0xB1>(v, v));    // lane ^ 1
    v = fmaxf(v, dpp_move<0x4E>(v, v));    // lane ^ 2
    v = fmaxf(v, dpp_move<0x141>(v, v));   // mirror within 8
    v = fmaxf(v, dpp_move<0x140>(v, v));   // mirror within 16
    return v;
}
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_move<0xB1>(v, v);
    v += dpp_move<0x4E>(v, v);
    v += dpp_move<0x141>(v, v);
    v += dpp_move<0x140>(v, v);
    return v;
}

// ---------------------------------------------------------------------------------------------
// Coalesced output of a wavefront's sub-tile.  The MFMA result layout gives each lane single
// elements of 32 different columns, so values are first laid out row-major in a wave-private
// LDS area (32 rows at a time, the operand stages are free by then) and then written with
// 16-byte stores: a wavefront store covers whole 256-byte row segments.
// `value(i, j, v, row, col)` yields the output for accumulator element v of block (i, j), whose
// global coordinates are (row, col).  All loops are fully unrolled so that the accumulators are
// only ever indexed with constants and stay in registers.
// ---------------------------------------------------------------------------------------------
// I0, I1 restrict the call to the 32-row blocks I0 .. I1-1 of the sub-tile (default: all of them).
template <class Cfg, class F, int I0 = 0, int I1 = Cfg::TM>
__device__ __forceinline__ void store_tile_bf16(char *smem, int wave, int lane, int row0, int col0, int row_limit,
                                                int col_limit /* multiple of 8 */, bf16_t *__restrict__ dst, long ld,
                                                F value)
{
    constexpr int RS = Cfg::WTN * 2 + 16;              // padded row stride in bytes
    constexpr int CPR = Cfg::WTN / 8;                   // 16-byte chunks per row
    constexpr int RPP = kWave / CPR;                    // rows per store pass
    static_assert(4 * 32 * RS <= Cfg::LDS_BYTES || Cfg::WM * Cfg::WN * 32 * RS <= Cfg::LDS_BYTES, "staging fits");
    char *stage = smem + wave * (32 * RS);
    __syncthreads();                                    // every wavefront is done reading operand tiles
#pragma unroll
    for (int i = I0; i < I1; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
#pragma unroll
            for (int j = 0; j < Cfg::TN; ++j) {
                const int c = j * 32 + (lane & 31);
                *reinterpret_cast<bf16_t *>(stage + r * RS + c * 2) = value(i, j, v, row0 + i * 32 + r, col0 + c);
            }
        }
        __syncthreads();
#pragma unroll
        for (int p = 0; p < 32 / RPP; ++p) {
            const int r = p * RPP + lane / CPR, ch = lane % CPR;
            const u32x4_t val = *reinterpret_cast<const u32x4_t *>(stage + r * RS + ch * 16);
            const int grow = row0 + i * 32 + r, gcol = col0 + ch * 8;
            if (grow < row_limit && gcol < col_limit)
                *reinterpret_cast<u32x4_t *>(dst + (size_t)grow * ld + gcol) = val;
        }
        __syncthreads();
    }
}

// Transposed bf16 output: dst[col * ld + row] = value(i, j, v, row, col).  A lane owns four consecutive
// rows of one column per accumulator group, so the sub-tile is laid out column-major in LDS (64 rows at
// a time, 8-byte writes) and leaves as 16-byte pieces of 128-byte column segments.
// row_limit and ld are multiples of 8; rows are written up to row_limit, columns up to col_limit.
// IP0, IP1 restrict the call to the 64-row passes IP0 .. IP1-1 (default: all of them).
template <class Cfg, class F, int IP0 = 0, int IP1 = Cfg::TM / 2>
__device__ __forceinline__ void store_tile_bf16_transposed(char *smem, int wave, int lane, int row0, int col0,
                                                           int row_limit, int col_limit, bf16_t *__restrict__ dst,
                                                           long ld, F value)
{
    static_assert(Cfg::TM % 2 == 0, "two 32-row blocks per pass");
    constexpr int CS = 64 * 2 + 16;                     // padded column stride in bytes (64 rows)
    static_assert(Cfg::WM * Cfg::WN * Cfg::WTN * CS <= Cfg::LDS_BYTES, "staging fits");
    char *stage = smem + wave * (Cfg::WTN * CS);
    __syncthreads();
#pragma unroll
    for (int ip = IP0; ip < IP1; ++ip) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii) {
            const int i = ip * 2 + ii;
#pragma unroll
            for (int j = 0; j < Cfg::TN; ++j) {
                const int c = j * 32 + (lane & 31);
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int r = 8 * gq + 4 * (lane >> 5);          // first of four consecutive rows
                    unsigned lo, hi;
                    {
                        const bf16_t a = value(i, j, gq * 4 + 0, row0 + i * 32 + r + 0, col0 + c);
                        const bf16_t b = value(i, j, gq * 4 + 1, row0 + i * 32 + r + 1, col0 + c);
                        lo = (unsigned)a | ((unsigned)b << 16);
                    }
                    {
                        const bf16_t a = value(i, j, gq * 4 + 2, row0 + i * 32 + r + 2, col0 + c);
                        const bf16_t b = value(i, j, gq * 4 + 3, row0 + i * 32 + r + 3, col0 + c);
                        hi = (unsigned)a | ((unsigned)b << 16);
                    }
                    typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
                    u32x2_t pk = {lo, hi};
                    *reinterpret_cast<u32x2_t *>(stage + c * CS + (ii * 32 + r) * 2) = pk;
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int p = 0; p < Cfg::WTN / 8; ++p) {
            const int c = p * 8 + (lane >> 3), ch = lane & 7;
            const u32x4_t val = *reinterpret_cast<const u32x4_t *>(stage + c * CS + ch * 16);
            const int grow = row0 + ip * 64 + ch * 8, gcol = col0 + c;
            if (grow < row_limit && gcol < col_limit)
                *reinterpret_cast<u32x4_t *>(dst + (size_t)gcol * ld + grow) = val;
        }
        __syncthreads();
    }
}

// fp32 variant: dst = value, or dst += value when `accumulate` is set (16-byte loads and stores).
template <class Cfg, class F>
__device__ __forceinline__ void store_tile_f32(char *smem, int wave, int lane, int row0, int col0, int row_limit,
                                               int col_limit /* multiple of 4 */, float *__restrict__ dst, long ld,
                                               bool accumulate, F value)
{
    typedef float f32x4_t __attribute__((ext_vector_type(4)));
    constexpr int RS = Cfg::WTN * 4 + 16;
    constexpr int CPR = Cfg::WTN / 4;
    constexpr int RPP = kWave / CPR;
    static_assert(Cfg::WM * Cfg::WN * 32 * RS <= Cfg::LDS_BYTES, "staging fits");
    char *stage = smem + wave * (32 * RS);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < Cfg::TM; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
#pragma unroll
            for (int j = 0; j < Cfg::TN; ++j) {
                const int c = j * 32 + (lane & 31);
                *reinterpret_cast<float *>(stage + r * RS + c * 4) = value(i, j, v, row0 + i * 32 + r, col0 + c);
            }
        }
        __syncthreads();
#pragma unroll
        for (int p = 0; p < 32 / RPP; ++p) {
            const int r = p * RPP + lane / CPR, ch = lane % CPR;
            f32x4_t val = *reinterpret_cast<const f32x4_t *>(stage + r * RS + ch * 16);
            const int grow = row0 + i * 32 + r, gcol = col0 + ch * 4;
            if (grow < row_limit && gcol < col_limit) {
                f32x4_t *q = reinterpret_cast<f32x4_t *>(dst + (size_t)grow * ld + gcol);
                if (accumulate) val += *q;
                *q = val;
            }
        }
        __syncthreads();
    }
}

// row / column of accumulator element v of block (i, j) for lane l, relative to the sub-tile origin
__device__ __forceinline__ int acc_row(int i, int v, int lane) { return i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }
__device__ __forceinline__ int acc_col(int j, int lane) { return j * 32 + (lane & 31); }

}  // namespace cph

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
    constexpr int GM = 8;
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
    // LDS position of that chunk: rows are 128 bytes, the 16-byte chunk index is XORed with row%8
    const int lds_w = lrow * 128 + ((lchunk ^ (lrow & 7)) << 4);

    // fragment reads: lane l reads row l%32 of a 32-row block, k-chunk 2*kk + l/32
    const int frag_row = lane & 31, frag_half = lane >> 5, frag_sw = lane & 7;
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

// Generic kernel: main loop + epilogue functor.  Epi::operator() receives the accumulators of one
// wavefront together with the global row/column of its sub-tile's origin.
template <class Cfg, class Epi>
__global__ void __launch_bounds__(Cfg::THREADS) k_gemm_nt(GemmOperands g, Epi epi)
{
    __shared__ __attribute__((aligned(16))) char smem[Cfg::LDS_BYTES];
    int tm, tn;
    if (!tile_of_block(blockIdx.x, gridDim.x, g.tiles_m, g.tiles_n, tm, tn)) return;
    f32x16_t acc[Cfg::TM][Cfg::TN];
    gemm_nt_mainloop<Cfg>(g, tm, tn, smem, acc);
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

// ---------------------------------------------------------------------------------------------
// Coalesced output of a wavefront's sub-tile.  The MFMA result layout gives each lane single
// elements of 32 different columns, so values are first laid out row-major in a wave-private
// LDS area (32 rows at a time, the operand stages are free by then) and then written with
// 16-byte stores: a wavefront store covers whole 256-byte row segments.
// `value(i, j, v, row, col)` yields the output for accumulator element v of block (i, j), whose
// global coordinates are (row, col).  All loops are fully unrolled so that the accumulators are
// only ever indexed with constants and stay in registers.
// ---------------------------------------------------------------------------------------------
template <class Cfg, class F>
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
    for (int i = 0; i < Cfg::TM; ++i) {
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

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
// WM x WN wavefronts split the tile; each wavefront issues 16x16x32 bf16 MFMAs on a
// (BM/WM) x (BN/WN) sub-tile whose fp32 accumulators stay in registers for the whole K loop.
// Operand tiles are fetched with 16-byte buffer loads (rows beyond M or N read as zero through
// the buffer descriptor's range check), staged through double-buffered LDS in an XOR-swizzled
// layout so that the 16-byte fragment reads of a wavefront are free of bank conflicts.
//
// K must be a multiple of 64; M and N are arbitrary.
//
// Either operand may instead be "K-major" (the contraction index is the slow one: A[K, lda] with the M output rows
// along its columns, likewise B[K, ldb]): the products of the backward pass that contract over rows (dU = dz^T Y,
// dW = dY^T H) or against a weight matrix stored the other way round (dY = dz U, dH = dY W) then need no
// transposed copy of anything.  A K-major tile is 64 k-rows of 256 columns; it is laid out in LDS so that gfx950's
// transposing LDS read (ds_read_b64_tr_b16: inside 16 lanes, 4 k-rows x 16 columns in, 4 k-values of one column
// per lane out) delivers MFMA operand fragments directly.  With both operands K-major K is arbitrary (rows past
// its end read as zero); otherwise K must still be a multiple of 64.
#pragma once

#include "cp_internal.hpp"
#include "tile_walk.hpp"

namespace cph {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

struct GemmOperands {
    const bf16_t *A;   // [M, lda]
    const bf16_t *B;   // [N, ldb]
    long lda, ldb;     // elements
    int M, N, K;       // K % 64 == 0 unless both operands are K-major
    int ka_rows, kb_rows;   // K-major operands: rows that exist (<= K; the rest of K reads as zero)
    int tiles_m, tiles_n;
    int gm;            // tile rows per group of the workgroup -> tile walk
};

// LDS layout of a K-major tile (64 k-rows x 256 columns).  Four consecutive k-rows (a quad) are interleaved in
// units of 32 bytes: the 16 columns [16 p, 16 p + 16) of the quad's rows t = 0..3 sit at p * 128 + t * 32, so the
// 4 x 32 bytes that 16 lanes hand to one transposing read are one 128-byte span; quads are 2 KB apart and every
// pair of quads is followed by 128 bytes of padding, which puts the quads of k-groups g and g + 1 (8 k-rows = two
// quads apart) into the two halves of the 256-byte bank cycle: a wavefront's read is free of bank conflicts.
// A direct global->LDS load instruction (64 lanes x 16 bytes = 1 KB, consecutive in LDS) fills half a quad: lane i
// fetches 8 columns [16 (8 e + i / 8) + 8 (i % 2), +8) of k-row (i % 8) / 2, i.e. 256 contiguous bytes of each of
// four rows; the four wavefronts of a pass fill two quads, and a pass advances by 4224 bytes.
constexpr int kKmPassBytes = 2 * 2048 + 128;
constexpr int kKmTileBytes = 8 * kKmPassBytes;

template <int BM_, int BN_, int WM_, int WN_, bool AKM_ = false, bool BKM_ = false, bool ABL_ = false, bool BBL_ = false>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, BK = 64;
    static constexpr bool AKM = AKM_, BKM = BKM_;     // operand is K-major
    static constexpr bool ABL = ABL_, BBL = BBL_;     // operand is stored tile by tile: [rows/256][K/64][256][64]
    static_assert(!(AKM_ && ABL_) && !(BKM_ && BBL_), "an operand is K-major or blocked, not both");
    static constexpr int THREADS = WM * WN * kWave;
    static constexpr int WTM = BM / WM, WTN = BN / WN;       // wavefront sub-tile
    static constexpr int TM16 = WTM / 16, TN16 = WTN / 16;   // 16x16 MFMA blocks per wavefront
    static constexpr int ROWS_PER_PASS = THREADS / 8;        // a pass moves one 16-byte chunk per thread
    static constexpr int A_PASSES = BM / ROWS_PER_PASS, B_PASSES = BN / ROWS_PER_PASS;
    static constexpr int A_BYTES = AKM_ ? kKmTileBytes : BM * BK * 2, B_BYTES = BKM_ ? kKmTileBytes : BN * BK * 2;
    static_assert(!(AKM_ || BKM_) || WM_ * WN_ == 4, "K-major operands: four wavefronts");
    static_assert((!AKM_ || BM_ == 256) && (!BKM_ || BN_ == 256), "a K-major tile has 256 columns");
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static_assert(BM % (WM * 64) == 0 && BN % (WN * 32) == 0, "wave tile must be a multiple of 64 rows x 32 columns");
    static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile rows must divide into load passes");
};

// Raw buffer descriptor for `bytes` bytes at `base` (no stride, range-checked).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// The same descriptor as four scalar words, and a direct global->LDS load of 16 bytes per lane spelled out, for the
// kernels with K-major operands.  Their fragments come from gfx950's transposing LDS read, and before every such
// read the compiler waits for all outstanding loads once it knows that loads into LDS are in flight (it cannot tell
// that they go to the other stage), which serialises the whole pipeline (measured: 3-5 times slower).  Loads
// issued this way are invisible to that bookkeeping; the main loop's own explicit waits (before the barrier that
// publishes a stage) are what orders them, exactly as for the other kernels.
typedef int i32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i32x4_t make_rsrc_words(const void *base, unsigned bytes)
{
    const unsigned long long p = reinterpret_cast<unsigned long long>(base);
    i32x4_t r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(p & 0xFFFFFFFFull));
    r[1] = __builtin_amdgcn_readfirstlane((int)((p >> 32) & 0xFFFFull));
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}
// lds_addr: LDS byte address of the wavefront's 1 KB destination (uniform); voff: per-lane byte offset (range-checked
// against the descriptor); soff: uniform byte offset (not range-checked)
__device__ __forceinline__ void load_lds_16_spelled_out(i32x4_t rsrc, unsigned lds_addr, unsigned voff, int soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory");
}

// Tile rows per group of that walk.  8 x 4 tiles in flight per XCD suit the vocabulary-wide products (125 or
// more tile columns; 16 rows per group cost them 10-25 %); the products with a d-wide output (16 tile columns)
// and y = W h run 2-5 % faster with 4 x 8, which re-reads their large A operand half as often (1, 2 and 8 rows per
// group cost dY 1.7-2.4 %, 2 and 8 cost dU 1.2-1.8 %).
constexpr int kGroupRowsWide = 8, kGroupRowsNarrow = 4;

// The main loop, with direct global->LDS loads (no staging registers, no LDS write instructions) and
// 16x16x32 MFMAs.  Each wavefront load instruction moves 64 x 16 bytes = 8 operand rows of 128 bytes into
// 1 KB of consecutive LDS; the XOR swizzle is realised by permuting which 16-byte chunk of its row each
// lane fetches.
// Why 16x16x32: on random bf16 data the matrix cores of this part are limited by power, not by issue rate,
// and that instruction delivers about 14 % more FLOP/s there than the 32x32x16 one (2.18 against 1.92
// PFLOP/s in a loop of nothing but MFMAs with this register tiling; the loop below gained 3-5 %).
// A K-step of 64 is two K-blocks of 32; a K-block is two phases, one per half of the wavefront's rows:
//   phase 0   rows half 0, k 0..31    + reads: A half 1 (k 0..31), B first half (k 32..63)   + 2nd half of the loads of tile kt+1
//   phase 1   rows half 1, k 0..31    + reads: B second half (k 32..63), A half 0 (k 32..63)
//   phase 2   rows half 0, k 32..63   + reads: A half 1 (k 32..63)
//   wait for tile kt+1, workgroup barrier
//   phase 3   rows half 1, k 32..63   + reads from tile kt+1: A half 0, B (k 0..31)          + 1st half of the loads of tile kt+2
// Memory instructions are issued one at a time between MFMAs (the order is pinned with scheduling
// barriers): a wavefront issues in order, so a cluster of loads would hold back its MFMAs.
// On return acc[i][j] holds the 16x16 block (i, j) of the wavefront's sub-tile: element v of lane l is
// row 4*(l/16) + v, column l%16 of that block.
template <class Cfg>
__device__ __forceinline__ void gemm_nt_mainloop_direct(const GemmOperands &g, int tm, int tn, char *smem,
                                                          f32x4_t (&acc)[Cfg::TM16][Cfg::TN16])
{
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, TM = Cfg::TM16, TN = Cfg::TN16;
    constexpr int HA = TM / 2, HB = TN / 2;                  // A fragments per row half, B fragments per read half
    constexpr int NLOAD = Cfg::A_PASSES + Cfg::B_PASSES;
    constexpr int NM = HA * TN;                              // MFMAs per phase
    // loads of a tile per phase, from the phase after the barrier that frees its stage: phases 3, 0, 1, 2.
    // Measured on the three large product shapes: 8/8/0/0 and 10/6/0/0 lead (the latter by about 1 %),
    // 12/4 loses 3-5 %, 16/0 and any load in phases 1 or 2 (less time to land) lose 10-30 %.
    constexpr int L3 = NLOAD * 5 / 8, L0 = NLOAD - L3, L1 = 0, L2 = 0;
    constexpr int NEARLY = L3;
    // The fragment reads of phase 2 are the last ones before the barrier, whose fence waits for every LDS read of the
    // wavefront: spread over the whole phase, the last of them was issued one matrix instruction before that wait and
    // the matrix pipe could run dry for an LDS latency per K-step.  They go into the first half of the phase (worth
    // 0.2-0.4 % on the three large shapes).
    constexpr int P2_SPAN = NM / 2;
    static_assert(BK == 64 && TM % 2 == 0 && TN % 2 == 0 && TN + HA <= NM && L2 >= 0, "schedule slots");
    typedef __attribute__((address_space(3))) void lds_void;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave / Cfg::WN) * Cfg::WTM;
    const int wn0 = (wave % Cfg::WN) * Cfg::WTN;

    const int m0 = tm * BM, n0 = tn * BN;
    const int rows_a = min(BM, g.M - m0), rows_b = min(BN, g.N - n0);
    // K-contiguous operand: one descriptor over the tile's rows, the K-step is a scalar byte offset.
    // K-major operand: a descriptor per K-step over its 64 k-rows from the tile's first column on (the whole
    // operand may exceed the 4 GiB a descriptor can address); k-rows past the operand's end are out of range and
    // read as zero, columns past M or N read whatever follows in the row and only reach accumulators that are
    // never stored.
    // bytes between two rows of the tile: the leading dimension, or 128 for a blocked operand
    const unsigned rsa = Cfg::ABL ? 128u : (unsigned)g.lda * 2u, rsb = Cfg::BBL ? 128u : (unsigned)g.ldb * 2u;
    // (a blocked operand's descriptor spans the whole panel of its tile row: all 256 rows of every block exist)
    const unsigned span_a = Cfg::ABL ? (unsigned)((size_t)BM * g.K * 2) : (unsigned)((size_t)rows_a * g.lda * 2);
    const unsigned span_b = Cfg::BBL ? (unsigned)((size_t)BN * g.K * 2) : (unsigned)((size_t)rows_b * g.ldb * 2);
    const __amdgpu_buffer_rsrc_t ra = make_rsrc(g.A + (size_t)m0 * g.lda, span_a);
    const __amdgpu_buffer_rsrc_t rb = make_rsrc(g.B + (size_t)n0 * g.ldb, span_b);
    // A K-major operand's descriptor is kept for the K-tile whose loads are being issued and moved on by one tile
    // (64 k-rows) at a time: a 64-bit add on the base and a choice among three sizes (a full tile, the operand's
    // last, partial one, nothing past its end).  Rebuilding it from the tile index cost a dozen scalar instructions
    // in one place, four times per K-step, which held the matrix instructions up by several percent.
    struct KmWalk {
        i32x4_t d;          // descriptor of tile `tile`
        int tile;
        unsigned step;      // bytes from one K-tile to the next
        int full_tiles;     // tiles with all 64 rows
        unsigned full, tail;
    };
    auto km_start = [&](const bf16_t *base, long ld, int col0, int krows) {
        KmWalk w;
        w.tile = 0;
        w.step = (unsigned)(BK * ld * 2);
        w.full_tiles = krows / BK;
        w.full = (unsigned)(((long)BK * ld - col0) * 2);
        const int rest = krows % BK;
        w.tail = rest > 0 ? (unsigned)(((long)rest * ld - col0) * 2) : 0u;
        w.d = make_rsrc_words(base + col0, w.full_tiles > 0 ? w.full : w.tail);
        return w;
    };
    auto km_advance = [&](KmWalk &w) {
        const unsigned long long at = (((unsigned long long)(unsigned)w.d[1] << 32) | (unsigned)w.d[0]) + w.step;
        ++w.tile;
        w.d[0] = (int)(unsigned)at;
        w.d[1] = (int)(unsigned)(at >> 32);
        w.d[2] = (int)(w.tile < w.full_tiles ? w.full : (w.tile == w.full_tiles ? w.tail : 0u));
    };
    KmWalk walk_a = km_start(g.A, g.lda, m0, g.ka_rows), walk_b = km_start(g.B, g.ldb, n0, g.kb_rows);
    constexpr bool kSpelledOut = Cfg::AKM || Cfg::BKM;
    const i32x4_t wa = make_rsrc_words(g.A + (size_t)m0 * g.lda, span_a);
    const i32x4_t wb = make_rsrc_words(g.B + (size_t)n0 * g.ldb, span_b);
    const unsigned lds_smem = __builtin_amdgcn_readfirstlane((unsigned)reinterpret_cast<unsigned long long>((lds_void *)smem));

    const int lrow = tid >> 3, pchunk = tid & 7;
    const int gchunk = pchunk ^ ((lrow >> 1) & 7);
    // K-major: k-row of the pass and first column that this thread fetches (see the layout above)
    const int km_row = (wave >> 1) * 4 + ((lane & 7) >> 1);
    const int km_col = ((wave & 1) * 8 + (lane >> 3)) * 16 + (lane & 1) * 8;
    const unsigned voff_a = Cfg::AKM ? (unsigned)km_row * (unsigned)g.lda * 2u + km_col * 2u
                                     : (unsigned)lrow * rsa + gchunk * 16u;
    const unsigned voff_b = Cfg::BKM ? (unsigned)km_row * (unsigned)g.ldb * 2u + km_col * 2u
                                     : (unsigned)lrow * rsb + gchunk * 16u;
    const unsigned pass_a = (unsigned)(Cfg::AKM ? 8 : Cfg::ROWS_PER_PASS) * rsa;
    const unsigned pass_b = (unsigned)(Cfg::BKM ? 8 : Cfg::ROWS_PER_PASS) * rsb;
    constexpr int lds_pass_a = Cfg::AKM ? kKmPassBytes : Cfg::ROWS_PER_PASS * 128;
    constexpr int lds_pass_b = Cfg::BKM ? kKmPassBytes : Cfg::ROWS_PER_PASS * 128;
    const int lds_wave = wave * 8 * 128;

    // fragment reads: lane l reads row l%16 of a 16-row block, 16-byte k-chunk 4*kb + l/16 of its 128-byte row
    const int frag_row = lane & 15, frag_q = lane >> 4, frag_sw = (lane >> 1) & 7;
    // K-major fragments: lane (g, s) = (lane / 16, lane % 16) of a transposing read addresses 8 bytes of k-row
    // s / 4 of a quad; k-group g is two quads (and one padding) further on; the 16-column block is a constant
    const int km_lane = frag_q * (2 * 2048 + 128) + frag_row * 8;
    const int lds_ra = Cfg::AKM ? km_lane + (wm0 / 16) * 128 : (wm0 + frag_row) * 128;
    const int lds_rb = Cfg::A_BYTES + (Cfg::BKM ? km_lane + (wn0 / 16) * 128 : (wn0 + frag_row) * 128);
    int coff[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) coff[kb] = ((kb * 4 + frag_q) ^ frag_sw) << 4;

    bf16x8_t fa[2][HA], fb[2][TN];

    // Everything that the descriptor's range check must see is in the vector offset (the scalar offset is added to
    // the address but not checked): the pass for both layouts.  The K-step is the scalar offset of a K-contiguous
    // operand and part of the descriptor's base for a K-major one.  Kernels with a K-major operand issue all their
    // loads spelled out (see load_lds_16_spelled_out).
    auto load_one = [&](int kt, int stage, int q) {
        // the K-step: 128 bytes along the row, or one block of BM (BN) rows x 128 bytes of a blocked operand
        const int soff = q < Cfg::A_PASSES ? kt * (Cfg::ABL ? BM * 128 : BK * 2) : kt * (Cfg::BBL ? BN * 128 : BK * 2);
        char *base = smem + stage * Cfg::STAGE_BYTES + lds_wave;
        const unsigned lbase = lds_smem + stage * Cfg::STAGE_BYTES + lds_wave;
        if (q < Cfg::A_PASSES) {
            if (Cfg::AKM)
                load_lds_16_spelled_out(walk_a.d, lbase + q * lds_pass_a, voff_a + q * pass_a, 0);       // tile kt == walk_a.tile
            else if (kSpelledOut)
                load_lds_16_spelled_out(wa, lbase + q * lds_pass_a, voff_a + q * pass_a, soff);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void *)(base + q * lds_pass_a), 16,
                                                         (int)(voff_a + q * pass_a), soff, 0, 0);
        } else {
            const int qb = q - Cfg::A_PASSES;
            if (Cfg::BKM)
                load_lds_16_spelled_out(walk_b.d, lbase + Cfg::A_BYTES + qb * lds_pass_b, voff_b + qb * pass_b, 0);
            else if (kSpelledOut)
                load_lds_16_spelled_out(wb, lbase + Cfg::A_BYTES + qb * lds_pass_b, voff_b + qb * pass_b, soff);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void *)(base + Cfg::A_BYTES + qb * lds_pass_b), 16,
                                                         (int)(voff_b + qb * pass_b), soff, 0, 0);
        }
    };
    // a fragment of a K-major tile: 16-column block `blk` of the wavefront, k-block kb: two transposing reads
    // (k-rows 0..3 and 4..7 of the lane's group of 8)
    auto read_km = [&](const char *st, int lane_base, int kb, int blk) {
        const char *p = st + lane_base + kb * (4 * kKmPassBytes) + blk * 128;
#if defined(__HIP_DEVICE_COMPILE__)
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(p));
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(p + 2048));
#else   // the host pass only parses this function
        const s16x4_t lo = *reinterpret_cast<const s16x4_t *>(p), hi = lo;
#endif
        return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto read_a = [&](const char *st, int kb, int buf, int half, int q) {
        if (Cfg::AKM) fa[buf][q] = read_km(st, lds_ra, kb, half * HA + q);
        else fa[buf][q] = *reinterpret_cast<const bf16x8_t *>(st + lds_ra + (half * HA + q) * 16 * 128 + coff[kb]);
    };
    auto read_b = [&](const char *st, int kb, int buf, int q) {
        if (Cfg::BKM) fb[buf][q] = read_km(st, lds_rb, kb, q);
        else fb[buf][q] = *reinterpret_cast<const bf16x8_t *>(st + lds_rb + q * 16 * 128 + coff[kb]);
    };
    auto mfma_one = [&](int abuf, int bbuf, int half, int idx) {
        const int i = idx / TN, j = idx % TN;
        // With K-major operands (fragments assembled from two 64-bit reads) the register allocator no longer keeps
        // the accumulators in place: it rotates them through copies between the two register files, several hundred
        // per K-step.  Spelling the instruction out with the accumulator tied to itself in the accumulation
        // registers and the fragments in vector registers gives the allocation the other kernels get by themselves.
        // The compiler still inserts the waits for the fragments' LDS reads (it sees the operands); what it cannot see
        // is that the instruction is a matrix instruction: uses of one accumulator are 64 instructions apart here, and
        // the wait states before the accumulators are read back are added after the loop (without them the epilogue
        // read accumulators that lacked the last K-block's contribution).
        if (Cfg::AKM || Cfg::BKM)
            asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0"
                         : "+a"(acc[half * HA + i][j])
                         : "v"(fa[abuf][i]), "v"(fb[bbuf][j]));
        else
            acc[half * HA + i][j] =
                __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[abuf][i], fb[bbuf][j], acc[half * HA + i][j], 0, 0, 0);
    };
    // the reads of the four phases, in the order the MFMAs that follow need them
    auto reads0 = [&](const char *st, const char *, int q) {       // A half 1 of k-block 0, then B first half of k-block 1
        if (q < HA) read_a(st, 0, 1, 1, q); else read_b(st, 1, 1, q - HA);
    };
    auto reads1 = [&](const char *st, const char *, int q) {       // B second half of k-block 1, then A half 0 of k-block 1
        if (q < HB) read_b(st, 1, 1, HB + q); else read_a(st, 1, 0, 0, q - HB);
    };
    auto reads2 = [&](const char *st, const char *, int q) { read_a(st, 1, 1, 1, q); };   // A half 1 of k-block 1
    auto reads3 = [&](const char *, const char *nx, int q) {       // next tile: A0, all of B, the rest of A half 0
        if (q == 0) read_a(nx, 0, 0, 0, 0);
        else if (q <= TN) read_b(nx, 0, 0, q - 1);
        else read_a(nx, 0, 0, 0, q - TN);
    };
#define CPH_PIN() __builtin_amdgcn_sched_barrier(0)
#define CPH_PHASE16(ABUF, BBUF, HALF, READS, NREAD, READ_SPAN, DO_LOAD, LOAD_KT, LOAD_STAGE, LOAD_Q0, LOAD_CNT) \
    _Pragma("unroll") for (int m = 0; m < NM; ++m) {                                               \
        mfma_one(ABUF, BBUF, HALF, m);                                                             \
        CPH_PIN();                                                                                 \
        if ((DO_LOAD) && (LOAD_CNT) > 0) {                                                         \
            _Pragma("unroll") for (int q = 0; q < (LOAD_CNT); ++q)                                 \
                if ((q * NM) / ((LOAD_CNT) > 0 ? (LOAD_CNT) : 1) == m) { load_one(LOAD_KT, LOAD_STAGE, (LOAD_Q0) + q); CPH_PIN(); } \
        }                                                                                          \
        _Pragma("unroll") for (int q = 0; q < (NREAD); ++q)                                        \
            if (((q + 1) * (READ_SPAN)) / (NREAD) - 1 == m) { READS(st, nx, q); CPH_PIN(); }       \
    }

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

    // No load is ever issued for a tile past the end of K: a late arrival would land in LDS while the
    // epilogue is using it.  The last two K-steps are therefore peeled off with their loads removed.
    const int KT = (g.K + BK - 1) / BK;
#pragma unroll
    for (int q = 0; q < NLOAD; ++q) load_one(0, 0, q);
    if (KT > 1) {
        if (Cfg::AKM) km_advance(walk_a);
        if (Cfg::BKM) km_advance(walk_b);
#pragma unroll
        for (int q = 0; q < NEARLY; ++q) load_one(1, 1, q);
        __builtin_amdgcn_s_waitcnt(0x0F70 | (NEARLY & 15) | ((NEARLY >> 4) << 14));   // vmcnt(NEARLY): tile 0 has landed
    } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);
    }
    __syncthreads();
    {
        const char *st = smem, *nx = smem;
        (void)st;
#pragma unroll
        for (int q = 0; q < TN + HA; ++q) reads3(st, nx, q);
    }

#define CPH_K_STEP_DIRECT16(KT_, LOAD_NEXT, LOAD_AFTER)                                            \
    {                                                                                              \
        const int cur = (KT_) & 1;                                                                 \
        const char *st = smem + cur * Cfg::STAGE_BYTES;                                            \
        const char *nx = smem + (cur ^ 1) * Cfg::STAGE_BYTES;                                      \
        CPH_PHASE16(0, 0, 0, reads0, HA + HB, NM, LOAD_NEXT, (KT_) + 1, cur ^ 1, L3, L0)           \
        CPH_PHASE16(1, 0, 1, reads1, HB + HA, NM, LOAD_NEXT, (KT_) + 1, cur ^ 1, L3 + L0, L1)      \
        CPH_PHASE16(0, 1, 0, reads2, HA, P2_SPAN, LOAD_NEXT, (KT_) + 1, cur ^ 1, L3 + L0 + L1, L2) \
        __builtin_amdgcn_s_waitcnt(0x0F70); /* vmcnt(0): tile kt+1 is complete in the other stage */ \
        __syncthreads();                                                                           \
        if (LOAD_AFTER) { /* the loads from here on are tile kt+2's */                             \
            if (Cfg::AKM) km_advance(walk_a);                                                      \
            if (Cfg::BKM) km_advance(walk_b);                                                      \
        }                                                                                          \
        CPH_PHASE16(1, 1, 1, reads3, TN + HA, NM, LOAD_AFTER, (KT_) + 2, cur, 0, NEARLY)           \
    }
    int kt = 0;
    for (; kt < KT - 2; ++kt) CPH_K_STEP_DIRECT16(kt, true, true)
    if (kt == KT - 2) {
        CPH_K_STEP_DIRECT16(kt, true, false)
        ++kt;
    }
    CPH_K_STEP_DIRECT16(kt, false, false)
    // The last matrix instructions above must have written their accumulators before anything reads them, and the
    // compiler does not know that they are matrix instructions: wait out their latency here, and pass every
    // accumulator through an (empty) volatile statement, which the compiler keeps behind that wait and ahead of
    // every later use of the accumulator.
    if (Cfg::AKM || Cfg::BKM) {
        asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) asm volatile("" : "+a"(acc[i][j]));
    }
#undef CPH_K_STEP_DIRECT16
#undef CPH_PHASE16
#undef CPH_PIN
}

// Generic kernel: main loop + epilogue functor.  Epi::run receives the accumulators of one wavefront
// together with the global row/column of its sub-tile's origin.
// One workgroup per output tile.  (A persistent variant, one workgroup per compute unit walking a fixed share
// of the tiles, was measured twice: it is no faster in isolation and slower inside the step, where a freshly
// dispatched workgroup goes to whichever compute unit is free first.)
// An epilogue that needs per-row values from global memory fetches them for the whole tile with one coalesced load
// at its start and parks them in LDS.  (Loaded where they are used they are a chain of exposed cache misses per
// tile while the matrix cores idle; requested before the main loop they cost the main loop 9 %: the registers
// they occupy across it change its schedule.)
// A side job rides along in the same launch: its `blocks` workgroups (a multiple of 8, so that the tile walk's
// view of the XCDs stays aligned) come first in the grid, run `run(job, smem)` and leave; small work that the
// launch does not depend on saves a launch of its own that way.
struct NoSideJob {
    static constexpr bool kActive = false;
    int blocks;
    __device__ void run(int, char *) const {}
};
template <class Cfg, class Epi, class Side>
__global__ void __launch_bounds__(Cfg::THREADS) k_gemm_nt(GemmOperands g, Epi epi, Side side)
{
    __shared__ __attribute__((aligned(16))) char smem[Cfg::LDS_BYTES];
    int bid = blockIdx.x;
    if (Side::kActive) {
        if (bid < side.blocks) {
            side.run(bid, smem);
            return;
        }
        bid -= side.blocks;
    }
    int tm, tn;
    if (!tile_of_block(bid, g.tiles_m, g.tiles_n, g.gm, tm, tn)) return;
    f32x4_t acc[Cfg::TM16][Cfg::TN16];
    gemm_nt_mainloop_direct<Cfg>(g, tm, tn, smem, acc);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row0 = tm * Cfg::BM + (wave / Cfg::WN) * Cfg::WTM;
    const int col0 = tn * Cfg::BN + (wave % Cfg::WN) * Cfg::WTN;
    epi.template run<Cfg>(acc, row0, col0, lane, wave, tn, smem);
}

template <class Cfg, class Epi, class Side = NoSideJob>
inline void launch_gemm_nt(const char *name, const bf16_t *A, long lda, int M, const bf16_t *B, long ldb, int N, int K,
                           const Epi &epi, hipStream_t st, int gm = kGroupRowsWide, const Side &side = Side{0},
                           int ka_rows = -1, int kb_rows = -1)
{
    ProfileScope prof(name, 2.0 * (double)M * (double)N * (double)K, st);
    GemmOperands g;
    g.A = A; g.B = B; g.lda = lda; g.ldb = ldb; g.M = M; g.N = N; g.K = K;
    g.ka_rows = ka_rows < 0 ? K : ka_rows; g.kb_rows = kb_rows < 0 ? K : kb_rows;
    g.tiles_m = (M + Cfg::BM - 1) / Cfg::BM;
    g.tiles_n = (N + Cfg::BN - 1) / Cfg::BN;
    g.gm = gm;
    const int extra = Side::kActive ? side.blocks : 0;
    k_gemm_nt<Cfg, Epi, Side><<<gemm_grid(g.tiles_m, g.tiles_n, g.gm) + extra, Cfg::THREADS, 0, st>>>(g, epi, side);
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
// elements of 16-column blocks, so values are first laid out row-major in a wave-private
// LDS area (32 rows at a time, the operand stages are free by then) and then written with
// 16-byte stores: a wavefront store covers whole 256-byte row segments.
// `value(i, j, v, row, col)` yields the output for accumulator element v of the 16x16 block (i, j), whose
// global coordinates are (row, col).  All loops are fully unrolled so that the accumulators are
// only ever indexed with constants and stay in registers.
// ---------------------------------------------------------------------------------------------

// row / column of accumulator element v of block (i, j) for lane l, relative to the sub-tile origin
__device__ __forceinline__ int acc_row(int i, int v, int lane) { return i * 16 + 4 * (lane >> 4) + v; }
__device__ __forceinline__ int acc_col(int j, int lane) { return j * 16 + (lane & 15); }

// P0, P1 restrict the call to the 32-row passes P0 .. P1-1 (default: all of them).  blocked: dst is stored block by
// block (blocked64_index) instead of row-major.
template <class Cfg, class F, int P0 = 0, int P1 = Cfg::WTM / 32>
__device__ __forceinline__ void store_tile_bf16(char *smem, int wave, int lane, int row0, int col0, int row_limit,
                                                int col_limit /* multiple of 8 */, bf16_t *__restrict__ dst, long ld,
                                                F value, bool blocked = false)
{
    constexpr int RS = Cfg::WTN * 2 + 16;              // padded row stride in bytes
    constexpr int CPR = Cfg::WTN / 8;                   // 16-byte chunks per row
    constexpr int RPP = kWave / CPR;                    // rows per store pass
    static_assert(Cfg::WM * Cfg::WN * 32 * RS <= Cfg::LDS_BYTES, "staging fits");
    char *stage = smem + wave * (32 * RS);
    // a lane's first output address; every later one is a compile-time multiple of the (uniform) row stride away,
    // which keeps 64-bit multiplies per store out of the vector unit
    // (blocked: the rows of one call lie in one block of 256 and an 8-column piece in one block of 64 columns)
    static_assert(Cfg::WTM <= 256 && 256 % Cfg::WTM == 0, "a wavefront's rows stay inside a block of 256");
    const size_t first_row = (size_t)(row0 + P0 * 32 + lane / CPR);
    const int first_col = col0 + (lane % CPR) * 8;
    bf16_t *out = dst + (blocked ? blocked64_index(first_row, first_col, ld) : first_row * ld + first_col);
    const size_t step = blocked ? (size_t)RPP * 64 : (size_t)RPP * ld;
    __syncthreads();                                    // every wavefront is done reading operand tiles
#pragma unroll
    for (int p = P0; p < P1; ++p) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii) {
            const int i = 2 * p + ii;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int r = 16 * ii + 4 * (lane >> 4) + v;
#pragma unroll
                for (int j = 0; j < Cfg::TN16; ++j) {
                    const int c = j * 16 + (lane & 15);
                    *reinterpret_cast<bf16_t *>(stage + r * RS + c * 2) = value(i, j, v, row0 + p * 32 + r, col0 + c);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 32 / RPP; ++q) {
            const int r = q * RPP + lane / CPR, ch = lane % CPR;
            const u32x4_t val = *reinterpret_cast<const u32x4_t *>(stage + r * RS + ch * 16);
            const int grow = row0 + p * 32 + r, gcol = col0 + ch * 8;
            if (grow < row_limit && gcol < col_limit)
                *reinterpret_cast<u32x4_t *>(out) = val;
            out += step;
        }
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);              // conversions of the next pass stay behind this one's stores
    }
}

// Two bf16 outputs of the same shape from one pass over the accumulators: pair(i, j, v) yields both values
// (first in the low half); one set of barriers and one staging round serve both.
template <class Cfg, class F>
__device__ __forceinline__ void store_tile_bf16_pair(char *smem, int wave, int lane, int row0, int col0, int row_limit,
                                                     int col_limit /* multiple of 8 */, bf16_t *__restrict__ dst0,
                                                     bf16_t *__restrict__ dst1, long ld, F pair)
{
    constexpr int RS = Cfg::WTN * 2 + 16;
    constexpr int CPR = Cfg::WTN / 8;
    constexpr int RPP = kWave / CPR;
    constexpr int REGION = Cfg::WM * Cfg::WN * 32 * RS;  // staging of one output
    static_assert(2 * REGION <= Cfg::LDS_BYTES, "staging fits");
    char *stage = smem + wave * (32 * RS);
    size_t off = (size_t)(row0 + lane / CPR) * ld + (col0 + (lane % CPR) * 8);            // as in store_tile_bf16
    const size_t step = (size_t)RPP * ld;
    __syncthreads();
#pragma unroll
    for (int p = 0; p < Cfg::WTM / 32; ++p) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii) {
            const int i = 2 * p + ii;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int r = 16 * ii + 4 * (lane >> 4) + v;
#pragma unroll
                for (int j = 0; j < Cfg::TN16; ++j) {
                    const int c = j * 16 + (lane & 15);
                    const uint32_t both = pair(i, j, v);
                    *reinterpret_cast<bf16_t *>(stage + r * RS + c * 2) = (bf16_t)(both & 0xFFFFu);
                    *reinterpret_cast<bf16_t *>(stage + REGION + r * RS + c * 2) = (bf16_t)(both >> 16);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 32 / RPP; ++q) {
            const int r = q * RPP + lane / CPR, ch = lane % CPR;
            const u32x4_t v0 = *reinterpret_cast<const u32x4_t *>(stage + r * RS + ch * 16);
            const u32x4_t v1 = *reinterpret_cast<const u32x4_t *>(stage + REGION + r * RS + ch * 16);
            const int grow = row0 + p * 32 + r, gcol = col0 + ch * 8;
            if (grow < row_limit && gcol < col_limit) {
                *reinterpret_cast<u32x4_t *>(dst0 + off) = v0;
                *reinterpret_cast<u32x4_t *>(dst1 + off) = v1;
            }
            off += step;
        }
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Transposed bf16 output: dst[col * ld + row] = value(i, j, v, row, col).  A lane owns four consecutive
// rows of one column per accumulator block, so the sub-tile is laid out column-major in LDS (64 rows at
// a time, 8-byte writes) and leaves as 16-byte pieces of 128-byte column segments.
// row_limit and ld are multiples of 8; rows are written up to row_limit, columns up to col_limit.
// IP0, IP1 restrict the call to the 64-row passes IP0 .. IP1-1 (default: all of them).
template <class Cfg, class F, int IP0 = 0, int IP1 = Cfg::WTM / 64>
__device__ __forceinline__ void store_tile_bf16_transposed(char *smem, int wave, int lane, int row0, int col0,
                                                           int row_limit, int col_limit, bf16_t *__restrict__ dst,
                                                           long ld, F value)
{
    static_assert(Cfg::WTM % 64 == 0, "four 16-row blocks per pass");
    constexpr int CS = 64 * 2 + 16;                     // padded column stride in bytes (64 rows)
    static_assert(Cfg::WM * Cfg::WN * Cfg::WTN * CS <= Cfg::LDS_BYTES, "staging fits");
    char *stage = smem + wave * (Cfg::WTN * CS);
    bf16_t *const out0 = dst + (size_t)(col0 + (lane >> 3)) * ld + (row0 + (lane & 7) * 8);         // as in store_tile_bf16
    const size_t step = (size_t)8 * ld;
    __syncthreads();
#pragma unroll
    for (int ip = IP0; ip < IP1; ++ip) {
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) {
            const int i = ip * 4 + ii;
            const int r = 16 * ii + 4 * (lane >> 4);                 // first of four consecutive rows
#pragma unroll
            for (int j = 0; j < Cfg::TN16; ++j) {
                const int c = j * 16 + (lane & 15);
                unsigned lo, hi;
                {
                    const bf16_t a = value(i, j, 0, row0 + ip * 64 + r + 0, col0 + c);
                    const bf16_t b = value(i, j, 1, row0 + ip * 64 + r + 1, col0 + c);
                    lo = (unsigned)a | ((unsigned)b << 16);
                }
                {
                    const bf16_t a = value(i, j, 2, row0 + ip * 64 + r + 2, col0 + c);
                    const bf16_t b = value(i, j, 3, row0 + ip * 64 + r + 3, col0 + c);
                    hi = (unsigned)a | ((unsigned)b << 16);
                }
                typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
                u32x2_t pk = {lo, hi};
                *reinterpret_cast<u32x2_t *>(stage + c * CS + r * 2) = pk;
            }
        }
        __syncthreads();
        bf16_t *out = out0 + ip * 64;
#pragma unroll
        for (int p = 0; p < Cfg::WTN / 8; ++p) {
            const int c = p * 8 + (lane >> 3), ch = lane & 7;
            const u32x4_t val = *reinterpret_cast<const u32x4_t *>(stage + c * CS + ch * 16);
            const int grow = row0 + ip * 64 + ch * 8, gcol = col0 + c;
            if (grow < row_limit && gcol < col_limit)
                *reinterpret_cast<u32x4_t *>(out) = val;
            out += step;
        }
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
    }
}

// fp32 variant: dst = value, or dst += value when `accumulate` is set (16-byte loads and stores).
template <class Cfg, class F>
__device__ __forceinline__ void store_tile_f32(char *smem, int wave, int lane, int row0, int col0, int row_limit,
                                               int col_limit /* multiple of 4 */, float *__restrict__ dst, long ld,
                                               bool accumulate, F value)
{
    constexpr int RS = Cfg::WTN * 4 + 16;
    constexpr int CPR = Cfg::WTN / 4;
    constexpr int RPP = kWave / CPR;
    static_assert(Cfg::WM * Cfg::WN * 32 * RS <= Cfg::LDS_BYTES, "staging fits");
    char *stage = smem + wave * (32 * RS);
    float *out = dst + (size_t)(row0 + lane / CPR) * ld + (col0 + (lane % CPR) * 4);          // as in store_tile_bf16
    const size_t step = (size_t)RPP * ld;
    __syncthreads();
#pragma unroll
    for (int p = 0; p < Cfg::WTM / 32; ++p) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii) {
            const int i = 2 * p + ii;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int r = 16 * ii + 4 * (lane >> 4) + v;
#pragma unroll
                for (int j = 0; j < Cfg::TN16; ++j) {
                    const int c = j * 16 + (lane & 15);
                    *reinterpret_cast<float *>(stage + r * RS + c * 4) = value(i, j, v, row0 + p * 32 + r, col0 + c);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 32 / RPP; ++q) {
            const int r = q * RPP + lane / CPR, ch = lane % CPR;
            f32x4_t val = *reinterpret_cast<const f32x4_t *>(stage + r * RS + ch * 16);
            const int grow = row0 + p * 32 + r, gcol = col0 + ch * 4;
            if (grow < row_limit && gcol < col_limit) {
                f32x4_t *o = reinterpret_cast<f32x4_t *>(out);
                if (accumulate) val += *o;
                *o = val;
            }
            out += step;
        }
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
    }
}

}  // namespace cph

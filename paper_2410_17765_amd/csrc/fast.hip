// Matrix-core path of the CP head loss (bf16 storage, d a multiple of 64).
//
// Forward:   gate -> Y = H W^T (hi/lo bf16) -> z = Y U^T with a running-statistics epilogue
//            (logits never stored) -> per-row log-normaliser and fp32 target logit -> mixture.
// Backward:  per bounded chunk of head rows: recompute z, epilogue writes dz in bf16 ->
//            dY = dz U and dU += dz^T Y; then dW = dY^T H, dH = dY W + G^T dg, dG = dg^T H.
// With CP_HEAD_KEEP_LOGITS the forward epilogue also keeps the logits as 16-bit floats and the backward
// pass reads them back instead of recomputing z (kept_logits.hpp).
// All products run through the one NT main loop of gemm_nt.hpp; operands that are not
// K-contiguous are transposed first (HBM-bound passes that cost a few percent of the GEMM time).
#include "gemm_nt.hpp"
#include "kept_logits.hpp"

#include <math.h>

namespace cph {

namespace {

typedef TileCfg<256, 256, 2, 2> Cfg;
// the same tile with the second, or both, operands K-major (the contraction index is their slow one)
typedef TileCfg<256, 256, 2, 2, false, true> CfgNN;
typedef TileCfg<256, 256, 2, 2, true, true> CfgTN;
// A stored in blocks of 256 rows x 64 columns (the chunk's logit gradients as the dY product reads them)
typedef TileCfg<256, 256, 2, 2, false, false, true, false> CfgBlockedA;
constexpr int kBlock = 256;


// ------------------------------------------------------------------------------------------
// epilogues
// ------------------------------------------------------------------------------------------

// bf16 store of the accumulators; optionally also the bf16 residual acc - bf16(acc), so that
// hi + lo carries the fp32 value to about 2^-17 relative.  N and ldc are multiples of 8.
struct EpiStoreBf16 {
    bf16_t *hi;
    bf16_t *lo;     // may be null
    long ldc;
    int M, N;
    template <class C>
    __device__ void run(f32x4_t (&acc)[C::TM16][C::TN16], int row0, int col0, int lane, int wave, int, char *smem) const
    {
        if (lo)
            store_tile_bf16_pair<C>(smem, wave, lane, row0, col0, M, N, hi, lo, ldc, [&](int i, int j, int v) {
                const float a = acc[i][j][v];
                const bf16_t h = f32_to_bf16(a);
                return (uint32_t)h | ((uint32_t)f32_to_bf16(a - bf16_to_f32(h)) << 16);
            });
        else
            store_tile_bf16<C>(smem, wave, lane, row0, col0, M, N, hi, ldc,
                               [&](int i, int j, int v, int, int) { return f32_to_bf16(acc[i][j][v]); });
    }
};

// fp32 store, optionally accumulating onto what is already there (chunked sums).  N, ldc multiples of 4.
struct EpiStoreF32 {
    float *C;
    long ldc;
    int M, N;
    int accumulate;
    template <class Cf>
    __device__ void run(f32x4_t (&acc)[Cf::TM16][Cf::TN16], int row0, int col0, int lane, int wave, int, char *smem) const
    {
        store_tile_f32<Cf>(smem, wave, lane, row0, col0, M, N, C, ldc, accumulate != 0,
                           [&](int i, int j, int v, int, int) { return acc[i][j][v]; });
    }
};

// The logits of the columns past the vocabulary (only the last tile column has any) are set to -inf once, so that
// the statistics below need no per-element test: -inf never wins a maximum and its exponential is zero (a row with no
// valid column keeps the maximum -inf and the reference 0, as before).  Uniform for the wavefront.
template <class C>
__device__ __forceinline__ void mask_columns_past_vocabulary(f32x4_t (&acc)[C::TM16][C::TN16], int col0, int lane, int V)
{
    if (col0 + C::WTN <= V) return;
#pragma unroll
    for (int j = 0; j < C::TN16; ++j)
        if (col0 + acc_col(j, lane) >= V) {
#pragma unroll
            for (int i = 0; i < C::TM16; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[i][j][v] = -INFINITY;
        }
}

// Running statistics of the logits (eq. 5 in log space): for every row of the wavefront's
// sub-tile the maximum and the sum of exp(z - max) over its columns.  One (max, sum) pair per
// row and per (tile column, wavefront column) goes to `part`; the logits themselves are dropped.
// A row of the sub-tile lives in one 16-lane group (its column blocks in the lane's registers), so a
// wavefront reduces four rows at a time with moves inside 16 lanes; the group's first lane writes the pair.
struct EpiRowStats {
    float2 *part;   // [M, parts]
    int parts;      // tiles_n * WN
    int M, V;
    template <class C>
    __device__ void run(f32x4_t (&acc)[C::TM16][C::TN16], int row0, int col0, int lane, int wave, int tn, char *) const
    {
        const int slot = tn * C::WN + (wave % C::WN);
        mask_columns_past_vocabulary<C>(acc, col0, lane, V);
#pragma unroll
        for (int i = 0; i < C::TM16; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float mx = -INFINITY;
#pragma unroll
                for (int j = 0; j < C::TN16; ++j) mx = fmaxf(mx, acc[i][j][v]);
                mx = row16_max(mx);
                const float ref = (mx == -INFINITY) ? 0.f : mx;
                float s = 0.f;
#pragma unroll
                for (int j = 0; j < C::TN16; ++j) s += __expf(acc[i][j][v] - ref);
                s = row16_sum(s);
                const int r = row0 + acc_row(i, v, lane);
                if ((lane & 15) == 0 && r < M)
                    part[(size_t)r * parts + slot] = make_float2(mx, (mx == -INFINITY) ? 0.f : s);
            }
    }
};

// The statistics of EpiRowStats, and the logits kept for the backward pass: zs[m, v] = fp16(z - ref) with ref
// the maximum of row m over the wavefront's 128 columns (the pair that goes to `part`).  Relative to that
// maximum the large probabilities of a row, which carry its gradient, sit near zero where fp16 resolves
// 2^-11 or better; a logit 16 below the maximum is kept to 2^-7, i.e. its probability to under one percent.
struct EpiRowStatsKeep {
    float2 *part;   // [M, parts]
    int parts;
    int M, V;
    uint16_t *zs;   // [M, ldzs]
    long ldzs;
    int Vp;         // columns of zs that are written (V rounded up to 64; those from V on hold junk)
    template <class C, int P>
    __device__ __forceinline__ void pass(f32x4_t (&acc)[C::TM16][C::TN16], int row0, int col0, int lane, int wave,
                                         int slot, char *smem) const
    {
#pragma unroll
        for (int i = 2 * P; i < 2 * P + 2; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float mx = -INFINITY;
#pragma unroll
                for (int j = 0; j < C::TN16; ++j) mx = fmaxf(mx, acc[i][j][v]);
                mx = row16_max(mx);
                const float ref = (mx == -INFINITY) ? 0.f : mx;
                float s = 0.f;
#pragma unroll
                for (int j = 0; j < C::TN16; ++j) {
                    acc[i][j][v] -= ref;
                    s += __expf(acc[i][j][v]);
                }
                s = row16_sum(s);
                const int r = row0 + acc_row(i, v, lane);
                if ((lane & 15) == 0 && r < M)
                    part[(size_t)r * parts + slot] = make_float2(mx, (mx == -INFINITY) ? 0.f : s);
            }
        auto half = [&](int i, int j, int v, int, int) { return f32_to_f16_bits(acc[i][j][v]); };
        store_tile_bf16<C, decltype(half), P, P + 1>(smem, wave, lane, row0, col0, M, Vp, zs, ldzs, half);
    }
    template <class C>
    __device__ void run(f32x4_t (&acc)[C::TM16][C::TN16], int row0, int col0, int lane, int wave, int tn, char *smem) const
    {
        static_assert(C::WTM == 128 && C::WTN == 128, "blocks of 128 columns, four passes of 32 rows");
        const int slot = tn * C::WN + (wave % C::WN);
        mask_columns_past_vocabulary<C>(acc, col0, lane, V);
        pass<C, 0>(acc, row0, col0, lane, wave, slot, smem);
        pass<C, 1>(acc, row0, col0, lane, wave, slot, smem);
        pass<C, 2>(acc, row0, col0, lane, wave, slot, smem);
        pass<C, 3>(acc, row0, col0, lane, wave, slot, smem);
    }
};

// Softmax gradient (derivative of eq. 8/9 with respect to the logits), written in bf16:
//   dz[m, v] = coef[m] * (exp(z - lse[m]) - 1[v = x_m]),  zero in the padding columns V..Vp-1;
// optionally also transposed (dzT[v, m], rows of the chunk padded with zeros up to Mcp), which is the
// operand layout of the dU product.
struct EpiDz {
    bf16_t *dZ;          // [Mc, Vp] for the chunk
    long ldz;
    bf16_t *dZt;         // [V, Mcp] or null
    long ldzt;
    const float4 *rowinfo;   // chunk-relative: {lse, coef (zero for dropped factors), target as int bits, -}
    int Mc, Mcp, V, Vp;
    int blocked;             // dZ is stored block by block (blocked64_index)
    template <class C>
    __device__ void run(f32x4_t (&acc)[C::TM16][C::TN16], int row0, int col0, int lane, int wave, int, char *smem) const
    {
        static_assert(C::WTM == 64 || C::WTM == 128, "sub-tiles of 64 or 128 rows");
        static_assert(C::WM * C::WN * C::WTN * (64 * 2 + 16) <= C::LDS_BYTES - C::BM * 16, "row values beyond the staging areas");
        // The row values of the tile's BM rows come in with one coalesced load, one row per thread, and are parked
        // in the last BM * 16 bytes of the LDS buffer, beyond every staging area of the stores below: loaded where
        // they are used, they were a chain of sixteen exposed cache misses per tile.
        static_assert(C::THREADS >= C::BM, "one row per thread");
        float4 *linfo = reinterpret_cast<float4 *>(smem + C::LDS_BYTES - C::BM * 16);
        const int trow = row0 - (wave / C::WN) * C::WTM + (int)threadIdx.x;       // this thread's row of the tile
        const float4 mine = rowinfo[trow < Mc ? trow : Mc - 1];
        __syncthreads();                                    // every wavefront is done reading operand tiles
        if ((int)threadIdx.x < C::BM) linfo[threadIdx.x] = mine;
        __syncthreads();
        const float4 *winfo = linfo + (wave / C::WN) * C::WTM;     // the rows of this wavefront's sub-tile
        // after convert() the even accumulator of a pair of rows holds both gradients as two bf16
        auto dz = [&](int i, int j, int v, int, int) {
            const uint32_t pk = __float_as_uint(acc[i][j][v & ~1]);
            return (bf16_t)((v & 1) ? (pk >> 16) : (pk & 0xFFFFu));
        };
        // 64 rows at a time: turn their logits into gradients in place and write them out at once, so that
        // the finished values do not stay in registers
        convert<C, 0>(acc, row0, col0, lane, winfo);
        store_tile_bf16<C, decltype(dz), 0, 2>(smem, wave, lane, row0, col0, Mc, Vp, dZ, ldz, dz, blocked != 0);
        if (dZt) store_tile_bf16_transposed<C, decltype(dz), 0, 1>(smem, wave, lane, row0, col0, Mcp, V, dZt, ldzt, dz);
        if (C::WTM > 64) {
            convert<C, 1>(acc, row0, col0, lane, winfo);
            store_tile_bf16<C, decltype(dz), 2, 4>(smem, wave, lane, row0, col0, Mc, Vp, dZ, ldz, dz, blocked != 0);
            if (dZt) store_tile_bf16_transposed<C, decltype(dz), 1, 2>(smem, wave, lane, row0, col0, Mcp, V, dZt, ldzt, dz);
        }
    }

    // Logits -> gradients for the 16-row blocks 4 IP .. 4 IP + 3, two consecutive rows at a time; the pair
    // is rounded to bf16 by one conversion and kept in the even row's accumulator.  The one-hot term touches
    // one element of a row, so it is a branch that a wavefront takes only where a target falls into its
    // columns.
    template <class C, int IP>
    __device__ __forceinline__ void convert(f32x4_t (&acc)[C::TM16][C::TN16], int row0, int col0, int lane,
                                            const float4 *winfo) const
    {
        const int lcol = col0 + (lane & 15);
        const bool ragged = col0 + 16 * C::TN16 > V;     // the same for the whole wavefront
#pragma unroll
        for (int i = 4 * IP; i < 4 * IP + 4; ++i) {
#pragma unroll
            for (int v = 0; v < 4; v += 2) {
                const int lrow = acc_row(i, v, lane);                // rows lrow and lrow + 1 of the sub-tile
                const int row = row0 + lrow;
                const float4 ra = winfo[lrow];                       // rows past the chunk hold the last row's values
                const float4 rb = winfo[lrow + 1];
                // rows past the chunk hold zero logits: coefficient 0 and offset 0 keep their product finite
                const float cfa = row < Mc ? ra.y : 0.f, cfb = row + 1 < Mc ? rb.y : 0.f;
                const float la = row < Mc ? ra.x : 0.f, lb = row + 1 < Mc ? rb.x : 0.f;
                float ga[C::TN16], gb[C::TN16];
#pragma unroll
                for (int j = 0; j < C::TN16; ++j) {
                    // z - lse first: exact where the logit is close to the log-normaliser (p close to 1)
                    ga[j] = cfa * __builtin_amdgcn_exp2f((acc[i][j][v] - la) * kLog2e);
                    gb[j] = cfb * __builtin_amdgcn_exp2f((acc[i][j][v + 1] - lb) * kLog2e);
                }
                const int xa = __float_as_int(ra.z) - lcol, xb = __float_as_int(rb.z) - lcol;   // 16 j at the target
                const bool ha = (xa & 15) == 0 && (unsigned)xa < 16u * C::TN16;
                const bool hb = (xb & 15) == 0 && (unsigned)xb < 16u * C::TN16;
                if (ha || hb) {
#pragma unroll
                    for (int j = 0; j < C::TN16; ++j) {
                        if (ha && xa == 16 * j) ga[j] -= cfa;
                        if (hb && xb == 16 * j) gb[j] -= cfb;
                    }
                }
                if (ragged) {
#pragma unroll
                    for (int j = 0; j < C::TN16; ++j)
                        if (lcol + 16 * j >= V) { ga[j] = 0.f; gb[j] = 0.f; }
                }
#pragma unroll
                for (int j = 0; j < C::TN16; ++j) acc[i][j][v] = __uint_as_float(f32x2_to_bf16x2(ga[j], gb[j]));
            }
            // keeps the per-row loads of the next block from being hoisted (they would spill registers)
            asm volatile("" ::: "memory");
        }
    }
};

// ------------------------------------------------------------------------------------------
// logit gradients from kept logits
// ------------------------------------------------------------------------------------------

// The gradient of EpiDz from the logits that EpiRowStatsKeep left behind instead of from a second product:
//   dz[m, v] = coef[m] * (exp(log P[m, v]) - 1[v = x_m]),  rowinfo as for EpiDz.
struct LossDzRule {
    static constexpr int RT = 2;
    __device__ __forceinline__ void operator()(int, int nrows, int col, int V, const float4 (&info)[2],
                                               const float (&lp)[2][8], float (&g)[2][8]) const
    {
#pragma unroll
        for (int h = 0; h < 2; ++h)
            if (h < nrows) {
                const float cf = info[h].y;
                const int x = __float_as_int(info[h].z) - col;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    float v = cf * __builtin_amdgcn_exp2f(lp[h][k] * kLog2e);
                    if (x == k) v -= cf;
                    g[h][k] = (col + k < V) ? v : 0.f;
                }
            }
    }
};

// ------------------------------------------------------------------------------------------
// small kernels around the GEMMs
// ------------------------------------------------------------------------------------------

// dst[c, r] = src[r, c] (bf16); dst rows are ldd long and columns R..Rp-1 are zero-filled.
__global__ void __launch_bounds__(kBlock) k_transpose_bf16(const bf16_t *__restrict__ src, long lds_, int R, int C,
                                                           bf16_t *__restrict__ dst, long ldd, int Rp, int tiles_c)
{
    __shared__ bf16_t tile[64][66];
    const int tc = blockIdx.x % tiles_c, tr = blockIdx.x / tiles_c;
    const int r0 = tr * 64, c0 = tc * 64;
    const int lx = threadIdx.x & 63, ly = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int r = r0 + i * 4 + ly, c = c0 + lx;
        tile[i * 4 + ly][lx] = (r < R && c < C) ? src[(size_t)r * lds_ + c] : (bf16_t)0;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int c = c0 + i * 4 + ly, r = r0 + lx;
        if (c < C && r < Rp) dst[(size_t)c * ldd + r] = tile[lx][i * 4 + ly];
    }
}

// The same with 16-byte accesses on both sides, for C a multiple of 64 and lds_, ldd, Rp multiples of 8 (and
// 16-byte aligned bases): a thread loads eight columns of a row at once, the tile crosses LDS, and a thread
// gathers eight rows of one column for a 16-byte store; a wavefront store covers 8 output rows x 128 bytes.
__global__ void __launch_bounds__(kBlock) k_transpose_bf16_wide(const bf16_t *__restrict__ src, long lds_, int R,
                                                                bf16_t *__restrict__ dst, long ldd, int Rp, int tiles_c)
{
    __shared__ uint32_t tile[64][33];                   // 64 rows x 64 bf16, one dword of padding per row
    const int tc = blockIdx.x % tiles_c, tr = blockIdx.x / tiles_c;
    const int r0 = tr * 64, c0 = tc * 64;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int id = threadIdx.x + kBlock * p, row = id >> 3, ch = id & 7;
        const int r = r0 + row;
        u32x4_t v = {0u, 0u, 0u, 0u};
        if (r < R) v = *reinterpret_cast<const u32x4_t *>(src + (size_t)r * lds_ + c0 + ch * 8);
#pragma unroll
        for (int w = 0; w < 4; ++w) tile[row][ch * 4 + w] = v[w];
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int id = threadIdx.x + kBlock * p, col = id >> 3, rg = id & 7;     // source column, group of 8 rows
        const int shift = (col & 1) * 16;
        u32x4_t v;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const uint32_t a = (tile[rg * 8 + 2 * w][col >> 1] >> shift) & 0xFFFFu;
            const uint32_t b = (tile[rg * 8 + 2 * w + 1][col >> 1] >> shift) & 0xFFFFu;
            v[w] = a | (b << 16);
        }
        const int r = r0 + rg * 8;
        if (r < Rp) *reinterpret_cast<u32x4_t *>(dst + (size_t)(c0 + col) * ldd + r) = v;
    }
}

void transpose_bf16(const bf16_t *src, long lds_, int R, int C, bf16_t *dst, long ldd, int Rp, hipStream_t st)
{
    ProfileScope prof("transpose", 2.0 * ((double)R * C + (double)Rp * C), st);   // work = bytes moved
    const int tiles_c = (C + 63) / 64, tiles_r = (Rp + 63) / 64;
    const bool wide = C % 64 == 0 && lds_ % 8 == 0 && ldd % 8 == 0 && Rp % 8 == 0 &&
                      (reinterpret_cast<uintptr_t>(src) & 15u) == 0 && (reinterpret_cast<uintptr_t>(dst) & 15u) == 0;
    if (wide)
        k_transpose_bf16_wide<<<(unsigned)((size_t)tiles_c * tiles_r), kBlock, 0, st>>>(src, lds_, R, dst, ldd, Rp, tiles_c);
    else
        k_transpose_bf16<<<(unsigned)((size_t)tiles_c * tiles_r), kBlock, 0, st>>>(src, lds_, R, C, dst, ldd, Rp, tiles_c);
}

// Per head row: combine the per-tile statistics into the log-normaliser (eq. 5), take the
// target logit as an fp32 dot product of U[x] with y = hi (+ lo), and form C = z[x] - lse (eq. 8).
// One wavefront per row.  part == NULL: the log-normaliser is read from lse_io instead of being
// computed.  X == NULL: only the log-normaliser is produced.  Ylo == NULL: y = hi.
__global__ void __launch_bounds__(kBlock) k_row_finish(size_t M, int d, int r, int parts,
                                                       const float2 *__restrict__ part,
                                                       const bf16_t *__restrict__ Yhi, const bf16_t *__restrict__ Ylo,
                                                       const bf16_t *__restrict__ U, const int32_t *__restrict__ X,
                                                       float *__restrict__ lse_io, float *__restrict__ C_out)
{
    const size_t m = (size_t)blockIdx.x * (kBlock / kWave) + (threadIdx.x >> 6);
    if (m >= M) return;
    const int lane = threadIdx.x & 63;
    float lse;
    if (part) {
        float mx = -INFINITY, l = 0.f;
        for (int p = lane; p < parts; p += kWave) {
            const float2 q = part[m * parts + p];
            if (q.x > mx) { l = l * __expf(mx - q.x) + q.y; mx = q.x; }
            else if (q.x != -INFINITY) l += q.y * __expf(q.x - mx);
        }
        const float Mx = wave_max(mx);
        const float L = wave_sum(mx == -INFINITY ? 0.f : l * __expf(mx - Mx));
        lse = Mx + logf(L);
        if (lane == 0) lse_io[m] = lse;
    } else {
        lse = lse_io[m];
    }
    if (!X) return;
    const int x = X[m / r];
    float zt = 0.f;
    if (x >= 0) {
        const bf16_t *u = U + (size_t)x * d, *yh = Yhi + m * d;
        if (Ylo) {
            const bf16_t *yl = Ylo + m * d;
            for (int k = lane; k < d; k += kWave)
                zt += bf16_to_f32(u[k]) * (bf16_to_f32(yh[k]) + bf16_to_f32(yl[k]));
        } else {
            for (int k = lane; k < d; k += kWave) zt += bf16_to_f32(u[k]) * bf16_to_f32(yh[k]);
        }
        zt = wave_sum(zt);
    }
    if (lane == 0) C_out[m] = (x >= 0) ? zt - lse : 0.f;
}

// ------------------------------------------------------------------------------------------
// draft step ("Sampling method"): small kernels around the two streaming GEMMs
// ------------------------------------------------------------------------------------------

__device__ __forceinline__ double wave_scan_inclusive(double v, int lane)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const double o = __shfl_up(v, off, kWave);
        if (lane >= off) v += o;
    }
    return v;
}

// fp32 dot product of two bf16 vectors of length d (a multiple of 64) over one wavefront, 16-byte loads
__device__ __forceinline__ float wave_dot_bf16(const bf16_t *__restrict__ a, const bf16_t *__restrict__ b, int d, int lane)
{
    const u32x4_t *pa = reinterpret_cast<const u32x4_t *>(a);
    const u32x4_t *pb = reinterpret_cast<const u32x4_t *>(b);
    float acc = 0.f;
    for (int k = lane; k < d / 8; k += kWave) {
        const u32x4_t x = pa[k], y = pb[k];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc += __uint_as_float(x[e] << 16) * __uint_as_float(y[e] << 16);
            acc += __uint_as_float(x[e] & 0xFFFF0000u) * __uint_as_float(y[e] & 0xFFFF0000u);
        }
    }
    return wave_sum(acc);
}

// gate (eq. 7) and the expert draw: log w = log_softmax(G h); a* = first a whose running sum of w
// (fp64) exceeds u, clamped to r-1.  One block per row of the batch, a wavefront per expert at a time.
// g_s: at least r floats of LDS.  uniforms = null: log w only.
constexpr int kWideBlock = 1024;
__device__ __forceinline__ void draft_gate_pick_row(size_t b, int nwaves, float *g_s, int d, int n, int r,
                                                    const bf16_t *__restrict__ H, const bf16_t *__restrict__ G,
                                                    const float *__restrict__ uniforms, float *__restrict__ logw,
                                                    int32_t *__restrict__ alpha)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int a = wave; a < r; a += nwaves) {
        const float p = wave_dot_bf16(G + (size_t)a * d, H + b * d, d, lane);
        if (lane == 0) g_s[a] = p;
    }
    __syncthreads();
    if (wave != 0) return;
    const float mine = lane < r ? g_s[lane] : -INFINITY;
    const float mx = wave_max(mine);
    const float s = wave_sum(lane < r ? expf(mine - mx) : 0.f);
    const float lse = mx + logf(s);
    const float w = lane < r ? expf(mine - lse) : 0.f;
    if (lane < r) logw[b * r + lane] = mine - lse;
    if (!uniforms) return;                      // log w only
    // inclusive running sum of w in expert order, fp64
    const double incl = wave_scan_inclusive((double)w, lane);
    const double u = (double)uniforms[b * (1 + n)];
    const unsigned long long crossed = __ballot(lane < r && incl > u);
    if (lane == 0) alpha[b] = crossed ? __ffsll((long long)crossed) - 1 : r - 1;
}
// It runs as a side job of the y product's launch (the two are independent: both read only H and weights), which
// saves the draft-type calls a launch: workgroup `job` of the first `blocks` (B rounded up to 8) takes row `job`.
struct GatePickSide {
    static constexpr bool kActive = true;
    int blocks;
    int B, d, n, r;
    const bf16_t *H, *G;
    const float *uniforms;
    float *logw;
    int32_t *alpha;
    __device__ void run(int job, char *smem) const
    {
        if (job >= B) return;
        draft_gate_pick_row((size_t)job, (int)(blockDim.x / kWave), reinterpret_cast<float *>(smem), d, n, r, H, G,
                            uniforms, logw, alpha);
    }
};

// Per (b, s): the log-normalisers of its r head rows from the per-segment statistics (eq. 5), then for
// the drawn expert's row the segment of the vocabulary in which the running sum of probabilities
// passes u: segment masses exp(max_j - lse) * sum_j accumulated in vocabulary order in fp64
// (lane-local runs, then a wavefront scan).  seg = -1 if the sum never passes u.
__global__ void __launch_bounds__(kWideBlock) k_draft_lse_segment(int n, int r, int parts, const float2 *__restrict__ part,
                                                              const int32_t *__restrict__ alpha,
                                                              const float *__restrict__ uniforms,
                                                              float *__restrict__ lse_out, int32_t *__restrict__ seg_out,
                                                              double *__restrict__ base_out)
{
    __shared__ float lse_s[64];
    const size_t bs = blockIdx.x;                 // b*n + s
    const size_t b = bs / n;
    const int s = (int)(bs % n);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int a = wave; a < r; a += kWideBlock / kWave) {
        const float2 *pm = part + (bs * r + a) * parts;
        float mx = -INFINITY, l = 0.f;
        for (int p = lane; p < parts; p += kWave) {
            const float2 q = pm[p];
            if (q.x > mx) { l = l * __expf(mx - q.x) + q.y; mx = q.x; }
            else if (q.x != -INFINITY) l += q.y * __expf(q.x - mx);
        }
        const float Mx = wave_max(mx);
        const float L = wave_sum(mx == -INFINITY ? 0.f : l * __expf(mx - Mx));
        const float lse = Mx + logf(L);
        if (lane == 0) { lse_out[bs * r + a] = lse; lse_s[a] = lse; }
    }
    __syncthreads();
    if (wave != 0) return;
    const int astar = alpha[b];
    const float l = lse_s[astar];
    const double u = (double)uniforms[b * (1 + n) + 1 + s];
    const float2 *pm = part + (bs * r + astar) * parts;
    const int per = (parts + kWave - 1) / kWave;  // consecutive segments per lane: lane order = vocabulary order
    const int lo = min(parts, lane * per), hi = min(parts, lo + per);
    double sum = 0.0;
    for (int j = lo; j < hi; ++j) {
        const float2 q = pm[j];
        sum += (q.x == -INFINITY) ? 0.0 : (double)(q.y * expf(q.x - l));
    }
    const double incl = wave_scan_inclusive(sum, lane);
    const unsigned long long crossed = __ballot(incl > u);
    if (crossed == 0ull) {
        if (lane == 0) { seg_out[bs] = -1; base_out[bs] = 0.0; }
        return;
    }
    const int first = __ffsll((long long)crossed) - 1;
    if (lane == first) {
        double c = incl - sum;
        int seg = hi - 1;
        for (int j = lo; j < hi; ++j) {
            const float2 q = pm[j];
            const double mj = (q.x == -INFINITY) ? 0.0 : (double)(q.y * expf(q.x - l));
            if (c + mj > u) { seg = j; break; }
            c += mj;
        }
        seg_out[bs] = seg;
        base_out[bs] = c;
    }
}

// Per (b, s): recompute the logits of the chosen segment (one wavefront per column, fp32 dot products
// of U rows with the bf16 y) and continue the scan token by token: first index whose running sum
// exceeds u; the last token of the segment if rounding between the two passes leaves none; V-1 if
// the running sum over the whole vocabulary never passed u.
constexpr int kPickBlock = 1024;
__global__ void __launch_bounds__(kPickBlock) k_draft_logits_pick(int d, int V, int n, int r, int seg_cols,
                                                                  const float *__restrict__ lse,
                                                                  const bf16_t *__restrict__ Y,
                                                                  const bf16_t *__restrict__ U,
                                                                  const int32_t *__restrict__ alpha,
                                                                  const int32_t *__restrict__ seg_in,
                                                                  const double *__restrict__ base_in,
                                                                  const float *__restrict__ uniforms,
                                                                  int32_t *__restrict__ tokens)
{
    __shared__ float p_s[256];
    const size_t bs = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int seg = seg_in[bs];
    if (seg < 0) {
        if (threadIdx.x == 0) tokens[bs] = V - 1;
        return;
    }
    const size_t m = bs * r + alpha[bs / n];
    const float l = lse[m];
    const int v0 = seg * seg_cols, cols = min(seg_cols, V - v0);
    // a wavefront owns up to four columns at a time and walks k for all of them together
    constexpr int NW = kPickBlock / kWave, CW = 4;
    const u32x4_t *yrow = reinterpret_cast<const u32x4_t *>(Y + m * d);
    for (int c0 = wave * CW; c0 < seg_cols; c0 += NW * CW) {
        float acc[CW] = {0.f, 0.f, 0.f, 0.f};
        const u32x4_t *urow[CW];
#pragma unroll
        for (int e = 0; e < CW; ++e)
            urow[e] = reinterpret_cast<const u32x4_t *>(U + (size_t)(v0 + min(c0 + e, cols - 1)) * d);
        for (int k = lane; k < d / 8; k += kWave) {
            const u32x4_t yv = yrow[k];
            u32x4_t uv[CW];
#pragma unroll
            for (int e = 0; e < CW; ++e) uv[e] = urow[e][k];
#pragma unroll
            for (int e = 0; e < CW; ++e)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc[e] += __uint_as_float(uv[e][q] << 16) * __uint_as_float(yv[q] << 16);
                    acc[e] += __uint_as_float(uv[e][q] & 0xFFFF0000u) * __uint_as_float(yv[q] & 0xFFFF0000u);
                }
        }
#pragma unroll
        for (int e = 0; e < CW; ++e) {
            const float z = wave_sum(acc[e]);
            if (lane == 0 && c0 + e < seg_cols) p_s[c0 + e] = (c0 + e < cols) ? expf(z - l) : 0.f;
        }
    }
    __syncthreads();
    if (wave != 0) return;
    const double u = (double)uniforms[(bs / n) * (1 + n) + 1 + (bs % n)];
    const int per = (seg_cols + kWave - 1) / kWave;
    const int lo = lane * per;
    double sum = 0.0;
    for (int i = lo; i < lo + per && i < cols; ++i) sum += (double)p_s[i];
    const double incl = base_in[bs] + wave_scan_inclusive(sum, lane);
    const unsigned long long crossed = __ballot(incl > u);
    if (crossed == 0ull) {
        if (lane == 0) tokens[bs] = v0 + cols - 1;
        return;
    }
    const int first = __ffsll((long long)crossed) - 1;
    if (lane == first) {
        double c = incl - sum;
        int tok = v0 + min(cols, lo + per) - 1;
        for (int i = lo; i < lo + per && i < cols; ++i) {
            c += (double)p_s[i];
            if (c > u) { tok = v0 + i; break; }
        }
        tokens[bs] = tok;
    }
}

// logq[b] = logsumexp_a( log w_a + sum_s (z_sa[tok_s] - lse_sa) ): eq. 9 at the drawn tuple over all experts
__global__ void __launch_bounds__(kWideBlock) k_draft_logq(int d, int n, int r, const float *__restrict__ logw,
                                                       const float *__restrict__ lse, const bf16_t *__restrict__ Y,
                                                       const bf16_t *__restrict__ U, const int32_t *__restrict__ tokens,
                                                       float *__restrict__ logq)
{
    __shared__ float C_s[64 * 64];
    const size_t b = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nr = n * r;
    for (int j = wave; j < nr; j += kWideBlock / kWave) {
        const size_t m = b * nr + j;
        const int tok = tokens[b * n + j / r];
        const float zt = wave_dot_bf16(U + (size_t)tok * d, Y + m * d, d, lane);
        if (lane == 0) C_s[j] = zt - lse[m];
    }
    __syncthreads();
    if (wave != 0) return;
    float a = -INFINITY;
    if (lane < r) {
        a = logw[b * r + lane];
        for (int s = 0; s < n; ++s) a += C_s[s * r + lane];
    }
    const float mx = wave_max(a);
    const float sum = wave_sum(lane < r ? expf(a - mx) : 0.f);
    if (lane == 0) logq[b] = mx + logf(sum);
}

// Log-normaliser (eq. 5) of one row from its per-segment statistics, by one wavefront.
__device__ __forceinline__ float row_lse_from_parts(const float2 *__restrict__ pm, int parts, int lane)
{
    // four independent loads per lane and step: the chain of rescalings is short, the loads overlap
    float mx = -INFINITY, l = 0.f;
    for (int p0 = 0; p0 < parts; p0 += 4 * kWave) {
        float2 qv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int p = p0 + i * kWave + lane;
            qv[i] = p < parts ? pm[p] : make_float2(-INFINITY, 0.f);
        }
        const float m4 = fmaxf(fmaxf(qv[0].x, qv[1].x), fmaxf(qv[2].x, qv[3].x));
        if (m4 == -INFINITY) continue;
        const float mn = fmaxf(mx, m4);
        float add = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) add += qv[i].y * __expf(qv[i].x - mn);     // exp(-inf) = 0 for empty segments
        l = l * __expf(mx - mn) + add;
        mx = mn;
    }
    const float Mx = wave_max(mx);
    const float L = wave_sum(mx == -INFINITY ? 0.f : l * __expf(mx - Mx));
    return Mx + logf(L);
}

__global__ void __launch_bounds__(kBlock) k_lse_from_parts(size_t rows, int parts, const float2 *__restrict__ part,
                                                           float *__restrict__ lse)
{
    const int lane = threadIdx.x & 63;
    const size_t row = (size_t)blockIdx.x * (kBlock / kWave) + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float v = row_lse_from_parts(part + row * parts, parts, lane);
    if (lane == 0) lse[row] = v;
}

// (max, sum of exp(z - max)) of one chunk of kStatCols columns of one row of stored fp32 logits
// (row stride ld, a multiple of 4): the per-segment statistics of eq. 5 for logits that are kept.
constexpr int kStatCols = 4096;
__global__ void __launch_bounds__(kBlock) k_row_stats_f32(int V, size_t ld, int parts, const float *__restrict__ z,
                                                          float2 *__restrict__ part)
{
    __shared__ float red_m[kBlock / kWave], red_l[kBlock / kWave];
    const size_t row = blockIdx.x;
    const int c0 = blockIdx.y * kStatCols;
    const float *zr = z + row * ld;
    float4 x[kStatCols / 4 / kBlock];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < kStatCols / 4 / kBlock; ++i) {
        const int c = c0 + (i * kBlock + threadIdx.x) * 4;
        x[i] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        if (c + 3 < V) {
            x[i] = *reinterpret_cast<const float4 *>(zr + c);
        } else if (c < V) {
            x[i].x = zr[c];
            if (c + 1 < V) x[i].y = zr[c + 1];
            if (c + 2 < V) x[i].z = zr[c + 2];
        }
        mx = fmaxf(fmaxf(mx, fmaxf(x[i].x, x[i].y)), fmaxf(x[i].z, x[i].w));
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    mx = wave_max(mx);
    if (lane == 0) red_m[wave] = mx;
    __syncthreads();
    float Mx = red_m[0];
#pragma unroll
    for (int w = 1; w < kBlock / kWave; ++w) Mx = fmaxf(Mx, red_m[w]);
    const float ref = (Mx == -INFINITY) ? 0.f : Mx;
    float l = 0.f;
#pragma unroll
    for (int i = 0; i < kStatCols / 4 / kBlock; ++i)
        l += __expf(x[i].x - ref) + __expf(x[i].y - ref) + __expf(x[i].z - ref) + __expf(x[i].w - ref);
    l = wave_sum(l);
    if (lane == 0) red_l[wave] = l;
    __syncthreads();
    if (threadIdx.x == 0) {
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < kBlock / kWave; ++w) L += red_l[w];
        part[row * parts + blockIdx.y] = make_float2(Mx, (Mx == -INFINITY) ? 0.f : L);
    }
}

// The paper's sequential scheme (eq. 11-13) for one row b of the batch, all n draws in one block.
// For step s the conditional is the mixture sum_a qhat_a P^(s)(. | a) with qhat = softmax(q),
// q_a = log w_a + sum_{k<s} log P^(k)(x_k | a).  It is sampled exactly like the single-expert draw of
// cp_head_draft_sample, with every mass replaced by its qhat-weighted sum over the r experts:
// segment masses from the GEMM's per-segment statistics (fp64, vocabulary order), then the logits of
// the crossing segment are recomputed for all r experts and the scan continues token by token.
// y of the step's r rows is staged in LDS when it fits (r*d <= 32768 elements), else read from memory.
constexpr int kSeqBlock = 1024;
constexpr int kSeqYElems = 32768;
__global__ void __launch_bounds__(kSeqBlock) k_draft_sequential(int d, int V, int n, int r, int parts, int seg_cols,
                                                                const float2 *__restrict__ part,
                                                                const bf16_t *__restrict__ Y,
                                                                const bf16_t *__restrict__ U,
                                                                const float *__restrict__ logw,
                                                                const float *__restrict__ uniforms,
                                                                int32_t *__restrict__ tokens, float *__restrict__ logq)
{
    __shared__ __attribute__((aligned(16))) bf16_t y_s[kSeqYElems];
    __shared__ float lse_s[64 * 64];
    __shared__ float z_s[64 * 128];
    __shared__ float q_s[64], qh_s[64];
    __shared__ double wave_tot[kSeqBlock / kWave];
    __shared__ double base_sh;
    __shared__ int cross_sh, seg_sh;
    const size_t b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NW = kSeqBlock / kWave;
    const int nr = n * r;
    const bool stage_y = r * d <= kSeqYElems;

    // log-normalisers of all n*r rows of this b (eq. 5)
    for (int j = wave; j < nr; j += NW) {
        const float v = row_lse_from_parts(part + (b * nr + j) * parts, parts, lane);
        if (lane == 0) lse_s[j] = v;
    }
    if (tid < r) q_s[tid] = logw[b * r + tid];
    __syncthreads();

    for (int s = 0; s < n; ++s) {
        const double u = (double)uniforms[b * n + s];
        const size_t row0 = (b * n + s) * r;             // first of the r head rows of this step
        if (wave == 0) {
            const float qa = lane < r ? q_s[lane] : -INFINITY;
            const float mx = wave_max(qa);
            const float qn = mx + logf(wave_sum(lane < r ? expf(qa - mx) : 0.f));
            if (lane < r) qh_s[lane] = expf(qa - qn);
        }
        if (tid == 0) cross_sh = 0x7FFFFFFF;
        if (stage_y) {
            const u32x4_t *src = reinterpret_cast<const u32x4_t *>(Y + row0 * d);
            u32x4_t *dst = reinterpret_cast<u32x4_t *>(y_s);
            for (int i = tid; i < r * d / 8; i += kSeqBlock) dst[i] = src[i];
        }
        __syncthreads();

        // mixture mass of every segment, running sum over the vocabulary in fp64
        const int per = (parts + kSeqBlock - 1) / kSeqBlock;
        const int lo = min(parts, tid * per), hi = min(parts, lo + per);
        double sum = 0.0;
        for (int j = lo; j < hi; ++j)
            for (int a = 0; a < r; ++a) {
                const float2 qv = part[(row0 + a) * parts + j];
                if (qv.x != -INFINITY) sum += (double)(qh_s[a] * qv.y * expf(qv.x - lse_s[s * r + a]));
            }
        double incl = wave_scan_inclusive(sum, lane);
        if (lane == kWave - 1) wave_tot[wave] = incl;
        __syncthreads();
        for (int w2 = 0; w2 < wave; ++w2) incl += wave_tot[w2];
        if (incl > u) atomicMin(&cross_sh, tid);
        __syncthreads();
        const bool forced = cross_sh == 0x7FFFFFFF;      // the running sum never passes u: last token
        if (forced) {
            if (tid == 0) { seg_sh = (V - 1) / seg_cols; base_sh = 0.0; }
        } else if (tid == cross_sh) {
            double c = incl - sum;
            int seg = hi - 1;
            for (int j = lo; j < hi; ++j) {
                double mj = 0.0;
                for (int a = 0; a < r; ++a) {
                    const float2 qv = part[(row0 + a) * parts + j];
                    if (qv.x != -INFINITY) mj += (double)(qh_s[a] * qv.y * expf(qv.x - lse_s[s * r + a]));
                }
                if (c + mj > u) { seg = j; break; }
                c += mj;
            }
            seg_sh = seg;
            base_sh = c;
        }
        __syncthreads();
        const int seg = seg_sh;
        const int v0 = seg * seg_cols, cols = min(seg_cols, V - v0);

        // logits of the segment for all r experts: a wavefront walks k for four columns and up to
        // eight experts together (the four loads of U per step are independent and stay in flight)
        const bf16_t *ybase = stage_y ? y_s : Y + row0 * d;
        constexpr int CW = 4, EW = 8;
        for (int c0 = wave * CW; c0 < cols; c0 += NW * CW) {
            const u32x4_t *urow[CW];
#pragma unroll
            for (int e = 0; e < CW; ++e)
                urow[e] = reinterpret_cast<const u32x4_t *>(U + (size_t)(v0 + min(c0 + e, cols - 1)) * d);
            for (int a0 = 0; a0 < r; a0 += EW) {
                float acc[EW][CW];
#pragma unroll
                for (int e = 0; e < EW; ++e)
#pragma unroll
                    for (int c = 0; c < CW; ++c) acc[e][c] = 0.f;
#pragma unroll 1
                for (int k = lane; k < d / 8; k += kWave) {
                    u32x4_t uv[CW];
#pragma unroll
                    for (int c = 0; c < CW; ++c) uv[c] = urow[c][k];
#pragma unroll
                    for (int e = 0; e < EW; ++e) {
                        // experts past r repeat the last one (their sums are dropped below)
                        const u32x4_t yv = reinterpret_cast<const u32x4_t *>(ybase + (size_t)min(a0 + e, r - 1) * d)[k];
#pragma unroll
                        for (int c = 0; c < CW; ++c)
#pragma unroll
                            for (int qd = 0; qd < 4; ++qd) {
                                acc[e][c] += __uint_as_float(uv[c][qd] << 16) * __uint_as_float(yv[qd] << 16);
                                acc[e][c] += __uint_as_float(uv[c][qd] & 0xFFFF0000u) * __uint_as_float(yv[qd] & 0xFFFF0000u);
                            }
                    }
                }
#pragma unroll
                for (int e = 0; e < EW; ++e)
#pragma unroll
                    for (int c = 0; c < CW; ++c) {
                        const float zz = wave_sum(acc[e][c]);
                        if (lane == 0 && a0 + e < r && c0 + c < cols) z_s[(a0 + e) * seg_cols + c0 + c] = zz;
                    }
            }
        }
        __syncthreads();

        if (wave == 0) {
            int tok;
            if (forced) {
                tok = V - 1;
            } else {
                const int per2 = (seg_cols + kWave - 1) / kWave;
                const int lo2 = lane * per2;
                double ps = 0.0;
                for (int i = lo2; i < lo2 + per2 && i < cols; ++i)
                    for (int a = 0; a < r; ++a) ps += (double)(qh_s[a] * expf(z_s[a * seg_cols + i] - lse_s[s * r + a]));
                const double in2 = base_sh + wave_scan_inclusive(ps, lane);
                const unsigned long long crossed = __ballot(in2 > u);
                if (crossed == 0ull) {
                    tok = v0 + cols - 1;
                } else {
                    const int first = __ffsll((long long)crossed) - 1;
                    int mine = v0 + min(cols, lo2 + per2) - 1;
                    if (lane == first) {
                        double c = in2 - ps;
                        for (int i = lo2; i < lo2 + per2 && i < cols; ++i) {
                            double pi = 0.0;
                            for (int a = 0; a < r; ++a)
                                pi += (double)(qh_s[a] * expf(z_s[a * seg_cols + i] - lse_s[s * r + a]));
                            c += pi;
                            if (c > u) { mine = v0 + i; break; }
                        }
                    }
                    tok = __shfl(mine, first, kWave);
                }
            }
            if (lane == 0) tokens[b * n + s] = tok;
            // expert log-weights take the log-probability of the drawn token (text under eq. 12)
            if (lane < r) q_s[lane] += z_s[lane * seg_cols + (tok - v0)] - lse_s[s * r + lane];
        }
        __syncthreads();
    }
    if (logq && wave == 0) {
        const float qa = lane < r ? q_s[lane] : -INFINITY;
        const float mx = wave_max(qa);
        const float sum = wave_sum(lane < r ? expf(qa - mx) : 0.f);
        if (lane == 0) logq[b] = mx + logf(sum);
    }
}

// Per head row {lse, coef = up_t * gamma[t, a] (zero for dropped factors), target}; dg[t, a] = up_t (w - gamma)
__global__ void k_bwd_coefficients(size_t M, int n, int r, const float *__restrict__ w, const float *__restrict__ gamma,
                                   const float *__restrict__ lse, const float *__restrict__ dloss, float scale,
                                   const int32_t *__restrict__ X, float4 *__restrict__ rowinfo, float *__restrict__ dg)
{
    const size_t m = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= M) return;
    const size_t t = m / ((size_t)n * r);
    const int a = (int)(m % r);
    const float up = dloss ? dloss[t] * scale : scale;
    const float gm = gamma[t * r + a];
    const int x = X[m / r];
    rowinfo[m] = make_float4(lse[m], (x >= 0) ? up * gm : 0.f, __int_as_float(x), 0.f);
    if ((m / r) % n == 0) dg[t * r + a] = up * (w[t * r + a] - gm);
}

// dH[t, j] += sum_a dg[t, a] G[a, j]
__global__ void k_add_gate_to_dh(size_t T, int d, int r, const bf16_t *__restrict__ G, const float *__restrict__ dg,
                                 float *__restrict__ dH)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= T * d) return;
    const size_t t = idx / d;
    const int j = (int)(idx % d);
    float acc = dH[idx];
    for (int a = 0; a < r; ++a) acc += dg[t * r + a] * bf16_to_f32(G[(size_t)a * d + j]);
    dH[idx] = acc;
}

// dG[a, j] = sum_t dg[t, a] H[t, j] in two deterministic stages: partial sums over chunks of 512
// positions (one thread per column j, eight experts at a time), then the chunks in increasing order.
constexpr int kGateChunk = 512;
__global__ void __launch_bounds__(kBlock) k_dgate_partial(size_t T, int d, int r, const bf16_t *__restrict__ H,
                                                          const float *__restrict__ dg, float *__restrict__ partial)
{
    const int j = blockIdx.x * kBlock + threadIdx.x;
    const size_t tc = blockIdx.y;
    if (j >= d) return;
    const size_t t0 = tc * kGateChunk, t1 = min(T, t0 + kGateChunk);
    for (int a0 = 0; a0 < r; a0 += 8) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (size_t t = t0; t < t1; ++t) {
            const float h = bf16_to_f32(H[t * d + j]);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (a0 + e < r) acc[e] += dg[t * r + a0 + e] * h;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (a0 + e < r) partial[(tc * r + a0 + e) * d + j] = acc[e];
    }
}
__global__ void k_dgate_reduce(int chunks, int d, int r, const float *__restrict__ partial, float *__restrict__ dG)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)r * d) return;
    float acc = 0.f;
    for (int c = 0; c < chunks; ++c) acc += partial[(size_t)c * r * d + idx];
    dG[idx] = acc;
}

// ------------------------------------------------------------------------------------------
// full heads (eq. 6 as printed: one V x d matrix F_sa per (s, a), no shared unembedding)
// Per-row quantities of this variant are kept head-major, index sa * T + t: every (s, a) runs its own
// products over the T positions, so its rows are contiguous for the epilogues above.
// ------------------------------------------------------------------------------------------

// One wavefront per (sa, t): log-normaliser from the statistics (eq. 5), target logit as an fp32 dot
// product of F_sa[x] with h (both bf16, so the products are exact), C = z[x] - lse (eq. 8).
__global__ void __launch_bounds__(kBlock) k_full_row_finish(size_t T, int d, int V, int n, int r, int parts,
                                                            const float2 *__restrict__ part,
                                                            const bf16_t *__restrict__ H, const bf16_t *__restrict__ F,
                                                            const int32_t *__restrict__ X, float *__restrict__ lse_out,
                                                            float *__restrict__ C_out)
{
    const size_t idx = (size_t)blockIdx.x * (kBlock / kWave) + (threadIdx.x >> 6);
    if (idx >= T * n * r) return;
    const int lane = threadIdx.x & 63;
    const size_t sa = idx / T, t = idx % T;
    const int s = (int)(sa / r), a = (int)(sa % r);
    const float lse = row_lse_from_parts(part + idx * parts, parts, lane);
    const int x = X[t * n + s];
    float zt = 0.f;
    if (x >= 0) zt = wave_dot_bf16(F + (sa * V + x) * d, H + t * d, d, lane);
    if (lane == 0) {
        lse_out[idx] = lse;
        C_out[(t * n + s) * r + a] = (x >= 0) ? zt - lse : 0.f;
    }
}

// Per (sa, t): {lse, coef = up_t * gamma[t, a] (zero for dropped factors), target}; dg[t, a] = up_t (w - gamma)
__global__ void k_full_bwd_coefficients(size_t T, int n, int r, const float *__restrict__ w,
                                        const float *__restrict__ gamma, const float *__restrict__ lse,
                                        const float *__restrict__ dloss, float scale, const int32_t *__restrict__ X,
                                        float4 *__restrict__ rowinfo, float *__restrict__ dg)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= T * n * r) return;
    const size_t sa = idx / T, t = idx % T;
    const int s = (int)(sa / r), a = (int)(sa % r);
    const float up = dloss ? dloss[t] * scale : scale;
    const float gm = gamma[t * r + a];
    const int x = X[t * n + s];
    rowinfo[idx] = make_float4(lse[idx], (x >= 0) ? up * gm : 0.f, __int_as_float(x), 0.f);
    if (s == 0) dg[t * r + a] = up * (w[t * r + a] - gm);
}

// ------------------------------------------------------------------------------------------
// workspace layouts
// ------------------------------------------------------------------------------------------

struct FwdWs {
    size_t logw, C, Ylo, part, total;
    int parts;
};
inline FwdWs fwd_ws(const cp_head_desc &ds)
{
    FwdWs f;
    const size_t M = (size_t)ds.T * ds.n * ds.r;
    f.parts = ((ds.V + Cfg::BN - 1) / Cfg::BN) * Cfg::WN;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    f.logw = take((size_t)ds.T * ds.r * 4);
    f.C = take(M * 4);
    f.Ylo = take(M * ds.d * 2);
    // with kept logits the statistics live in ctx: the backward pass needs the maxima again
    f.part = (ds.flags & CP_HEAD_KEEP_LOGITS) ? off : take(M * f.parts * sizeof(float2));
    f.total = off;
    return f;
}

// Rows of logit gradients held at a time: about 4 GiB of bf16 at V = 32000, i.e. 65536 rows.  Measured on the
// headline step: 2 GiB 450.4 ms, 4 GiB 447.9, 8 GiB 448.3 (the dU product gains from fewer accumulation passes
// over its fp32 output, the dz product loses about half of that).  A larger vocabulary keeps at least 32768
// rows, up to 8 GiB of them: the rows of a chunk are the contraction length of its dU product, and at 8192 rows
// (2 GiB at V = 128256) that product ran at 1.08 PFLOP/s against 1.25 at 32768.  The count is a multiple of 16
// tiles of 256 rows where possible, so that the d-wide products of a chunk (16 tile columns at d = 4096) fill
// all 256 compute units in whole rounds.
inline size_t bwd_chunk_rows(const cp_head_desc &ds)
{
    const size_t M = (size_t)ds.T * ds.n * ds.r;
    const size_t Vp = round_up((size_t)ds.V, 64);
    size_t rows = ((size_t)1 << 32) / (Vp * 2);
    if (rows < 32768) {
        const size_t cap = ((size_t)1 << 33) / (Vp * 2);
        rows = cap < 32768 ? cap : 32768;
    }
    if (rows >= 16 * (size_t)Cfg::BM) rows = rows / (16 * Cfg::BM) * (16 * Cfg::BM);
    else rows = rows / Cfg::BM * Cfg::BM;
    if (rows < (size_t)Cfg::BM || (ds.flags & CP_HEAD_MIN_WORKSPACE)) rows = Cfg::BM;
    return rows < M ? rows : (M ? M : 1);
}

struct BwdWs {
    size_t coef, dg, dGpart, Ut, Wt, dY, dZ, dZt, Yt, total;
    size_t Vp, chunk, chunk_p;
    size_t ldV, ldM, ldN;   // leading dimensions of the transposed operands (K padded to 64, plus 64)
};
inline BwdWs bwd_ws(const cp_head_desc &ds)
{
    BwdWs b;
    const size_t T = (size_t)ds.T, nrd = (size_t)ds.n * ds.r * ds.d, M = T * ds.n * ds.r;
    b.Vp = round_up((size_t)ds.V, 64);
    b.chunk = bwd_chunk_rows(ds);
    b.chunk_p = round_up(b.chunk, 64);
    b.ldV = b.Vp + 64; b.ldM = b.chunk_p + 64; b.ldN = nrd + 64;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    b.coef = take(M * 16);
    b.dg = take(T * ds.r * 4);
    b.dGpart = take(((T + kGateChunk - 1) / kGateChunk) * ds.r * ds.d * 4);
    b.Ut = take((size_t)ds.d * b.ldV * 2);
    b.Wt = take((size_t)ds.d * b.ldN * 2);
    b.dY = take(M * ds.d * 2);
    b.dZ = take(round_up(b.chunk, 256) * b.Vp * 2);   // stored in blocks of 256 rows x 64 columns
    b.dZt = take((size_t)ds.V * b.ldM * 2);
    b.Yt = take((size_t)ds.d * b.ldM * 2);
    b.total = off;
    return b;
}

// Saved-for-backward buffer of the full-head calls: [lse nr*T f32, head-major][w T*r][gamma T*r]
struct FullCtx {
    size_t lse, w, gamma, zpart, zs, total;
    size_t Vp;
    int parts;
    bool keep;      // CP_HEAD_KEEP_LOGITS: statistics and logits of all rows (head-major, like lse) stay in ctx
};
inline FullCtx full_ctx(const cp_head_desc &ds)
{
    FullCtx c;
    const size_t M = (size_t)ds.T * ds.n * ds.r, Tr = (size_t)ds.T * ds.r;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    c.lse = take(M * 4);
    c.w = take(Tr * 4);
    c.gamma = take(Tr * 4);
    c.keep = (ds.flags & CP_HEAD_KEEP_LOGITS) != 0 && use_fast_path(ds);
    c.Vp = round_up((size_t)ds.V, 64);
    c.parts = ((ds.V + Cfg::BN - 1) / Cfg::BN) * Cfg::WN;
    c.zpart = c.zs = off;
    if (c.keep) {
        c.zpart = take(M * c.parts * sizeof(float2));
        c.zs = take(M * c.Vp * 2);
    }
    c.total = off;
    return c;
}

struct FullFwdWs {
    size_t logw, C, part, total;
    int parts;
};
inline FullFwdWs full_fwd_ws(const cp_head_desc &ds)
{
    FullFwdWs f;
    const size_t M = (size_t)ds.T * ds.n * ds.r;
    f.parts = ((ds.V + Cfg::BN - 1) / Cfg::BN) * Cfg::WN;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    f.logw = take((size_t)ds.T * ds.r * 4);
    f.C = take(M * 4);
    f.part = (ds.flags & CP_HEAD_KEEP_LOGITS) ? off : take(M * f.parts * sizeof(float2));   // else in ctx
    f.total = off;
    return f;
}

// Positions whose logit gradients (for one head at a time) are held together: about 2 GiB of bf16
inline size_t full_chunk_rows(const cp_head_desc &ds)
{
    const size_t Vp = round_up((size_t)ds.V, 64);
    size_t rows = ((size_t)1 << 31) / (Vp * 2);
    rows = rows / Cfg::BM * Cfg::BM;
    if (rows < (size_t)Cfg::BM || (ds.flags & CP_HEAD_MIN_WORKSPACE)) rows = Cfg::BM;
    const size_t T = (size_t)ds.T;
    return rows < T ? rows : (T ? T : 1);
}

struct FullBwdWs {
    size_t coef, dg, dGpart, Ht, dZ, dZt, total;
    size_t Vp, Tp, chunk, chunk_p;
    size_t ldT, ldM;
};
inline FullBwdWs full_bwd_ws(const cp_head_desc &ds)
{
    FullBwdWs b;
    const size_t T = (size_t)ds.T, M = T * ds.n * ds.r;
    b.Vp = round_up((size_t)ds.V, 64);
    b.Tp = round_up(T, 64);
    b.chunk = full_chunk_rows(ds);
    b.chunk_p = round_up(b.chunk, 64);
    b.ldT = b.Tp + 64; b.ldM = b.chunk_p + 64;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    b.coef = take(M * 16);
    b.dg = take(T * ds.r * 4);
    b.dGpart = take(((T + kGateChunk - 1) / kGateChunk) * ds.r * ds.d * 4);
    b.Ht = take((size_t)ds.d * b.ldT * 2);
    b.dZ = take(b.chunk * b.Vp * 2);
    b.dZt = take((size_t)ds.V * b.ldM * 2);
    b.total = off;
    return b;
}

inline bool dims_fit(const cp_head_desc &ds)
{
    // the GEMM addresses rows of a tile with 32-bit byte offsets and counts rows in int
    const size_t nrd = (size_t)ds.n * ds.r * ds.d, M = (size_t)ds.T * ds.n * ds.r;
    const size_t max_ld = (nrd > (size_t)ds.V + 64 ? nrd : (size_t)ds.V + 64) + 64;
    return M < ((size_t)1 << 31) && nrd < ((size_t)1 << 31) && max_ld * 2 * 256 < ((size_t)1 << 32) &&
           ((size_t)ds.T + 128) * 2 * 256 < ((size_t)1 << 32);
}

}  // namespace

// rows of a 64-row tile: the draft GEMMs with at most this many rows stream their big operand with
// two 80 KB workgroups per compute unit instead of one 128 KB workgroup
typedef TileCfg<64, 256, 1, 4> CfgSkinny;
// rows up to which the z product of a draft-type call uses the 64-row tile (several tile rows then share the
// slices of U through L2: their workgroups are neighbours in the tile walk)
#ifndef CPH_SKINNY_ROWS
#define CPH_SKINNY_ROWS 64
#endif
constexpr int kSkinnyRows = CPH_SKINNY_ROWS;
// z = U y for the few rows of a draft-type call: picks the tile by the number of rows
template <class Epi>
inline void launch_z_streamed(const char *name, const bf16_t *Y, int d, int rows, const bf16_t *U, int V, const Epi &epi,
                              hipStream_t st)
{
    if (rows <= kSkinnyRows) launch_gemm_nt<CfgSkinny>(name, Y, d, rows, U, d, V, d, epi, st, kSkinnyRows / CfgSkinny::BM);
    else launch_gemm_nt<Cfg>(name, Y, d, rows, U, d, V, d, epi, st);
}
// y = W_sa h for the first `heads` of the n r head matrices (bf16, rounded: part of the draft distribution's
// definition), with the gate (and the expert draw, if uniforms is given) as the launch's side job
inline void launch_y_with_gate(const char *name, const cp_head_desc &ds, const bf16_t *H, const bf16_t *W, const bf16_t *G,
                               const float *uniforms, bf16_t *Y, float *logw, int32_t *alpha, int heads, hipStream_t st)
{
    const int B = (int)ds.T, d = ds.d, cols = heads * d;
    const GatePickSide side{(B + 7) / 8 * 8, B, d, ds.n, ds.r, H, G, uniforms, logw, alpha};
    const EpiStoreBf16 epi{Y, nullptr, (long)cols, B, cols};
    if (B <= CfgSkinny::BM) launch_gemm_nt<CfgSkinny>(name, H, d, B, W, d, cols, d, epi, st, kGroupRowsWide, side);
    else launch_gemm_nt<Cfg>(name, H, d, B, W, d, cols, d, epi, st, kGroupRowsWide, side);
}
// statistics segments (pairs per row, columns per segment) of that choice
inline void z_segments(int rows, int V, int &parts, int &seg_cols)
{
    if (rows <= kSkinnyRows) {
        parts = ((V + CfgSkinny::BN - 1) / CfgSkinny::BN) * CfgSkinny::WN;
        seg_cols = CfgSkinny::WTN;
    } else {
        parts = ((V + Cfg::BN - 1) / Cfg::BN) * Cfg::WN;
        seg_cols = Cfg::WTN;
    }
}

struct DraftWs {
    size_t logw, Y, part, lse, seg, base, total;
    int parts_max;
};
inline DraftWs draft_ws(const cp_head_desc &ds)
{
    DraftWs f;
    const size_t M = (size_t)ds.T * ds.n * ds.r;
    f.parts_max = ((ds.V + Cfg::BN - 1) / Cfg::BN) * CfgSkinny::WN;   // the finer of the two segmentations
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    f.logw = take((size_t)ds.T * ds.r * 4);
    f.Y = take(M * ds.d * 2);
    f.part = take(M * f.parts_max * sizeof(float2));
    f.lse = take(M * 4);
    f.seg = take((size_t)ds.T * ds.n * 4);
    f.base = take((size_t)ds.T * ds.n * 8);
    f.total = off;
    return f;
}

struct FirstTokenWs {
    size_t logw, Y, z, lse, part, total;
    size_t V4;
    int parts;
};
inline FirstTokenWs first_token_ws(const cp_head_desc &ds)
{
    FirstTokenWs f;
    const size_t rows = (size_t)ds.T * ds.r;
    f.V4 = round_up((size_t)ds.V, 4);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    f.logw = take(rows * 4);
    f.Y = take(rows * ds.d * 2);
    f.z = take(rows * f.V4 * 4);
    f.lse = take(rows * 4);
    f.parts = (ds.V + kStatCols - 1) / kStatCols;
    f.part = take(rows * f.parts * sizeof(float2));
    f.total = off;
    return f;
}

size_t fast_workspace_bytes(const cp_head_desc &ds, int op)
{
    if (op == CP_HEAD_OP_LOSS_FWD) return fwd_ws(ds).total;
    if (op == CP_HEAD_OP_LOSS_BWD) return bwd_ws(ds).total;
    if (op == CP_HEAD_OP_FIRST_TOKEN) return first_token_ws(ds).total;
    if (op == CP_HEAD_OP_FULL_LOSS_FWD) return full_fwd_ws(ds).total;
    if (op == CP_HEAD_OP_FULL_LOSS_BWD) return full_bwd_ws(ds).total;
    return draft_ws(ds).total;   // both draft calls
}

// Everything of the forward pass that is per head row: gate (eq. 7), y, the statistics of z, the
// log-normalisers (eq. 5) and C (eq. 8).  `out` receives where the results live in ctx and ws.
int fast_fwd_rows(const cp_head_desc &ds, const void *Hv, const void *Wv, const void *Uv, const void *Gv,
                  const int32_t *X, void *ctx, void *ws, FastFwdBuffers *out, hipStream_t st)
{
    if (!dims_fit(ds)) return CP_HEAD_ERR_UNSUPPORTED;
    const bf16_t *H = (const bf16_t *)Hv, *W = (const bf16_t *)Wv, *U = (const bf16_t *)Uv;
    const CtxLayout cl = ctx_layout(ds, true);
    const FwdWs f = fwd_ws(ds);
    const int T = (int)ds.T, d = ds.d, V = ds.V;
    const size_t M = (size_t)T * ds.n * ds.r;
    const int nrd = ds.n * ds.r * d;
    float *lse = at<float>(ctx, cl.lse), *w = at<float>(ctx, cl.w), *gamma = at<float>(ctx, cl.gamma);
    bf16_t *Y = at<bf16_t>(ctx, cl.Y);
    float *logw = at<float>(ws, f.logw), *C = at<float>(ws, f.C);
    bf16_t *Ylo = at<bf16_t>(ws, f.Ylo);
    float2 *part = cl.keep ? at<float2>(ctx, cl.zpart) : at<float2>(ws, f.part);
    if (cl.keep && (cl.parts != f.parts || kKeptTile != Cfg::WTN)) return CP_HEAD_ERR_UNSUPPORTED;

    launch_gate(ds, Hv, Gv, logw, w, st);                                                      // eq. 7
    launch_gemm_nt<Cfg>("gemm_y", H, d, T, W, d, nrd, d, EpiStoreBf16{Y, Ylo, (long)nrd, T, nrd}, st, kGroupRowsNarrow);   // y = W_sa h
    if (cl.keep)                                                                               // z = U y, statistics, z kept
        launch_gemm_nt<Cfg>("gemm_z_stats_keep", Y, d, (int)M, U, d, V, d,
                            EpiRowStatsKeep{part, f.parts, (int)M, V, at<uint16_t>(ctx, cl.zs), (long)cl.Vp, (int)cl.Vp}, st);
    else
        launch_gemm_nt<Cfg>("gemm_z_stats", Y, d, (int)M, U, d, V, d, EpiRowStats{part, f.parts, (int)M, V}, st);  // z = U y, statistics
    k_row_finish<<<blocks_for(M, kBlock / kWave), kBlock, 0, st>>>(M, d, ds.r, f.parts, part, Y, Ylo, U, X, lse, C);
    out->lse = lse; out->w = w; out->gamma = gamma; out->logw = logw; out->C = C; out->Y = Y;
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

int fast_loss_fwd(const cp_head_desc &ds, const void *Hv, const void *Wv, const void *Uv, const void *Gv,
                  const int32_t *X, float *loss, void *ctx, void *ws, size_t, hipStream_t st)
{
    if (ds.T == 0) return CP_HEAD_OK;
    FastFwdBuffers b;
    const int rc = fast_fwd_rows(ds, Hv, Wv, Uv, Gv, X, ctx, ws, &b, st);
    if (rc != CP_HEAD_OK) return rc;
    launch_mixture(ds, b.logw, b.C, loss, b.gamma, -1.f, st);                                        // eq. 9
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

// Which operand layout each product of the backward pass uses.  The main loop reads a K-major operand (the
// contraction index is its slow one) with gfx950's transposing LDS read, which needs no transposed copy of anything
// but costs the loop 4-5 % per K-major operand (two 64-bit reads per fragment instead of one 128-bit read: twice the
// LDS instructions and LDS busy time for the same bytes; measured at the headline size: dY 97.3 -> 101.2 ms per step
// with U K-major, dU 99.6 -> 109.9 with dz and Y K-major, dH 12.5 -> 13.0, dW 12.7 -> 13.7).  A transposed copy is
// an HBM-bound pass that costs less than that wherever the product is vocabulary-sized (dz^T from the dz epilogue 5.3
// ms per step, Y^T 2.7, U^T 0.1, W^T 0.5), so those products keep the K-contiguous form; dW = dY^T H is the one
// whose transposed copies (4.3 GB of dY: 1.8 ms) cost more than its K-major loop (1.0 ms), and they were 4.3 GB of
// workspace.

// The backward pass below dY: dH = dY W + G^T dg, dW = dY^T H, dG = dg^T H.  Wt: scratch for W^T [d, n r d + 64];
// dGpart: the partial sums of the two-stage gate gradient.
static int bwd_below_dy(const cp_head_desc &ds, const bf16_t *H, const bf16_t *W, const bf16_t *G, const bf16_t *dY,
                        const float *dg, float *dH, float *dW, float *dG, bf16_t *Wt, float *dGpart, hipStream_t st)
{
    const int d = ds.d, r = ds.r;
    const size_t T = (size_t)ds.T, nrd = (size_t)ds.n * r * d;
    const long ldN = (long)nrd + 64;
    // dH = dY W + G^T dg   (contraction over (s, a, k))
    transpose_bf16(W, d, (int)nrd, d, Wt, ldN, (int)nrd, st);         // Wt[d, nrd]
    launch_gemm_nt<Cfg>("gemm_dh", dY, (long)nrd, (int)T, Wt, ldN, d, (int)nrd, EpiStoreF32{dH, (long)d, (int)T, d, 0}, st,
                        kGroupRowsNarrow);
    k_add_gate_to_dh<<<blocks_for(T * d, kBlock), kBlock, 0, st>>>(T, d, r, G, dg, dH);
    if (dW)
        // dW_sa = dY_sa^T H   (contraction over positions: both operands K-major, any number of positions)
        launch_gemm_nt<CfgTN>("gemm_dw", dY, (long)nrd, (int)nrd, H, d, d, (int)T, EpiStoreF32{dW, (long)d, (int)nrd, d, 0}, st,
                              kGroupRowsNarrow);
    if (dG) {
        const unsigned chunks = (unsigned)((T + kGateChunk - 1) / kGateChunk);
        k_dgate_partial<<<dim3(blocks_for((size_t)d, kBlock), chunks), kBlock, 0, st>>>(T, d, r, H, dg, dGpart);
        k_dgate_reduce<<<blocks_for((size_t)r * d, kBlock), kBlock, 0, st>>>((int)chunks, d, r, dGpart, dG);
    }
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

// dY = dz U and dU (+)= dz^T Y for one chunk of head rows whose dz (and, if dU is wanted, dz^T) is in place.
// dZ is stored block by block (blocked64_index, ld = Vp): its rows are 2 Vp bytes apart otherwise, a tile's K-step
// touches 256 separate cache lines of it, and the product, which streams the chunk's 4 GiB of it from HBM, runs 4 %
// slower.  Ut: U^T [d, Vp + 64]; Yt: scratch for the chunk's Y^T [d, Mcp + 64].
static void bwd_chunk_products(const cp_head_desc &ds, const bf16_t *dZ, const bf16_t *dZt, long ldM, const bf16_t *Yc,
                               int Mc, const bf16_t *Ut, bf16_t *Yt, bf16_t *dYc, float *dU, bool accumulate, hipStream_t st)
{
    const int d = ds.d, V = ds.V;
    const int Vp = (int)round_up((size_t)V, 64), Mcp = (int)round_up((size_t)Mc, 64);
    const long ldV = (long)Vp + 64;
    // dY = dz U   (contraction over the vocabulary)
    launch_gemm_nt<CfgBlockedA>("gemm_dy", dZ, Vp, Mc, Ut, ldV, d, Vp, EpiStoreBf16{dYc, nullptr, (long)d, Mc, d}, st,
                                kGroupRowsNarrow);
    if (dU) {
        // dU += dz^T Y   (contraction over the rows of the chunk)
        transpose_bf16(Yc, d, Mc, d, Yt, ldM, Mcp, st);               // Yt[d, Mcp]
        launch_gemm_nt<Cfg>("gemm_du", dZt, ldM, V, Yt, ldM, d, Mcp, EpiStoreF32{dU, (long)d, V, d, accumulate ? 1 : 0}, st,
                            kGroupRowsNarrow);
    }
}

// The backward pass below the logit gradients: per bounded chunk of head rows `dz_launch` writes dz
// (bf16, row-major and, if dU is wanted, transposed), then dY = dz U and dU += dz^T Y; afterwards
// dW = dY^T H, dH = dY W + G^T dg and dG = dg^T H.  dg[T,r] must already hold the gate gradients.
int fast_bwd_from_dz(const cp_head_desc &ds, const void *Hv, const void *Wv, const void *Uv, const void *Gv,
                     const void *Yv, const float *dg, float *dH, float *dW, float *dU, float *dG, void *ws,
                     FastDzLaunch dz_launch, void *user, hipStream_t st)
{
    const int d = ds.d, V = ds.V, r = ds.r, n = ds.n;
    const bf16_t *H = (const bf16_t *)Hv, *W = (const bf16_t *)Wv, *U = (const bf16_t *)Uv, *G = (const bf16_t *)Gv;
    const bf16_t *Y = (const bf16_t *)Yv;
    const BwdWs b = bwd_ws(ds);
    const size_t T = (size_t)ds.T, M = T * n * r;
    bf16_t *Ut = at<bf16_t>(ws, b.Ut), *Wt = at<bf16_t>(ws, b.Wt), *dY = at<bf16_t>(ws, b.dY);
    bf16_t *dZ = at<bf16_t>(ws, b.dZ), *dZt = at<bf16_t>(ws, b.dZt), *Yt = at<bf16_t>(ws, b.Yt);
    const int Vp = (int)b.Vp;

    transpose_bf16(U, d, V, d, Ut, (long)b.ldV, Vp, st);              // Ut[d, Vp]
    int first = 1;
    for (size_t m0 = 0; m0 < M; m0 += b.chunk) {
        const int Mc = (int)((M - m0 < b.chunk) ? M - m0 : b.chunk);
        const int Mcp = (int)round_up((size_t)Mc, 64);
        const bf16_t *Yc = Y + m0 * d;
        // recompute z for the chunk; the epilogue turns it into dz (bf16); the tiles over V also
        // cover the padding columns V..Vp-1, which the epilogue zero-fills
        dz_launch(user, Yc, Mc, Mcp, m0, dZ, (long)Vp, true, dU ? dZt : nullptr, (long)b.ldM, st);
        bwd_chunk_products(ds, dZ, dZt, (long)b.ldM, Yc, Mc, Ut, Yt, dY + m0 * d, dU, !first, st);
        first = 0;
    }
    return bwd_below_dy(ds, H, W, G, dY, dg, dH, dW, dG, Wt, at<float>(ws, b.dGpart), st);
}

bool fast_dims_fit(const cp_head_desc &ds) { return dims_fit(ds); }

namespace {
struct LossDzArgs {
    const bf16_t *U;
    const float4 *rowinfo;
    int d, V;
};
// dz of the training loss: dz[m, v] = coef[m] (exp(z - lse[m]) - 1[v = x_m])
void loss_dz_launch(void *user, const bf16_t *Yc, int Mc, int Mcp, size_t m0, bf16_t *dZ, long ldz, bool dz_blocked,
                    bf16_t *dZt, long ldzt, hipStream_t st)
{
    const LossDzArgs *a = static_cast<const LossDzArgs *>(user);
    launch_gemm_nt<Cfg>("gemm_z_dz", Yc, a->d, Mc, a->U, a->d, a->V, a->d,
                        EpiDz{dZ, ldz, dZt, ldzt, a->rowinfo + m0, Mc, Mcp, a->V, (int)ldz, dz_blocked ? 1 : 0}, st);
}

struct KeptDzArgs {
    KeptLogits kept;         // zs [M, Vp], part [M, parts]
    const float4 *rowinfo;
    int V;
};
// the same dz from the logits kept by the forward pass
void kept_dz_launch(void *user, const bf16_t *, int Mc, int Mcp, size_t m0, bf16_t *dZ, long ldz, bool dz_blocked,
                    bf16_t *dZt, long ldzt, hipStream_t st)
{
    const KeptDzArgs *a = static_cast<const KeptDzArgs *>(user);
    launch_dz_from_kept(a->kept, m0, a->rowinfo + m0, LossDzRule{}, Mc, Mcp, a->V, dZ, ldz, dz_blocked, dZt, ldzt, st);
}
}  // namespace

int fast_loss_bwd(const cp_head_desc &ds, const void *Hv, const void *Wv, const void *Uv, const void *Gv,
                  const int32_t *X, const float *dloss, float scale, const void *ctx, float *dH, float *dW,
                  float *dU, float *dG, void *ws, size_t, hipStream_t st)
{
    const int d = ds.d, V = ds.V, r = ds.r, n = ds.n;
    const size_t nrd = (size_t)n * r * d;
    if (ds.T == 0) {
        launch_fill_zero(dW, nrd * d, st);
        launch_fill_zero(dU, (size_t)V * d, st);
        launch_fill_zero(dG, (size_t)r * d, st);
        return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
    }
    if (!dims_fit(ds)) return CP_HEAD_ERR_UNSUPPORTED;
    const CtxLayout cl = ctx_layout(ds, true);
    const BwdWs b = bwd_ws(ds);
    const size_t M = (size_t)ds.T * n * r;
    const float *lse = at<float>(ctx, cl.lse), *w = at<float>(ctx, cl.w), *gamma = at<float>(ctx, cl.gamma);
    float4 *rowinfo = at<float4>(ws, b.coef);
    float *dg = at<float>(ws, b.dg);
    k_bwd_coefficients<<<blocks_for(M, kBlock), kBlock, 0, st>>>(M, n, r, w, gamma, lse, dloss, scale, X, rowinfo, dg);
    if (cl.keep) {
        KeptDzArgs kept{KeptLogits{at<uint16_t>(ctx, cl.zs), at<float2>(ctx, cl.zpart), (long)cl.Vp, cl.parts}, rowinfo, V};
        return fast_bwd_from_dz(ds, Hv, Wv, Uv, Gv, at<bf16_t>(ctx, cl.Y), dg, dH, dW, dU, dG, ws, kept_dz_launch, &kept, st);
    }
    LossDzArgs args{(const bf16_t *)Uv, rowinfo, d, V};
    return fast_bwd_from_dz(ds, Hv, Wv, Uv, Gv, at<bf16_t>(ctx, cl.Y), dg, dH, dW, dU, dG, ws, loss_dz_launch, &args, st);
}

// ------------------------------------------------------------------------------------------
// training step in one call: loss and gradients, one chunk of positions at a time
// ------------------------------------------------------------------------------------------

// Positions per chunk: whole positions whose head rows fit the backward pass's bound on logit-sized buffers.
struct StepWs {
    size_t logw, w, gamma, dg, dGpart, Ut, Wt, dY, C, lse, coef, Yc, Ylo, part, zs, dZ, dZt, Yt, total;
    size_t Vp, pos, rows, ldM;
    int parts;
};
inline StepWs step_ws(const cp_head_desc &ds)
{
    StepWs f;
    const size_t T = (size_t)ds.T, nr = (size_t)ds.n * ds.r, M = T * nr, nrd = nr * ds.d;
    f.Vp = round_up((size_t)ds.V, 64);
    f.parts = ((ds.V + Cfg::BN - 1) / Cfg::BN) * Cfg::WN;
    f.pos = bwd_chunk_rows(ds) / nr;
    if (f.pos < 1) f.pos = 1;
    if (f.pos > T) f.pos = T ? T : 1;
    f.rows = f.pos * nr;
    f.ldM = round_up(f.rows, 64) + 64;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    f.logw = take(T * ds.r * 4);
    f.w = take(T * ds.r * 4);
    f.gamma = take(T * ds.r * 4);
    f.dg = take(T * ds.r * 4);
    f.dGpart = take(((T + kGateChunk - 1) / kGateChunk) * ds.r * ds.d * 4);
    f.Ut = take((size_t)ds.d * (f.Vp + 64) * 2);
    f.Wt = take((size_t)ds.d * (nrd + 64) * 2);
    f.dY = take(M * ds.d * 2);
    f.C = take(f.rows * 4);
    f.lse = take(f.rows * 4);
    f.coef = take(f.rows * 16);
    f.Yc = take(f.rows * ds.d * 2);
    f.Ylo = take(f.rows * ds.d * 2);
    f.part = take(f.rows * f.parts * sizeof(float2));
    f.zs = take(f.rows * f.Vp * 2);
    f.dZ = take(round_up(f.rows, 256) * f.Vp * 2);   // stored in blocks of 256 rows x 64 columns
    f.dZt = take((size_t)ds.V * f.ldM * 2);
    f.Yt = take((size_t)ds.d * f.ldM * 2);
    f.total = off;
    return f;
}
size_t fast_step_workspace_bytes(const cp_head_desc &ds) { return step_ws(ds).total; }

// Forward and backward interleaved per chunk of positions.  The logits of a chunk are kept as 16-bit floats (as
// with CP_HEAD_KEEP_LOGITS, but for one chunk: the buffer does not grow with T) from the product that forms their
// statistics to the pass that turns them into gradients a few launches later, so U y is multiplied once per step.
int fast_loss_step(const cp_head_desc &ds, const void *Hv, const void *Wv, const void *Uv, const void *Gv,
                   const int32_t *X, const float *dloss, float scale, float *loss, float *dH, float *dW, float *dU,
                   float *dG, void *ws, hipStream_t st)
{
    const int d = ds.d, V = ds.V, r = ds.r, n = ds.n;
    const size_t nr = (size_t)n * r, nrd = nr * d, T = (size_t)ds.T;
    if (T == 0) {
        launch_fill_zero(dW, nrd * d, st);
        launch_fill_zero(dU, (size_t)V * d, st);
        launch_fill_zero(dG, (size_t)r * d, st);
        return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
    }
    if (!dims_fit(ds) || kKeptTile != Cfg::WTN) return CP_HEAD_ERR_UNSUPPORTED;
    const bf16_t *H = (const bf16_t *)Hv, *W = (const bf16_t *)Wv, *U = (const bf16_t *)Uv, *G = (const bf16_t *)Gv;
    const StepWs f = step_ws(ds);
    float *logw = at<float>(ws, f.logw), *w = at<float>(ws, f.w), *gamma = at<float>(ws, f.gamma), *dg = at<float>(ws, f.dg);
    float *C = at<float>(ws, f.C), *lse = at<float>(ws, f.lse);
    float4 *rowinfo = at<float4>(ws, f.coef);
    bf16_t *dY = at<bf16_t>(ws, f.dY), *Yc = at<bf16_t>(ws, f.Yc), *Ylo = at<bf16_t>(ws, f.Ylo), *dZ = at<bf16_t>(ws, f.dZ);
    float2 *part = at<float2>(ws, f.part);
    uint16_t *zs = at<uint16_t>(ws, f.zs);
    const int Vp = (int)f.Vp;

    bf16_t *Ut = at<bf16_t>(ws, f.Ut), *dZt = at<bf16_t>(ws, f.dZt), *Yt = at<bf16_t>(ws, f.Yt);
    launch_gate(ds, Hv, Gv, logw, w, st);                                                             // eq. 7, all positions
    transpose_bf16(U, d, V, d, Ut, (long)f.Vp + 64, Vp, st);                                          // Ut[d, Vp]
    int first = 1;
    for (size_t t0 = 0; t0 < T; t0 += f.pos) {
        const size_t P = (T - t0 < f.pos) ? T - t0 : f.pos;
        const size_t m0 = t0 * nr;
        const int Mc = (int)(P * nr), Mcp = (int)round_up((size_t)Mc, 64);
        cp_head_desc sub = ds;
        sub.T = (int64_t)P;
        const int32_t *Xc = X + t0 * n;
        // forward of the chunk: y, statistics of z with the logits kept, log-normalisers and C (eq. 5, 8), mixture (eq. 9)
        launch_gemm_nt<Cfg>("gemm_y", H + t0 * d, d, (int)P, W, d, (int)nrd, d, EpiStoreBf16{Yc, Ylo, (long)nrd, (int)P, (int)nrd}, st,
                            kGroupRowsNarrow);
        launch_gemm_nt<Cfg>("gemm_z_stats_keep", Yc, d, Mc, U, d, V, d, EpiRowStatsKeep{part, f.parts, Mc, V, zs, (long)Vp, Vp}, st);
        k_row_finish<<<blocks_for((size_t)Mc, kBlock / kWave), kBlock, 0, st>>>((size_t)Mc, d, r, f.parts, part, Yc, Ylo, U, Xc, lse, C);
        launch_mixture(sub, logw + t0 * r, C, loss + t0, gamma + t0 * r, -1.f, st);
        // backward of the chunk down to dY and dU
        k_bwd_coefficients<<<blocks_for((size_t)Mc, kBlock), kBlock, 0, st>>>((size_t)Mc, n, r, w + t0 * r, gamma + t0 * r, lse,
                                                                            dloss ? dloss + t0 : nullptr, scale, Xc, rowinfo,
                                                                            dg + t0 * r);
        launch_dz_from_kept(KeptLogits{zs, part, (long)Vp, f.parts}, 0, rowinfo, LossDzRule{}, Mc, Mcp, V, dZ, (long)Vp, true,
                            dU ? dZt : nullptr, (long)f.ldM, st);
        bwd_chunk_products(ds, dZ, dZt, (long)f.ldM, Yc, Mc, Ut, Yt, dY + m0 * d, dU, !first, st);
        first = 0;
    }
    return bwd_below_dy(ds, H, W, G, dY, dg, dH, dW, dG, at<bf16_t>(ws, f.Wt), at<float>(ws, f.dGpart), st);
}

int fast_draft(const cp_head_desc &ds, const void *Hv, const void *Wv, const void *Uv, const void *Gv,
               const float *uniforms, int32_t *alpha, int32_t *tokens, float *logq, void *ws, size_t,
               hipStream_t st)
{
    if (ds.T == 0) return CP_HEAD_OK;
    if (!dims_fit(ds)) return CP_HEAD_ERR_UNSUPPORTED;
    const bf16_t *H = (const bf16_t *)Hv, *W = (const bf16_t *)Wv, *U = (const bf16_t *)Uv, *G = (const bf16_t *)Gv;
    const DraftWs f = draft_ws(ds);
    const int B = (int)ds.T, d = ds.d, V = ds.V, n = ds.n, r = ds.r;
    const size_t M = (size_t)B * n * r;
    float *logw = at<float>(ws, f.logw), *lse = at<float>(ws, f.lse);
    bf16_t *Y = at<bf16_t>(ws, f.Y);
    float2 *part = at<float2>(ws, f.part);
    int32_t *seg = at<int32_t>(ws, f.seg);
    double *base = at<double>(ws, f.base);
    const unsigned rows = (unsigned)(B * n);

    // y = W_sa h, rounded to bf16 (part of the draft distribution's definition); streams W once.  The gate and the
    // expert draw (eq. 7, a* ~ w) ride along as the launch's first workgroups.
    launch_y_with_gate("draft_gemm_y", ds, H, W, G, uniforms, Y, logw, alpha, n * r, st);
    // z = U y for all B*n*r rows with running statistics; streams U once, logits are not stored
    int parts, seg_cols;
    z_segments((int)M, V, parts, seg_cols);
    launch_z_streamed("draft_gemm_z", Y, d, (int)M, U, V, EpiRowStats{part, parts, (int)M, V}, st);
    {
        ProfileScope prof("draft_lse_segment", (double)M * parts * 8, st);
        k_draft_lse_segment<<<rows, kWideBlock, 0, st>>>(n, r, parts, part, alpha, uniforms, lse, seg, base);
    }
    {
        ProfileScope prof("draft_logits_pick", (double)rows * seg_cols * d * 2, st);
        k_draft_logits_pick<<<rows, kPickBlock, 0, st>>>(d, V, n, r, seg_cols, lse, Y, U, alpha, seg, base, uniforms,
                                                        tokens);
    }
    if (logq) {
        ProfileScope prof("draft_logq", (double)M * d * 4, st);
        k_draft_logq<<<(unsigned)B, kWideBlock, 0, st>>>(d, n, r, logw, lse, Y, U, tokens, logq);
    }
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

int fast_first_token(const cp_head_desc &ds, const void *Hv, const void *Wv, const void *Uv, const void *Gv,
                     float *logp, void *ws, hipStream_t st)
{
    if (ds.T == 0) return CP_HEAD_OK;
    if (!dims_fit(ds)) return CP_HEAD_ERR_UNSUPPORTED;
    const bf16_t *H = (const bf16_t *)Hv, *W = (const bf16_t *)Wv, *U = (const bf16_t *)Uv, *G = (const bf16_t *)Gv;
    const FirstTokenWs f = first_token_ws(ds);
    const int B = (int)ds.T, d = ds.d, V = ds.V, r = ds.r;
    const int rows = B * r, V4 = (int)f.V4;
    float *logw = at<float>(ws, f.logw), *z = at<float>(ws, f.z), *lse = at<float>(ws, f.lse);
    bf16_t *Y = at<bf16_t>(ws, f.Y);
    // first head only: its matrices are the first r blocks of W, so y has rows (b, a); the gate (eq. 7) rides along
    launch_y_with_gate("first_gemm_y", ds, H, W, G, nullptr, Y, logw, nullptr, r, st);
    // the r rows of logits per b are the output's own size: they are stored once (fp32), read once for
    // their log-normalisers and once for the mixture
    launch_z_streamed("first_gemm_z", Y, d, rows, U, V, EpiStoreF32{z, (long)V4, rows, V4, 0}, st);
    ProfileScope prof("first_mix", (double)rows * V * 8 + (double)B * V * 4, st);
    float2 *part = at<float2>(ws, f.part);
    k_row_stats_f32<<<dim3((unsigned)rows, (unsigned)f.parts), kBlock, 0, st>>>(V, (size_t)V4, f.parts, z, part);
    k_lse_from_parts<<<blocks_for((size_t)rows, kBlock / kWave), kBlock, 0, st>>>((size_t)rows, f.parts, part, lse);
    launch_first_token_mix(ds, z, (size_t)V4, lse, logw, logp, st);                         // eq. 11
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

int fast_draft_sequential(const cp_head_desc &ds, const void *Hv, const void *Wv, const void *Uv, const void *Gv,
                          const float *uniforms, int32_t *tokens, float *logq, void *ws, hipStream_t st)
{
    if (ds.T == 0) return CP_HEAD_OK;
    if (!dims_fit(ds)) return CP_HEAD_ERR_UNSUPPORTED;
    const bf16_t *H = (const bf16_t *)Hv, *W = (const bf16_t *)Wv, *U = (const bf16_t *)Uv, *G = (const bf16_t *)Gv;
    const DraftWs f = draft_ws(ds);
    const int B = (int)ds.T, d = ds.d, V = ds.V, n = ds.n, r = ds.r;
    const size_t M = (size_t)B * n * r;
    float *logw = at<float>(ws, f.logw);
    bf16_t *Y = at<bf16_t>(ws, f.Y);
    float2 *part = at<float2>(ws, f.part);
    launch_y_with_gate("seq_gemm_y", ds, H, W, G, nullptr, Y, logw, nullptr, n * r, st);          // y and the gate (eq. 7)
    int parts, seg_cols;
    z_segments((int)M, V, parts, seg_cols);
    launch_z_streamed("seq_gemm_z", Y, d, (int)M, U, V, EpiRowStats{part, parts, (int)M, V}, st);
    ProfileScope prof("seq_draw", (double)B * n * r * seg_cols * d * 2, st);
    k_draft_sequential<<<(unsigned)B, kSeqBlock, 0, st>>>(d, V, n, r, parts, seg_cols, part, Y, U, logw, uniforms, tokens,
                                                          logq);                                             // eq. 11-13
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

// ------------------------------------------------------------------------------------------
// full heads: loss forward and backward
// ------------------------------------------------------------------------------------------

size_t fast_full_ctx_bytes(const cp_head_desc &ds) { return full_ctx(ds).total; }

int fast_full_loss_fwd(const cp_head_desc &ds, const void *Hv, const void *Fv, const void *Gv, const int32_t *X,
                       float *loss, void *ctx, void *ws, hipStream_t st)
{
    if (ds.T == 0) return CP_HEAD_OK;
    if (!dims_fit(ds)) return CP_HEAD_ERR_UNSUPPORTED;
    const bf16_t *H = (const bf16_t *)Hv, *F = (const bf16_t *)Fv;
    const FullCtx cl = full_ctx(ds);
    const FullFwdWs f = full_fwd_ws(ds);
    const int T = (int)ds.T, d = ds.d, V = ds.V, nr = ds.n * ds.r;
    const size_t M = (size_t)T * nr;
    float *lse = at<float>(ctx, cl.lse), *w = at<float>(ctx, cl.w), *gamma = at<float>(ctx, cl.gamma);
    float *logw = at<float>(ws, f.logw), *C = at<float>(ws, f.C);
    float2 *part = cl.keep ? at<float2>(ctx, cl.zpart) : at<float2>(ws, f.part);
    uint16_t *zs = at<uint16_t>(ctx, cl.zs);
    launch_gate(ds, Hv, Gv, logw, w, st);                                                       // eq. 7
    for (int sa = 0; sa < nr; ++sa) {                                                           // z_sa = F_sa h (eq. 6), statistics
        if (cl.keep)
            launch_gemm_nt<Cfg>("full_gemm_z_stats_keep", H, d, T, F + (size_t)sa * V * d, d, V, d,
                                EpiRowStatsKeep{part + (size_t)sa * T * f.parts, f.parts, T, V,
                                                zs + (size_t)sa * T * cl.Vp, (long)cl.Vp, (int)cl.Vp}, st);
        else
            launch_gemm_nt<Cfg>("full_gemm_z_stats", H, d, T, F + (size_t)sa * V * d, d, V, d,
                                EpiRowStats{part + (size_t)sa * T * f.parts, f.parts, T, V}, st);
    }
    k_full_row_finish<<<blocks_for(M, kBlock / kWave), kBlock, 0, st>>>((size_t)T, d, V, ds.n, ds.r, f.parts, part, H, F, X,
                                                                        lse, C);             // eq. 5, 8
    launch_mixture(ds, logw, C, loss, gamma, -1.f, st);                                         // eq. 9
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

int fast_full_loss_bwd(const cp_head_desc &ds, const void *Hv, const void *Fv, const void *Gv, const int32_t *X,
                       const float *dloss, float scale, const void *ctx, float *dH, float *dF, float *dG, void *ws,
                       hipStream_t st)
{
    const int d = ds.d, V = ds.V, r = ds.r, n = ds.n, nr = n * r;
    if (ds.T == 0) {
        if (dF) launch_fill_zero(dF, (size_t)nr * V * d, st);
        if (dG) launch_fill_zero(dG, (size_t)r * d, st);
        return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
    }
    if (!dims_fit(ds)) return CP_HEAD_ERR_UNSUPPORTED;
    const bf16_t *H = (const bf16_t *)Hv, *F = (const bf16_t *)Fv, *G = (const bf16_t *)Gv;
    const FullCtx cl = full_ctx(ds);
    const FullBwdWs b = full_bwd_ws(ds);
    const size_t T = (size_t)ds.T, M = T * nr;
    const float *lse = at<float>(ctx, cl.lse), *w = at<float>(ctx, cl.w), *gamma = at<float>(ctx, cl.gamma);
    float4 *rowinfo = at<float4>(ws, b.coef);
    float *dg = at<float>(ws, b.dg);
    bf16_t *Ht = at<bf16_t>(ws, b.Ht);
    bf16_t *dZ = at<bf16_t>(ws, b.dZ), *dZt = at<bf16_t>(ws, b.dZt);
    const int Vp = (int)b.Vp, Tp = (int)b.Tp;
    const long ldT = (long)b.ldT, ldM = (long)b.ldM;

    k_full_bwd_coefficients<<<blocks_for(M, kBlock), kBlock, 0, st>>>(T, n, r, w, gamma, lse, dloss, scale, X, rowinfo, dg);
    if (dF) transpose_bf16(H, d, (int)T, d, Ht, ldT, Tp, st);         // Ht[d, Tp]
    int first_chunk = 1;
    for (size_t t0 = 0; t0 < T; t0 += b.chunk) {
        const int Tc = (int)((T - t0 < b.chunk) ? T - t0 : b.chunk);
        const int Tcp = (int)round_up((size_t)Tc, 64);
        const bf16_t *Hc = H + t0 * d;
        for (int sa = 0; sa < nr; ++sa) {
            const bf16_t *Fsa = F + (size_t)sa * V * d;
            // dz (bf16), also transposed, from the kept logits of these positions, or from z_sa recomputed
            if (cl.keep) {
                KeptDzArgs kept{KeptLogits{at<uint16_t>(ctx, cl.zs), at<float2>(ctx, cl.zpart), (long)cl.Vp, cl.parts}, rowinfo, V};
                kept_dz_launch(&kept, nullptr, Tc, Tcp, (size_t)sa * T + t0, dZ, (long)Vp, false, dF ? dZt : nullptr, ldM, st);
            } else {
                launch_gemm_nt<Cfg>("full_gemm_z_dz", Hc, d, Tc, Fsa, d, V, d,
                                    EpiDz{dZ, (long)Vp, dF ? dZt : nullptr, ldM, rowinfo + (size_t)sa * T + t0, Tc, Tcp, V, Vp, 0}, st);
            }
            // dH += dz F_sa   (contraction over the vocabulary; F_sa as it is stored is K-major for this product, and
            // a transposed copy of every head matrix per chunk would cost more than the K-major loop does)
            launch_gemm_nt<CfgNN>("full_gemm_dh", dZ, Vp, Tc, Fsa, d, d, Vp,
                                  EpiStoreF32{dH + t0 * d, (long)d, Tc, d, sa ? 1 : 0}, st, kGroupRowsNarrow, NoSideJob{0}, -1, V);
            // dF_sa += dz^T H   (contraction over the positions of the chunk)
            if (dF)
                launch_gemm_nt<Cfg>("full_gemm_df", dZt, ldM, V, Ht + t0, ldT, d, Tcp,
                                    EpiStoreF32{dF + (size_t)sa * V * d, (long)d, V, d, first_chunk ? 0 : 1}, st,
                                    kGroupRowsNarrow);
        }
        first_chunk = 0;
    }
    k_add_gate_to_dh<<<blocks_for(T * d, kBlock), kBlock, 0, st>>>(T, d, r, G, dg, dH);       // + G^T dg
    if (dG) {
        float *part = at<float>(ws, b.dGpart);
        const unsigned chunks = (unsigned)((T + kGateChunk - 1) / kGateChunk);
        k_dgate_partial<<<dim3(blocks_for((size_t)d, kBlock), chunks), kBlock, 0, st>>>(T, d, r, H, dg, part);
        k_dgate_reduce<<<blocks_for((size_t)r * d, kBlock), kBlock, 0, st>>>((int)chunks, d, r, part, dG);
    }
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

}  // namespace cph

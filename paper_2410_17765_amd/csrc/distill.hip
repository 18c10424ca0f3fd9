// Head-only fine-tuning loss ("Fine tuning", eq. 14 and the discounted sum after it): the matrix-core path
// (bf16, d % 64 == 0, r in {1, 2, 4, 8}) and, at the end of the file, the plain fp32 path for every other shape.
//
// Reading of the paper's open points (the same as the CPU checker's):
//   p^d_k[v] = sum_a qhat^(k)_a P^(k)(v | a),  qhat^(k) = softmax_a(log w_a + sum_{j<k} C_ja)   (eq. 13, true prefix)
//   p^c_k    = softmax(TZ[t,k,:])                                                              (teacher, an input)
//   L_k      = beta KL(p^c_k || p^d_k) - (1 - beta) log p^d_k[x_k],   loss[t] = sum_k disc^(k-1) L_k
//
// The per-token distribution p^d_k is a mixture over the r experts, so its logarithm couples the r head rows
// of one (t, k).  Those rows are adjacent (m = (t n + k) r + a) and, for r in {1, 2, 4, 8}, sit in the four
// accumulator registers a lane holds of one 16x16 block of the MFMA result (and, for r = 8, in two neighbouring
// 16-lane groups):
// the epilogues below form log p^d_k[v] inside the tile, with no logits stored.
//
// Forward:  the per-row part of the training loss (gate, y, statistics of z, lse, C) -> teacher log-normalisers
//           -> expert weights qhat per token -> a second product z = Y U^T whose epilogue accumulates, per row,
//           S_a = sum_v p^c[v] rho_a[v] and, per token, KL(p^c || p^d) -> per-position loss and the row
//           coefficients of the backward pass.
// Backward: a third product whose epilogue writes dz = c1 P - c3 p^c rho + c2 1[v = x] in bf16; everything
//           below dz is the training loss's backward pass.
// With CP_HEAD_KEEP_LOGITS the first product keeps its logits (kept_logits.hpp) and the second and third
// products become HBM-bound passes over them: k_distill_kl_kept and k_dz_from_kept<DistillDzRule>.
#include "gemm_nt.hpp"
#include "kept_logits.hpp"

#include <math.h>

namespace cph {

namespace {

typedef TileCfg<256, 256, 2, 2> Cfg;
constexpr int kBlock = 256;

// ------------------------------------------------------------------------------------------
// small kernels
// ------------------------------------------------------------------------------------------

// log-normaliser of every teacher row TZ[g, :], one block per row
template <typename TT>
__global__ void __launch_bounds__(kBlock) k_teacher_lse(int V, const TT *__restrict__ TZ, float *__restrict__ tlse)
{
    __shared__ float red[kBlock / kWave];
    const size_t g = blockIdx.x;
    const TT *row = TZ + g * V;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float mx = -INFINITY;
    for (int v = threadIdx.x; v < V; v += kBlock) mx = fmaxf(mx, ld_f32(row, v));
    mx = wave_max(mx);
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    float Mx = red[0];
#pragma unroll
    for (int w = 1; w < kBlock / kWave; ++w) Mx = fmaxf(Mx, red[w]);
    __syncthreads();
    float l = 0.f;
    for (int v = threadIdx.x; v < V; v += kBlock) l += expf(ld_f32(row, v) - Mx);
    l = wave_sum(l);
    if (lane == 0) red[wave] = l;
    __syncthreads();
    if (threadIdx.x == 0) {
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < kBlock / kWave; ++w) L += red[w];
        tlse[g] = Mx + logf(L);
    }
}

// Per position: the expert weights of every token's conditional (eq. 13 under the true prefix) and what
// follows from the target column alone.  rowa[m] = {lse, log qhat}; rhox[m] = qhat_a P_a[x] / p^d[x];
// ce[t, k] = -log p^d_k[x_k].  A dropped token (x < 0) gets log qhat = 0, rhox = 0, ce = 0.  r <= MAXR.
template <int MAXR>
__global__ void k_distill_weights(size_t T, int n, int r, const float *__restrict__ logw, const float *__restrict__ C,
                                  const float *__restrict__ lse, const int32_t *__restrict__ X,
                                  float2 *__restrict__ rowa, float *__restrict__ rhox, float *__restrict__ ce)
{
    const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    float q[MAXR];
    for (int a = 0; a < r; ++a) q[a] = logw[t * r + a];
    for (int k = 0; k < n; ++k) {
        const size_t m0 = (t * n + k) * r;
        const int x = X[t * n + k];
        if (x < 0) {
            for (int a = 0; a < r; ++a) { rowa[m0 + a] = make_float2(lse[m0 + a], 0.f); rhox[m0 + a] = 0.f; }
            ce[t * n + k] = 0.f;
            continue;
        }
        float mx = q[0];
        for (int a = 1; a < r; ++a) mx = fmaxf(mx, q[a]);
        float s = 0.f;
        for (int a = 0; a < r; ++a) s += expf(q[a] - mx);
        const float qn = mx + logf(s);
        float px = 0.f;
        for (int a = 0; a < r; ++a) px += expf(q[a] - qn + C[m0 + a]);
        for (int a = 0; a < r; ++a) {
            rowa[m0 + a] = make_float2(lse[m0 + a], q[a] - qn);
            rhox[m0 + a] = expf(q[a] - qn + C[m0 + a]) / px;
            q[a] += C[m0 + a];
        }
        ce[t * n + k] = -logf(px);
    }
}

// sums of the per-tile partial pairs of one row, one wavefront per row
__global__ void __launch_bounds__(kBlock) k_sum_parts(size_t M, int parts, const float2 *__restrict__ part,
                                                      float2 *__restrict__ out)
{
    const size_t m = (size_t)blockIdx.x * (kBlock / kWave) + (threadIdx.x >> 6);
    if (m >= M) return;
    const int lane = threadIdx.x & 63;
    float a = 0.f, b = 0.f;
    for (int p = lane; p < parts; p += kWave) {
        const float2 v = part[m * parts + p];
        a += v.x;
        b += v.y;
    }
    a = wave_sum(a);
    b = wave_sum(b);
    if (lane == 0) out[m] = make_float2(a, b);
}

// Per position: the loss and the row coefficients of the backward pass (for an upstream gradient of one):
//   R_a = beta S_a + (1 - beta) rhox_a,  dq_ka = g_k (qhat_a - R_a),  D_ka = sum_{k' > k} dq_k'a
//   c1[m] = g_k R_a - D_ka,  c2[m] = D_ka - (1 - beta) g_k rhox_a,  c3[t, k] = beta g_k,  dgsum[t, a] = sum_k dq_ka
// with g_k = disc^k for a kept token and 0 for a dropped one.  r <= MAXR.
template <int MAXR>
__global__ void k_distill_finish(size_t T, int n, int r, float beta, float disc, const int32_t *__restrict__ X,
                                 const float2 *__restrict__ rowa, const float *__restrict__ rhox,
                                 const float *__restrict__ ce, const float2 *__restrict__ SK,
                                 float *__restrict__ loss, float *__restrict__ c1, float *__restrict__ c2,
                                 float *__restrict__ c3, float *__restrict__ dgsum)
{
    const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    float D[MAXR];
    for (int a = 0; a < r; ++a) D[a] = 0.f;
    // last token to first, so that D accumulates the tokens after k
    float total = 0.f;
    for (int k = n - 1; k >= 0; --k) {
        const size_t m0 = (t * n + k) * r;
        const bool kept = X[t * n + k] >= 0;
        const float g = !kept ? 0.f : (k == 0 ? 1.f : powf(disc, (float)k));
        if (kept) total += g * (beta * SK[m0].y + (1.f - beta) * ce[t * n + k]);
        for (int a = 0; a < r; ++a) {
            const float R = beta * SK[m0 + a].x + (1.f - beta) * rhox[m0 + a];
            c1[m0 + a] = kept ? g * R - D[a] : 0.f;
            c2[m0 + a] = kept ? D[a] - (1.f - beta) * g * rhox[m0 + a] : 0.f;
            if (kept) D[a] += g * (expf(rowa[m0 + a].y) - R);
        }
        c3[t * n + k] = beta * g;
    }
    for (int a = 0; a < r; ++a) dgsum[t * r + a] = D[a];
    loss[t] = total;
}

// Backward row information: rowinfo[m] = {lse, log qhat, up c1, up c2}, grp[t n + k] = {tlse, up c3, x, -},
// dg[t, a] = up dgsum[t, a];  up = dloss[t] * scale (or scale)
__global__ void k_distill_bwd_rows(size_t M, int n, int r, const float2 *__restrict__ rowa, const float *__restrict__ c1,
                                   const float *__restrict__ c2, const float *__restrict__ c3,
                                   const float *__restrict__ tlse, const float *__restrict__ dgsum,
                                   const float *__restrict__ dloss, float scale, const int32_t *__restrict__ X,
                                   float4 *__restrict__ rowinfo, float4 *__restrict__ grp, float *__restrict__ dg)
{
    const size_t m = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= M) return;
    const size_t g = m / r, t = g / n;
    const int a = (int)(m % r);
    const float up = dloss ? dloss[t] * scale : scale;
    const float2 ra = rowa[m];
    rowinfo[m] = make_float4(ra.x, ra.y, up * c1[m], up * c2[m]);
    if (a == 0) grp[g] = make_float4(tlse[g], up * c3[g], __int_as_float(X[g]), 0.f);
    if (g % n == 0) dg[t * r + a] = up * dgsum[t * r + a];
}

// ------------------------------------------------------------------------------------------
// epilogues
// ------------------------------------------------------------------------------------------

// log of the mixture over the R experts of a token, for the four registers jj (four consecutive rows) of a block:
// l[jj] = log(qhat_a P_a[v]) of this lane's column; on return lm[jj] = log sum_a exp(l_a) of jj's group.
template <int R>
__device__ __forceinline__ void group_log_mixture(const float (&l)[4], float (&lm)[4])
{
    if (R == 1) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) lm[jj] = l[jj];
    } else if (R == 2) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const float mx = fmaxf(l[2 * p], l[2 * p + 1]);
            const float v = mx + __logf(__expf(l[2 * p] - mx) + __expf(l[2 * p + 1] - mx));
            lm[2 * p] = v;
            lm[2 * p + 1] = v;
        }
    } else {
        float mx = fmaxf(fmaxf(l[0], l[1]), fmaxf(l[2], l[3]));
        if (R == 8) mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));            // the other four rows: neighbouring 16-lane group
        float s = __expf(l[0] - mx) + __expf(l[1] - mx) + __expf(l[2] - mx) + __expf(l[3] - mx);
        if (R == 8) s += __shfl_xor(s, 16, kWave);
        const float v = mx + __logf(s);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) lm[jj] = v;
    }
}

// Second forward product: per row S_a = sum_v p^c[v] rho_a[v] and per token KL(p^c || p^d), as per-tile
// partial sums {S, KL} in part[M, parts] (every row of a token carries the token's KL).
template <int R>
struct EpiDistillStats {
    float2 *part;
    int parts;
    const float2 *rowa;      // [M] {lse, log qhat}
    const bf16_t *TZ;        // [M / R, V]
    const float *tlse;       // [M / R]
    int M, V;
    template <class C>
    __device__ void run(f32x4_t (&acc)[C::TM16][C::TN16], int row0, int col0, int lane, int wave, int tn, char *smem) const
    {
        const int slot = tn * C::WN + (wave % C::WN);
        // {lse, log qhat, teacher log-normaliser} of the tile's BM rows: one coalesced load, one row per thread, parked
        // in LDS (the operand stages are free by now); loaded per block they were a chain of exposed cache misses
        static_assert(C::THREADS >= C::BM, "one row per thread");
        float4 *linfo = reinterpret_cast<float4 *>(smem);
        {
            const int trow = min(row0 - (wave / C::WN) * C::WTM + (int)threadIdx.x, M - 1);
            const float2 ra = rowa[trow];
            const float tl = tlse[trow / R];
            __syncthreads();                                // every wavefront is done reading operand tiles
            if ((int)threadIdx.x < C::BM) linfo[threadIdx.x] = make_float4(ra.x, ra.y, tl, 0.f);
            __syncthreads();
        }
        const float4 *winfo = linfo + (wave / C::WN) * C::WTM;
#pragma unroll
        for (int i = 0; i < C::TM16; ++i) {
            const int lbase = 16 * i + 4 * (lane >> 4);
            const int rbase = row0 + lbase;
            float lse_[4], lq_[4], tl_[4];
            size_t trow_[4];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int rc = min(rbase + jj, M - 1);
                const float4 ri = winfo[lbase + jj];
                lse_[jj] = ri.x;
                lq_[jj] = ri.y;
                tl_[jj] = ri.z;
                trow_[jj] = (size_t)(rc / R) * V;
            }
            float S[4] = {0.f, 0.f, 0.f, 0.f}, KL[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < C::TN16; ++j) {
                const int col = col0 + acc_col(j, lane);
                const bool cv = col < V;
                const int cc = cv ? col : V - 1;
                float l[4], lm[4];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) l[jj] = acc[i][j][jj] - lse_[jj] + lq_[jj];
                group_log_mixture<R>(l, lm);
                float lpc[4];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    if (R >= 4 && jj > 0) lpc[jj] = lpc[0];                      // one token per four rows
                    else if (R == 2 && (jj & 1)) lpc[jj] = lpc[jj - 1];
                    else lpc[jj] = bf16_to_f32(TZ[trow_[jj] + cc]) - tl_[jj];
                }
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const float pc = cv ? __expf(lpc[jj]) : 0.f;
                    S[jj] += pc * __expf(l[jj] - lm[jj]);
                    KL[jj] += pc * (lpc[jj] - lm[jj]);
                }
            }
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const float s = row16_sum(S[jj]), kl = row16_sum(KL[jj]);
                const int row = rbase + jj;
                if ((lane & 15) == 0 && row < M) part[(size_t)row * parts + slot] = make_float2(s, kl);
            }
        }
    }
};

// Third product (backward): dz = c1 P - c3 p^c rho + c2 1[v = x] in bf16, row-major and transposed.
template <int R>
struct EpiDzDistill {
    bf16_t *dZ;
    long ldz;
    bf16_t *dZt;             // or null
    long ldzt;
    const float4 *rowinfo;   // chunk-relative [Mc] {lse, log qhat, c1, c2} (upstream gradient folded in)
    const float4 *grp;       // chunk-relative [Mc / R] {tlse, c3, target as int bits, -}
    const bf16_t *TZ;        // chunk-relative [Mc / R, V]; Mc / R * V < 2^31
    int Mc, Mcp, V, Vp;
    int blocked;             // dZ is stored block by block (blocked64_index)
    template <class C>
    __device__ void run(f32x4_t (&acc)[C::TM16][C::TN16], int row0, int col0, int lane, int wave, int, char *smem) const
    {
        static_assert(C::WTM == 64 || C::WTM == 128, "sub-tiles of 64 or 128 rows");
        constexpr int RG = R < 4 ? R : 4;        // rows of one token among the four registers of a block
        constexpr int NG = 4 / RG;               // tokens among them
        auto dz = [&](int i, int j, int v, int, int) { return f32_to_bf16(acc[i][j][v]); };
        // The row values of the tile's BM rows and the token values of each row's token come in with one coalesced
        // load each, one row per thread, and are parked in the last BM * 32 bytes of the LDS buffer, beyond every
        // staging area of the stores below: loaded where they are used, they were a chain of exposed cache misses.
        static_assert(C::THREADS >= C::BM, "one row per thread");
        static_assert(C::WM * C::WN * C::WTN * (64 * 2 + 16) <= C::LDS_BYTES - C::BM * 32, "row values beyond the staging areas");
        float4 *linfo = reinterpret_cast<float4 *>(smem + C::LDS_BYTES - C::BM * 32), *lgrp = linfo + C::BM;
        {
            const int trow = row0 - (wave / C::WN) * C::WTM + (int)threadIdx.x;   // this thread's row of the tile
            const int crow = trow < Mc ? trow : Mc - 1;
            const float4 mine = rowinfo[crow], gmine = grp[crow / R];
            __syncthreads();                                // every wavefront is done reading operand tiles
            if ((int)threadIdx.x < C::BM) {
                linfo[threadIdx.x] = mine;
                lgrp[threadIdx.x] = gmine;
            }
            __syncthreads();
        }
        const float4 *winfo = linfo + (wave / C::WN) * C::WTM, *wgrp = lgrp + (wave / C::WN) * C::WTM;
        // 64 rows at a time: turn their logits into gradients and write them out at once, so that the
        // finished values do not stay in registers
        convert<C, RG, NG, 0>(acc, row0, col0, lane, winfo, wgrp);
        store_tile_bf16<C, decltype(dz), 0, 2>(smem, wave, lane, row0, col0, Mc, Vp, dZ, ldz, dz, blocked != 0);
        if (dZt) store_tile_bf16_transposed<C, decltype(dz), 0, 1>(smem, wave, lane, row0, col0, Mcp, V, dZt, ldzt, dz);
        if (C::WTM > 64) {
            convert<C, RG, NG, 1>(acc, row0, col0, lane, winfo, wgrp);
            store_tile_bf16<C, decltype(dz), 2, 4>(smem, wave, lane, row0, col0, Mc, Vp, dZ, ldz, dz, blocked != 0);
            if (dZt) store_tile_bf16_transposed<C, decltype(dz), 1, 2>(smem, wave, lane, row0, col0, Mcp, V, dZt, ldzt, dz);
        }
    }

    // logits -> gradients, in place, for the 16-row blocks 4 IP .. 4 IP + 3
    template <class C, int RG, int NG, int IP>
    __device__ __forceinline__ void convert(f32x4_t (&acc)[C::TM16][C::TN16], int row0, int col0, int lane,
                                            const float4 *winfo, const float4 *wgrp) const
    {
        const bf16_t *__restrict__ tz = TZ;
#pragma unroll
        for (int i = 4 * IP; i < 4 * IP + 4; ++i) {
            const int lbase = 16 * i + 4 * (lane >> 4);      // first of the lane's four rows, in the sub-tile
            const int rbase = row0 + lbase;
            float lse_[4], lq_[4], c1_[4], c2_[4];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int row = rbase + jj;
                const float4 ri = winfo[lbase + jj];         // rows past the chunk hold the last row's values
                lse_[jj] = ri.x;
                lq_[jj] = ri.y;
                c1_[jj] = row < Mc ? ri.z : 0.f;
                c2_[jj] = row < Mc ? ri.w : 0.f;
            }
            float tl_[NG], c3_[NG];
            int x_[NG], toff_[NG];
#pragma unroll
            for (int gi = 0; gi < NG; ++gi) {
                const int row = rbase + gi * RG;
                const int g = min(row, Mc - 1) / R;
                const float4 gv = wgrp[lbase + gi * RG];
                tl_[gi] = gv.x;
                c3_[gi] = row < Mc ? gv.y : 0.f;
                x_[gi] = __float_as_int(gv.z);
                toff_[gi] = g * V;
            }
#pragma unroll
            for (int j = 0; j < C::TN16; ++j) {
                const int col = col0 + acc_col(j, lane);
                const bool cv = col < V;
                const int cc = cv ? col : V - 1;
                float l[4], lm[4];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) l[jj] = acc[i][j][jj] - lse_[jj] + lq_[jj];
                group_log_mixture<R>(l, lm);
#pragma unroll
                for (int gi = 0; gi < NG; ++gi) {
                    const float lpc = bf16_to_f32(tz[toff_[gi] + cc]) - tl_[gi];
#pragma unroll
                    for (int e = 0; e < RG; ++e) {
                        const int jj = gi * RG + e;
                        const float P = __expf(l[jj] - lq_[jj]);
                        const float g = c1_[jj] * P - c3_[gi] * __expf(lpc + l[jj] - lm[jj]) + (col == x_[gi] ? c2_[jj] : 0.f);
                        acc[i][j][jj] = cv ? g : 0.f;
                    }
                }
            }
            // keeps the row loads of later blocks from being hoisted (they would spill registers)
            asm volatile("" ::: "memory");
        }
    }
};

// ------------------------------------------------------------------------------------------
// the same two passes over kept logits
// ------------------------------------------------------------------------------------------

// teacher logits of 8 consecutive columns; columns from V on read as the last valid one (and are not used)
__device__ __forceinline__ void load_teacher8(const bf16_t *__restrict__ trow, int col, int V, float (&tz)[8])
{
    const bf16_t *p = trow + col;
    if (col + 8 <= V && (reinterpret_cast<uintptr_t>(p) & 15u) == 0) {
        const u32x4_t raw = *reinterpret_cast<const u32x4_t *>(p);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            tz[2 * k] = __uint_as_float(raw[k] << 16);
            tz[2 * k + 1] = __uint_as_float(raw[k] & 0xFFFF0000u);
        }
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) tz[k] = bf16_to_f32(trow[col + k < V ? col + k : V - 1]);
    }
}

template <int R>
__device__ __forceinline__ float log_mixture(const float (&l)[R])
{
    float mx = l[0];
#pragma unroll
    for (int a = 1; a < R; ++a) mx = fmaxf(mx, l[a]);
    float s = 0.f;
#pragma unroll
    for (int a = 0; a < R; ++a) s += __expf(l[a] - mx);
    return mx + __logf(s);
}

// What EpiDistillStats accumulates, from the kept logits: one workgroup per token g, a thread takes 8 columns
// of the token's R rows at a time; SK[g R + a] = {S_a, KL}.
template <int R>
__global__ void __launch_bounds__(kBlock) k_distill_kl_kept(KeptLogits kept, int V, int Vp, const float2 *__restrict__ rowa,
                                                            const bf16_t *__restrict__ TZ, const float *__restrict__ tlse,
                                                            float2 *__restrict__ SK)
{
    __shared__ float red[kBlock / kWave][R + 1];
    const size_t g = blockIdx.x;
    float lse_[R], lq_[R], S[R];
#pragma unroll
    for (int a = 0; a < R; ++a) {
        const float2 ra = rowa[g * R + a];
        lse_[a] = ra.x;
        lq_[a] = ra.y;
        S[a] = 0.f;
    }
    const float tl = tlse[g];
    const bf16_t *trow = TZ + g * (size_t)V;
    float kl = 0.f;
    for (int col = (int)threadIdx.x * 8; col < Vp && col < V; col += kBlock * 8) {
        float lp[R][8], tz[8];
#pragma unroll
        for (int a = 0; a < R; ++a) kept_log_probs(kept, g * R + a, col, lse_[a], lp[a]);
        load_teacher8(trow, col, V, tz);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            if (col + k >= V) continue;
            float l[R];
#pragma unroll
            for (int a = 0; a < R; ++a) l[a] = lp[a][k] + lq_[a];
            const float lm = log_mixture<R>(l);
            const float lpc = tz[k] - tl;
            const float pc = __expf(lpc);
            kl += pc * (lpc - lm);
#pragma unroll
            for (int a = 0; a < R; ++a) S[a] += pc * __expf(l[a] - lm);
        }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    kl = wave_sum(kl);
#pragma unroll
    for (int a = 0; a < R; ++a) S[a] = wave_sum(S[a]);
    if (lane == 0) {
#pragma unroll
        for (int a = 0; a < R; ++a) red[wave][a] = S[a];
        red[wave][R] = kl;
    }
    __syncthreads();
    if ((int)threadIdx.x < R) {
        float s = 0.f, k = 0.f;
        for (int w = 0; w < kBlock / kWave; ++w) {
            s += red[w][threadIdx.x];
            k += red[w][R];
        }
        SK[g * R + threadIdx.x] = make_float2(s, k);
    }
}

// The gradient of EpiDzDistill for a thread's rows of k_dz_from_kept: whole tokens (R rows each; a chunk starts
// and ends on a token).  rowinfo {lse, log qhat, c1, c2}; grp and TZ chunk-relative as for EpiDzDistill.
template <int R>
struct DistillDzRule {
    static constexpr int RT = R < 2 ? 2 : R;
    const float4 *grp;
    const bf16_t *TZ;
    __device__ __forceinline__ void operator()(int row, int nrows, int col, int V, const float4 (&info)[RT],
                                               const float (&lp)[RT][8], float (&g)[RT][8]) const
    {
#pragma unroll
        for (int gi = 0; gi < RT / R; ++gi) {
            if (gi * R >= nrows) continue;
            const size_t tok = (size_t)(row / R + gi);
            const float4 gv = grp[tok];
            const float tl = gv.x, c3 = gv.y;
            const int x = __float_as_int(gv.z) - col;
            float tz[8];
            load_teacher8(TZ + tok * (size_t)V, col, V, tz);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (col + k >= V) continue;
                float l[R];
#pragma unroll
                for (int e = 0; e < R; ++e) l[e] = lp[gi * R + e][k] + info[gi * R + e].y;
                const float lm = log_mixture<R>(l);
                const float lpc = tz[k] - tl;
#pragma unroll
                for (int e = 0; e < R; ++e) {
                    const int h = gi * R + e;
                    g[h][k] = info[h].z * __expf(lp[h][k]) - c3 * __expf(lpc + l[e] - lm) + (x == k ? info[h].w : 0.f);
                }
            }
        }
    }
};

// ------------------------------------------------------------------------------------------
// buffers
// ------------------------------------------------------------------------------------------

// ctx: the training loss's ctx, then {rowa [M] float2, c1 [M], c2 [M], c3 [T n], tlse [T n], dgsum [T r]}
struct DistillCtx {
    size_t base, rowa, c1, c2, c3, tlse, dgsum, total;
};
bool on_matrix_cores(const cp_head_desc &ds)
{
    return use_fast_path(ds) && (ds.r == 1 || ds.r == 2 || ds.r == 4 || ds.r == 8);
}
}  // namespace
bool distill_on_matrix_cores(const cp_head_desc &ds) { return on_matrix_cores(ds); }
namespace {
DistillCtx distill_ctx(const cp_head_desc &ds)
{
    DistillCtx c;
    const size_t M = (size_t)ds.T * ds.n * ds.r, Tn = (size_t)ds.T * ds.n, Tr = (size_t)ds.T * ds.r;
    size_t off = ctx_layout(ds, on_matrix_cores(ds)).total;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    c.base = 0;
    c.rowa = take(M * 8);
    c.c1 = take(M * 4);
    c.c2 = take(M * 4);
    c.c3 = take(Tn * 4);
    c.tlse = take(Tn * 4);
    c.dgsum = take(Tr * 4);
    c.total = off;
    return c;
}

// forward workspace: the training loss's, then {rhox [M], ce [T n], SK [M] float2, part [M, parts] float2}
struct DistillFwdWs {
    size_t rhox, ce, SK, part, total;
    int parts;
};
DistillFwdWs distill_fwd_ws(const cp_head_desc &ds)
{
    DistillFwdWs f;
    const size_t M = (size_t)ds.T * ds.n * ds.r, Tn = (size_t)ds.T * ds.n;
    f.parts = ((ds.V + Cfg::BN - 1) / Cfg::BN) * Cfg::WN;
    size_t off = align_up(fast_workspace_bytes(ds, CP_HEAD_OP_LOSS_FWD));
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    f.rhox = take(M * 4);
    f.ce = take(Tn * 4);
    f.SK = take(M * 8);
    f.part = (ds.flags & CP_HEAD_KEEP_LOGITS) ? off : take(M * f.parts * sizeof(float2));   // no second product then
    f.total = off;
    return f;
}

// backward workspace: the training loss's, then {rowinfo [M] float4, grp [T n] float4, dg [T r]}
struct DistillBwdWs {
    size_t rowinfo, grp, dg, total;
};
DistillBwdWs distill_bwd_ws(const cp_head_desc &ds)
{
    DistillBwdWs b;
    const size_t M = (size_t)ds.T * ds.n * ds.r, Tn = (size_t)ds.T * ds.n, Tr = (size_t)ds.T * ds.r;
    size_t off = align_up(fast_workspace_bytes(ds, CP_HEAD_OP_LOSS_BWD));
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    b.rowinfo = take(M * 16);
    b.grp = take(Tn * 16);
    b.dg = take(Tr * 4);
    b.total = off;
    return b;
}

template <int R>
void launch_stats(const cp_head_desc &ds, const bf16_t *Y, const bf16_t *U, float2 *part, int parts,
                  const float2 *rowa, const bf16_t *TZ, const float *tlse, hipStream_t st)
{
    const int M = (int)((size_t)ds.T * ds.n * ds.r);
    launch_gemm_nt<Cfg>("distill_gemm_z_kl", Y, ds.d, M, U, ds.d, ds.V, ds.d,
                        EpiDistillStats<R>{part, parts, rowa, TZ, tlse, M, ds.V}, st);
}

struct DistillDzArgs {
    const bf16_t *U, *TZ;
    const float4 *rowinfo, *grp;
    int d, V, r;
};
template <int R>
void distill_dz_launch(void *user, const bf16_t *Yc, int Mc, int Mcp, size_t m0, bf16_t *dZ, long ldz, bool dz_blocked,
                       bf16_t *dZt, long ldzt, hipStream_t st)
{
    const DistillDzArgs *a = static_cast<const DistillDzArgs *>(user);
    launch_gemm_nt<Cfg>("distill_gemm_z_dz", Yc, a->d, Mc, a->U, a->d, a->V, a->d,
                        EpiDzDistill<R>{dZ, ldz, dZt, ldzt, a->rowinfo + m0, a->grp + m0 / R, a->TZ + (m0 / R) * a->V, Mc, Mcp,
                                        a->V, (int)ldz, dz_blocked ? 1 : 0},
                        st);
}

template <int R>
void launch_kl_kept(const cp_head_desc &ds, const KeptLogits &kept, const float2 *rowa, const bf16_t *TZ, const float *tlse,
                    float2 *SK, hipStream_t st)
{
    const size_t Tn = (size_t)ds.T * ds.n;
    // algorithmic traffic: kept logits and teacher logits read once
    ProfileScope scope("distill_kl_kept", ((double)Tn * R * kept.ld + (double)Tn * ds.V) * 2.0, st);
    k_distill_kl_kept<R><<<(unsigned)Tn, kBlock, 0, st>>>(kept, ds.V, (int)kept.ld, rowa, TZ, tlse, SK);
}

struct DistillKeptArgs {
    KeptLogits kept;
    const bf16_t *TZ;
    const float4 *rowinfo, *grp;
    int V;
};
template <int R>
void distill_kept_dz_launch(void *user, const bf16_t *, int Mc, int Mcp, size_t m0, bf16_t *dZ, long ldz, bool dz_blocked,
                            bf16_t *dZt, long ldzt, hipStream_t st)
{
    const DistillKeptArgs *a = static_cast<const DistillKeptArgs *>(user);
    launch_dz_from_kept(a->kept, m0, a->rowinfo + m0, DistillDzRule<R>{a->grp + m0 / R, a->TZ + (m0 / R) * a->V}, Mc, Mcp,
                        a->V, dZ, ldz, dz_blocked, dZt, ldzt, st);
}

int mfma_distill_fwd(const cp_head_desc &ds, const void *H, const void *W, const void *Uv, const void *G,
                     const int32_t *X, const void *TZv, float beta, float disc, float *loss, void *ctx, void *ws,
                     hipStream_t st)
{
    if (ds.T == 0) return CP_HEAD_OK;
    FastFwdBuffers fb;
    const int rc = fast_fwd_rows(ds, H, W, Uv, G, X, ctx, ws, &fb, st);      // gate, y, statistics, lse, C (eq. 5-8)
    if (rc != CP_HEAD_OK) return rc;
    const bf16_t *U = (const bf16_t *)Uv, *TZ = (const bf16_t *)TZv;
    const DistillCtx dc = distill_ctx(ds);
    const DistillFwdWs f = distill_fwd_ws(ds);
    const size_t T = (size_t)ds.T, M = T * ds.n * ds.r, Tn = T * ds.n;
    float2 *rowa = at<float2>(ctx, dc.rowa);
    float *c1 = at<float>(ctx, dc.c1), *c2 = at<float>(ctx, dc.c2), *c3 = at<float>(ctx, dc.c3);
    float *tlse = at<float>(ctx, dc.tlse), *dgsum = at<float>(ctx, dc.dgsum);
    float *rhox = at<float>(ws, f.rhox), *ce = at<float>(ws, f.ce);
    float2 *SK = at<float2>(ws, f.SK), *part = at<float2>(ws, f.part);

    k_teacher_lse<bf16_t><<<(unsigned)Tn, kBlock, 0, st>>>(ds.V, TZ, tlse);
    k_distill_weights<8><<<blocks_for(T, kBlock), kBlock, 0, st>>>(T, ds.n, ds.r, fb.logw, fb.C, fb.lse, X, rowa, rhox, ce);
    const CtxLayout cl = ctx_layout(ds, true);
    if (cl.keep) {
        const KeptLogits kept{at<uint16_t>(ctx, cl.zs), at<float2>(ctx, cl.zpart), (long)cl.Vp, cl.parts};
        switch (ds.r) {
        case 1: launch_kl_kept<1>(ds, kept, rowa, TZ, tlse, SK, st); break;
        case 2: launch_kl_kept<2>(ds, kept, rowa, TZ, tlse, SK, st); break;
        case 4: launch_kl_kept<4>(ds, kept, rowa, TZ, tlse, SK, st); break;
        default: launch_kl_kept<8>(ds, kept, rowa, TZ, tlse, SK, st); break;
        }
    } else {
        switch (ds.r) {
        case 1: launch_stats<1>(ds, fb.Y, U, part, f.parts, rowa, TZ, tlse, st); break;
        case 2: launch_stats<2>(ds, fb.Y, U, part, f.parts, rowa, TZ, tlse, st); break;
        case 4: launch_stats<4>(ds, fb.Y, U, part, f.parts, rowa, TZ, tlse, st); break;
        default: launch_stats<8>(ds, fb.Y, U, part, f.parts, rowa, TZ, tlse, st); break;
        }
        k_sum_parts<<<blocks_for(M, kBlock / kWave), kBlock, 0, st>>>(M, f.parts, part, SK);
    }
    k_distill_finish<8><<<blocks_for(T, kBlock), kBlock, 0, st>>>(T, ds.n, ds.r, beta, disc, X, rowa, rhox, ce, SK, loss, c1,
                                                                  c2, c3, dgsum);
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

int mfma_distill_bwd(const cp_head_desc &ds, const void *H, const void *W, const void *Uv, const void *G,
                     const int32_t *X, const void *TZv, const float *dloss, float scale, const void *ctx, float *dH,
                     float *dW, float *dU, float *dG, void *ws, hipStream_t st)
{
    const size_t nrd = (size_t)ds.n * ds.r * ds.d;
    if (ds.T == 0) {
        launch_fill_zero(dW, nrd * ds.d, st);
        launch_fill_zero(dU, (size_t)ds.V * ds.d, st);
        launch_fill_zero(dG, (size_t)ds.r * ds.d, st);
        return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
    }
    if (!fast_dims_fit(ds)) return CP_HEAD_ERR_UNSUPPORTED;
    const DistillCtx dc = distill_ctx(ds);
    const DistillBwdWs b = distill_bwd_ws(ds);
    const CtxLayout cl = ctx_layout(ds, true);
    const size_t M = (size_t)ds.T * ds.n * ds.r;
    const float2 *rowa = at<float2>(ctx, dc.rowa);
    const float *c1 = at<float>(ctx, dc.c1), *c2 = at<float>(ctx, dc.c2), *c3 = at<float>(ctx, dc.c3);
    const float *tlse = at<float>(ctx, dc.tlse), *dgsum = at<float>(ctx, dc.dgsum);
    float4 *rowinfo = at<float4>(ws, b.rowinfo), *grp = at<float4>(ws, b.grp);
    float *dg = at<float>(ws, b.dg);
    k_distill_bwd_rows<<<blocks_for(M, kBlock), kBlock, 0, st>>>(M, ds.n, ds.r, rowa, c1, c2, c3, tlse, dgsum, dloss, scale, X,
                                                                 rowinfo, grp, dg);
    if (cl.keep) {
        DistillKeptArgs kargs{KeptLogits{at<uint16_t>(ctx, cl.zs), at<float2>(ctx, cl.zpart), (long)cl.Vp, cl.parts},
                              (const bf16_t *)TZv, rowinfo, grp, ds.V};
        FastDzLaunch kfn = ds.r == 1 ? distill_kept_dz_launch<1> : ds.r == 2 ? distill_kept_dz_launch<2>
                         : ds.r == 4 ? distill_kept_dz_launch<4> : distill_kept_dz_launch<8>;
        return fast_bwd_from_dz(ds, H, W, Uv, G, at<bf16_t>(ctx, cl.Y), dg, dH, dW, dU, dG, ws, kfn, &kargs, st);
    }
    DistillDzArgs args{(const bf16_t *)Uv, (const bf16_t *)TZv, rowinfo, grp, ds.d, ds.V, ds.r};
    FastDzLaunch fn = ds.r == 1 ? distill_dz_launch<1> : ds.r == 2 ? distill_dz_launch<2>
                    : ds.r == 4 ? distill_dz_launch<4> : distill_dz_launch<8>;
    return fast_bwd_from_dz(ds, H, W, Uv, G, at<bf16_t>(ctx, cl.Y), dg, dH, dW, dU, dG, ws, fn, &args, st);
}


// ------------------------------------------------------------------------------------------
// plain fp32 path: any r <= 64, any d, fp32 or bf16 storage.  The logits of one chunk of rows are written
// out in fp32 and the per-token mixture is formed from them by one block per token.
// ------------------------------------------------------------------------------------------
constexpr int kMaxRank = 64;

// One block per token g = g0 + blockIdx.x of the chunk whose logits are zc[(gi r + a), V]:
// SK[g r + a] = {S_a, KL} with S_a = sum_v p^c[v] rho_a[v], KL = sum_v p^c[v] (log p^c[v] - log p^d[v]).
// Lane a of every wavefront accumulates S_a (r <= 64).
template <typename TT>
__global__ void __launch_bounds__(kBlock) k_distill_kl_plain(int V, int r, size_t g0, const float *__restrict__ zc,
                                                             const float2 *__restrict__ rowa, const TT *__restrict__ TZ,
                                                             const float *__restrict__ tlse, float2 *__restrict__ SK)
{
    __shared__ float lse_s[kMaxRank], lq_s[kMaxRank], S_s[kBlock / kWave][kMaxRank], kl_s[kBlock / kWave];
    const size_t gi = blockIdx.x, g = g0 + gi;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if ((int)threadIdx.x < r) {
        const float2 ra = rowa[g * r + threadIdx.x];
        lse_s[threadIdx.x] = ra.x;
        lq_s[threadIdx.x] = ra.y;
    }
    __syncthreads();
    const float tl = tlse[g];
    const float *zrow = zc + gi * r * (size_t)V;
    const TT *trow = TZ + g * (size_t)V;
    float Sacc = 0.f, kl = 0.f;
    // every lane of a wavefront runs the same number of rounds, so that the sums over lanes see all of them
    for (int v0 = wave * kWave; v0 < V; v0 += kBlock) {
        const int v = v0 + lane;
        const bool cv = v < V;
        const int vc = cv ? v : V - 1;
        float mx = -INFINITY;
        for (int a = 0; a < r; ++a) mx = fmaxf(mx, zrow[(size_t)a * V + vc] - lse_s[a] + lq_s[a]);
        float sum = 0.f;
        for (int a = 0; a < r; ++a) sum += expf(zrow[(size_t)a * V + vc] - lse_s[a] + lq_s[a] - mx);
        const float lm = mx + logf(sum);
        const float lpc = ld_f32(trow, (size_t)vc) - tl;
        const float pc = cv ? expf(lpc) : 0.f;
        kl += pc * (lpc - lm);
        for (int a = 0; a < r; ++a) {
            const float s = wave_sum(pc * expf(zrow[(size_t)a * V + vc] - lse_s[a] + lq_s[a] - lm));
            if (lane == a) Sacc += s;
        }
    }
    kl = wave_sum(kl);
    S_s[wave][lane] = Sacc;
    if (lane == 0) kl_s[wave] = kl;
    __syncthreads();
    if ((int)threadIdx.x < r) {
        float S = 0.f, K = 0.f;
        for (int w = 0; w < kBlock / kWave; ++w) { S += S_s[w][threadIdx.x]; K += kl_s[w]; }
        SK[g * r + threadIdx.x] = make_float2(S, K);
    }
}

// One block per token of the chunk: the chunk's logits in dZ become, in place,
// dz = c1 P - c3 p^c rho + c2 1[v = x] (every entry is read and written by the same thread).
template <typename TT>
__global__ void __launch_bounds__(kBlock) k_distill_dz_plain(int V, int r, size_t g0, float *__restrict__ dZ,
                                                             const float4 *__restrict__ rowinfo,
                                                             const float4 *__restrict__ grp, const TT *__restrict__ TZ)
{
    __shared__ float4 ri_s[kMaxRank];
    const size_t gi = blockIdx.x, g = g0 + gi;
    if ((int)threadIdx.x < r) ri_s[threadIdx.x] = rowinfo[g * r + threadIdx.x];
    __syncthreads();
    const float4 gv = grp[g];
    const float tl = gv.x, c3 = gv.y;
    const int x = __float_as_int(gv.z);
    float *zrow = dZ + gi * r * (size_t)V;
    const TT *trow = TZ + g * (size_t)V;
    for (int v = threadIdx.x; v < V; v += kBlock) {
        float mx = -INFINITY;
        for (int a = 0; a < r; ++a) mx = fmaxf(mx, zrow[(size_t)a * V + v] - ri_s[a].x + ri_s[a].y);
        float sum = 0.f;
        for (int a = 0; a < r; ++a) sum += expf(zrow[(size_t)a * V + v] - ri_s[a].x + ri_s[a].y - mx);
        const float lm = mx + logf(sum);
        const float lpc = ld_f32(trow, (size_t)v) - tl;
        for (int a = 0; a < r; ++a) {
            const float4 ri = ri_s[a];
            const float lP = zrow[(size_t)a * V + v] - ri.x;
            zrow[(size_t)a * V + v] = ri.z * expf(lP) - c3 * expf(lpc + lP + ri.y - lm) + (v == x ? ri.w : 0.f);
        }
    }
}

// forward workspace: the plain training loss's, then {rhox [M], ce [T n], SK [M] float2, zc [chunk, V]}
struct PlainFwdWs {
    size_t rhox, ce, SK, zc, total;
};
PlainFwdWs plain_fwd_ws(const cp_head_desc &ds)
{
    PlainFwdWs f;
    const size_t M = (size_t)ds.T * ds.n * ds.r, Tn = (size_t)ds.T * ds.n;
    size_t off = align_up(generic_workspace_bytes(ds, CP_HEAD_OP_LOSS_FWD));
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    f.rhox = take(M * 4);
    f.ce = take(Tn * 4);
    f.SK = take(M * 8);
    f.zc = take(generic_bwd_chunk_rows(ds) * ds.V * 4);
    f.total = off;
    return f;
}
DistillBwdWs plain_bwd_ws(const cp_head_desc &ds)
{
    DistillBwdWs b;
    const size_t M = (size_t)ds.T * ds.n * ds.r, Tn = (size_t)ds.T * ds.n, Tr = (size_t)ds.T * ds.r;
    size_t off = align_up(generic_workspace_bytes(ds, CP_HEAD_OP_LOSS_BWD));
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    b.rowinfo = take(M * 16);
    b.grp = take(Tn * 16);
    b.dg = take(Tr * 4);
    b.total = off;
    return b;
}

template <typename TT>
int plain_distill_fwd(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                      const int32_t *X, const TT *TZ, float beta, float disc, float *loss, void *ctx, void *ws,
                      hipStream_t st)
{
    GenericFwdBuffers fb;
    const int rc = generic_fwd_rows(ds, H, W, U, G, X, ctx, ws, &fb, st);
    if (rc != CP_HEAD_OK) return rc;
    const DistillCtx dc = distill_ctx(ds);
    const PlainFwdWs f = plain_fwd_ws(ds);
    const size_t T = (size_t)ds.T, M = T * ds.n * ds.r, Tn = T * ds.n;
    float2 *rowa = at<float2>(ctx, dc.rowa);
    float *c1 = at<float>(ctx, dc.c1), *c2 = at<float>(ctx, dc.c2), *c3 = at<float>(ctx, dc.c3);
    float *tlse = at<float>(ctx, dc.tlse), *dgsum = at<float>(ctx, dc.dgsum);
    float *rhox = at<float>(ws, f.rhox), *ce = at<float>(ws, f.ce), *zc = at<float>(ws, f.zc);
    float2 *SK = at<float2>(ws, f.SK);
    k_teacher_lse<TT><<<(unsigned)Tn, kBlock, 0, st>>>(ds.V, TZ, tlse);
    k_distill_weights<kMaxRank><<<blocks_for(T, kBlock), kBlock, 0, st>>>(T, ds.n, ds.r, fb.logw, fb.C, fb.lse, X, rowa,
                                                                          rhox, ce);
    const size_t chunk = generic_bwd_chunk_rows(ds);
    for (size_t m0 = 0; m0 < M; m0 += chunk) {
        const size_t Mc = (M - m0 < chunk) ? M - m0 : chunk;
        generic_logits_rows(ds, U, fb.Y, m0, Mc, zc, st);
        k_distill_kl_plain<TT><<<(unsigned)(Mc / ds.r), kBlock, 0, st>>>(ds.V, ds.r, m0 / ds.r, zc, rowa, TZ, tlse, SK);
    }
    k_distill_finish<kMaxRank><<<blocks_for(T, kBlock), kBlock, 0, st>>>(T, ds.n, ds.r, beta, disc, X, rowa, rhox, ce, SK,
                                                                         loss, c1, c2, c3, dgsum);
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

template <typename TT>
struct PlainDzArgs {
    const cp_head_desc *ds;
    const void *U;
    const float *Y;
    const TT *TZ;
    const float4 *rowinfo, *grp;
};
template <typename TT>
void plain_dz_launch(void *user, size_t m0, size_t Mc, float *dZ, hipStream_t st)
{
    const PlainDzArgs<TT> *a = static_cast<const PlainDzArgs<TT> *>(user);
    const cp_head_desc &ds = *a->ds;
    generic_logits_rows(ds, a->U, a->Y, m0, Mc, dZ, st);
    k_distill_dz_plain<TT><<<(unsigned)(Mc / ds.r), kBlock, 0, st>>>(ds.V, ds.r, m0 / ds.r, dZ, a->rowinfo, a->grp, a->TZ);
}

template <typename TT>
int plain_distill_bwd(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                      const int32_t *X, const TT *TZ, const float *dloss, float scale, const void *ctx, float *dH,
                      float *dW, float *dU, float *dG, void *ws, hipStream_t st)
{
    const DistillCtx dc = distill_ctx(ds);
    const DistillBwdWs b = plain_bwd_ws(ds);
    const CtxLayout cl = ctx_layout(ds, false);
    const size_t M = (size_t)ds.T * ds.n * ds.r;
    const float2 *rowa = at<float2>(ctx, dc.rowa);
    const float *c1 = at<float>(ctx, dc.c1), *c2 = at<float>(ctx, dc.c2), *c3 = at<float>(ctx, dc.c3);
    const float *tlse = at<float>(ctx, dc.tlse), *dgsum = at<float>(ctx, dc.dgsum);
    float4 *rowinfo = at<float4>(ws, b.rowinfo), *grp = at<float4>(ws, b.grp);
    float *dg = at<float>(ws, b.dg);
    k_distill_bwd_rows<<<blocks_for(M, kBlock), kBlock, 0, st>>>(M, ds.n, ds.r, rowa, c1, c2, c3, tlse, dgsum, dloss, scale, X,
                                                                 rowinfo, grp, dg);
    PlainDzArgs<TT> args{&ds, U, at<float>(ctx, cl.Y), TZ, rowinfo, grp};
    return generic_bwd_from_dz(ds, H, W, U, G, at<float>(ctx, cl.Y), dg, dH, dW, dU, dG, ws, plain_dz_launch<TT>, &args, st);
}

}  // namespace

// The plain path keeps no logits: there the flag is dropped before any layout is computed.
static cp_head_desc without_kept_logits(cp_head_desc ds)
{
    if (!on_matrix_cores(ds)) ds.flags &= ~CP_HEAD_KEEP_LOGITS;
    return ds;
}

size_t distill_ctx_bytes(const cp_head_desc &ds) { return distill_ctx(without_kept_logits(ds)).total; }
size_t distill_workspace_bytes(const cp_head_desc &ds_in, int op)
{
    const cp_head_desc ds = without_kept_logits(ds_in);
    if (on_matrix_cores(ds)) return op == CP_HEAD_OP_DISTILL_FWD ? distill_fwd_ws(ds).total : distill_bwd_ws(ds).total;
    return op == CP_HEAD_OP_DISTILL_FWD ? plain_fwd_ws(ds).total : plain_bwd_ws(ds).total;
}

int distill_loss_fwd(const cp_head_desc &ds_in, const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X, const void *TZ, float beta, float disc, float *loss, void *ctx, void *ws,
                     hipStream_t st)
{
    const cp_head_desc ds = without_kept_logits(ds_in);
    if (ds.T == 0) return CP_HEAD_OK;
    if (on_matrix_cores(ds)) return mfma_distill_fwd(ds, H, W, U, G, X, TZ, beta, disc, loss, ctx, ws, st);
    if (ds.dtype == CP_HEAD_FP32)
        return plain_distill_fwd<float>(ds, H, W, U, G, X, (const float *)TZ, beta, disc, loss, ctx, ws, st);
    return plain_distill_fwd<bf16_t>(ds, H, W, U, G, X, (const bf16_t *)TZ, beta, disc, loss, ctx, ws, st);
}

int distill_loss_bwd(const cp_head_desc &ds_in, const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X, const void *TZ, const float *dloss, float scale, const void *ctx, float *dH,
                     float *dW, float *dU, float *dG, void *ws, hipStream_t st)
{
    const cp_head_desc ds = without_kept_logits(ds_in);
    if (ds.T == 0) {
        launch_fill_zero(dW, (size_t)ds.n * ds.r * ds.d * ds.d, st);
        launch_fill_zero(dU, (size_t)ds.V * ds.d, st);
        launch_fill_zero(dG, (size_t)ds.r * ds.d, st);
        return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
    }
    if (on_matrix_cores(ds)) return mfma_distill_bwd(ds, H, W, U, G, X, TZ, dloss, scale, ctx, dH, dW, dU, dG, ws, st);
    if (ds.dtype == CP_HEAD_FP32)
        return plain_distill_bwd<float>(ds, H, W, U, G, X, (const float *)TZ, dloss, scale, ctx, dH, dW, dU, dG, ws, st);
    return plain_distill_bwd<bf16_t>(ds, H, W, U, G, X, (const bf16_t *)TZ, dloss, scale, ctx, dH, dW, dU, dG, ws, st);
}

}  // namespace cph

// Plain fp32 path of the CP head: correct for every shape and storage type, no
// tiling.  It serves fp32 storage and shapes the matrix-core path does not take,
// and its per-position bookkeeping kernels (gate, mixture, expert draw) are
// shared with that path.  One thread block per head row (t, s, a) or one thread
// per output element; every sum runs in a fixed order, so results are reproducible.
//
// Head rows are ordered m = (t*n + s)*r + a, so X[m / r] is the row's target and
// m / (n*r) its position.
#include "cp_internal.hpp"

#include <math.h>

#include <algorithm>

namespace cph {

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;


// ------------------------------------------------------------------------------------------
// gate: logw = log_softmax(G h), w = exp(logw)      (eq. 7)
// one wavefront per position; lane a ends up holding g_a
// ------------------------------------------------------------------------------------------
template <typename TIn>
__global__ void __launch_bounds__(kWave) k_gate(int d, int r, const TIn *__restrict__ H, const TIn *__restrict__ G,
                                                float *__restrict__ logw, float *__restrict__ w)
{
    const size_t t = blockIdx.x;
    const int lane = threadIdx.x;
    const TIn *h = H + t * d;
    float mine = -INFINITY;
    for (int a = 0; a < r; ++a) {
        float p = 0.f;
        for (int k = lane; k < d; k += kWave) p += ld_f32(G, (size_t)a * d + k) * ld_f32(h, k);
        p = wave_sum(p);
        if (lane == a) mine = p;
    }
    const float mx = wave_max(mine);
    const float s = wave_sum(lane < r ? expf(mine - mx) : 0.f);
    const float lse = mx + logf(s);
    if (lane < r) {
        logw[t * r + lane] = mine - lse;
        w[t * r + lane] = expf(mine - lse);
    }
}

// ------------------------------------------------------------------------------------------
// y = W_sa h for one head row m = (t, s, a); optional rounding of y to bf16
// ------------------------------------------------------------------------------------------
template <typename TIn>
__global__ void __launch_bounds__(kBlock) k_y_generic(int d, int nr, const TIn *__restrict__ H,
                                                      const TIn *__restrict__ W, float *__restrict__ Y, int round_y)
{
    extern __shared__ float hs[];
    const size_t m = blockIdx.x;
    const size_t t = m / nr;
    const int sa = (int)(m % nr);
    for (int k = threadIdx.x; k < d; k += kBlock) hs[k] = ld_f32(H, t * d + k);
    __syncthreads();
    const TIn *Wsa = W + (size_t)sa * d * d;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    for (int k = wave; k < d; k += kWavesPerBlock) {
        float p = 0.f;
        for (int j = lane; j < d; j += kWave) p += ld_f32(Wsa, (size_t)k * d + j) * hs[j];
        p = wave_sum(p);
        if (lane == 0) Y[m * d + k] = round_y ? bf16_to_f32(f32_to_bf16(p)) : p;
    }
}

// ------------------------------------------------------------------------------------------
// z = U y for one head row; running (max, sum exp) over the vocabulary gives the
// log-normaliser (eq. 5); C = z[x] - lse (eq. 8).  Block b serves row m0 + b; lse and C are indexed by the row,
// z_out (written only if not NULL) by the block.
// ------------------------------------------------------------------------------------------
template <typename TIn>
__global__ void __launch_bounds__(kBlock) k_zstats_generic(int d, int V, int r, size_t m0, const TIn *__restrict__ U,
                                                           const float *__restrict__ Y, const int32_t *__restrict__ X,
                                                           float *__restrict__ lse_out, float *__restrict__ C_out,
                                                           float *__restrict__ z_out)
{
    extern __shared__ float ys[];
    __shared__ float red_m[kWavesPerBlock], red_l[kWavesPerBlock], red_zt;
    const size_t m = m0 + blockIdx.x;
    for (int k = threadIdx.x; k < d; k += kBlock) ys[k] = Y[m * d + k];
    if (threadIdx.x == 0) red_zt = 0.f;
    __syncthreads();
    const int x = X ? X[m / r] : -1;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    float mx = -INFINITY, l = 0.f;
    for (int v = wave; v < V; v += kWavesPerBlock) {
        float p = 0.f;
        for (int k = lane; k < d; k += kWave) p += ld_f32(U, (size_t)v * d + k) * ys[k];
        const float z = wave_sum(p);
        if (z_out && lane == 0) z_out[(size_t)blockIdx.x * V + v] = z;
        if (z > mx) { l = l * expf(mx - z) + 1.f; mx = z; }
        else l += expf(z - mx);
        if (v == x && lane == 0) red_zt = z;
    }
    if (lane == 0) { red_m[wave] = mx; red_l[wave] = l; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float Mx = red_m[0];
        for (int i = 1; i < kWavesPerBlock; ++i) Mx = fmaxf(Mx, red_m[i]);
        float L = 0.f;
        for (int i = 0; i < kWavesPerBlock; ++i) L += red_l[i] * expf(red_m[i] - Mx);
        const float lse = Mx + logf(L);
        if (lse_out) lse_out[m] = lse;
        if (C_out) C_out[m] = (x >= 0) ? red_zt - lse : 0.f;
    }
}

// ------------------------------------------------------------------------------------------
// mixture over experts (eq. 9) and the posterior gamma_a = exp(a_a - L); one wavefront per position
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kWave) k_mixture(int n, int r, const float *__restrict__ logw,
                                                   const float *__restrict__ C, float *__restrict__ loss,
                                                   float *__restrict__ gamma, float sign)
{
    const size_t t = blockIdx.x;
    const int lane = threadIdx.x;
    float a = -INFINITY;
    if (lane < r) {
        a = logw[t * r + lane];
        for (int s = 0; s < n; ++s) a += C[(t * n + s) * r + lane];
    }
    const float mx = wave_max(a);
    const float sum = wave_sum(lane < r ? expf(a - mx) : 0.f);
    const float L = mx + logf(sum);
    if (lane == 0) loss[t] = sign * L;   // -L: the loss; +L: the joint log-probability
    if (gamma && lane < r) gamma[t * r + lane] = expf(a - L);
}

// ------------------------------------------------------------------------------------------
// backward pieces
// ------------------------------------------------------------------------------------------

__global__ void k_fill_zero(size_t count, float *__restrict__ p)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0.f;
}

// dg[t,a] = up_t (w_a - gamma_a): derivative of eq. 9 with respect to the gate pre-activations
__global__ void k_dgate(size_t Tr, int r, const float *__restrict__ w, const float *__restrict__ gamma,
                        const float *__restrict__ dloss, float scale, float *__restrict__ dg)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= Tr) return;
    const float up = dloss ? dloss[i / r] * scale : scale;
    dg[i] = up * (w[i] - gamma[i]);
}

// dz[v] = up_t gamma_a (softmax(z)[v] - 1[v = x]) for the rows m0 .. m0+gridDim.x-1
template <typename TIn>
__global__ void __launch_bounds__(kBlock) k_dz_generic(int d, int V, int n, int r, size_t m0,
                                                       const TIn *__restrict__ U, const float *__restrict__ Y,
                                                       const int32_t *__restrict__ X, const float *__restrict__ lse,
                                                       const float *__restrict__ gamma,
                                                       const float *__restrict__ dloss, float scale,
                                                       float *__restrict__ dZ)
{
    extern __shared__ float ys[];
    const size_t mc = blockIdx.x, m = m0 + mc;
    for (int k = threadIdx.x; k < d; k += kBlock) ys[k] = Y[m * d + k];
    __syncthreads();
    const size_t t = m / ((size_t)n * r);
    const int a = (int)(m % r);
    const int x = X[m / r];
    const float up = dloss ? dloss[t] * scale : scale;
    const float coef = up * gamma[t * r + a];
    const float l = lse[m];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    for (int v = wave; v < V; v += kWavesPerBlock) {
        float p = 0.f;
        for (int k = lane; k < d; k += kWave) p += ld_f32(U, (size_t)v * d + k) * ys[k];
        const float z = wave_sum(p);
        if (lane == 0) dZ[mc * V + v] = (x < 0) ? 0.f : coef * (expf(z - l) - (v == x ? 1.f : 0.f));
    }
}

// dY[m,k] = sum_v dZ[mc,v] U[v,k]
template <typename TIn>
__global__ void __launch_bounds__(kBlock) k_dy_generic(int d, int V, size_t m0, size_t Mc,
                                                       const TIn *__restrict__ U, const float *__restrict__ dZ,
                                                       float *__restrict__ dY)
{
    const size_t idx = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= Mc * d) return;
    const size_t mc = idx / d;
    const int k = (int)(idx % d);
    float acc = 0.f;
    for (int v = 0; v < V; ++v) acc += dZ[mc * V + v] * ld_f32(U, (size_t)v * d + k);
    dY[(m0 + mc) * d + k] = acc;
}

// dU[v,k] (+)= sum_mc dZ[mc,v] Y[m0+mc,k]
__global__ void __launch_bounds__(kBlock) k_du_generic(int d, int V, size_t m0, size_t Mc,
                                                       const float *__restrict__ dZ, const float *__restrict__ Y,
                                                       float *__restrict__ dU, int accumulate)
{
    const size_t idx = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= (size_t)V * d) return;
    const size_t v = idx / d;
    const int k = (int)(idx % d);
    float acc = accumulate ? dU[idx] : 0.f;
    for (size_t mc = 0; mc < Mc; ++mc) acc += dZ[mc * V + v] * Y[(m0 + mc) * d + k];
    dU[idx] = acc;
}

// dW[sa,k,j] = sum_t dY[(t,sa),k] H[t,j]
template <typename TIn>
__global__ void __launch_bounds__(kBlock) k_dw_generic(size_t T, int d, int nr, const TIn *__restrict__ H,
                                                       const float *__restrict__ dY, float *__restrict__ dW)
{
    const size_t idx = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= (size_t)nr * d * d) return;
    const int j = (int)(idx % d);
    const size_t sak = idx / d;
    const size_t sa = sak / d;
    const int k = (int)(sak % d);
    float acc = 0.f;
    for (size_t t = 0; t < T; ++t) acc += dY[(t * nr + sa) * d + k] * ld_f32(H, t * d + j);
    dW[idx] = acc;
}

// dH[t,j] = sum_{sa,k} dY[(t,sa),k] W[sa,k,j] + sum_a dg[t,a] G[a,j]
template <typename TIn>
__global__ void __launch_bounds__(kBlock) k_dh_generic(size_t T, int d, int nr, int r, const TIn *__restrict__ W,
                                                       const TIn *__restrict__ G, const float *__restrict__ dY,
                                                       const float *__restrict__ dg, float *__restrict__ dH)
{
    const size_t idx = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= T * d) return;
    const size_t t = idx / d;
    const int j = (int)(idx % d);
    float acc = 0.f;
    for (int sa = 0; sa < nr; ++sa)
        for (int k = 0; k < d; ++k) acc += dY[(t * nr + sa) * d + k] * ld_f32(W, ((size_t)sa * d + k) * d + j);
    for (int a = 0; a < r; ++a) acc += dg[t * r + a] * ld_f32(G, (size_t)a * d + j);
    dH[idx] = acc;
}

// dG[a,j] = sum_t dg[t,a] H[t,j]
template <typename TIn>
__global__ void __launch_bounds__(kBlock) k_dg_generic(size_t T, int d, int r, const TIn *__restrict__ H,
                                                       const float *__restrict__ dg, float *__restrict__ dG)
{
    const size_t idx = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= (size_t)r * d) return;
    const int a = (int)(idx / d);
    const int j = (int)(idx % d);
    float acc = 0.f;
    for (size_t t = 0; t < T; ++t) acc += dg[t * r + a] * ld_f32(H, t * d + j);
    dG[idx] = acc;
}

// ------------------------------------------------------------------------------------------
// draft pieces
// ------------------------------------------------------------------------------------------

// expert draw: first a with cdf_w[a] > u, running sum in fp64, clamp to r-1
__global__ void k_pick_alpha(size_t B, int n, int r, const float *__restrict__ w, const float *__restrict__ uniforms,
                             int32_t *__restrict__ alpha)
{
    const size_t b = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const double u = (double)uniforms[b * (1 + n)];
    double c = 0.0;
    int pick = r - 1;
    bool found = false;
    for (int a = 0; a < r; ++a) {
        c += (double)w[b * r + a];
        if (!found && c > u) { pick = a; found = true; }
    }
    alpha[b] = pick;
}

// token draw for (b, s) from the stored logits of row (b, s, a*): thread i owns a contiguous
// segment of the vocabulary; segment sums in fp64, then one thread walks the segment sums and
// the owner of the crossing segment walks its tokens.
__global__ void __launch_bounds__(kBlock) k_sample_generic(int V, int n, int r, const float *__restrict__ z,
                                                           const float *__restrict__ lse,
                                                           const int32_t *__restrict__ alpha,
                                                           const float *__restrict__ uniforms,
                                                           int32_t *__restrict__ tokens)
{
    __shared__ double seg_sum[kBlock];
    __shared__ double base;
    __shared__ int chosen;
    const size_t bs = blockIdx.x;            // b*n + s
    const size_t b = bs / n;
    const int s = (int)(bs % n);
    const size_t row = bs * r + alpha[b];
    const float *zr = z + row * V;
    const float l = lse[row];
    const double u = (double)uniforms[b * (1 + n) + 1 + s];
    const int seg = (V + kBlock - 1) / kBlock;
    const int lo = min(V, (int)threadIdx.x * seg), hi = min(V, lo + seg);
    double sum = 0.0;
    for (int v = lo; v < hi; ++v) sum += (double)expf(zr[v] - l);
    seg_sum[threadIdx.x] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        double c = 0.0;
        int pick = -1;
        for (int i = 0; i < kBlock; ++i) {
            if (c + seg_sum[i] > u) { pick = i; break; }
            c += seg_sum[i];
        }
        chosen = pick;
        base = c;
        if (pick < 0) tokens[bs] = V - 1;
    }
    __syncthreads();
    if ((int)threadIdx.x == chosen) {
        double c = base;
        int tok = hi - 1;
        for (int v = lo; v < hi; ++v) {
            c += (double)expf(zr[v] - l);
            if (c > u) { tok = v; break; }
        }
        tokens[bs] = tok;
    }
}

// logq[b] = logsumexp_a( logw_a + sum_s (z_sa[tok_s] - lse_sa) )    (eq. 9 at the drawn tuple)
__global__ void __launch_bounds__(kWave) k_logq_generic(int V, int n, int r, const float *__restrict__ logw,
                                                        const float *__restrict__ z, const float *__restrict__ lse,
                                                        const int32_t *__restrict__ tokens, float *__restrict__ logq)
{
    const size_t b = blockIdx.x;
    const int lane = threadIdx.x;
    float a = -INFINITY;
    if (lane < r) {
        a = logw[b * r + lane];
        for (int s = 0; s < n; ++s) {
            const size_t row = (b * n + s) * r + lane;
            a += z[row * V + tokens[b * n + s]] - lse[row];
        }
    }
    const float mx = wave_max(a);
    const float sum = wave_sum(lane < r ? expf(a - mx) : 0.f);
    if (lane == 0) logq[b] = mx + logf(sum);
}

// The paper's sequential scheme (eq. 11-13) from stored logits, one block per row b of the batch: for every
// token the conditional sum_a qhat_a P^(s)(. | a) is scanned in vocabulary order (thread i owns a contiguous
// run of tokens, run sums in fp64), then the expert log-weights take the drawn token's log-probabilities.
__global__ void __launch_bounds__(kBlock) k_sample_sequential_generic(int V, int n, int r, const float *__restrict__ z,
                                                                      const float *__restrict__ lse,
                                                                      const float *__restrict__ logw,
                                                                      const float *__restrict__ uniforms,
                                                                      int32_t *__restrict__ tokens,
                                                                      float *__restrict__ logq)
{
    __shared__ double seg_sum[kBlock];
    __shared__ double base;
    __shared__ float q_s[64], qh_s[64];
    __shared__ int chosen, tok_sh;
    const size_t b = blockIdx.x;
    const int tid = threadIdx.x;
    if (tid < r) q_s[tid] = logw[b * r + tid];
    __syncthreads();
    for (int s = 0; s < n; ++s) {
        const size_t row0 = (b * n + s) * r;
        const double u = (double)uniforms[b * n + s];
        if (tid == 0) {
            float mx = q_s[0];
            for (int a = 1; a < r; ++a) mx = fmaxf(mx, q_s[a]);
            float sm = 0.f;
            for (int a = 0; a < r; ++a) sm += expf(q_s[a] - mx);
            const float qn = mx + logf(sm);
            for (int a = 0; a < r; ++a) qh_s[a] = expf(q_s[a] - qn);
        }
        __syncthreads();
        const int seg = (V + kBlock - 1) / kBlock;
        const int lo = min(V, tid * seg), hi = min(V, lo + seg);
        double sum = 0.0;
        for (int v = lo; v < hi; ++v) {
            float p = 0.f;
            for (int a = 0; a < r; ++a) p += qh_s[a] * expf(z[(row0 + a) * V + v] - lse[row0 + a]);
            sum += (double)p;
        }
        seg_sum[tid] = sum;
        __syncthreads();
        if (tid == 0) {
            double c = 0.0;
            int pick = -1;
            for (int i = 0; i < kBlock; ++i) {
                if (c + seg_sum[i] > u) { pick = i; break; }
                c += seg_sum[i];
            }
            chosen = pick;
            base = c;
            if (pick < 0) tok_sh = V - 1;
        }
        __syncthreads();
        if (tid == chosen) {
            double c = base;
            int tok = hi - 1;
            for (int v = lo; v < hi; ++v) {
                float p = 0.f;
                for (int a = 0; a < r; ++a) p += qh_s[a] * expf(z[(row0 + a) * V + v] - lse[row0 + a]);
                c += (double)p;
                if (c > u) { tok = v; break; }
            }
            tok_sh = tok;
        }
        __syncthreads();
        const int tok = tok_sh;
        if (tid == 0) tokens[b * n + s] = tok;
        if (tid < r) q_s[tid] += z[(row0 + tid) * V + tok] - lse[row0 + tid];
        __syncthreads();
    }
    if (logq && tid == 0) {
        float mx = q_s[0];
        for (int a = 1; a < r; ++a) mx = fmaxf(mx, q_s[a]);
        float sm = 0.f;
        for (int a = 0; a < r; ++a) sm += expf(q_s[a] - mx);
        logq[b] = mx + logf(sm);
    }
}

// ------------------------------------------------------------------------------------------
// full heads (eq. 6 as printed): z_sa = F_sa h with one V x d matrix per (s, a); rows m = (t n + s) r + a
// ------------------------------------------------------------------------------------------

// running statistics of z = F_sa h for one head row, C = z[x] - lse; with dZ != NULL (backward) the
// second sweep writes dz[v] = coef (softmax(z)[v] - 1[v = x]) for chunk row m - m0 instead
template <typename TIn>
__global__ void __launch_bounds__(kBlock) k_full_row_generic(int d, int V, int n, int r, size_t m0,
                                                             const TIn *__restrict__ H, const TIn *__restrict__ F,
                                                             const int32_t *__restrict__ X, float *__restrict__ lse_io,
                                                             float *__restrict__ C_out,
                                                             const float *__restrict__ gamma,
                                                             const float *__restrict__ dloss, float scale,
                                                             float *__restrict__ dZ)
{
    extern __shared__ float hs[];
    __shared__ float red_m[kWavesPerBlock], red_l[kWavesPerBlock], red_zt;
    const size_t mc = blockIdx.x, m = m0 + mc;
    const int nr = n * r;
    const size_t t = m / nr;
    const int sa = (int)(m % nr), a = sa % r;
    for (int k = threadIdx.x; k < d; k += kBlock) hs[k] = ld_f32(H, t * d + k);
    if (threadIdx.x == 0) red_zt = 0.f;
    __syncthreads();
    const TIn *Fsa = F + (size_t)sa * V * d;
    const int x = X[m / r];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    if (!dZ) {
        float mx = -INFINITY, l = 0.f;
        for (int v = wave; v < V; v += kWavesPerBlock) {
            float p = 0.f;
            for (int k = lane; k < d; k += kWave) p += ld_f32(Fsa, (size_t)v * d + k) * hs[k];
            const float z = wave_sum(p);
            if (z > mx) { l = l * expf(mx - z) + 1.f; mx = z; }
            else l += expf(z - mx);
            if (v == x && lane == 0) red_zt = z;
        }
        if (lane == 0) { red_m[wave] = mx; red_l[wave] = l; }
        __syncthreads();
        if (threadIdx.x == 0) {
            float Mx = red_m[0];
            for (int i = 1; i < kWavesPerBlock; ++i) Mx = fmaxf(Mx, red_m[i]);
            float L = 0.f;
            for (int i = 0; i < kWavesPerBlock; ++i) L += red_l[i] * expf(red_m[i] - Mx);
            const float lse = Mx + logf(L);
            lse_io[m] = lse;
            C_out[m] = (x >= 0) ? red_zt - lse : 0.f;
        }
    } else {
        const float up = dloss ? dloss[t] * scale : scale;
        const float coef = up * gamma[t * r + a];
        const float l = lse_io[m];
        for (int v = wave; v < V; v += kWavesPerBlock) {
            float p = 0.f;
            for (int k = lane; k < d; k += kWave) p += ld_f32(Fsa, (size_t)v * d + k) * hs[k];
            const float z = wave_sum(p);
            if (lane == 0) dZ[mc * V + v] = (x < 0) ? 0.f : coef * (expf(z - l) - (v == x ? 1.f : 0.f));
        }
    }
}

// dF[sa,v,j] (+)= sum over the positions t0 .. t0+Tc-1 of dZ[(t - t0) nr + sa, v] H[t, j]
template <typename TIn>
__global__ void __launch_bounds__(kBlock) k_df_generic(int d, int V, int nr, size_t t0, size_t Tc,
                                                       const TIn *__restrict__ H, const float *__restrict__ dZ,
                                                       float *__restrict__ dF, int accumulate)
{
    const size_t idx = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= (size_t)nr * V * d) return;
    const int j = (int)(idx % d);
    const size_t sav = idx / d;
    const int v = (int)(sav % V);
    const size_t sa = sav / V;
    float acc = accumulate ? dF[idx] : 0.f;
    for (size_t tc = 0; tc < Tc; ++tc) acc += dZ[(tc * nr + sa) * V + v] * ld_f32(H, (t0 + tc) * d + j);
    dF[idx] = acc;
}

// dH[t,j] = sum_{sa,v} dZ[(t - t0) nr + sa, v] F[sa,v,j] + sum_a dg[t,a] G[a,j] for the positions of the chunk
template <typename TIn>
__global__ void __launch_bounds__(kBlock) k_dh_full_generic(int d, int V, int nr, int r, size_t t0, size_t Tc,
                                                            const TIn *__restrict__ F, const TIn *__restrict__ G,
                                                            const float *__restrict__ dZ, const float *__restrict__ dg,
                                                            float *__restrict__ dH)
{
    const size_t idx = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= Tc * d) return;
    const size_t tc = idx / d, t = t0 + tc;
    const int j = (int)(idx % d);
    float acc = 0.f;
    for (int sa = 0; sa < nr; ++sa)
        for (int v = 0; v < V; ++v) acc += dZ[(tc * nr + sa) * V + v] * ld_f32(F, ((size_t)sa * V + v) * d + j);
    for (int a = 0; a < r; ++a) acc += dg[t * r + a] * ld_f32(G, (size_t)a * d + j);
    dH[t * d + j] = acc;
}

// ------------------------------------------------------------------------------------------
// next-token distribution (eq. 11) and the balancing statistic (eq. 10)
// ------------------------------------------------------------------------------------------

// logp[b, v] = logsumexp_a( logw[b,a] + z[(b*r+a), v] - lse[b*r+a] )      (eq. 11 in log space)
__global__ void __launch_bounds__(kBlock) k_first_token_mix(int V, int r, size_t ld, const float *__restrict__ z,
                                                            const float *__restrict__ lse,
                                                            const float *__restrict__ logw, float *__restrict__ logp)
{
    const int v = blockIdx.y * kBlock + threadIdx.x;
    const size_t b = blockIdx.x;
    if (v >= V) return;
    float mx = -INFINITY, l = 0.f;
    for (int a = 0; a < r; ++a) {
        const size_t row = b * r + a;
        const float x = logw[row] + z[row * ld + v] - lse[row];
        if (x > mx) { l = l * expf(mx - x) + 1.f; mx = x; }
        else l += expf(x - mx);
    }
    logp[b * (size_t)V + v] = mx + logf(l);
}

// eq. 10, first stage: argmax_a of the gate pre-activations per position (first index on ties; the
// softmax is monotone), histogram per block in LDS, then integer atomics (exact, order-independent)
template <typename TIn>
__global__ void __launch_bounds__(kBlock) k_aux_argmax(size_t T, int d, int r, const TIn *__restrict__ H,
                                                       const TIn *__restrict__ G, unsigned long long *__restrict__ counts)
{
    __shared__ unsigned int hist[64];
    if (threadIdx.x < 64) hist[threadIdx.x] = 0;
    __syncthreads();
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    for (size_t t = (size_t)blockIdx.x * kWavesPerBlock + wave; t < T; t += (size_t)gridDim.x * kWavesPerBlock) {
        const TIn *h = H + t * d;
        float best = -INFINITY;
        int arg = 0;
        for (int a = 0; a < r; ++a) {
            float p = 0.f;
            for (int k = lane; k < d; k += kWave) p += ld_f32(G, (size_t)a * d + k) * ld_f32(h, k);
            p = wave_sum(p);
            if (p > best) { best = p; arg = a; }
        }
        if (lane == 0) atomicAdd(&hist[arg], 1u);
    }
    __syncthreads();
    if ((int)threadIdx.x < r && hist[threadIdx.x]) atomicAdd(&counts[threadIdx.x], (unsigned long long)hist[threadIdx.x]);
}

__global__ void k_fill_zero_u64(int count, unsigned long long *__restrict__ p)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0ull;
}

// eq. 10, second stage: L_aux = sum_a (n_a / N - 1/r)^2
__global__ void __launch_bounds__(kWave) k_aux_finish(size_t T, int r, const unsigned long long *__restrict__ counts,
                                                      float *__restrict__ laux)
{
    const int lane = threadIdx.x;
    float dev = 0.f;
    if (lane < r) dev = (T ? (float)((double)counts[lane] / (double)T) : 0.f) - 1.f / (float)r;
    const float s = wave_sum(dev * dev);
    if (lane == 0) *laux = s;
}

// rows of the dZ chunk on this path: about 512 MiB of fp32 logit gradients at a time (256 rows with the
// least-workspace flag), and the r rows of one token never split over two chunks
inline size_t generic_chunk_rows(const cp_head_desc &ds)
{
    const size_t M = (size_t)ds.T * ds.n * ds.r;
    size_t rows = ((size_t)1 << 27) / (size_t)ds.V;
    if (ds.flags & CP_HEAD_MIN_WORKSPACE) rows = 256;
    rows = rows / ds.r * ds.r;
    if (rows < (size_t)ds.r) rows = (size_t)ds.r;
    return rows < M ? rows : (M ? M : (size_t)ds.r);
}

struct GenericWs {
    size_t logw, C, dY, dZ, dg, w, Y, z, lse, total;
};

inline GenericWs generic_ws(const cp_head_desc &ds, int op)
{
    GenericWs g = {};
    const size_t M = (size_t)ds.T * ds.n * ds.r, Tr = (size_t)ds.T * ds.r;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    if (op == CP_HEAD_OP_LOSS_FWD) {
        g.logw = take(Tr * 4);
        g.C = take(M * 4);
    } else if (op == CP_HEAD_OP_LOSS_BWD) {
        g.dY = take(M * ds.d * 4);
        g.dZ = take(generic_chunk_rows(ds) * ds.V * 4);
        g.dg = take(Tr * 4);
    } else {
        g.logw = take(Tr * 4);
        g.w = take(Tr * 4);
        g.Y = take(M * ds.d * 4);
        g.z = take(M * ds.V * 4);
        g.lse = take(M * 4);
    }
    g.total = off;
    return g;
}


template <typename TIn>
int loss_fwd_t(const cp_head_desc &ds, const TIn *H, const TIn *W, const TIn *U, const TIn *G, const int32_t *X,
               float *loss, void *ctx, void *ws, hipStream_t st)
{
    const CtxLayout cl = ctx_layout(ds, false);
    const GenericWs g = generic_ws(ds, CP_HEAD_OP_LOSS_FWD);
    const size_t M = (size_t)ds.T * ds.n * ds.r;
    float *lse = at<float>(ctx, cl.lse), *w = at<float>(ctx, cl.w), *gamma = at<float>(ctx, cl.gamma);
    float *Y = at<float>(ctx, cl.Y);
    float *logw = at<float>(ws, g.logw), *C = at<float>(ws, g.C);
    const size_t lds = (size_t)ds.d * sizeof(float);
    k_gate<TIn><<<(unsigned)ds.T, kWave, 0, st>>>(ds.d, ds.r, H, G, logw, w);
    k_y_generic<TIn><<<(unsigned)M, kBlock, lds, st>>>(ds.d, ds.n * ds.r, H, W, Y, 0);
    k_zstats_generic<TIn><<<(unsigned)M, kBlock, lds, st>>>(ds.d, ds.V, ds.r, 0, U, Y, X, lse, C, nullptr);
    k_mixture<<<(unsigned)ds.T, kWave, 0, st>>>(ds.n, ds.r, logw, C, loss, gamma, -1.f);
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

// Everything below the logit gradients, shared by the training loss and the fine-tuning loss: `fn` fills dZ with
// the gradients of the rows [m0, m0 + Mc) of one chunk, which is then contracted into dY and dU; dW, dH, dG follow.
template <typename TIn>
int bwd_from_dz_t(const cp_head_desc &ds, const TIn *H, const TIn *W, const TIn *U, const TIn *G, const float *Y,
                  const float *dg, float *dH, float *dW, float *dU, float *dG, void *ws, GenericDzLaunch fn, void *user,
                  hipStream_t st)
{
    const GenericWs g = generic_ws(ds, CP_HEAD_OP_LOSS_BWD);
    const size_t T = (size_t)ds.T, M = T * ds.n * ds.r;
    float *dY = at<float>(ws, g.dY), *dZ = at<float>(ws, g.dZ);
    const size_t chunk = generic_chunk_rows(ds);
    int first = 1;
    for (size_t m0 = 0; m0 < M; m0 += chunk) {
        const size_t Mc = (M - m0 < chunk) ? M - m0 : chunk;
        fn(user, m0, Mc, dZ, st);
        k_dy_generic<TIn><<<blocks_for(Mc * ds.d, kBlock), kBlock, 0, st>>>(ds.d, ds.V, m0, Mc, U, dZ, dY);
        if (dU)
            k_du_generic<<<blocks_for((size_t)ds.V * ds.d, kBlock), kBlock, 0, st>>>(ds.d, ds.V, m0, Mc, dZ, Y, dU,
                                                                                    first ? 0 : 1);
        first = 0;
    }
    if (dW)
        k_dw_generic<TIn><<<blocks_for((size_t)ds.n * ds.r * ds.d * ds.d, kBlock), kBlock, 0, st>>>(T, ds.d,
                                                                                                  ds.n * ds.r, H, dY, dW);
    k_dh_generic<TIn><<<blocks_for(T * ds.d, kBlock), kBlock, 0, st>>>(T, ds.d, ds.n * ds.r, ds.r, W, G, dY, dg, dH);
    if (dG) k_dg_generic<TIn><<<blocks_for((size_t)ds.r * ds.d, kBlock), kBlock, 0, st>>>(T, ds.d, ds.r, H, dg, dG);
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

template <typename TIn>
struct LossDzArgs {
    const cp_head_desc *ds;
    const TIn *U;
    const float *Y, *lse, *gamma, *dloss;
    const int32_t *X;
    float scale;
};
template <typename TIn>
void loss_dz_launch(void *user, size_t m0, size_t Mc, float *dZ, hipStream_t st)
{
    const LossDzArgs<TIn> *a = static_cast<const LossDzArgs<TIn> *>(user);
    const cp_head_desc &ds = *a->ds;
    k_dz_generic<TIn><<<(unsigned)Mc, kBlock, (size_t)ds.d * sizeof(float), st>>>(ds.d, ds.V, ds.n, ds.r, m0, a->U, a->Y, a->X,
                                                                                  a->lse, a->gamma, a->dloss, a->scale, dZ);
}

template <typename TIn>
int loss_bwd_t(const cp_head_desc &ds, const TIn *H, const TIn *W, const TIn *U, const TIn *G, const int32_t *X,
               const float *dloss, float scale, const void *ctx, float *dH, float *dW, float *dU, float *dG,
               void *ws, hipStream_t st)
{
    const CtxLayout cl = ctx_layout(ds, false);
    const GenericWs g = generic_ws(ds, CP_HEAD_OP_LOSS_BWD);
    const size_t Tr = (size_t)ds.T * ds.r;
    const float *lse = at<float>(ctx, cl.lse), *w = at<float>(ctx, cl.w), *gamma = at<float>(ctx, cl.gamma);
    const float *Y = at<float>(ctx, cl.Y);
    float *dg = at<float>(ws, g.dg);
    k_dgate<<<blocks_for(Tr, kBlock), kBlock, 0, st>>>(Tr, ds.r, w, gamma, dloss, scale, dg);
    LossDzArgs<TIn> args{&ds, U, Y, lse, gamma, dloss, X, scale};
    return bwd_from_dz_t<TIn>(ds, H, W, U, G, Y, dg, dH, dW, dU, dG, ws, loss_dz_launch<TIn>, &args, st);
}

template <typename TIn>
int draft_t(const cp_head_desc &ds, const TIn *H, const TIn *W, const TIn *U, const TIn *G, const float *uniforms,
            int32_t *alpha, int32_t *tokens, float *logq, void *ws, hipStream_t st)
{
    const GenericWs g = generic_ws(ds, CP_HEAD_OP_DRAFT);
    const size_t B = (size_t)ds.T, M = B * ds.n * ds.r;
    float *logw = at<float>(ws, g.logw), *w = at<float>(ws, g.w), *Y = at<float>(ws, g.Y);
    float *z = at<float>(ws, g.z), *lse = at<float>(ws, g.lse);
    const size_t lds = (size_t)ds.d * sizeof(float);
    const int round_y = ds.dtype == CP_HEAD_BF16 ? 1 : 0;
    k_gate<TIn><<<(unsigned)B, kWave, 0, st>>>(ds.d, ds.r, H, G, logw, w);
    k_pick_alpha<<<blocks_for(B, kWave), kWave, 0, st>>>(B, ds.n, ds.r, w, uniforms, alpha);
    k_y_generic<TIn><<<(unsigned)M, kBlock, lds, st>>>(ds.d, ds.n * ds.r, H, W, Y, round_y);
    k_zstats_generic<TIn><<<(unsigned)M, kBlock, lds, st>>>(ds.d, ds.V, ds.r, 0, U, Y, nullptr, lse, nullptr, z);
    k_sample_generic<<<(unsigned)(B * ds.n), kBlock, 0, st>>>(ds.V, ds.n, ds.r, z, lse, alpha, uniforms, tokens);
    if (logq) k_logq_generic<<<(unsigned)B, kWave, 0, st>>>(ds.V, ds.n, ds.r, logw, z, lse, tokens, logq);
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

template <typename TIn>
int draft_sequential_t(const cp_head_desc &ds, const TIn *H, const TIn *W, const TIn *U, const TIn *G,
                       const float *uniforms, int32_t *tokens, float *logq, void *ws, hipStream_t st)
{
    const GenericWs g = generic_ws(ds, CP_HEAD_OP_DRAFT);
    const size_t B = (size_t)ds.T, M = B * ds.n * ds.r;
    float *logw = at<float>(ws, g.logw), *w = at<float>(ws, g.w), *Y = at<float>(ws, g.Y);
    float *z = at<float>(ws, g.z), *lse = at<float>(ws, g.lse);
    const size_t lds = (size_t)ds.d * sizeof(float);
    const int round_y = ds.dtype == CP_HEAD_BF16 ? 1 : 0;
    k_gate<TIn><<<(unsigned)B, kWave, 0, st>>>(ds.d, ds.r, H, G, logw, w);
    k_y_generic<TIn><<<(unsigned)M, kBlock, lds, st>>>(ds.d, ds.n * ds.r, H, W, Y, round_y);
    k_zstats_generic<TIn><<<(unsigned)M, kBlock, lds, st>>>(ds.d, ds.V, ds.r, 0, U, Y, nullptr, lse, nullptr, z);
    k_sample_sequential_generic<<<(unsigned)B, kBlock, 0, st>>>(ds.V, ds.n, ds.r, z, lse, logw, uniforms, tokens, logq);
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

}  // namespace

int generic_draft_sequential(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                             const float *uniforms, int32_t *tokens, float *logq, void *ws, hipStream_t st)
{
    if (ds.T == 0) return CP_HEAD_OK;
    if (ds.dtype == CP_HEAD_FP32)
        return draft_sequential_t<float>(ds, (const float *)H, (const float *)W, (const float *)U, (const float *)G,
                                         uniforms, tokens, logq, ws, st);
    return draft_sequential_t<bf16_t>(ds, (const bf16_t *)H, (const bf16_t *)W, (const bf16_t *)U, (const bf16_t *)G,
                                      uniforms, tokens, logq, ws, st);
}

size_t generic_workspace_bytes(const cp_head_desc &ds, int op) { return generic_ws(ds, op).total; }

size_t generic_bwd_chunk_rows(const cp_head_desc &ds) { return generic_chunk_rows(ds); }

namespace {
template <typename TIn>
void fwd_rows_t(const cp_head_desc &ds, const TIn *H, const TIn *W, const TIn *U, const TIn *G, const int32_t *X,
                const GenericFwdBuffers &b, hipStream_t st)
{
    const size_t M = (size_t)ds.T * ds.n * ds.r, lds = (size_t)ds.d * sizeof(float);
    k_gate<TIn><<<(unsigned)ds.T, kWave, 0, st>>>(ds.d, ds.r, H, G, b.logw, b.w);
    k_y_generic<TIn><<<(unsigned)M, kBlock, lds, st>>>(ds.d, ds.n * ds.r, H, W, b.Y, 0);
    k_zstats_generic<TIn><<<(unsigned)M, kBlock, lds, st>>>(ds.d, ds.V, ds.r, 0, U, b.Y, X, b.lse, b.C, nullptr);
}
}  // namespace

int generic_fwd_rows(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X, void *ctx, void *ws, GenericFwdBuffers *out, hipStream_t st)
{
    const CtxLayout cl = ctx_layout(ds, false);
    const GenericWs g = generic_ws(ds, CP_HEAD_OP_LOSS_FWD);
    GenericFwdBuffers b;
    b.lse = at<float>(ctx, cl.lse);
    b.w = at<float>(ctx, cl.w);
    b.gamma = at<float>(ctx, cl.gamma);
    b.Y = at<float>(ctx, cl.Y);
    b.logw = at<float>(ws, g.logw);
    b.C = at<float>(ws, g.C);
    if (ds.dtype == CP_HEAD_FP32)
        fwd_rows_t<float>(ds, (const float *)H, (const float *)W, (const float *)U, (const float *)G, X, b, st);
    else
        fwd_rows_t<bf16_t>(ds, (const bf16_t *)H, (const bf16_t *)W, (const bf16_t *)U, (const bf16_t *)G, X, b, st);
    *out = b;
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

void generic_logits_rows(const cp_head_desc &ds, const void *U, const float *Y, size_t m0, size_t Mc, float *z,
                         hipStream_t st)
{
    const size_t lds = (size_t)ds.d * sizeof(float);
    if (ds.dtype == CP_HEAD_FP32)
        k_zstats_generic<float><<<(unsigned)Mc, kBlock, lds, st>>>(ds.d, ds.V, ds.r, m0, (const float *)U, Y, nullptr,
                                                                   nullptr, nullptr, z);
    else
        k_zstats_generic<bf16_t><<<(unsigned)Mc, kBlock, lds, st>>>(ds.d, ds.V, ds.r, m0, (const bf16_t *)U, Y, nullptr,
                                                                    nullptr, nullptr, z);
}

int generic_bwd_from_dz(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                        const float *Y, const float *dg, float *dH, float *dW, float *dU, float *dG, void *ws,
                        GenericDzLaunch fn, void *user, hipStream_t st)
{
    if (ds.dtype == CP_HEAD_FP32)
        return bwd_from_dz_t<float>(ds, (const float *)H, (const float *)W, (const float *)U, (const float *)G, Y, dg,
                                    dH, dW, dU, dG, ws, fn, user, st);
    return bwd_from_dz_t<bf16_t>(ds, (const bf16_t *)H, (const bf16_t *)W, (const bf16_t *)U, (const bf16_t *)G, Y, dg,
                                 dH, dW, dU, dG, ws, fn, user, st);
}

int generic_loss_fwd(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X, float *loss, void *ctx, void *ws, hipStream_t st)
{
    if (ds.T == 0) return CP_HEAD_OK;
    if (ds.dtype == CP_HEAD_FP32)
        return loss_fwd_t<float>(ds, (const float *)H, (const float *)W, (const float *)U, (const float *)G, X, loss,
                                 ctx, ws, st);
    return loss_fwd_t<bf16_t>(ds, (const bf16_t *)H, (const bf16_t *)W, (const bf16_t *)U, (const bf16_t *)G, X, loss,
                              ctx, ws, st);
}

void launch_fill_zero(float *p, size_t count, hipStream_t st)
{
    if (p && count) k_fill_zero<<<blocks_for(count, kBlock), kBlock, 0, st>>>(count, p);
}

int generic_loss_bwd(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X, const float *dloss, float scale, const void *ctx, float *dH, float *dW,
                     float *dU, float *dG, void *ws, hipStream_t st)
{
    if (ds.T == 0) {   // empty batch: the weight gradients are empty sums
        launch_fill_zero(dW, (size_t)ds.n * ds.r * ds.d * ds.d, st);
        launch_fill_zero(dU, (size_t)ds.V * ds.d, st);
        launch_fill_zero(dG, (size_t)ds.r * ds.d, st);
        return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
    }
    if (ds.dtype == CP_HEAD_FP32)
        return loss_bwd_t<float>(ds, (const float *)H, (const float *)W, (const float *)U, (const float *)G, X, dloss,
                                 scale, ctx, dH, dW, dU, dG, ws, st);
    return loss_bwd_t<bf16_t>(ds, (const bf16_t *)H, (const bf16_t *)W, (const bf16_t *)U, (const bf16_t *)G, X,
                              dloss, scale, ctx, dH, dW, dU, dG, ws, st);
}

int generic_draft(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                  const float *uniforms, int32_t *alpha, int32_t *tokens, float *logq, void *ws, hipStream_t st)
{
    if (ds.T == 0) return CP_HEAD_OK;
    if (ds.dtype == CP_HEAD_FP32)
        return draft_t<float>(ds, (const float *)H, (const float *)W, (const float *)U, (const float *)G, uniforms,
                              alpha, tokens, logq, ws, st);
    return draft_t<bf16_t>(ds, (const bf16_t *)H, (const bf16_t *)W, (const bf16_t *)U, (const bf16_t *)G, uniforms,
                           alpha, tokens, logq, ws, st);
}

// ---- first-token marginal on the plain path: z of the r first-head rows is stored, then mixed
struct GenericFirstWs {
    size_t logw, w, Y, z, lse, total;
};
static GenericFirstWs generic_first_ws(const cp_head_desc &ds)
{
    GenericFirstWs g;
    const size_t rows = (size_t)ds.T * ds.r;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    g.logw = take(rows * 4);
    g.w = take(rows * 4);
    g.Y = take(rows * ds.d * 4);
    g.z = take(rows * ds.V * 4);
    g.lse = take(rows * 4);
    g.total = off;
    return g;
}
size_t generic_first_token_workspace_bytes(const cp_head_desc &ds) { return generic_first_ws(ds).total; }

void launch_first_token_mix(const cp_head_desc &ds, const float *z, size_t ld, const float *lse, const float *logw,
                            float *logp, hipStream_t st)
{
    if (ds.T == 0) return;
    k_first_token_mix<<<dim3((unsigned)ds.T, blocks_for((size_t)ds.V, kBlock)), kBlock, 0, st>>>(
        ds.V, ds.r, ld, z, lse, logw, logp);
}

template <typename TIn>
static int first_token_t(const cp_head_desc &ds, const TIn *H, const TIn *W, const TIn *U, const TIn *G, float *logp,
                         void *ws, hipStream_t st)
{
    const GenericFirstWs g = generic_first_ws(ds);
    const size_t rows = (size_t)ds.T * ds.r;
    float *logw = at<float>(ws, g.logw), *w = at<float>(ws, g.w), *Y = at<float>(ws, g.Y);
    float *z = at<float>(ws, g.z), *lse = at<float>(ws, g.lse);
    const size_t lds = (size_t)ds.d * sizeof(float);
    const int round_y = ds.dtype == CP_HEAD_BF16 ? 1 : 0;
    k_gate<TIn><<<(unsigned)ds.T, kWave, 0, st>>>(ds.d, ds.r, H, G, logw, w);
    // the first head's matrices are the first r blocks of W, so its rows are (b, a) with nr = r
    k_y_generic<TIn><<<(unsigned)rows, kBlock, lds, st>>>(ds.d, ds.r, H, W, Y, round_y);
    k_zstats_generic<TIn><<<(unsigned)rows, kBlock, lds, st>>>(ds.d, ds.V, ds.r, 0, U, Y, nullptr, lse, nullptr, z);
    launch_first_token_mix(ds, z, (size_t)ds.V, lse, logw, logp, st);
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

int generic_first_token(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                        float *logp, void *ws, hipStream_t st)
{
    if (ds.T == 0) return CP_HEAD_OK;
    if (ds.dtype == CP_HEAD_FP32)
        return first_token_t<float>(ds, (const float *)H, (const float *)W, (const float *)U, (const float *)G, logp, ws, st);
    return first_token_t<bf16_t>(ds, (const bf16_t *)H, (const bf16_t *)W, (const bf16_t *)U, (const bf16_t *)G, logp, ws,
                                 st);
}

int aux_balance(const cp_head_desc &ds, const void *H, const void *G, int64_t *counts, float *laux, hipStream_t st)
{
    unsigned long long *c = reinterpret_cast<unsigned long long *>(counts);
    k_fill_zero_u64<<<1, 64, 0, st>>>(ds.r, c);
    if (ds.T > 0) {
        const unsigned blocks = (unsigned)std::min<size_t>(((size_t)ds.T + kWavesPerBlock - 1) / kWavesPerBlock, 4096);
        if (ds.dtype == CP_HEAD_FP32)
            k_aux_argmax<float><<<blocks, kBlock, 0, st>>>((size_t)ds.T, ds.d, ds.r, (const float *)H, (const float *)G, c);
        else
            k_aux_argmax<bf16_t><<<blocks, kBlock, 0, st>>>((size_t)ds.T, ds.d, ds.r, (const bf16_t *)H,
                                                            (const bf16_t *)G, c);
    }
    k_aux_finish<<<1, kWave, 0, st>>>((size_t)ds.T, ds.r, c, laux);
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

// ---- full heads on the plain path
struct GenericFullWs {
    size_t logw, C, dg, dZ, total;
    size_t chunk_pos;
};
static GenericFullWs generic_full_ws(const cp_head_desc &ds)
{
    GenericFullWs g;
    const size_t T = (size_t)ds.T, nr = (size_t)ds.n * ds.r;
    // whole positions per chunk: at most 512 MiB of fp32 logit gradients at a time, at least one position
    size_t pos = ((size_t)1 << 27) / ((size_t)ds.V * nr);
    if (pos < 1) pos = 1;
    g.chunk_pos = pos < T ? pos : (T ? T : 1);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    g.logw = take(T * ds.r * 4);
    g.C = take(T * nr * 4);
    g.dg = take(T * ds.r * 4);
    g.dZ = take(g.chunk_pos * nr * ds.V * 4);
    g.total = off;
    return g;
}
size_t generic_full_workspace_bytes(const cp_head_desc &ds) { return generic_full_ws(ds).total; }

template <typename TIn>
static int full_fwd_t(const cp_head_desc &ds, const TIn *H, const TIn *F, const TIn *G, const int32_t *X, float *loss,
                      void *ctx, void *ws, hipStream_t st)
{
    const CtxLayout cl = ctx_layout(ds, false);      // lse, w, gamma at the same offsets; no y is kept
    const GenericFullWs g = generic_full_ws(ds);
    const size_t M = (size_t)ds.T * ds.n * ds.r;
    float *lse = at<float>(ctx, cl.lse), *w = at<float>(ctx, cl.w), *gamma = at<float>(ctx, cl.gamma);
    float *logw = at<float>(ws, g.logw), *C = at<float>(ws, g.C);
    const size_t lds = (size_t)ds.d * sizeof(float);
    k_gate<TIn><<<(unsigned)ds.T, kWave, 0, st>>>(ds.d, ds.r, H, G, logw, w);
    k_full_row_generic<TIn><<<(unsigned)M, kBlock, lds, st>>>(ds.d, ds.V, ds.n, ds.r, 0, H, F, X, lse, C, nullptr, nullptr,
                                                              0.f, nullptr);
    k_mixture<<<(unsigned)ds.T, kWave, 0, st>>>(ds.n, ds.r, logw, C, loss, gamma, -1.f);
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

template <typename TIn>
static int full_bwd_t(const cp_head_desc &ds, const TIn *H, const TIn *F, const TIn *G, const int32_t *X,
                      const float *dloss, float scale, const void *ctx, float *dH, float *dF, float *dG, void *ws,
                      hipStream_t st)
{
    const CtxLayout cl = ctx_layout(ds, false);
    const GenericFullWs g = generic_full_ws(ds);
    const size_t T = (size_t)ds.T, Tr = T * ds.r;
    const int nr = ds.n * ds.r;
    float *lse = const_cast<float *>(at<float>(ctx, cl.lse));
    const float *w = at<float>(ctx, cl.w), *gamma = at<float>(ctx, cl.gamma);
    float *dg = at<float>(ws, g.dg), *dZ = at<float>(ws, g.dZ);
    const size_t lds = (size_t)ds.d * sizeof(float);
    k_dgate<<<blocks_for(Tr, kBlock), kBlock, 0, st>>>(Tr, ds.r, w, gamma, dloss, scale, dg);
    int first = 1;
    for (size_t t0 = 0; t0 < T; t0 += g.chunk_pos) {
        const size_t Tc = (T - t0 < g.chunk_pos) ? T - t0 : g.chunk_pos;
        k_full_row_generic<TIn><<<(unsigned)(Tc * nr), kBlock, lds, st>>>(ds.d, ds.V, ds.n, ds.r, t0 * nr, H, F, X, lse,
                                                                          nullptr, gamma, dloss, scale, dZ);
        k_dh_full_generic<TIn><<<blocks_for(Tc * ds.d, kBlock), kBlock, 0, st>>>(ds.d, ds.V, nr, ds.r, t0, Tc, F, G, dZ,
                                                                                 dg, dH);
        if (dF)
            k_df_generic<TIn><<<blocks_for((size_t)nr * ds.V * ds.d, kBlock), kBlock, 0, st>>>(ds.d, ds.V, nr, t0, Tc, H,
                                                                                               dZ, dF, first ? 0 : 1);
        first = 0;
    }
    if (dG) k_dg_generic<TIn><<<blocks_for((size_t)ds.r * ds.d, kBlock), kBlock, 0, st>>>(T, ds.d, ds.r, H, dg, dG);
    return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
}

int generic_full_loss_fwd(const cp_head_desc &ds, const void *H, const void *F, const void *G, const int32_t *X,
                          float *loss, void *ctx, void *ws, hipStream_t st)
{
    if (ds.T == 0) return CP_HEAD_OK;
    if (ds.dtype == CP_HEAD_FP32)
        return full_fwd_t<float>(ds, (const float *)H, (const float *)F, (const float *)G, X, loss, ctx, ws, st);
    return full_fwd_t<bf16_t>(ds, (const bf16_t *)H, (const bf16_t *)F, (const bf16_t *)G, X, loss, ctx, ws, st);
}

int generic_full_loss_bwd(const cp_head_desc &ds, const void *H, const void *F, const void *G, const int32_t *X,
                          const float *dloss, float scale, const void *ctx, float *dH, float *dF, float *dG, void *ws,
                          hipStream_t st)
{
    if (ds.T == 0) {
        launch_fill_zero(dF, (size_t)ds.n * ds.r * ds.V * ds.d, st);
        launch_fill_zero(dG, (size_t)ds.r * ds.d, st);
        return hipGetLastError() == hipSuccess ? CP_HEAD_OK : CP_HEAD_ERR_LAUNCH;
    }
    if (ds.dtype == CP_HEAD_FP32)
        return full_bwd_t<float>(ds, (const float *)H, (const float *)F, (const float *)G, X, dloss, scale, ctx, dH, dF, dG,
                                 ws, st);
    return full_bwd_t<bf16_t>(ds, (const bf16_t *)H, (const bf16_t *)F, (const bf16_t *)G, X, dloss, scale, ctx, dH, dF,
                              dG, ws, st);
}

void launch_gate(const cp_head_desc &ds, const void *H, const void *G, float *logw, float *w, hipStream_t st)
{
    if (ds.T == 0) return;
    if (ds.dtype == CP_HEAD_FP32)
        k_gate<float><<<(unsigned)ds.T, kWave, 0, st>>>(ds.d, ds.r, (const float *)H, (const float *)G, logw, w);
    else
        k_gate<bf16_t><<<(unsigned)ds.T, kWave, 0, st>>>(ds.d, ds.r, (const bf16_t *)H, (const bf16_t *)G, logw, w);
}

void launch_mixture(const cp_head_desc &ds, const float *logw, const float *C, float *out, float *gamma,
                    float sign, hipStream_t st)
{
    if (ds.T == 0) return;
    k_mixture<<<(unsigned)ds.T, kWave, 0, st>>>(ds.n, ds.r, logw, C, out, gamma, sign);
}

void launch_pick_alpha(const cp_head_desc &ds, const float *w, const float *uniforms, int32_t *alpha, hipStream_t st)
{
    if (ds.T == 0) return;
    k_pick_alpha<<<blocks_for((size_t)ds.T, kWave), kWave, 0, st>>>((size_t)ds.T, ds.n, ds.r, w, uniforms, alpha);
}

}  // namespace cph

/*
 * CP multi-token-prediction head: plain fp64 CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, by-the-definition
 * implementation that the GPU library is checked against.  It shares no code
 * with the GPU library, is never linked into it, and must not be used as a
 * fallback by any product path.
 *
 * What is computed (paper sections "Overall concept", "Training procedure",
 * "Sampling method", "Fine tuning"):
 *
 *   gate            w      = softmax(G h)                          (eq. 7)
 *   reduced head    y_sa   = W_sa h ,  z_sa = U y_sa               (shared-unembedding
 *                                                                   head of "Fine tuning")
 *   factor          P^(s)(x | a) = softmax(z_sa)_x                 (eq. 5, eq. 6)
 *   log factor      C_sa   = z_sa[x_s] - logsumexp_v z_sa[v]       (eq. 8)
 *   joint           L      = logsumexp_a( log w_a + sum_s C_sa )   (eq. 2, eq. 9)
 *   loss            loss   = -L   (per position, nats)
 *   full head       z_sa   = F_sa h, F_sa of size V x d            (eq. 6 as printed; full_loss_*)
 *
 * The backward pass is the analytic derivative of the lines above (the paper
 * leaves it to automatic differentiation); it is pinned by finite differences
 * in the tests.
 *
 * Everything is double precision, loops only, no blocking or fusion.  Inputs
 * arrive either as float (CPO_IN_T=float: values that are exact in the storage
 * type, widened on the fly) or as double (for finite-difference tests); the
 * file is compiled once per input type.
 *
 * Threads: positions are independent, so loops over positions (and, in the
 * second phase of the backward pass, over output rows) carry an OpenMP
 * pragma.  Each output element is still a sum in one fixed order.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef CPO_IN_T
#define CPO_IN_T double
#endif
#ifndef CPO_PREFIX
#define CPO_PREFIX cpo_f64_
#endif
#define CPO_CAT2(a, b) a##b
#define CPO_CAT(a, b) CPO_CAT2(a, b)
#define CPO(name) CPO_CAT(CPO_PREFIX, name)

typedef CPO_IN_T in_t;

typedef struct {
    int64_t T;        /* positions (loss) or batch size B (draft) */
    int32_t d, V, n, r;
    int32_t round_y;  /* 0: y kept in fp64; 1: y rounded to bfloat16 (nearest-even) before z = U y */
} cpo_shape;

/* ------------------------------------------------------------------------- */
/* small helpers                                                              */
/* ------------------------------------------------------------------------- */

/* Nearest bfloat16 (8 significant bits), ties to even; normal range only. */
static double round_to_bf16(double v)
{
    if (v == 0.0 || !isfinite(v)) return v;
    int e;
    double m = frexp(v, &e);             /* v = m * 2^e, 0.5 <= |m| < 1 */
    double q = nearbyint(ldexp(m, 8));   /* default rounding mode: ties to even */
    return ldexp(q, e - 8);
}

/* max + log sum exp(x - max) */
static double logsumexp(const double *x, int64_t len)
{
    double mx = x[0];
    for (int64_t i = 1; i < len; ++i) if (x[i] > mx) mx = x[i];
    double s = 0.0;
    for (int64_t i = 0; i < len; ++i) s += exp(x[i] - mx);
    return mx + log(s);
}

/* eq. 7 in log space: logw = g - logsumexp(g), g = G h */
static void gate_logw(const cpo_shape *sh, const in_t *h, const in_t *G, double *logw)
{
    for (int a = 0; a < sh->r; ++a) {
        double g = 0.0;
        for (int k = 0; k < sh->d; ++k) g += (double)G[(size_t)a * sh->d + k] * (double)h[k];
        logw[a] = g;
    }
    double lse = logsumexp(logw, sh->r);
    for (int a = 0; a < sh->r; ++a) logw[a] -= lse;
}

/*
 * y = W_sa h  (W_sa is d x d, row = output feature).
 * With round_y the result is rounded to bfloat16.  Rounding is discontinuous: an element that lies
 * within accumulation error of a rounding midpoint may legitimately land on either neighbour in an
 * implementation that accumulates in fp32.  For tests of such cases the exact y can be returned
 * (y_exact, may be NULL) and a caller-chosen nudge (may be NULL) is added before rounding.
 */
static void head_y_ex(const cpo_shape *sh, const in_t *h, const in_t *W, int s, int a,
                      const double *nudge, double *y_exact, double *y)
{
    const in_t *Wsa = W + ((size_t)s * sh->r + a) * sh->d * sh->d;
    for (int k = 0; k < sh->d; ++k) {
        double acc = 0.0;
        for (int j = 0; j < sh->d; ++j) acc += (double)Wsa[(size_t)k * sh->d + j] * (double)h[j];
        if (y_exact) y_exact[k] = acc;
        if (nudge) acc += nudge[k];
        y[k] = sh->round_y ? round_to_bf16(acc) : acc;
    }
}

static void head_y(const cpo_shape *sh, const in_t *h, const in_t *W, int s, int a, double *y)
{
    head_y_ex(sh, h, W, s, a, NULL, NULL, y);
}

/* z = U y  (U is V x d) */
static void head_z(const cpo_shape *sh, const in_t *U, const double *y, double *z)
{
    for (int v = 0; v < sh->V; ++v) {
        double acc = 0.0;
        for (int k = 0; k < sh->d; ++k) acc += (double)U[(size_t)v * sh->d + k] * y[k];
        z[v] = acc;
    }
}

/* ------------------------------------------------------------------------- */
/* loss forward                                                               */
/* ------------------------------------------------------------------------- */

/*
 * Per-position negative joint log-likelihood (eq. 9 with the sign flipped).
 *   H[T,d] W[n,r,d,d] U[V,d] G[r,d]; X[T,n] targets, X<0 drops that factor.
 *   loss[T]; optional (may be NULL): logw[T,r], C[T,n,r] (eq. 8),
 *   lse[T,n,r] (log normaliser of each factor, eq. 5).
 * Returns 0, or -1 on allocation failure / bad shape.
 */
int CPO(loss_fwd)(const cpo_shape *sh, const in_t *H, const in_t *W, const in_t *U, const in_t *G,
                  const int32_t *X, double *loss, double *logw_out, double *C_out, double *lse_out)
{
    if (sh->T < 0 || sh->d <= 0 || sh->V <= 0 || sh->n <= 0 || sh->r <= 0) return -1;
    const int d = sh->d, V = sh->V, n = sh->n, r = sh->r;
    int fail = 0;
#pragma omp parallel
    {
        double *y = malloc(sizeof(double) * d);
        double *z = malloc(sizeof(double) * V);
        double *logw = malloc(sizeof(double) * r);
        double *a = malloc(sizeof(double) * r);
        if (!y || !z || !logw || !a) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t t = 0; t < sh->T; ++t) {
                const in_t *h = H + (size_t)t * d;
                gate_logw(sh, h, G, logw);
                for (int al = 0; al < r; ++al) a[al] = logw[al];
                for (int s = 0; s < n; ++s) {
                    for (int al = 0; al < r; ++al) {
                        head_y(sh, h, W, s, al, y);
                        head_z(sh, U, y, z);
                        double lse = logsumexp(z, V);
                        int32_t x = X[(size_t)t * n + s];
                        double C = (x >= 0) ? z[x] - lse : 0.0;       /* eq. 8 */
                        a[al] += C;
                        size_t idx = ((size_t)t * n + s) * r + al;
                        if (C_out) C_out[idx] = C;
                        if (lse_out) lse_out[idx] = lse;
                    }
                }
                loss[t] = -logsumexp(a, r);                            /* eq. 9 */
                if (logw_out) for (int al = 0; al < r; ++al) logw_out[(size_t)t * r + al] = logw[al];
            }
        }
        free(y); free(z); free(logw); free(a);
    }
    return fail ? -1 : 0;
}

/*
 * Joint probability by the second line of eq. 9, written naively in
 * probability space: sum_a w_a prod_s softmax(z_sa)[x_s].  Only sensible for
 * small problems (it exists to pin the log-space routine above).
 */
int CPO(joint_prob_naive)(const cpo_shape *sh, const in_t *H, const in_t *W, const in_t *U, const in_t *G,
                          const int32_t *X, double *prob)
{
    const int d = sh->d, V = sh->V, n = sh->n, r = sh->r;
    double *y = malloc(sizeof(double) * d), *z = malloc(sizeof(double) * V), *g = malloc(sizeof(double) * r);
    if (!y || !z || !g) { free(y); free(z); free(g); return -1; }
    for (int64_t t = 0; t < sh->T; ++t) {
        const in_t *h = H + (size_t)t * d;
        double gsum = 0.0;
        for (int al = 0; al < r; ++al) {
            double acc = 0.0;
            for (int k = 0; k < d; ++k) acc += (double)G[(size_t)al * d + k] * (double)h[k];
            g[al] = exp(acc);
            gsum += g[al];
        }
        double total = 0.0;
        for (int al = 0; al < r; ++al) {
            double term = g[al] / gsum;                                /* w_a, eq. 7 */
            for (int s = 0; s < n; ++s) {
                const int x = X[(size_t)t * n + s];
                if (x < 0) continue;                                   /* a dropped factor, as in loss_fwd */
                head_y(sh, h, W, s, al, y);
                head_z(sh, U, y, z);
                double zsum = 0.0;
                for (int v = 0; v < V; ++v) zsum += exp(z[v]);
                term *= exp(z[x]) / zsum;                              /* eq. 6 */
            }
            total += term;                                             /* eq. 2 */
        }
        prob[t] = total;
    }
    free(y); free(z); free(g);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* loss backward                                                              */
/* ------------------------------------------------------------------------- */

/*
 * Gradients of sum_t dloss[t] * loss[t] with respect to H, W, U, G.
 *
 * With a_al = log w_al + sum_s C_s,al and L = logsumexp_al a_al, loss = -L:
 *   gamma_al      = exp(a_al - L)                      (posterior over experts)
 *   dloss/dz_sa[v] = gamma_al * (softmax(z_sa)[v] - 1[v = x_s])
 *   dloss/dg_al    = w_al - gamma_al                    (g = G h, log w = log_softmax g)
 * and everything below z, g is linear: dy = U^T dz, dU = dz (x) y, dW_sa = dy (x) h,
 * dG = dg (x) h, dh = sum_sa W_sa^T dy_sa + G^T dg.
 *
 * Phase 1 (per position) stores dz, y and dy; phase 2 forms the weight
 * gradients as plain sums over positions in increasing t.  Memory therefore
 * grows with T*n*r*V: this routine is meant for the small T used in tests.
 *
 * dH[T,d], dW[n,r,d,d], dU[V,d], dG[r,d] are overwritten; any may be NULL.
 * dloss may be NULL (all ones).
 */
int CPO(loss_bwd)(const cpo_shape *sh, const in_t *H, const in_t *W, const in_t *U, const in_t *G,
                  const int32_t *X, const double *dloss,
                  double *dH, double *dW, double *dU, double *dG)
{
    if (sh->round_y) return -1;   /* the derivative is defined for the unrounded map only */
    const int d = sh->d, V = sh->V, n = sh->n, r = sh->r;
    const int64_t T = sh->T;
    const size_t nr = (size_t)n * r;
    double *dz_all = malloc(sizeof(double) * (size_t)T * nr * V);
    double *y_all = malloc(sizeof(double) * (size_t)T * nr * d);
    double *dy_all = malloc(sizeof(double) * (size_t)T * nr * d);
    double *dg_all = malloc(sizeof(double) * (size_t)T * r);
    if (!dz_all || !y_all || !dy_all || !dg_all) { free(dz_all); free(y_all); free(dy_all); free(dg_all); return -1; }
    int fail = 0;

    /* phase 1: everything that belongs to one position */
#pragma omp parallel
    {
        double *z = malloc(sizeof(double) * V);
        double *logw = malloc(sizeof(double) * r);
        double *a = malloc(sizeof(double) * r);
        double *lse = malloc(sizeof(double) * nr);
        if (!z || !logw || !a || !lse) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t t = 0; t < T; ++t) {
                const in_t *h = H + (size_t)t * d;
                const double up = dloss ? dloss[t] : 1.0;
                gate_logw(sh, h, G, logw);
                for (int al = 0; al < r; ++al) a[al] = logw[al];
                /* forward, keeping y and (temporarily) z - lse in the dz slot */
                for (int s = 0; s < n; ++s)
                    for (int al = 0; al < r; ++al) {
                        size_t row = ((size_t)t * n + s) * r + al;
                        double *y = y_all + row * d;
                        double *dz = dz_all + row * V;
                        head_y(sh, h, W, s, al, y);
                        head_z(sh, U, y, z);
                        double l = logsumexp(z, V);
                        lse[(size_t)s * r + al] = l;
                        for (int v = 0; v < V; ++v) dz[v] = z[v] - l;   /* log P^(s)(v | al) */
                        int32_t x = X[(size_t)t * n + s];
                        if (x >= 0) a[al] += dz[x];
                    }
                double L = logsumexp(a, r);
                for (int al = 0; al < r; ++al) {
                    double gamma = exp(a[al] - L);
                    dg_all[(size_t)t * r + al] = up * (exp(logw[al]) - gamma);
                    for (int s = 0; s < n; ++s) {
                        size_t row = ((size_t)t * n + s) * r + al;
                        double *dz = dz_all + row * V;
                        int32_t x = X[(size_t)t * n + s];
                        if (x < 0) {
                            for (int v = 0; v < V; ++v) dz[v] = 0.0;    /* dropped factor */
                        } else {
                            for (int v = 0; v < V; ++v) dz[v] = up * gamma * exp(dz[v]);
                            dz[x] -= up * gamma;
                        }
                        /* dy = U^T dz */
                        double *dy = dy_all + row * d;
                        for (int k = 0; k < d; ++k) {
                            double acc = 0.0;
                            for (int v = 0; v < V; ++v) acc += (double)U[(size_t)v * d + k] * dz[v];
                            dy[k] = acc;
                        }
                    }
                }
                if (dH) {
                    double *dh = dH + (size_t)t * d;
                    for (int j = 0; j < d; ++j) {
                        double acc = 0.0;
                        for (int s = 0; s < n; ++s)
                            for (int al = 0; al < r; ++al) {
                                const in_t *Wsa = W + ((size_t)s * r + al) * d * d;
                                const double *dy = dy_all + (((size_t)t * n + s) * r + al) * d;
                                for (int k = 0; k < d; ++k) acc += (double)Wsa[(size_t)k * d + j] * dy[k];
                            }
                        for (int al = 0; al < r; ++al)
                            acc += (double)G[(size_t)al * d + j] * dg_all[(size_t)t * r + al];
                        dh[j] = acc;
                    }
                }
            }
        }
        free(z); free(logw); free(a); free(lse);
    }

    /* phase 2: sums over positions */
    if (!fail && dW) {
#pragma omp parallel for schedule(static)
        for (int64_t sak = 0; sak < (int64_t)nr * d; ++sak) {   /* (s, al, k) */
            size_t sa = (size_t)sak / d;
            int k = (int)(sak % d);
            double *out = dW + (size_t)sak * d;
            for (int j = 0; j < d; ++j) out[j] = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                double dyk = dy_all[((size_t)t * nr + sa) * d + k];
                const in_t *h = H + (size_t)t * d;
                for (int j = 0; j < d; ++j) out[j] += dyk * (double)h[j];
            }
        }
    }
    if (!fail && dU) {
#pragma omp parallel for schedule(static)
        for (int v = 0; v < V; ++v) {
            double *out = dU + (size_t)v * d;
            for (int k = 0; k < d; ++k) out[k] = 0.0;
            for (size_t row = 0; row < (size_t)T * nr; ++row) {
                double dzv = dz_all[row * V + v];
                const double *y = y_all + row * d;
                for (int k = 0; k < d; ++k) out[k] += dzv * y[k];
            }
        }
    }
    if (!fail && dG) {
        for (int al = 0; al < r; ++al)
            for (int j = 0; j < d; ++j) {
                double acc = 0.0;
                for (int64_t t = 0; t < T; ++t) acc += dg_all[(size_t)t * r + al] * (double)H[(size_t)t * d + j];
                dG[(size_t)al * d + j] = acc;
            }
    }
    free(dz_all); free(y_all); free(dy_all); free(dg_all);
    return fail ? -1 : 0;
}

/* ------------------------------------------------------------------------- */
/* draft sampling                                                             */
/* ------------------------------------------------------------------------- */

/* first index whose running sum exceeds u, clamped to the last index */
static int inverse_cdf(const double *p, int len, double u, double *cdf_out)
{
    int pick = -1;
    double c = 0.0;
    for (int i = 0; i < len; ++i) {
        c += p[i];
        if (cdf_out) cdf_out[i] = c;
        if (pick < 0 && c > u) pick = i;
    }
    return pick < 0 ? len - 1 : pick;
}

/*
 * Draw one expert index and then n tokens per row ("Sampling method"; the
 * two-stage draw has exactly the joint of eq. 2, whose chain of conditionals
 * the paper's sequential scheme walks through).
 *
 *   uniforms[B,1+n] in [0,1): column 0 picks the expert, column 1+s token s.
 *   alpha_in : NULL, or B forced expert indices (then column 0 is ignored).
 *   alpha[B], tokens[B,n]: the draw.  logq[B] (may be NULL): eq. 9 evaluated at
 *   the drawn tuple, over all experts.
 *   cdf_w[B,r], cdf_tok[B,n,V] (may be NULL): the running sums the draw used.
 *   y_exact[B,n,r,d] (may be NULL): y before rounding; y_nudge[B,n,r,d] (may be NULL): added to y
 *   before rounding (see head_y_ex).
 *
 * Inverse-CDF convention: index order, first index with cdf > u, clamp to last.
 */
int CPO(draft_sample)(const cpo_shape *sh, const in_t *H, const in_t *W, const in_t *U, const in_t *G,
                      const double *uniforms, const int32_t *alpha_in,
                      int32_t *alpha, int32_t *tokens, double *logq, double *cdf_w, double *cdf_tok,
                      double *y_exact, const double *y_nudge)
{
    const int d = sh->d, V = sh->V, n = sh->n, r = sh->r;
    const size_t nr = (size_t)n * r;
    int fail = 0;
#pragma omp parallel
    {
        double *y = malloc(sizeof(double) * d);
        double *zs = malloc(sizeof(double) * nr * V);     /* z - lse for every (s, al) */
        double *p = malloc(sizeof(double) * (V > r ? V : r));
        double *logw = malloc(sizeof(double) * r);
        double *a = malloc(sizeof(double) * r);
        if (!y || !zs || !p || !logw || !a) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t b = 0; b < sh->T; ++b) {
                const in_t *h = H + (size_t)b * d;
                const double *u = uniforms + (size_t)b * (1 + n);
                gate_logw(sh, h, G, logw);
                for (int al = 0; al < r; ++al) p[al] = exp(logw[al]);
                int astar = inverse_cdf(p, r, u[0], cdf_w ? cdf_w + (size_t)b * r : NULL);
                if (alpha_in) astar = alpha_in[b];
                alpha[b] = astar;
                for (int s = 0; s < n; ++s)
                    for (int al = 0; al < r; ++al) {
                        double *z = zs + ((size_t)s * r + al) * V;
                        size_t row = ((size_t)b * n + s) * r + al;
                        head_y_ex(sh, h, W, s, al, y_nudge ? y_nudge + row * d : NULL,
                                  y_exact ? y_exact + row * d : NULL, y);
                        head_z(sh, U, y, z);
                        double l = logsumexp(z, V);
                        for (int v = 0; v < V; ++v) z[v] -= l;
                    }
                for (int al = 0; al < r; ++al) a[al] = logw[al];
                for (int s = 0; s < n; ++s) {
                    const double *lp = zs + ((size_t)s * r + astar) * V;
                    for (int v = 0; v < V; ++v) p[v] = exp(lp[v]);
                    int tok = inverse_cdf(p, V, u[1 + s], cdf_tok ? cdf_tok + ((size_t)b * n + s) * V : NULL);
                    tokens[(size_t)b * n + s] = tok;
                    for (int al = 0; al < r; ++al) a[al] += zs[((size_t)s * r + al) * V + tok];
                }
                if (logq) logq[b] = logsumexp(a, r);
            }
        }
        free(y); free(zs); free(p); free(logw); free(a);
    }
    return fail ? -1 : 0;
}

/*
 * The paper's sequential scheme, one step: the distribution of token s of one
 * position given the already drawn tokens prefix[0..s-1].  Eq. 11 is s = 0.
 * For s > 0 the printed equations omit the factor of the new token and the
 * normaliser; the reading taken here is the conditional that the joint of
 * eq. 2 implies,
 *   P(x_s | x_<s)  =  sum_a  q_a P^(s)(x_s | a),
 *   q_a  proportional to  w_a prod_{k<s} P^(k)(x_k | a),
 * i.e. the expert log-weights are updated with log P^(k)(x_k | a) after each
 * draw, as the text under eq. 12 describes.
 * prob[V] receives the distribution for position t.
 */
int CPO(sequential_conditional)(const cpo_shape *sh, const in_t *H, const in_t *W, const in_t *U, const in_t *G,
                                int64_t t, int s, const int32_t *prefix, double *prob)
{
    const int d = sh->d, V = sh->V, r = sh->r;
    double *y = malloc(sizeof(double) * d), *z = malloc(sizeof(double) * V);
    double *q = malloc(sizeof(double) * r);
    if (!y || !z || !q) { free(y); free(z); free(q); return -1; }
    const in_t *h = H + (size_t)t * d;
    gate_logw(sh, h, G, q);
    for (int k = 0; k < s; ++k)
        for (int al = 0; al < r; ++al) {
            head_y(sh, h, W, k, al, y);
            head_z(sh, U, y, z);
            q[al] += z[prefix[k]] - logsumexp(z, V);
        }
    double qn = logsumexp(q, r);
    for (int v = 0; v < V; ++v) prob[v] = 0.0;
    for (int al = 0; al < r; ++al) {
        head_y(sh, h, W, s, al, y);
        head_z(sh, U, y, z);
        double l = logsumexp(z, V);
        for (int v = 0; v < V; ++v) prob[v] += exp(q[al] - qn + z[v] - l);
    }
    free(y); free(z); free(q);
    return 0;
}

/*
 * First-token marginal (eq. 11) in log space: logp[b, v] = log sum_a w_a P^(1)(v | a).
 * logp[B,V].  y_nudge[B,r,d] (may be NULL) is added to the first head's y before rounding, as in
 * draft_sample (the two admissible roundings of an element on a rounding tie).
 */
int CPO(first_token_logprob)(const cpo_shape *sh, const in_t *H, const in_t *W, const in_t *U, const in_t *G,
                             const double *y_nudge, double *logp)
{
    const int d = sh->d, V = sh->V, r = sh->r;
    int fail = 0;
#pragma omp parallel
    {
        double *y = malloc(sizeof(double) * d), *z = malloc(sizeof(double) * (size_t)r * V);
        double *logw = malloc(sizeof(double) * r), *t = malloc(sizeof(double) * r);
        if (!y || !z || !logw || !t) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t b = 0; b < sh->T; ++b) {
                const in_t *h = H + (size_t)b * d;
                gate_logw(sh, h, G, logw);
                for (int al = 0; al < r; ++al) {
                    double *za = z + (size_t)al * V;
                    head_y_ex(sh, h, W, 0, al, y_nudge ? y_nudge + ((size_t)b * r + al) * d : NULL, NULL, y);
                    head_z(sh, U, y, za);
                    double l = logsumexp(za, V);
                    for (int v = 0; v < V; ++v) za[v] -= l;          /* log P^(1)(v | al) */
                }
                for (int v = 0; v < V; ++v) {
                    for (int al = 0; al < r; ++al) t[al] = logw[al] + z[(size_t)al * V + v];
                    logp[(size_t)b * V + v] = logsumexp(t, r);
                }
            }
        }
        free(y); free(z); free(logw); free(t);
    }
    return fail ? -1 : 0;
}

/*
 * The paper's sequential scheme ("Sampling method", eq. 11-13 with the reading documented at
 * sequential_conditional): x_1 is drawn from the first-token marginal, then each x_s from
 *   P(x_s | x_<s) = sum_a qhat_a P^(s)(x_s | a),   qhat = softmax(q),
 *   q_a = log w_a + sum_{k<s} log P^(k)(x_k | a)
 * ("updating the unnormalized logits of the experts").  One uniform per token: uniforms[B,n].
 * tokens[B,n]; logq[B] (may be NULL) = logsumexp_a q_a after the last draw, the joint
 * log-probability (eq. 9) of the drawn tuple; cdf[B,n,V] (may be NULL): the running sums used.
 * Inverse-CDF convention as in draft_sample; y_nudge[B,n,r,d] (may be NULL) as in draft_sample.
 */
int CPO(draft_sample_sequential)(const cpo_shape *sh, const in_t *H, const in_t *W, const in_t *U, const in_t *G,
                                 const double *uniforms, const double *y_nudge, int32_t *tokens, double *logq,
                                 double *cdf)
{
    const int d = sh->d, V = sh->V, n = sh->n, r = sh->r;
    int fail = 0;
#pragma omp parallel
    {
        double *y = malloc(sizeof(double) * d), *lp = malloc(sizeof(double) * (size_t)r * V);
        double *p = malloc(sizeof(double) * V), *q = malloc(sizeof(double) * r);
        if (!y || !lp || !p || !q) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t b = 0; b < sh->T; ++b) {
                const in_t *h = H + (size_t)b * d;
                gate_logw(sh, h, G, q);
                for (int s = 0; s < n; ++s) {
                    for (int al = 0; al < r; ++al) {
                        double *za = lp + (size_t)al * V;
                        head_y_ex(sh, h, W, s, al,
                                  y_nudge ? y_nudge + (((size_t)b * n + s) * r + al) * d : NULL, NULL, y);
                        head_z(sh, U, y, za);
                        double l = logsumexp(za, V);
                        for (int v = 0; v < V; ++v) za[v] -= l;      /* log P^(s)(v | al) */
                    }
                    double qn = logsumexp(q, r);
                    for (int v = 0; v < V; ++v) {
                        double acc = 0.0;
                        for (int al = 0; al < r; ++al) acc += exp(q[al] - qn + lp[(size_t)al * V + v]);
                        p[v] = acc;
                    }
                    int tok = inverse_cdf(p, V, uniforms[(size_t)b * n + s], cdf ? cdf + ((size_t)b * n + s) * V : NULL);
                    tokens[(size_t)b * n + s] = tok;
                    for (int al = 0; al < r; ++al) q[al] += lp[(size_t)al * V + tok];
                }
                if (logq) logq[b] = logsumexp(q, r);
            }
        }
        free(y); free(lp); free(p); free(q);
    }
    return fail ? -1 : 0;
}

/*
 * Auxiliary balancing statistic (eq. 10): counts[a] = number of positions whose largest gate weight is
 * expert a (first index on ties), and L_aux = sum_a (counts[a]/T - 1/r)^2.
 */
int CPO(aux_balance)(const cpo_shape *sh, const in_t *H, const in_t *G, int64_t *counts, double *laux)
{
    const int d = sh->d, r = sh->r;
    double *logw = malloc(sizeof(double) * r);
    if (!logw) return -1;
    for (int a = 0; a < r; ++a) counts[a] = 0;
    for (int64_t t = 0; t < sh->T; ++t) {
        gate_logw(sh, H + (size_t)t * d, G, logw);
        int best = 0;
        for (int a = 1; a < r; ++a) if (logw[a] > logw[best]) best = a;
        counts[best] += 1;
    }
    double acc = 0.0;
    for (int a = 0; a < r; ++a) {
        double dev = (sh->T > 0 ? (double)counts[a] / (double)sh->T : 0.0) - 1.0 / r;
        acc += dev * dev;
    }
    *laux = acc;
    free(logw);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* full heads (eq. 6 as printed): one V x d matrix per (s, a), no shared unembedding */
/* ------------------------------------------------------------------------- */

/* z = F_sa h, F[n,r,V,d] */
static void full_head_z(const cpo_shape *sh, const in_t *h, const in_t *F, int s, int a, double *z)
{
    const in_t *Fsa = F + ((size_t)s * sh->r + a) * sh->V * sh->d;
    for (int v = 0; v < sh->V; ++v) {
        double acc = 0.0;
        for (int k = 0; k < sh->d; ++k) acc += (double)Fsa[(size_t)v * sh->d + k] * (double)h[k];
        z[v] = acc;
    }
}

/*
 * Loss forward with full heads: P^(s)(. | a) = softmax(F_sa h) (eq. 6), the rest as in loss_fwd
 * (eq. 7, 8, 9).  H[T,d] F[n,r,V,d] G[r,d] X[T,n]; loss[T]; optional logw[T,r], C[T,n,r], lse[T,n,r].
 */
int CPO(full_loss_fwd)(const cpo_shape *sh, const in_t *H, const in_t *F, const in_t *G, const int32_t *X,
                       double *loss, double *logw_out, double *C_out, double *lse_out)
{
    if (sh->T < 0 || sh->d <= 0 || sh->V <= 0 || sh->n <= 0 || sh->r <= 0) return -1;
    const int d = sh->d, V = sh->V, n = sh->n, r = sh->r;
    int fail = 0;
#pragma omp parallel
    {
        double *z = malloc(sizeof(double) * V), *logw = malloc(sizeof(double) * r), *a = malloc(sizeof(double) * r);
        if (!z || !logw || !a) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t t = 0; t < sh->T; ++t) {
                const in_t *h = H + (size_t)t * d;
                gate_logw(sh, h, G, logw);
                for (int al = 0; al < r; ++al) a[al] = logw[al];
                for (int s = 0; s < n; ++s)
                    for (int al = 0; al < r; ++al) {
                        full_head_z(sh, h, F, s, al, z);
                        double lse = logsumexp(z, V);
                        int32_t x = X[(size_t)t * n + s];
                        double C = (x >= 0) ? z[x] - lse : 0.0;       /* eq. 8 */
                        a[al] += C;
                        size_t idx = ((size_t)t * n + s) * r + al;
                        if (C_out) C_out[idx] = C;
                        if (lse_out) lse_out[idx] = lse;
                    }
                loss[t] = -logsumexp(a, r);                            /* eq. 9 */
                if (logw_out) for (int al = 0; al < r; ++al) logw_out[(size_t)t * r + al] = logw[al];
            }
        }
        free(z); free(logw); free(a);
    }
    return fail ? -1 : 0;
}

/*
 * Gradients of sum_t dloss[t] * loss[t] with full heads: with gamma, dz and dg as in loss_bwd,
 *   dF_sa = sum_t dz_tsa (x) h_t ,  dG = sum_t dg_t (x) h_t ,  dh_t = sum_sa F_sa^T dz_tsa + G^T dg_t.
 * dH[T,d], dF[n,r,V,d], dG[r,d] are overwritten; any may be NULL; dloss may be NULL (all ones).
 * Stores dz for every (t, s, a): small T only.
 */
int CPO(full_loss_bwd)(const cpo_shape *sh, const in_t *H, const in_t *F, const in_t *G, const int32_t *X,
                       const double *dloss, double *dH, double *dF, double *dG)
{
    const int d = sh->d, V = sh->V, n = sh->n, r = sh->r;
    const int64_t T = sh->T;
    const size_t nr = (size_t)n * r;
    double *dz_all = malloc(sizeof(double) * ((size_t)T * nr * V + 1));
    double *dg_all = malloc(sizeof(double) * ((size_t)T * r + 1));
    if (!dz_all || !dg_all) { free(dz_all); free(dg_all); return -1; }
    int fail = 0;
#pragma omp parallel
    {
        double *z = malloc(sizeof(double) * V), *logw = malloc(sizeof(double) * r), *a = malloc(sizeof(double) * r);
        if (!z || !logw || !a) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t t = 0; t < T; ++t) {
                const in_t *h = H + (size_t)t * d;
                const double up = dloss ? dloss[t] : 1.0;
                gate_logw(sh, h, G, logw);
                for (int al = 0; al < r; ++al) a[al] = logw[al];
                for (int s = 0; s < n; ++s)
                    for (int al = 0; al < r; ++al) {
                        double *dz = dz_all + (((size_t)t * n + s) * r + al) * V;
                        full_head_z(sh, h, F, s, al, z);
                        double l = logsumexp(z, V);
                        for (int v = 0; v < V; ++v) dz[v] = z[v] - l;   /* log P^(s)(v | al) for now */
                        int32_t x = X[(size_t)t * n + s];
                        if (x >= 0) a[al] += dz[x];
                    }
                double L = logsumexp(a, r);
                for (int al = 0; al < r; ++al) {
                    double gamma = exp(a[al] - L);
                    dg_all[(size_t)t * r + al] = up * (exp(logw[al]) - gamma);
                    for (int s = 0; s < n; ++s) {
                        double *dz = dz_all + (((size_t)t * n + s) * r + al) * V;
                        int32_t x = X[(size_t)t * n + s];
                        if (x < 0) {
                            for (int v = 0; v < V; ++v) dz[v] = 0.0;
                        } else {
                            for (int v = 0; v < V; ++v) dz[v] = up * gamma * exp(dz[v]);
                            dz[x] -= up * gamma;
                        }
                    }
                }
                if (dH) {
                    double *dh = dH + (size_t)t * d;
                    for (int j = 0; j < d; ++j) {
                        double acc = 0.0;
                        for (size_t sa = 0; sa < nr; ++sa) {
                            const in_t *Fsa = F + sa * V * d;
                            const double *dz = dz_all + ((size_t)t * nr + sa) * V;
                            for (int v = 0; v < V; ++v) acc += (double)Fsa[(size_t)v * d + j] * dz[v];
                        }
                        for (int al = 0; al < r; ++al)
                            acc += (double)G[(size_t)al * d + j] * dg_all[(size_t)t * r + al];
                        dh[j] = acc;
                    }
                }
            }
        }
        free(z); free(logw); free(a);
    }
    if (!fail && dF) {
#pragma omp parallel for schedule(static)
        for (int64_t sav = 0; sav < (int64_t)nr * V; ++sav) {   /* (s, al, v) */
            size_t sa = (size_t)sav / V;
            int v = (int)(sav % V);
            double *out = dF + (size_t)sav * d;
            for (int j = 0; j < d; ++j) out[j] = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                double dzv = dz_all[((size_t)t * nr + sa) * V + v];
                const in_t *h = H + (size_t)t * d;
                for (int j = 0; j < d; ++j) out[j] += dzv * (double)h[j];
            }
        }
    }
    if (!fail && dG) {
        for (int al = 0; al < r; ++al)
            for (int j = 0; j < d; ++j) {
                double acc = 0.0;
                for (int64_t t = 0; t < T; ++t) acc += dg_all[(size_t)t * r + al] * (double)H[(size_t)t * d + j];
                dG[(size_t)al * d + j] = acc;
            }
    }
    free(dz_all); free(dg_all);
    return fail ? -1 : 0;
}

/* ------------------------------------------------------------------------- */
/* head-only fine-tuning loss ("Fine tuning", eq. 14 and the sum after it)    */
/* ------------------------------------------------------------------------- */

/*
 * The paper leaves open what the k-th token's distribution p^d is conditioned on, the direction of the
 * KL term and the discount.  Reading taken here:
 *   p^d_k[v] = P(x_k = v | x_<k) = sum_a qhat^(k)_a P^(k)(v | a),  qhat^(k) = softmax_a(log w_a + sum_{j<k} C_ja)
 *              (the conditional of eq. 13 under the true prefix x_<k);
 *   p^c_k    = softmax(TZ[t,k,:]), the distribution of the original head, supplied by the caller;
 *   L_k      = beta * KL(p^c_k || p^d_k) + (1 - beta) * (-log p^d_k[x_k])
 *              (arguments read as (prediction, target) in both terms of eq. 14);
 *   loss[t]  = sum_{k=1..n} disc^(k-1) L_k.
 * With beta = 0 and disc = 1 the chain of conditionals multiplies to the joint, so the loss is that of
 * loss_fwd.  A negative target drops token k's term; its factor then leaves the expert weights unchanged.
 *
 * TZ[T,n,V] teacher logits.  loss[T]; optional kl[T,n], ce[T,n] (zero for dropped tokens).
 */
int CPO(distill_loss_fwd)(const cpo_shape *sh, const in_t *H, const in_t *W, const in_t *U, const in_t *G,
                          const int32_t *X, const in_t *TZ, double beta, double disc,
                          double *loss, double *kl_out, double *ce_out)
{
    const int d = sh->d, V = sh->V, n = sh->n, r = sh->r;
    int fail = 0;
#pragma omp parallel
    {
        double *y = malloc(sizeof(double) * d), *lp = malloc(sizeof(double) * (size_t)r * V);
        double *lpc = malloc(sizeof(double) * V), *q = malloc(sizeof(double) * r);
        if (!y || !lp || !lpc || !q) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t t = 0; t < sh->T; ++t) {
                const in_t *h = H + (size_t)t * d;
                gate_logw(sh, h, G, q);
                double total = 0.0, weight = 1.0;
                for (int k = 0; k < n; ++k, weight *= disc) {
                    const int32_t x = X[(size_t)t * n + k];
                    double kl = 0.0, ce = 0.0;
                    if (x >= 0) {
                        for (int al = 0; al < r; ++al) {
                            double *za = lp + (size_t)al * V;
                            head_y(sh, h, W, k, al, y);
                            head_z(sh, U, y, za);
                            double l = logsumexp(za, V);
                            for (int v = 0; v < V; ++v) za[v] -= l;                  /* log P^(k)(v | al) */
                        }
                        const in_t *tz = TZ + ((size_t)t * n + k) * V;
                        for (int v = 0; v < V; ++v) lpc[v] = (double)tz[v];
                        double lt = logsumexp(lpc, V);
                        for (int v = 0; v < V; ++v) lpc[v] -= lt;                    /* log p^c_k[v] */
                        double qn = logsumexp(q, r);
                        for (int v = 0; v < V; ++v) {
                            double m = 0.0;
                            for (int al = 0; al < r; ++al) m += exp(q[al] - qn + lp[(size_t)al * V + v]);
                            kl += exp(lpc[v]) * (lpc[v] - log(m));
                            if (v == x) ce = -log(m);
                        }
                        total += weight * (beta * kl + (1.0 - beta) * ce);
                        for (int al = 0; al < r; ++al) q[al] += lp[(size_t)al * V + x];
                    }
                    if (kl_out) kl_out[(size_t)t * n + k] = kl;
                    if (ce_out) ce_out[(size_t)t * n + k] = ce;
                }
                loss[t] = total;
            }
        }
        free(y); free(lp); free(lpc); free(q);
    }
    return fail ? -1 : 0;
}

/*
 * Gradients of sum_t dloss[t] * loss[t] for distill_loss_fwd (the teacher logits are constants).
 * With g_k = disc^(k-1) (zero for a dropped token), rho_a[v] = qhat_a P_a[v] / p^d[v] (expert posterior
 * given token v), S_a = sum_v p^c[v] rho_a[v] and R_a = beta S_a + (1 - beta) rho_a[x_k], all for token k:
 *   dL/dq^(k)_a = g_k (qhat_a - R_a)                 q^(k)_a = log w_a + sum_{j<k} C_ja
 *   dL/dz_ka[v] = g_k ( R_a P_a[v] - beta p^c[v] rho_a[v] - (1 - beta) rho_a[x_k] 1[v = x_k] )
 *                 + D_ka (1[v = x_k] - P_a[v]),      D_ka = sum_{k' > k} dL/dq^(k')_a   (through C_ka)
 *   dL/dg_a     = sum_k dL/dq^(k)_a                  (these sum to zero over a, so the log-softmax of the
 *                                                     gate passes them through unchanged)
 * and below z, g everything is linear as in loss_bwd.  dH, dW, dU, dG overwritten; any may be NULL.
 */
int CPO(distill_loss_bwd)(const cpo_shape *sh, const in_t *H, const in_t *W, const in_t *U, const in_t *G,
                          const int32_t *X, const in_t *TZ, double beta, double disc, const double *dloss,
                          double *dH, double *dW, double *dU, double *dG)
{
    if (sh->round_y) return -1;
    const int d = sh->d, V = sh->V, n = sh->n, r = sh->r;
    const int64_t T = sh->T;
    const size_t nr = (size_t)n * r;
    double *dz_all = malloc(sizeof(double) * ((size_t)T * nr * V + 1));
    double *y_all = malloc(sizeof(double) * ((size_t)T * nr * d + 1));
    double *dy_all = malloc(sizeof(double) * ((size_t)T * nr * d + 1));
    double *dg_all = malloc(sizeof(double) * ((size_t)T * r + 1));
    if (!dz_all || !y_all || !dy_all || !dg_all) { free(dz_all); free(y_all); free(dy_all); free(dg_all); return -1; }
    int fail = 0;
#pragma omp parallel
    {
        double *lpc = malloc(sizeof(double) * V), *q = malloc(sizeof(double) * r), *qh = malloc(sizeof(double) * r);
        double *m = malloc(sizeof(double) * V);
        double *dq = malloc(sizeof(double) * nr);      /* dL/dq^(k)_a */
        double *Rk = malloc(sizeof(double) * nr), *rhox = malloc(sizeof(double) * nr);
        if (!lpc || !q || !qh || !m || !dq || !Rk || !rhox) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t t = 0; t < T; ++t) {
                const in_t *h = H + (size_t)t * d;
                const double up = dloss ? dloss[t] : 1.0;
                gate_logw(sh, h, G, q);
                double weight = 1.0;
                /* forward sweep over the tokens: dz_all holds log P, then the first part of dz */
                for (int k = 0; k < n; ++k, weight *= disc) {
                    const int32_t x = X[(size_t)t * n + k];
                    for (int al = 0; al < r; ++al) {
                        size_t row = ((size_t)t * n + k) * r + al;
                        double *y = y_all + row * d, *lp = dz_all + row * V;
                        head_y(sh, h, W, k, al, y);
                        head_z(sh, U, y, lp);
                        double l = logsumexp(lp, V);
                        for (int v = 0; v < V; ++v) lp[v] -= l;
                    }
                    if (x < 0) {
                        for (int al = 0; al < r; ++al) {
                            dq[(size_t)k * r + al] = 0.0; Rk[(size_t)k * r + al] = 0.0; rhox[(size_t)k * r + al] = 0.0;
                            double *lp = dz_all + (((size_t)t * n + k) * r + al) * V;
                            for (int v = 0; v < V; ++v) lp[v] = 0.0;                 /* dropped: no gradient */
                        }
                        continue;
                    }
                    const in_t *tz = TZ + ((size_t)t * n + k) * V;
                    for (int v = 0; v < V; ++v) lpc[v] = (double)tz[v];
                    double lt = logsumexp(lpc, V);
                    for (int v = 0; v < V; ++v) lpc[v] -= lt;
                    double qn = logsumexp(q, r);
                    for (int al = 0; al < r; ++al) qh[al] = exp(q[al] - qn);
                    for (int v = 0; v < V; ++v) {
                        double acc = 0.0;
                        for (int al = 0; al < r; ++al)
                            acc += qh[al] * exp(dz_all[(((size_t)t * n + k) * r + al) * V + v]);
                        m[v] = acc;                                                  /* p^d_k[v] */
                    }
                    for (int al = 0; al < r; ++al) {
                        double *lp = dz_all + (((size_t)t * n + k) * r + al) * V;
                        double S = 0.0;
                        for (int v = 0; v < V; ++v) S += exp(lpc[v]) * qh[al] * exp(lp[v]) / m[v];
                        double rx = qh[al] * exp(lp[x]) / m[x];
                        double R = beta * S + (1.0 - beta) * rx;
                        Rk[(size_t)k * r + al] = R;
                        rhox[(size_t)k * r + al] = rx;
                        dq[(size_t)k * r + al] = weight * (qh[al] - R);
                        q[al] += lp[x];                                              /* C_ka enters later tokens */
                        /* first part of dz, g_k ( R P - beta p^c rho - (1-beta) rho[x] 1[v=x] ), replaces log P in the slot */
                        for (int v = 0; v < V; ++v) {
                            double P = exp(lp[v]);
                            double rho = qh[al] * P / m[v];
                            double val = weight * (R * P - beta * exp(lpc[v]) * rho);
                            if (v == x) val -= weight * (1.0 - beta) * rx;
                            lp[v] = val;
                        }
                    }
                }
                /* second part: D_ka (1[v = x_k] - P_ka[v]), known once every later token has been seen;
                 * P is formed again from y (the slot no longer holds log P) */
                for (int k = 0; k < n; ++k) {
                    const int32_t x = X[(size_t)t * n + k];
                    if (x < 0) continue;
                    for (int al = 0; al < r; ++al) {
                        double D = 0.0;
                        for (int k2 = k + 1; k2 < n; ++k2) D += dq[(size_t)k2 * r + al];
                        size_t row = ((size_t)t * n + k) * r + al;
                        double *dz = dz_all + row * V;
                        head_z(sh, U, y_all + row * d, m);                           /* m is free by now: z_ka */
                        double l = logsumexp(m, V);
                        for (int v = 0; v < V; ++v) dz[v] -= D * exp(m[v] - l);
                        dz[x] += D;
                    }
                }
                for (int al = 0; al < r; ++al) {
                    double acc = 0.0;
                    for (int k = 0; k < n; ++k) acc += dq[(size_t)k * r + al];
                    dg_all[(size_t)t * r + al] = up * acc;
                }
                for (int k = 0; k < n; ++k)
                    for (int al = 0; al < r; ++al) {
                        size_t row = ((size_t)t * n + k) * r + al;
                        double *dz = dz_all + row * V, *dy = dy_all + row * d;
                        for (int v = 0; v < V; ++v) dz[v] *= up;
                        for (int j = 0; j < d; ++j) {
                            double acc = 0.0;
                            for (int v = 0; v < V; ++v) acc += (double)U[(size_t)v * d + j] * dz[v];
                            dy[j] = acc;
                        }
                    }
                if (dH) {
                    double *dh = dH + (size_t)t * d;
                    for (int j = 0; j < d; ++j) {
                        double acc = 0.0;
                        for (size_t sa = 0; sa < nr; ++sa) {
                            const in_t *Wsa = W + sa * d * d;
                            const double *dy = dy_all + ((size_t)t * nr + sa) * d;
                            for (int kk = 0; kk < d; ++kk) acc += (double)Wsa[(size_t)kk * d + j] * dy[kk];
                        }
                        for (int al = 0; al < r; ++al)
                            acc += (double)G[(size_t)al * d + j] * dg_all[(size_t)t * r + al];
                        dh[j] = acc;
                    }
                }
            }
        }
        free(lpc); free(q); free(qh); free(m); free(dq); free(Rk); free(rhox);
    }
    if (!fail && dW) {
#pragma omp parallel for schedule(static)
        for (int64_t sak = 0; sak < (int64_t)nr * d; ++sak) {
            size_t sa = (size_t)sak / d;
            int kk = (int)(sak % d);
            double *out = dW + (size_t)sak * d;
            for (int j = 0; j < d; ++j) out[j] = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                double dyk = dy_all[((size_t)t * nr + sa) * d + kk];
                const in_t *h = H + (size_t)t * d;
                for (int j = 0; j < d; ++j) out[j] += dyk * (double)h[j];
            }
        }
    }
    if (!fail && dU) {
#pragma omp parallel for schedule(static)
        for (int v = 0; v < V; ++v) {
            double *out = dU + (size_t)v * d;
            for (int j = 0; j < d; ++j) out[j] = 0.0;
            for (size_t row = 0; row < (size_t)T * nr; ++row) {
                double dzv = dz_all[row * V + v];
                const double *y = y_all + row * d;
                for (int j = 0; j < d; ++j) out[j] += dzv * y[j];
            }
        }
    }
    if (!fail && dG) {
        for (int al = 0; al < r; ++al)
            for (int j = 0; j < d; ++j) {
                double acc = 0.0;
                for (int64_t t = 0; t < T; ++t) acc += dg_all[(size_t)t * r + al] * (double)H[(size_t)t * d + j];
                dG[(size_t)al * d + j] = acc;
            }
    }
    free(dz_all); free(y_all); free(dy_all); free(dg_all);
    return fail ? -1 : 0;
}

/* For tests of the rounding helper. */
double CPO(round_to_bf16)(double v) { return round_to_bf16(v); }

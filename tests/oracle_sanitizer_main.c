/*
 * Host-only sanitizer run of the CPU oracle: this file includes the oracle's C source, is built with
 * -fsanitize=address,undefined by tests/test_oracle_sanitizers.py and calls every entry point once on a
 * tiny problem whose buffers are heap blocks of exactly the documented sizes, so that a read or write one
 * element past any of them, a leak, or undefined arithmetic aborts the run.  It checks no values (the
 * pins do); it prints "ok" and returns 0 if every call returned 0.
 */
#include "cp_oracle.c"

#include <stdio.h>

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform01(void)
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}
static in_t *random_block(size_t count, double scale)
{
    in_t *p = malloc(sizeof(in_t) * count);
    for (size_t i = 0; i < count; ++i) p[i] = (in_t)((uniform01() * 2.0 - 1.0) * scale);
    return p;
}
static double *doubles(size_t count) { return malloc(sizeof(double) * (count ? count : 1)); }

int main(void)
{
    const int T = 5, d = 6, V = 7, n = 3, r = 3;
    int bad = 0;
    for (int round_y = 0; round_y < 2; ++round_y) {
        cpo_shape sh = {T, d, V, n, r, round_y};
        in_t *H = random_block((size_t)T * d, 1.0), *W = random_block((size_t)n * r * d * d, 0.4);
        in_t *U = random_block((size_t)V * d, 0.6), *G = random_block((size_t)r * d, 0.4);
        in_t *F = random_block((size_t)n * r * V * d, 0.4), *TZ = random_block((size_t)T * n * V, 1.5);
        int32_t *X = malloc(sizeof(int32_t) * T * n), *alpha = malloc(sizeof(int32_t) * T);
        int32_t *tokens = malloc(sizeof(int32_t) * T * n);
        for (int i = 0; i < T * n; ++i) X[i] = (int32_t)(uniform01() * V);
        X[1] = -1;                                            /* a dropped factor */
        double *loss = doubles(T), *logw = doubles((size_t)T * r), *C = doubles((size_t)T * n * r);
        double *lse = doubles((size_t)T * n * r), *prob = doubles(V > T ? V : T), *dloss = doubles(T);
        double *dH = doubles((size_t)T * d), *dW = doubles((size_t)n * r * d * d), *dU = doubles((size_t)V * d);
        double *dG = doubles((size_t)r * d), *dF = doubles((size_t)n * r * V * d);
        double *u = doubles((size_t)T * (1 + n)), *logq = doubles(T), *cdf_w = doubles((size_t)T * r);
        double *cdf_tok = doubles((size_t)T * n * V), *y_exact = doubles((size_t)T * n * r * d);
        double *nudge = doubles((size_t)T * n * r * d), *logp = doubles((size_t)T * V);
        double *kl = doubles((size_t)T * n), *ce = doubles((size_t)T * n), laux = 0.0;
        int64_t counts[3];
        for (int i = 0; i < T * (1 + n); ++i) u[i] = uniform01();
        for (int i = 0; i < T; ++i) dloss[i] = uniform01();
        for (int i = 0; i < T * n * r * d; ++i) nudge[i] = 1e-4 * (uniform01() - 0.5);

        bad |= CPO(loss_fwd)(&sh, H, W, U, G, X, loss, logw, C, lse);
        bad |= CPO(loss_fwd)(&sh, H, W, U, G, X, loss, NULL, NULL, NULL);
        bad |= CPO(draft_sample)(&sh, H, W, U, G, u, NULL, alpha, tokens, logq, cdf_w, cdf_tok, y_exact, nudge);
        bad |= CPO(draft_sample)(&sh, H, W, U, G, u, alpha, alpha, tokens, NULL, NULL, NULL, NULL, NULL);
        bad |= CPO(sequential_conditional)(&sh, H, W, U, G, T - 1, 2, tokens, prob);
        bad |= CPO(first_token_logprob)(&sh, H, W, U, G, nudge, logp);
        bad |= CPO(draft_sample_sequential)(&sh, H, W, U, G, u, nudge, tokens, logq, cdf_tok);
        bad |= CPO(aux_balance)(&sh, H, G, counts, &laux);
        if (!round_y) {
            bad |= CPO(joint_prob_naive)(&sh, H, W, U, G, X, prob);
            bad |= CPO(loss_bwd)(&sh, H, W, U, G, X, dloss, dH, dW, dU, dG);
            bad |= CPO(loss_bwd)(&sh, H, W, U, G, X, NULL, dH, NULL, NULL, NULL);
            bad |= CPO(full_loss_fwd)(&sh, H, F, G, X, loss, logw, C, lse);
            bad |= CPO(full_loss_bwd)(&sh, H, F, G, X, dloss, dH, dF, dG);
            bad |= CPO(distill_loss_fwd)(&sh, H, W, U, G, X, TZ, 0.7, 0.9, loss, kl, ce);
            bad |= CPO(distill_loss_bwd)(&sh, H, W, U, G, X, TZ, 0.7, 0.9, dloss, dH, dW, dU, dG);
        }
        /* an empty batch touches nothing */
        cpo_shape empty = {0, d, V, n, r, round_y};
        bad |= CPO(loss_fwd)(&empty, H, W, U, G, X, loss, NULL, NULL, NULL);
        free(H); free(W); free(U); free(G); free(F); free(TZ); free(X); free(alpha); free(tokens);
        free(loss); free(logw); free(C); free(lse); free(prob); free(dloss); free(dH); free(dW); free(dU); free(dG);
        free(dF); free(u); free(logq); free(cdf_w); free(cdf_tok); free(y_exact); free(nudge); free(logp);
        free(kl); free(ce);
    }
    (void)CPO(round_to_bf16)(1.00390625);
    if (bad) { fprintf(stderr, "an oracle call failed\n"); return 1; }
    puts("ok");
    return 0;
}

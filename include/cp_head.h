/*
 * cp_head.h - C ABI of the MI355X (gfx950) CP multi-token-prediction head.
 *
 * The head models the joint distribution of the next n tokens after a position
 * as a rank-r canonical (CP) mixture (paper eq. 2):
 *
 *     P(x_1..x_n | h) = sum_a  w_a  prod_s  P^(s)(x_s | a)
 *     w               = softmax(G h)                               (eq. 7)
 *     P^(s)(. | a)    = softmax(U (W_sa h))                        (eq. 6, with the
 *                        shared-unembedding head of section "Fine tuning")
 *
 * Tensors (all dense, row-major, DEVICE pointers owned by the caller):
 *     H[T,d]       hidden states, one row per position
 *     W[n,r,d,d]   W[s,a] is d x d, y = W[s,a] h  (row = output feature)
 *     U[V,d]       shared unembedding
 *     G[r,d]       gate
 *     X[T,n]       int32 targets, X[t,s] = token s+1 steps after position t;
 *                  a negative entry drops that factor (no loss term, no gradient);
 *                  entries >= V are undefined behaviour
 * H, W, U, G have the storage type named by cp_head_desc.dtype; all arithmetic
 * accumulates in fp32.
 *
 * General rules for every entry point:
 *   - the library allocates no memory and keeps no state between calls: the
 *     caller supplies `ctx` (values saved by the forward pass for the backward
 *     pass) and `workspace` (scratch, contents undefined afterwards), sized by
 *     the two query functions; both must be 256-byte aligned;
 *   - every call only enqueues work on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and never synchronises;
 *   - the return value is CP_HEAD_OK or a negative error code; on error nothing
 *     was enqueued, except CP_HEAD_ERR_LAUNCH which reports a failed launch;
 *   - results are deterministic: no floating-point atomics are used.
 *
 * Limits: 1 <= r <= 64, 1 <= n <= 64, d >= 1, V >= 1, T >= 0, T*n*r*max(d,V) < 2^62.
 * The matrix-core path is taken for dtype = bf16 with d a multiple of 64; other
 * shapes and fp32 storage run on a plain fp32 path (correct for any shape, slow).
 */
#ifndef CP_HEAD_H
#define CP_HEAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CP_HEAD_FP32 = 0,   /* H, W, U, G are float */
    CP_HEAD_BF16 = 1    /* H, W, U, G are bfloat16 (raw 16-bit patterns) */
};

enum {
    CP_HEAD_FORCE_GENERIC = 1,  /* flags bit 0: use the plain fp32 path even where the
                                   matrix-core path applies (a second opinion in tests) */
    CP_HEAD_MIN_WORKSPACE = 2,  /* flags bit 1: the backward pass holds logit gradients for one
                                   tile of 256 head rows at a time (least workspace, slower)
                                   instead of its default of 32768 rows or 4 GiB worth of them,
                                   whichever is more, up to 8 GiB (0.5 GiB on the plain path) */
    CP_HEAD_KEEP_LOGITS = 4     /* flags bit 2, off by default (by default no logit is ever stored).
                                   Matrix-core path of the three loss call pairs only (cp_head_loss_,
                                   cp_head_full_loss_, cp_head_distill_loss_ fwd / bwd; ignored on the
                                   plain path and by the other calls): the forward pass keeps every logit
                                   in ctx as a 16-bit float relative to the maximum of its row over a
                                   block of 128 columns (T*n*r*roundup(V,64)*2 bytes plus 16 bytes per row
                                   and 256 columns), and the backward pass reads them back instead of
                                   multiplying U y a second time.  Trades HBM capacity for a quarter of
                                   the backward pass's matrix work; set it in the desc of both calls of a
                                   pair or of neither. */
};

enum {
    CP_HEAD_OK = 0,
    CP_HEAD_ERR_INVALID_ARG = -1,     /* null pointer, bad dimension, misaligned buffer */
    CP_HEAD_ERR_UNSUPPORTED = -2,     /* shape or dtype outside the stated limits */
    CP_HEAD_ERR_WORKSPACE = -3,       /* workspace_bytes smaller than the query reports */
    CP_HEAD_ERR_LAUNCH = -4,          /* a kernel launch failed (hipGetLastError) */
    CP_HEAD_ERR_STATIC_SCRATCH = -5   /* cp_head_draft_sample_static: the shape needs more scratch than
                                         CP_HEAD_STATIC_SCRATCH_BYTES */
};

enum {
    CP_HEAD_OP_LOSS_FWD = 0, CP_HEAD_OP_LOSS_BWD = 1, CP_HEAD_OP_DRAFT = 2,
    CP_HEAD_OP_FIRST_TOKEN = 3, CP_HEAD_OP_DRAFT_SEQUENTIAL = 4, CP_HEAD_OP_AUX_BALANCE = 5,
    CP_HEAD_OP_FULL_LOSS_FWD = 6, CP_HEAD_OP_FULL_LOSS_BWD = 7,
    CP_HEAD_OP_DISTILL_FWD = 8, CP_HEAD_OP_DISTILL_BWD = 9,
    CP_HEAD_OP_LOSS_FWD_BWD = 10
};

typedef struct cp_head_desc {
    int64_t T;        /* positions (loss calls) or batch size B (draft call) */
    int32_t d;        /* hidden size */
    int32_t V;        /* vocabulary size */
    int32_t n;        /* future tokens per position */
    int32_t r;        /* CP rank = number of experts */
    int32_t dtype;    /* CP_HEAD_FP32 or CP_HEAD_BF16 */
    int32_t flags;    /* OR of CP_HEAD_FORCE_GENERIC, CP_HEAD_MIN_WORKSPACE, CP_HEAD_KEEP_LOGITS, or 0 */
} cp_head_desc;

/* Human-readable text for an error code (static storage). */
const char *cp_head_strerror(int code);

/*
 * Bytes of `ctx` that cp_head_loss_fwd fills and cp_head_loss_bwd reads: the
 * log-normaliser of every factor (eq. 5), the gate weights (eq. 7), the
 * posterior over experts, and the projected states y = W_sa h; with
 * CP_HEAD_KEEP_LOGITS also the logits.  Host-only.
 */
int cp_head_ctx_bytes(const cp_head_desc *desc, size_t *bytes);

/*
 * Bytes of scratch `workspace` that operation `op` (CP_HEAD_OP_*) needs for
 * this shape.  Host-only.  The size is bounded in the number of positions for
 * the logit-sized buffers: logits and their gradients are only ever held for a
 * bounded chunk of rows, never for all T*n*r rows (CP_HEAD_KEEP_LOGITS keeps
 * the logits of all rows, but in ctx, not here).
 */
int cp_head_workspace_bytes(const cp_head_desc *desc, int op, size_t *bytes);

/*
 * Training loss, forward (section "Training procedure", eq. 8 and eq. 9):
 *     C_sa    = z_sa[X[t,s]] - logsumexp_v z_sa[v],   z_sa = U (W_sa h_t)
 *     loss[t] = -logsumexp_a( log w_a + sum_s C_sa )          (nats, no reduction)
 * loss[T] is fp32, overwritten.  ctx receives what the backward pass needs.
 * Precision on the matrix-core path (bf16 storage): the log-normalisers are formed from logits of y
 * rounded to bf16 (a matrix-core operand), the target logit z_sa[X[t,s]] from y kept to about fp32
 * (bf16 value plus bf16 residual).  exp(-loss) is therefore the joint of eq. 2 only up to that
 * mixed rounding: within 2e-3 of the unrounded value at the workloads' shapes.  -logq that
 * cp_head_draft_sample reports for the same tokens takes every term from the rounded y and
 * differs from loss by the rounding of the n target logits: rms about 1.1e-3 sqrt(n) for logits
 * of unit scale, below 1e-2 at n = 4.  The backward pass differentiates the function with the
 * rounded y throughout.
 */
int cp_head_loss_fwd(const cp_head_desc *desc,
                     const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X,
                     float *loss,
                     void *ctx, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Training loss, backward: gradients of  sum_t dloss[t] * loss[t]  (the
 * derivative of eq. 9 through eq. 8, 6 and 7).  `ctx` must come from
 * cp_head_loss_fwd on the same desc and inputs.  dloss[T] is fp32; NULL means
 * dloss[t] = scale for all t (otherwise `scale` multiplies dloss).
 * Outputs are fp32 and OVERWRITTEN: dH[T,d], dW[n,r,d,d], dU[V,d], dG[r,d].
 * dU may be NULL (frozen unembedding: that product is skipped); dW and dG may
 * be NULL too; dH is required.
 */
int cp_head_loss_bwd(const cp_head_desc *desc,
                     const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X,
                     const float *dloss, float scale,
                     const void *ctx,
                     float *dH, float *dW, float *dU, float *dG,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * Training loss and its gradients in one call (section "Training procedure", eq. 9 and its derivative), for
 * training loops in which the loss is the last node of the graph, so that the upstream gradient is known
 * before the forward pass: dloss[T] / scale as in cp_head_loss_bwd.  loss[T] and the gradients are exactly
 * what cp_head_loss_fwd followed by cp_head_loss_bwd return (same kernels, same arithmetic); no ctx is needed,
 * the workspace is sized by cp_head_workspace_bytes with CP_HEAD_OP_LOSS_FWD_BWD.
 * What the single call buys on the matrix-core path: forward and backward are interleaved per chunk of
 * positions, and the logits of a chunk are kept as 16-bit floats from the product that forms their statistics to
 * the pass that turns them into gradients a few launches later.  U y is therefore multiplied once per step
 * instead of twice, as with CP_HEAD_KEEP_LOGITS, but the kept logits are those of one chunk only: at most 4 GiB
 * (8 GiB for vocabularies whose 32768 rows need more), however many positions the batch has.  The logits do
 * reach HBM in this call, one bounded chunk at a time; the pair of calls above with flags = 0 never stores one.
 * dU, dW, dG may be NULL as in cp_head_loss_bwd; loss and dH are required.  CP_HEAD_KEEP_LOGITS is ignored.
 */
int cp_head_loss_fwd_bwd(const cp_head_desc *desc,
                         const void *H, const void *W, const void *U, const void *G,
                         const int32_t *X,
                         const float *dloss, float scale,
                         float *loss,
                         float *dH, float *dW, float *dU, float *dG,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * Draft step for self-speculative decoding (section "Sampling method"): for
 * each of the B = desc->T rows of H draw an expert a* ~ w and then, for every
 * s, a token from P^(s)(. | a*).  The pair of draws has exactly the joint of
 * eq. 2, i.e. the distribution the paper's sequential scheme (eq. 11-13)
 * samples from.  The library holds no random-number generator:
 *     uniforms[B,1+n]  fp32 in [0,1): column 0 draws the expert, column 1+s token s.
 * Inverse-CDF convention: index order, the first index whose running sum
 * exceeds u, clamped to the last index.  With bf16 storage y = W_sa h is
 * rounded to bf16 (nearest-even) before z = U y: that rounding is part of the
 * sampled distribution's definition.
 * Outputs: alpha[B] int32, tokens[B,n] int32, logq[B] fp32 (may be NULL) =
 * log of eq. 2 at the drawn tuple, summed over all experts, every logit taken from the
 * rounded y (so -logq and cp_head_loss_fwd at the same tokens differ by the rounding of
 * the n target logits: see cp_head_loss_fwd).
 */
int cp_head_draft_sample(const cp_head_desc *desc,
                         const void *H, const void *W, const void *U, const void *G,
                         const float *uniforms,
                         int32_t *alpha, int32_t *tokens, float *logq,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same draft step for callers that cannot hand over or allocate a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  The scratch memory the kernels need
 * lives in a static device array inside the library, CP_HEAD_STATIC_SCRATCH_BYTES per GPU, held until
 * the process ends; the call allocates nothing (no device, host or library allocation; leave the
 * timing hook below switched off, which creates events).  Arguments and results are those of
 * cp_head_draft_sample, bit for bit.  A shape whose cp_head_workspace_bytes(desc, CP_HEAD_OP_DRAFT)
 * exceeds CP_HEAD_STATIC_SCRATCH_BYTES is refused with CP_HEAD_ERR_STATIC_SCRATCH and nothing is
 * enqueued (48 MiB holds B = 64 rows at d = 4096, V = 128256, n = 4, r = 8).  The first call on a
 * device looks up that device's copy of the array (make it outside any graph capture); all calls on
 * one GPU share the array, so calls that overlap on one GPU (different streams or threads) race:
 * serialise them.  Nothing in the array has to start at zero and nothing is kept between calls.
 */
#define CP_HEAD_STATIC_SCRATCH_BYTES ((size_t)48 << 20)
int cp_head_draft_sample_static(const cp_head_desc *desc,
                                const void *H, const void *W, const void *U, const void *G,
                                const float *uniforms,
                                int32_t *alpha, int32_t *tokens, float *logq,
                                void *stream);

/*
 * First-token marginal (eq. 11), in log space, for each of the B = desc->T rows of H:
 *     logp[b, v] = log sum_a w_a P^(1)(v | a)
 * This is the distribution of the next token under the head (the one a speculative verifier or
 * the first-token loss needs).  logp[B,V] fp32, overwritten.  With bf16 storage y is rounded to
 * bf16 as in cp_head_draft_sample.
 */
int cp_head_first_token_logprob(const cp_head_desc *desc,
                                const void *H, const void *W, const void *U, const void *G,
                                float *logp,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * The paper's own sequential sampling scheme (section "Sampling method", eq. 11-13): x_1 is drawn
 * from the first-token marginal and each further x_s from
 *     P(x_s | x_<s) = sum_a qhat_a P^(s)(x_s | a),  qhat = softmax(q),
 *     q_a = log w_a + sum_{k<s} log P^(k)(x_k | a)
 * (the expert log-weights are updated after every draw; the printed eq. 12/13 omit the new token's
 * factor and the normaliser).  It samples the same joint (eq. 2) as cp_head_draft_sample but
 * needs no expert draw: uniforms[B,n] fp32 in [0,1), one per token; inverse-CDF convention and
 * the bf16 rounding of y as in cp_head_draft_sample.  Outputs: tokens[B,n] int32, logq[B] fp32
 * (may be NULL) = joint log-probability of the drawn tuple.
 */
int cp_head_draft_sample_sequential(const cp_head_desc *desc,
                                    const void *H, const void *W, const void *U, const void *G,
                                    const float *uniforms,
                                    int32_t *tokens, float *logq,
                                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * Auxiliary balancing statistic (section "Auxilary load balancing loss", eq. 10) over the
 * T = desc->T positions of H: counts[a] = number of positions whose largest gate weight is
 * expert a (first index on ties), laux = sum_a (counts[a]/T - 1/r)^2.  counts[r] int64 and
 * laux[1] fp32 are device buffers, overwritten.  The statistic is piecewise constant in the
 * parameters, so no gradient is defined.  d, V, n of desc other than d and r are ignored.
 */
int cp_head_aux_balance(const cp_head_desc *desc, const void *H, const void *G,
                        int64_t *counts, float *laux,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * Full heads (eq. 6 as printed): every (s, a) has its own V x d matrix and there is no shared
 * unembedding,
 *     P^(s)(. | a) = softmax(F_sa h),      F[n,r,V,d] in the storage type of desc->dtype,
 * the parameterisation the paper trains from scratch; gate, eq. 8 and eq. 9 as in cp_head_loss_fwd.
 * cp_head_full_ctx_bytes sizes the `ctx` these two calls share (log-normalisers, gate weights,
 * posterior); workspaces are sized by cp_head_workspace_bytes with CP_HEAD_OP_FULL_LOSS_FWD / _BWD.
 * Forward: loss[T] fp32, overwritten.  Backward: gradients of sum_t dloss[t] * loss[t] (dloss and
 * scale as in cp_head_loss_bwd); dH[T,d] (required), dF[n,r,V,d] and dG[r,d] (either may be NULL)
 * are fp32 and overwritten.  Logits are recomputed head by head for a bounded chunk of positions;
 * nothing of size T*n*r*V is ever stored, unless CP_HEAD_KEEP_LOGITS asks for it (then ctx holds them).
 */
int cp_head_full_ctx_bytes(const cp_head_desc *desc, size_t *bytes);
int cp_head_full_loss_fwd(const cp_head_desc *desc,
                          const void *H, const void *F, const void *G,
                          const int32_t *X,
                          float *loss,
                          void *ctx, void *workspace, size_t workspace_bytes, void *stream);
int cp_head_full_loss_bwd(const cp_head_desc *desc,
                          const void *H, const void *F, const void *G,
                          const int32_t *X,
                          const float *dloss, float scale,
                          const void *ctx,
                          float *dH, float *dF, float *dG,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Head-only fine-tuning loss (section "Fine tuning", eq. 14 and the discounted sum after it) for the
 * shared-unembedding heads, against the logits of the original head.  The paper leaves open what the
 * k-th token's distribution is conditioned on, the direction of the KL term and the discount; the
 * reading implemented is
 *     p^d_k[v] = P(x_k = v | x_<k) = sum_a qhat^(k)_a P^(k)(v | a)    (eq. 13 under the true prefix X[t, <k])
 *     p^c_k    = softmax(TZ[t, k, :])                                 (TZ[T,n,V]: teacher logits, storage type)
 *     L_k      = beta * KL(p^c_k || p^d_k) - (1 - beta) * log p^d_k[X[t,k]]
 *     loss[t]  = sum_{k=0..n-1} discount^k L_k
 * (the paper sets beta = 0.9; with beta = 0 and discount = 1 the loss equals cp_head_loss_fwd's).
 * A negative target drops token k's term and leaves the expert weights of later tokens unchanged.
 * cp_head_distill_ctx_bytes sizes the `ctx` shared by the two calls; workspaces are sized by
 * cp_head_workspace_bytes with CP_HEAD_OP_DISTILL_FWD / _BWD.  Backward: gradients of
 * sum_t dloss[t] * loss[t] with TZ constant; dloss/scale and the outputs as in cp_head_loss_bwd
 * (dU = NULL for the frozen unembedding of fine tuning).  Every entry of TZ must be finite, also in the
 * rows of dropped tokens.  For bf16 storage with d a multiple of 64 and r in {1, 2, 4, 8} no logits are
 * stored: the mixture over the experts is formed inside the tiles of two further vocabulary-sized
 * products on the matrix cores (with CP_HEAD_KEEP_LOGITS: the first product keeps its logits in ctx
 * and the two further ones become memory-bound passes over them).  Every other shape and fp32 storage
 * run on the plain fp32 path, which keeps the fp32 logits of one chunk of rows at a time in the workspace.
 */
int cp_head_distill_ctx_bytes(const cp_head_desc *desc, size_t *bytes);
int cp_head_distill_loss_fwd(const cp_head_desc *desc,
                             const void *H, const void *W, const void *U, const void *G,
                             const int32_t *X, const void *TZ, float beta, float discount,
                             float *loss,
                             void *ctx, void *workspace, size_t workspace_bytes, void *stream);
int cp_head_distill_loss_bwd(const cp_head_desc *desc,
                             const void *H, const void *W, const void *U, const void *G,
                             const int32_t *X, const void *TZ,
                             const float *dloss, float scale,
                             const void *ctx,
                             float *dH, float *dW, float *dU, float *dG,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * Optional per-kernel timing for benchmarks (not part of the method).  While
 * enabled, every large launch inside the three calls above is bracketed by a
 * pair of events on the stream it is launched on.  cp_head_profile_read waits
 * for those events, folds them by kernel name (launch count, total
 * milliseconds, total work: FLOPs for the matrix products, bytes for the
 * transposes), clears the list and writes up to max_entries rows; *count
 * receives the number of distinct names.  Not thread-safe; the event objects
 * are the only thing the library ever creates.
 */
typedef struct cp_head_kernel_time {
    char name[32];
    int32_t launches;
    double total_ms;
    double total_work;
} cp_head_kernel_time;

int cp_head_profile_enable(int on);
int cp_head_profile_read(cp_head_kernel_time *out, int max_entries, int *count);

#ifdef __cplusplus
}
#endif
#endif /* CP_HEAD_H */

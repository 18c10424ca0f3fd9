// Internal declarations shared by the translation units of libcphead.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "cp_head.h"

namespace cph {

typedef uint16_t bf16_t;   // raw bfloat16 bit pattern

constexpr int kWave = 64;

// ---------------------------------------------------------------- device helpers
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

constexpr float kLog2e = 1.4426950408889634f;

// fp32 -> bf16, round to nearest even: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32)
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    return __builtin_bit_cast(bf16_t, (__bf16)f);
}
// two fp32 values -> two bf16 in one register (a in the low half), one conversion instruction
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float a, float b)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ float ld_f32(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float ld_f32(const bf16_t *p, size_t i) { return bf16_to_f32(p[i]); }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

// ---------------------------------------------------------------- host-side layout
inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline unsigned blocks_for(size_t n, int per) { return (unsigned)((n + per - 1) / per); }
template <typename T>
inline T *at(void *base, size_t off) { return reinterpret_cast<T *>(static_cast<char *>(base) + off); }
template <typename T>
inline const T *at(const void *base, size_t off) { return reinterpret_cast<const T *>(static_cast<const char *>(base) + off); }

// Saved-for-backward buffer: [lse M f32][w T*r f32][gamma T*r f32][Y M*d], and on the matrix-core path with
// CP_HEAD_KEEP_LOGITS also [zpart M*parts float2][zs M*Vp fp16]: the (maximum, sum of exponentials) of every
// row over each block of 128 columns, and the logits relative to that maximum.
struct CtxLayout {
    size_t lse, w, gamma, Y, zpart, zs, total;
    size_t Vp;      // row length of zs
    int parts;      // blocks of 128 columns per row (two per 256-column tile)
    bool keep;
};
// Y is fp32 on the generic path and bf16 on the matrix-core path.
inline CtxLayout ctx_layout(const cp_head_desc &ds, bool fast)
{
    CtxLayout c;
    size_t M = (size_t)ds.T * ds.n * ds.r, Tr = (size_t)ds.T * ds.r;
    size_t off = 0;
    c.lse = off;   off = align_up(off + M * 4);
    c.w = off;     off = align_up(off + Tr * 4);
    c.gamma = off; off = align_up(off + Tr * 4);
    c.Y = off;     off = align_up(off + M * ds.d * (fast ? 2 : 4));
    c.keep = fast && (ds.flags & CP_HEAD_KEEP_LOGITS);
    c.Vp = round_up((size_t)ds.V, 64);
    c.parts = ((ds.V + 255) / 256) * 2;
    c.zpart = c.zs = off;
    if (c.keep) {
        c.zpart = off; off = align_up(off + M * c.parts * 8);
        c.zs = off;    off = align_up(off + M * c.Vp * 2);
    }
    c.total = off;
    return c;
}

inline bool use_fast_path(const cp_head_desc &ds)
{
    return ds.dtype == CP_HEAD_BF16 && (ds.d % 64) == 0 && !(ds.flags & CP_HEAD_FORCE_GENERIC);
}

// ---------------------------------------------------------------- generic (plain fp32) path
size_t generic_workspace_bytes(const cp_head_desc &ds, int op);
int generic_loss_fwd(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X, float *loss, void *ctx, void *ws, hipStream_t st);
int generic_loss_bwd(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X, const float *dloss, float scale, const void *ctx,
                     float *dH, float *dW, float *dU, float *dG, void *ws, hipStream_t st);
int generic_draft(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                  const float *uniforms, int32_t *alpha, int32_t *tokens, float *logq, void *ws, hipStream_t st);

// Pieces of the plain path that the fine-tuning loss builds on.  generic_fwd_rows runs the per-row part of the
// training loss's forward pass (gate, y, lse, C) into ctx / ws laid out as for generic_loss_fwd;
// generic_logits_rows writes the fp32 logits of the rows [m0, m0 + Mc) to z[Mc, V]; generic_bwd_from_dz runs the
// training loss's backward pass below the logit gradients, which `fn` produces one chunk of
// generic_bwd_chunk_rows() rows (a multiple of r) at a time.  ws is laid out as for generic_loss_bwd.
struct GenericFwdBuffers {
    float *lse, *w, *gamma, *Y, *logw, *C;
};
int generic_fwd_rows(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X, void *ctx, void *ws, GenericFwdBuffers *out, hipStream_t st);
void generic_logits_rows(const cp_head_desc &ds, const void *U, const float *Y, size_t m0, size_t Mc, float *z,
                         hipStream_t st);
size_t generic_bwd_chunk_rows(const cp_head_desc &ds);
typedef void (*GenericDzLaunch)(void *user, size_t m0, size_t Mc, float *dZ, hipStream_t st);
int generic_bwd_from_dz(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                        const float *Y, const float *dg, float *dH, float *dW, float *dU, float *dG, void *ws,
                        GenericDzLaunch fn, void *user, hipStream_t st);

int generic_draft_sequential(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                             const float *uniforms, int32_t *tokens, float *logq, void *ws, hipStream_t st);
size_t generic_full_workspace_bytes(const cp_head_desc &ds);
int generic_full_loss_fwd(const cp_head_desc &ds, const void *H, const void *F, const void *G, const int32_t *X,
                          float *loss, void *ctx, void *ws, hipStream_t st);
int generic_full_loss_bwd(const cp_head_desc &ds, const void *H, const void *F, const void *G, const int32_t *X,
                          const float *dloss, float scale, const void *ctx, float *dH, float *dF, float *dG, void *ws,
                          hipStream_t st);
size_t generic_first_token_workspace_bytes(const cp_head_desc &ds);
int generic_first_token(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                        float *logp, void *ws, hipStream_t st);
int aux_balance(const cp_head_desc &ds, const void *H, const void *G, int64_t *counts, float *laux, hipStream_t st);
// logp = logsumexp_a(logw + z - lse) from stored first-head logits z[(b,a), ld] and their log-normalisers
void launch_first_token_mix(const cp_head_desc &ds, const float *z, size_t ld, const float *lse, const float *logw,
                            float *logp, hipStream_t st);

// Kernels of the generic path that the matrix-core path reuses (fp32 bookkeeping per position).
void launch_gate(const cp_head_desc &ds, const void *H, const void *G, float *logw, float *w, hipStream_t st);
// out[t] = sign * logsumexp_a(logw + sum_s C): sign = -1 gives the loss, +1 the joint log-probability
void launch_mixture(const cp_head_desc &ds, const float *logw, const float *C, float *out, float *gamma,
                    float sign, hipStream_t st);
void launch_fill_zero(float *p, size_t count, hipStream_t st);
void launch_pick_alpha(const cp_head_desc &ds, const float *w, const float *uniforms, int32_t *alpha,
                       hipStream_t st);

// ---------------------------------------------------------------- optional per-kernel timing
// While profiling is switched on (cp_head_profile_enable), a ProfileScope brackets a launch with a
// pair of events on the launch stream and remembers the work it stands for.
bool profile_begin(const char *name, double work, hipStream_t st);   // whether a record was opened
void profile_end(hipStream_t st);
struct ProfileScope {
    hipStream_t st;
    bool open;
    ProfileScope(const char *name, double work, hipStream_t s) : st(s), open(profile_begin(name, work, s)) {}
    ~ProfileScope() { if (open) profile_end(st); }
};

// ---------------------------------------------------------------- matrix-core path
size_t fast_workspace_bytes(const cp_head_desc &ds, int op);
int fast_loss_fwd(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                  const int32_t *X, float *loss, void *ctx, void *ws, size_t ws_bytes, hipStream_t st);
int fast_loss_bwd(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                  const int32_t *X, const float *dloss, float scale, const void *ctx,
                  float *dH, float *dW, float *dU, float *dG, void *ws, size_t ws_bytes, hipStream_t st);
size_t fast_step_workspace_bytes(const cp_head_desc &ds);
int fast_loss_step(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                   const int32_t *X, const float *dloss, float scale, float *loss, float *dH, float *dW, float *dU,
                   float *dG, void *ws, hipStream_t st);
int fast_draft(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
               const float *uniforms, int32_t *alpha, int32_t *tokens, float *logq, void *ws, size_t ws_bytes,
               hipStream_t st);
int fast_first_token(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G, float *logp,
                     void *ws, hipStream_t st);
int fast_draft_sequential(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                          const float *uniforms, int32_t *tokens, float *logq, void *ws, hipStream_t st);

// Pieces of the matrix-core loss path that other losses over the same heads build on.
struct FastFwdBuffers {
    float *lse, *w, *gamma;   // in ctx: log-normalisers [M], gate weights and posterior [T, r]
    float *logw, *C;          // in the forward workspace: log w [T, r], C [M] (eq. 8)
    bf16_t *Y;                // in ctx: y [M, d]
};
int fast_fwd_rows(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                  const int32_t *X, void *ctx, void *ws, FastFwdBuffers *out, hipStream_t st);
// writes dz for rows m0 .. m0+Mc-1 of the chunk whose y is Yc: dZ[Mc, ldz] (dz_blocked: stored in blocks of 256 rows x
// 64 columns instead of row-major) and, unless null, dZt[V, ldzt]
typedef void (*FastDzLaunch)(void *user, const bf16_t *Yc, int Mc, int Mcp, size_t m0, bf16_t *dZ, long ldz, bool dz_blocked,
                             bf16_t *dZt, long ldzt, hipStream_t st);
int fast_bwd_from_dz(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                     const void *Y, const float *dg, float *dH, float *dW, float *dU, float *dG, void *ws,
                     FastDzLaunch dz_launch, void *user, hipStream_t st);
bool fast_dims_fit(const cp_head_desc &ds);

size_t fast_full_ctx_bytes(const cp_head_desc &ds);
int fast_full_loss_fwd(const cp_head_desc &ds, const void *H, const void *F, const void *G, const int32_t *X,
                       float *loss, void *ctx, void *ws, hipStream_t st);
int fast_full_loss_bwd(const cp_head_desc &ds, const void *H, const void *F, const void *G, const int32_t *X,
                       const float *dloss, float scale, const void *ctx, float *dH, float *dF, float *dG, void *ws,
                       hipStream_t st);

// ---------------------------------------------------------------- fine-tuning (distillation) loss
// matrix-core path for bf16, d % 64 == 0, r in {1, 2, 4, 8}; the plain path otherwise
bool distill_on_matrix_cores(const cp_head_desc &ds);   // the fine-tuning loss's own path selector
size_t distill_ctx_bytes(const cp_head_desc &ds);
size_t distill_workspace_bytes(const cp_head_desc &ds, int op);
int distill_loss_fwd(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X, const void *TZ, float beta, float disc, float *loss, void *ctx, void *ws,
                     hipStream_t st);
int distill_loss_bwd(const cp_head_desc &ds, const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X, const void *TZ, const float *dloss, float scale, const void *ctx, float *dH,
                     float *dW, float *dU, float *dG, void *ws, hipStream_t st);

}  // namespace cph

// C ABI of libcphead.so: argument checks, path selection, dispatch.
#include "cp_internal.hpp"

#include <stdio.h>

#include <mutex>
#include <string>
#include <vector>

using namespace cph;

// ---------------------------------------------------------------- optional per-kernel timing
namespace {
struct ProfileRecord {
    const char *name;
    double work;
    hipEvent_t start, stop;
};
bool g_profile_on = false;
std::vector<ProfileRecord> g_profile;
}  // namespace

namespace cph {
// Returns whether a record was pushed: only then may profile_end record its stop event.
bool profile_begin(const char *name, double work, hipStream_t st)
{
    if (!g_profile_on) return false;
    ProfileRecord rec{name, work, nullptr, nullptr};
    if (hipEventCreate(&rec.start) != hipSuccess) return false;
    if (hipEventCreate(&rec.stop) != hipSuccess) {
        (void)hipEventDestroy(rec.start);
        return false;
    }
    if (hipEventRecord(rec.start, st) != hipSuccess) {
        (void)hipEventDestroy(rec.start);
        (void)hipEventDestroy(rec.stop);
        return false;
    }
    g_profile.push_back(rec);
    return true;
}
void profile_end(hipStream_t st)
{
    if (g_profile.empty()) return;
    ProfileRecord &rec = g_profile.back();
    if (hipEventRecord(rec.stop, st) != hipSuccess) {          // a record without a stop event is dropped
        (void)hipEventDestroy(rec.start);
        (void)hipEventDestroy(rec.stop);
        g_profile.pop_back();
    }
}
}  // namespace cph

namespace {

constexpr int kMaxRank = 64;
constexpr int kMaxHeads = 64;
constexpr int kMaxGenericD = 16000;   // the plain path keeps one fp32 row of length d in LDS

int check_desc(const cp_head_desc *ds)
{
    if (!ds) return CP_HEAD_ERR_INVALID_ARG;
    if (ds->T < 0 || ds->d < 1 || ds->V < 1 || ds->n < 1 || ds->r < 1) return CP_HEAD_ERR_INVALID_ARG;
    if (ds->dtype != CP_HEAD_FP32 && ds->dtype != CP_HEAD_BF16) return CP_HEAD_ERR_UNSUPPORTED;
    if (ds->r > kMaxRank || ds->n > kMaxHeads) return CP_HEAD_ERR_UNSUPPORTED;
    const double rows = (double)ds->T * ds->n * ds->r;
    if (rows * (double)(ds->d > ds->V ? ds->d : ds->V) >= 4.6e18) return CP_HEAD_ERR_UNSUPPORTED;
    if (rows >= 2147483647.0) return CP_HEAD_ERR_UNSUPPORTED;   // one thread block per head row
    if (!use_fast_path(*ds) && ds->d > kMaxGenericD) return CP_HEAD_ERR_UNSUPPORTED;
    return CP_HEAD_OK;
}

// The fine-tuning loss runs ranks other than 1, 2, 4, 8 on the plain path even where the training loss would use
// the matrix cores, so the plain path's limit on d applies to it by its own path selector.
bool distill_shape_supported(const cp_head_desc &ds)
{
    return distill_on_matrix_cores(ds) || ds.d <= kMaxGenericD;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 255u) != 0; }

// The single-call training step on the plain path is the forward call followed by the backward call, with the
// saved-for-backward buffer carved out of the workspace.
size_t plain_step_ctx_bytes(const cp_head_desc &ds) { return (ctx_layout(ds, false).total + 255) / 256 * 256; }
size_t plain_step_workspace_bytes(const cp_head_desc &ds)
{
    const size_t f = generic_workspace_bytes(ds, CP_HEAD_OP_LOSS_FWD), b = generic_workspace_bytes(ds, CP_HEAD_OP_LOSS_BWD);
    return plain_step_ctx_bytes(ds) + (f > b ? f : b);
}

size_t workspace_need(const cp_head_desc &ds, int op)
{
    if (op == CP_HEAD_OP_LOSS_FWD_BWD) return use_fast_path(ds) ? fast_step_workspace_bytes(ds) : plain_step_workspace_bytes(ds);
    if (op == CP_HEAD_OP_AUX_BALANCE) return 256;   // none needed; a token size keeps the calling pattern uniform
    if (op == CP_HEAD_OP_FULL_LOSS_FWD || op == CP_HEAD_OP_FULL_LOSS_BWD)
        return use_fast_path(ds) ? fast_workspace_bytes(ds, op) : generic_full_workspace_bytes(ds);
    if (op == CP_HEAD_OP_DISTILL_FWD || op == CP_HEAD_OP_DISTILL_BWD)
        return distill_workspace_bytes(ds, op);
    if (use_fast_path(ds)) return fast_workspace_bytes(ds, op);
    if (op == CP_HEAD_OP_FIRST_TOKEN) return generic_first_token_workspace_bytes(ds);
    if (op == CP_HEAD_OP_DRAFT_SEQUENTIAL) return generic_workspace_bytes(ds, CP_HEAD_OP_DRAFT);   // same buffers
    return generic_workspace_bytes(ds, op);
}


// ---------------------------------------------------------------- scratch for callers that cannot allocate
// One array per GPU (every device that loads the code object holds its own copy at its own address), used by
// cp_head_draft_sample_static in place of a caller's workspace.  In host code the array's name is only a handle for
// the symbol lookup: the device address is resolved once per device, with that device current, and kept; kernels
// and every other use take that pointer.
constexpr size_t kStaticScratchBytes = CP_HEAD_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[CP_HEAD_STATIC_SCRATCH_BYTES];
namespace {
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

int static_scratch_of_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CP_HEAD_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return CP_HEAD_ERR_LAUNCH;
        if (reinterpret_cast<uintptr_t>(ptr) & 255u) return CP_HEAD_ERR_LAUNCH;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return CP_HEAD_OK;
}

}  // namespace

extern "C" {

const char *cp_head_strerror(int code)
{
    switch (code) {
    case CP_HEAD_OK: return "ok";
    case CP_HEAD_ERR_INVALID_ARG: return "invalid argument (null pointer, bad dimension or misaligned buffer)";
    case CP_HEAD_ERR_UNSUPPORTED: return "unsupported shape or storage type";
    case CP_HEAD_ERR_WORKSPACE: return "workspace too small";
    case CP_HEAD_ERR_LAUNCH: return "kernel launch failed";
    case CP_HEAD_ERR_STATIC_SCRATCH: return "shape needs more scratch than the library's static buffer holds";
    default: return "unknown error code";
    }
}

int cp_head_profile_enable(int on)
{
    g_profile_on = on != 0;
    return CP_HEAD_OK;
}

int cp_head_profile_read(cp_head_kernel_time *out, int max_entries, int *count)
{
    if (!count || (max_entries > 0 && !out)) return CP_HEAD_ERR_INVALID_ARG;
    // fold the records by kernel name, in order of first appearance
    std::vector<cp_head_kernel_time> rows;
    for (ProfileRecord &rec : g_profile) {
        float ms = 0.f;
        const bool timed = hipEventSynchronize(rec.stop) == hipSuccess &&
                           hipEventElapsedTime(&ms, rec.start, rec.stop) == hipSuccess;
        (void)hipEventDestroy(rec.start);
        (void)hipEventDestroy(rec.stop);
        if (!timed) continue;                                    // never fold an unmeasured launch into the averages
        size_t i = 0;
        for (; i < rows.size(); ++i)
            if (std::string(rows[i].name) == rec.name) break;
        if (i == rows.size()) {
            cp_head_kernel_time row = {};
            snprintf(row.name, sizeof(row.name), "%s", rec.name);
            rows.push_back(row);
        }
        rows[i].launches += 1;
        rows[i].total_ms += ms;
        rows[i].total_work += rec.work;
    }
    g_profile.clear();
    *count = (int)rows.size();
    for (int i = 0; i < max_entries && i < (int)rows.size(); ++i) out[i] = rows[i];
    return CP_HEAD_OK;
}

int cp_head_ctx_bytes(const cp_head_desc *desc, size_t *bytes)
{
    if (!bytes) return CP_HEAD_ERR_INVALID_ARG;
    const int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    *bytes = ctx_layout(*desc, use_fast_path(*desc)).total;
    return CP_HEAD_OK;
}

int cp_head_workspace_bytes(const cp_head_desc *desc, int op, size_t *bytes)
{
    if (!bytes) return CP_HEAD_ERR_INVALID_ARG;
    const int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (op < CP_HEAD_OP_LOSS_FWD || op > CP_HEAD_OP_LOSS_FWD_BWD) return CP_HEAD_ERR_INVALID_ARG;
    if ((op == CP_HEAD_OP_DISTILL_FWD || op == CP_HEAD_OP_DISTILL_BWD) && !distill_shape_supported(*desc))
        return CP_HEAD_ERR_UNSUPPORTED;
    *bytes = workspace_need(*desc, op);
    return CP_HEAD_OK;
}

int cp_head_loss_fwd(const cp_head_desc *desc, const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X, float *loss, void *ctx, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!W || !U || !G) return CP_HEAD_ERR_INVALID_ARG;
    if (desc->T > 0 && (!H || !X || !loss)) return CP_HEAD_ERR_INVALID_ARG;
    if (!ctx || !workspace || misaligned(ctx) || misaligned(workspace)) return CP_HEAD_ERR_INVALID_ARG;
    const bool fast = use_fast_path(*desc);
    const size_t need = fast ? fast_workspace_bytes(*desc, CP_HEAD_OP_LOSS_FWD)
                             : generic_workspace_bytes(*desc, CP_HEAD_OP_LOSS_FWD);
    if (workspace_bytes < need) return CP_HEAD_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (fast) return fast_loss_fwd(*desc, H, W, U, G, X, loss, ctx, workspace, workspace_bytes, st);
    return generic_loss_fwd(*desc, H, W, U, G, X, loss, ctx, workspace, st);
}

int cp_head_loss_bwd(const cp_head_desc *desc, const void *H, const void *W, const void *U, const void *G,
                     const int32_t *X, const float *dloss, float scale, const void *ctx, float *dH, float *dW,
                     float *dU, float *dG, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!W || !U || !G) return CP_HEAD_ERR_INVALID_ARG;
    if (desc->T > 0 && (!H || !X || !dH)) return CP_HEAD_ERR_INVALID_ARG;
    if (!ctx || !workspace || misaligned(ctx) || misaligned(workspace)) return CP_HEAD_ERR_INVALID_ARG;
    const bool fast = use_fast_path(*desc);
    const size_t need = fast ? fast_workspace_bytes(*desc, CP_HEAD_OP_LOSS_BWD)
                             : generic_workspace_bytes(*desc, CP_HEAD_OP_LOSS_BWD);
    if (workspace_bytes < need) return CP_HEAD_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (fast)
        return fast_loss_bwd(*desc, H, W, U, G, X, dloss, scale, ctx, dH, dW, dU, dG, workspace, workspace_bytes, st);
    return generic_loss_bwd(*desc, H, W, U, G, X, dloss, scale, ctx, dH, dW, dU, dG, workspace, st);
}

int cp_head_loss_fwd_bwd(const cp_head_desc *desc, const void *H, const void *W, const void *U, const void *G,
                         const int32_t *X, const float *dloss, float scale, float *loss, float *dH, float *dW, float *dU,
                         float *dG, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!W || !U || !G) return CP_HEAD_ERR_INVALID_ARG;
    if (desc->T > 0 && (!H || !X || !loss || !dH)) return CP_HEAD_ERR_INVALID_ARG;
    if (!workspace || misaligned(workspace)) return CP_HEAD_ERR_INVALID_ARG;
    if (workspace_bytes < workspace_need(*desc, CP_HEAD_OP_LOSS_FWD_BWD)) return CP_HEAD_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (use_fast_path(*desc)) return fast_loss_step(*desc, H, W, U, G, X, dloss, scale, loss, dH, dW, dU, dG, workspace, st);
    void *ctx = workspace;
    void *ws = static_cast<char *>(workspace) + plain_step_ctx_bytes(*desc);
    rc = generic_loss_fwd(*desc, H, W, U, G, X, loss, ctx, ws, st);
    if (rc != CP_HEAD_OK) return rc;
    return generic_loss_bwd(*desc, H, W, U, G, X, dloss, scale, ctx, dH, dW, dU, dG, ws, st);
}

int cp_head_draft_sample(const cp_head_desc *desc, const void *H, const void *W, const void *U, const void *G,
                         const float *uniforms, int32_t *alpha, int32_t *tokens, float *logq, void *workspace,
                         size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!W || !U || !G) return CP_HEAD_ERR_INVALID_ARG;
    if (desc->T > 0 && (!H || !uniforms || !alpha || !tokens)) return CP_HEAD_ERR_INVALID_ARG;
    if (!workspace || misaligned(workspace)) return CP_HEAD_ERR_INVALID_ARG;
    const bool fast = use_fast_path(*desc);
    const size_t need = fast ? fast_workspace_bytes(*desc, CP_HEAD_OP_DRAFT)
                             : generic_workspace_bytes(*desc, CP_HEAD_OP_DRAFT);
    if (workspace_bytes < need) return CP_HEAD_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (fast) return fast_draft(*desc, H, W, U, G, uniforms, alpha, tokens, logq, workspace, workspace_bytes, st);
    return generic_draft(*desc, H, W, U, G, uniforms, alpha, tokens, logq, workspace, st);
}

int cp_head_draft_sample_static(const cp_head_desc *desc, const void *H, const void *W, const void *U, const void *G,
                                const float *uniforms, int32_t *alpha, int32_t *tokens, float *logq, void *stream)
{
    int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!W || !U || !G) return CP_HEAD_ERR_INVALID_ARG;
    if (desc->T > 0 && (!H || !uniforms || !alpha || !tokens)) return CP_HEAD_ERR_INVALID_ARG;
    const bool fast = use_fast_path(*desc);
    const size_t need = fast ? fast_workspace_bytes(*desc, CP_HEAD_OP_DRAFT)
                             : generic_workspace_bytes(*desc, CP_HEAD_OP_DRAFT);
    if (need > kStaticScratchBytes) return CP_HEAD_ERR_STATIC_SCRATCH;
    void *ws = nullptr;
    rc = static_scratch_of_current_device(&ws);
    if (rc != CP_HEAD_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (fast) return fast_draft(*desc, H, W, U, G, uniforms, alpha, tokens, logq, ws, kStaticScratchBytes, st);
    return generic_draft(*desc, H, W, U, G, uniforms, alpha, tokens, logq, ws, st);
}

int cp_head_first_token_logprob(const cp_head_desc *desc, const void *H, const void *W, const void *U, const void *G,
                                float *logp, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!W || !U || !G) return CP_HEAD_ERR_INVALID_ARG;
    if (desc->T > 0 && (!H || !logp)) return CP_HEAD_ERR_INVALID_ARG;
    if (!workspace || misaligned(workspace)) return CP_HEAD_ERR_INVALID_ARG;
    if (workspace_bytes < workspace_need(*desc, CP_HEAD_OP_FIRST_TOKEN)) return CP_HEAD_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (use_fast_path(*desc)) return fast_first_token(*desc, H, W, U, G, logp, workspace, st);
    return generic_first_token(*desc, H, W, U, G, logp, workspace, st);
}

int cp_head_draft_sample_sequential(const cp_head_desc *desc, const void *H, const void *W, const void *U,
                                    const void *G, const float *uniforms, int32_t *tokens, float *logq,
                                    void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!W || !U || !G) return CP_HEAD_ERR_INVALID_ARG;
    if (desc->T > 0 && (!H || !uniforms || !tokens)) return CP_HEAD_ERR_INVALID_ARG;
    if (!workspace || misaligned(workspace)) return CP_HEAD_ERR_INVALID_ARG;
    if (workspace_bytes < workspace_need(*desc, CP_HEAD_OP_DRAFT_SEQUENTIAL)) return CP_HEAD_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (use_fast_path(*desc)) return fast_draft_sequential(*desc, H, W, U, G, uniforms, tokens, logq, workspace, st);
    return generic_draft_sequential(*desc, H, W, U, G, uniforms, tokens, logq, workspace, st);
}

int cp_head_aux_balance(const cp_head_desc *desc, const void *H, const void *G, int64_t *counts, float *laux,
                        void *workspace, size_t workspace_bytes, void *stream)
{
    (void)workspace;
    (void)workspace_bytes;
    int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!G || !counts || !laux) return CP_HEAD_ERR_INVALID_ARG;
    if (desc->T > 0 && !H) return CP_HEAD_ERR_INVALID_ARG;
    return aux_balance(*desc, H, G, counts, laux, static_cast<hipStream_t>(stream));
}

int cp_head_full_ctx_bytes(const cp_head_desc *desc, size_t *bytes)
{
    if (!bytes) return CP_HEAD_ERR_INVALID_ARG;
    const int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    *bytes = fast_full_ctx_bytes(*desc);
    return CP_HEAD_OK;
}

int cp_head_full_loss_fwd(const cp_head_desc *desc, const void *H, const void *F, const void *G, const int32_t *X,
                          float *loss, void *ctx, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!F || !G) return CP_HEAD_ERR_INVALID_ARG;
    if (desc->T > 0 && (!H || !X || !loss)) return CP_HEAD_ERR_INVALID_ARG;
    if (!ctx || !workspace || misaligned(ctx) || misaligned(workspace)) return CP_HEAD_ERR_INVALID_ARG;
    if (workspace_bytes < workspace_need(*desc, CP_HEAD_OP_FULL_LOSS_FWD)) return CP_HEAD_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (use_fast_path(*desc)) return fast_full_loss_fwd(*desc, H, F, G, X, loss, ctx, workspace, st);
    return generic_full_loss_fwd(*desc, H, F, G, X, loss, ctx, workspace, st);
}

int cp_head_full_loss_bwd(const cp_head_desc *desc, const void *H, const void *F, const void *G, const int32_t *X,
                          const float *dloss, float scale, const void *ctx, float *dH, float *dF, float *dG,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!F || !G) return CP_HEAD_ERR_INVALID_ARG;
    if (desc->T > 0 && (!H || !X || !dH)) return CP_HEAD_ERR_INVALID_ARG;
    if (!ctx || !workspace || misaligned(ctx) || misaligned(workspace)) return CP_HEAD_ERR_INVALID_ARG;
    if (workspace_bytes < workspace_need(*desc, CP_HEAD_OP_FULL_LOSS_BWD)) return CP_HEAD_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (use_fast_path(*desc)) return fast_full_loss_bwd(*desc, H, F, G, X, dloss, scale, ctx, dH, dF, dG, workspace, st);
    return generic_full_loss_bwd(*desc, H, F, G, X, dloss, scale, ctx, dH, dF, dG, workspace, st);
}

int cp_head_distill_ctx_bytes(const cp_head_desc *desc, size_t *bytes)
{
    if (!bytes) return CP_HEAD_ERR_INVALID_ARG;
    const int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!distill_shape_supported(*desc)) return CP_HEAD_ERR_UNSUPPORTED;
    *bytes = distill_ctx_bytes(*desc);
    return CP_HEAD_OK;
}

int cp_head_distill_loss_fwd(const cp_head_desc *desc, const void *H, const void *W, const void *U, const void *G,
                             const int32_t *X, const void *TZ, float beta, float discount, float *loss, void *ctx,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!W || !U || !G) return CP_HEAD_ERR_INVALID_ARG;
    if (desc->T > 0 && (!H || !X || !TZ || !loss)) return CP_HEAD_ERR_INVALID_ARG;
    if (!(beta >= 0.f && beta <= 1.f) || !(discount >= 0.f)) return CP_HEAD_ERR_INVALID_ARG;
    if (!ctx || !workspace || misaligned(ctx) || misaligned(workspace)) return CP_HEAD_ERR_INVALID_ARG;
    if (!distill_shape_supported(*desc)) return CP_HEAD_ERR_UNSUPPORTED;
    if (workspace_bytes < workspace_need(*desc, CP_HEAD_OP_DISTILL_FWD)) return CP_HEAD_ERR_WORKSPACE;
    return distill_loss_fwd(*desc, H, W, U, G, X, TZ, beta, discount, loss, ctx, workspace,
                            static_cast<hipStream_t>(stream));
}

int cp_head_distill_loss_bwd(const cp_head_desc *desc, const void *H, const void *W, const void *U, const void *G,
                             const int32_t *X, const void *TZ, const float *dloss, float scale, const void *ctx,
                             float *dH, float *dW, float *dU, float *dG, void *workspace, size_t workspace_bytes,
                             void *stream)
{
    int rc = check_desc(desc);
    if (rc != CP_HEAD_OK) return rc;
    if (!W || !U || !G) return CP_HEAD_ERR_INVALID_ARG;
    if (desc->T > 0 && (!H || !X || !TZ || !dH)) return CP_HEAD_ERR_INVALID_ARG;
    if (!ctx || !workspace || misaligned(ctx) || misaligned(workspace)) return CP_HEAD_ERR_INVALID_ARG;
    if (!distill_shape_supported(*desc)) return CP_HEAD_ERR_UNSUPPORTED;
    if (workspace_bytes < workspace_need(*desc, CP_HEAD_OP_DISTILL_BWD)) return CP_HEAD_ERR_WORKSPACE;
    return distill_loss_bwd(*desc, H, W, U, G, X, TZ, dloss, scale, ctx, dH, dW, dU, dG, workspace,
                            static_cast<hipStream_t>(stream));
}

}  // extern "C"

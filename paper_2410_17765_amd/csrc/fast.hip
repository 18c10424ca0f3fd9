// Matrix-core path (placeholder until the MFMA kernels land).
#include "cp_internal.hpp"
namespace cph {
size_t fast_workspace_bytes(const cp_head_desc &, int) { return 256; }
int fast_loss_fwd(const cp_head_desc &, const void *, const void *, const void *, const void *, const int32_t *, float *, void *, void *, size_t, hipStream_t) { return CP_HEAD_ERR_UNSUPPORTED; }
int fast_loss_bwd(const cp_head_desc &, const void *, const void *, const void *, const void *, const int32_t *, const float *, float, const void *, float *, float *, float *, float *, void *, size_t, hipStream_t) { return CP_HEAD_ERR_UNSUPPORTED; }
int fast_draft(const cp_head_desc &, const void *, const void *, const void *, const void *, const float *, int32_t *, int32_t *, float *, void *, size_t, hipStream_t) { return CP_HEAD_ERR_UNSUPPORTED; }
}

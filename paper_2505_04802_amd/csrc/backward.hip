// Entry points of the training-side kernels (gradients); the chain rule applied to
// the operations of ORBIT-2 Sec. 4.1 / 4.2.
#include <string>

#include "common.h"

using namespace reslim;

extern "C" int tiles_attention_bwd_workspace_bytes(const reslim_ctx *c, int32_t batch, size_t *out) {
  if (!c || !out || batch < 1) return RESLIM_EINVAL;
  *out = tiles_attention_bwd_ws_bytes(c, batch);
  return RESLIM_OK;
}

extern "C" int tiles_attention_bwd(reslim_ctx *c, const void *qkv, const void *out, const float *lse, const void *d_out,
                                   void *d_qkv, int32_t batch, void *workspace, size_t ws_bytes, void *hip_stream) {
  const char *fn = "tiles_attention_bwd";
  if (!c) return RESLIM_EINVAL;
  if (!qkv || !out || !lse || !d_out || !d_qkv) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  int rc = check_common(c, fn, batch, nullptr, 0, false);
  if (rc != RESLIM_OK) return rc;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255))
    return set_error(c, RESLIM_EWORKSPACE, std::string(fn) + ": workspace null or not 256-byte aligned");
  if (ws_bytes < tiles_attention_bwd_ws_bytes(c, batch))
    return set_error(c, RESLIM_EWORKSPACE, std::string(fn) + ": workspace smaller than tiles_attention_bwd_workspace_bytes()");
  RESLIM_TRY("launch", launch_tiles_attention_bwd(c, qkv, out, lse, d_out, d_qkv, batch, workspace, false,
                                                  static_cast<hipStream_t>(hip_stream)));
  return RESLIM_OK;
}

// Entry points that chain the kernels: embed, block, head, forward
// (ORBIT-2 Sec. 4.1 data flow, applied tile-wise as in Sec. 4.2).
#include <algorithm>

#include "common.h"

namespace reslim {

// Workspace layout (all offsets 256-byte aligned), M = batch * n_h, Mi = batch * N:
//   X    float [M, D]                  residual stream (reslim_forward only)
//   A    act   [M, D]                  LayerNorm output / attention output / aggregated values
//   big  max( act [M, max(3D, R)],     qkv, then the feed-forward hidden layer
//             float [Mi, D],           embedded tokens before the tile-major gather
//             float [Mi, head_out] )   head projection before un-patchify
Workspace plan_workspace(const reslim_ctx *c, int batch, void *base) {
  const size_t M = static_cast<size_t>(batch) * c->n_h, Mi = static_cast<size_t>(batch) * c->N;
  const size_t D = c->cfg.embed_dim, es = act_size(c);
  const size_t x_b = align256(M * D * sizeof(float));
  const size_t a_b = align256(M * D * es);
  size_t big_b = M * std::max<size_t>(3 * D, c->R) * es;
  big_b = std::max(big_b, Mi * D * sizeof(float));
  big_b = std::max(big_b, Mi * static_cast<size_t>(c->head_out) * sizeof(float));
  big_b = align256(big_b);
  Workspace w;
  unsigned char *p = static_cast<unsigned char *>(base);
  w.X = reinterpret_cast<float *>(p);
  w.A = p + x_b;
  w.big = p + x_b + a_b;
  w.total = x_b + a_b + big_b;
  return w;
}

static int check_common(reslim_ctx *c, const char *fn, int batch, const void *ws, size_t ws_bytes, bool need_ws) {
  if (batch < 1 || batch > 65535) return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": batch must be in [1, 65535]");
  if (static_cast<int64_t>(batch) * c->n_h > INT32_MAX)
    return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": batch * tokens exceeds int32 row indexing");
  if (need_ws) {
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255)) return set_error(c, RESLIM_EWORKSPACE, std::string(fn) + ": workspace null or not 256-byte aligned");
    if (ws_bytes < plan_workspace(c, batch, nullptr).total)
      return set_error(c, RESLIM_EWORKSPACE, std::string(fn) + ": workspace smaller than reslim_workspace_bytes()");
  }
  return RESLIM_OK;
}

static int hip_fail(reslim_ctx *c, const char *fn, const char *what, hipError_t e) {
  return set_error(c, RESLIM_EHIP, std::string(fn) + ": " + what + ": " + hipGetErrorString(e));
}

#define RESLIM_TRY(what, expr)                                   \
  do {                                                           \
    hipError_t e_ = (expr);                                      \
    if (e_ != hipSuccess) return hip_fail(c, fn, what, e_);      \
  } while (0)

static int embed_impl(reslim_ctx *c, const char *fn, const float *x, float *tokens, int batch, const Workspace &w, hipStream_t st) {
  const int D = c->cfg.embed_dim, dt = c->cfg.dtype;
  const int Mi = batch * c->N;
  RESLIM_TRY("embed_agg", launch_embed_agg(c, x, w.A, batch, st));
  RESLIM_TRY("aggregation output GEMM",
             launch_gemm(dt, EPI_BIAS_TAB_F32, w.A, c->d_agg_wo, c->d_zero_bias, w.big, D, c->d_pos_res, c->N, Mi, D, D, st));
  RESLIM_TRY("gather", launch_gather_rows(static_cast<const float *>(w.big), c->d_gather, tokens, batch, c->n_h, c->N, D, st));
  return RESLIM_OK;
}

static int block_impl(reslim_ctx *c, const char *fn, int layer, float *X, int batch, const Workspace &w, hipStream_t st) {
  const int D = c->cfg.embed_dim, R = c->R, dt = c->cfg.dtype;
  const int M = static_cast<int>(batch * c->n_h);
  const LayerWeights &lw = c->layers[layer];
  RESLIM_TRY("LN1", launch_layernorm(dt, X, nullptr, 0, 0, lw.ln1_g, lw.ln1_b, w.A, M, D, st));
  RESLIM_TRY("QKV GEMM", launch_gemm(dt, EPI_BIAS_ACT, w.A, lw.w_qkv, lw.b_qkv, w.big, 3 * D, nullptr, 0, M, 3 * D, D, st));
  RESLIM_TRY("tile attention", launch_tiles_attention(c, w.big, w.A, batch, st));
  RESLIM_TRY("proj GEMM", launch_gemm(dt, EPI_BIAS_RESADD_F32, w.A, lw.w_proj, lw.b_proj, X, D, nullptr, 0, M, D, D, st));
  RESLIM_TRY("LN2", launch_layernorm(dt, X, nullptr, 0, 0, lw.ln2_g, lw.ln2_b, w.A, M, D, st));
  RESLIM_TRY("FC1 GEMM", launch_gemm(dt, EPI_BIAS_GELU_ACT, w.A, lw.w_fc1, lw.b_fc1, w.big, R, nullptr, 0, M, R, D, st));
  RESLIM_TRY("FC2 GEMM", launch_gemm(dt, EPI_BIAS_RESADD_F32, w.big, lw.w_fc2, lw.b_fc2, X, D, nullptr, 0, M, D, R, st));
  return RESLIM_OK;
}

static int head_impl(reslim_ctx *c, const char *fn, const float *x, const float *tokens, float *y, int batch, const Workspace &w, hipStream_t st) {
  const int D = c->cfg.embed_dim, dt = c->cfg.dtype;
  const int Mi = batch * c->N;
  RESLIM_TRY("final LN", launch_layernorm(dt, tokens, c->d_interior_src, c->N, c->n_h, c->d_lnf_g, c->d_lnf_b, w.A, Mi, D, st));
  RESLIM_TRY("head GEMM", launch_gemm(dt, EPI_BIAS_F32, w.A, c->d_w_head, c->d_b_head, w.big, c->head_out, nullptr, 0, Mi, c->head_out, D, st));
  RESLIM_TRY("residual path", launch_residual_unpatchify(c, x, w.big, 0, y, batch, st));
  return RESLIM_OK;
}

}  // namespace reslim

using namespace reslim;

extern "C" int reslim_tokens_per_sample(const reslim_ctx *ctx, int64_t *n_h_out) {
  if (!ctx || !n_h_out) return RESLIM_EINVAL;
  *n_h_out = ctx->n_h;
  return RESLIM_OK;
}

extern "C" int reslim_workspace_bytes(const reslim_ctx *ctx, int32_t batch, size_t *out) {
  if (!ctx || !out || batch < 1) return RESLIM_EINVAL;
  *out = plan_workspace(ctx, batch, nullptr).total;
  return RESLIM_OK;
}

extern "C" int reslim_flop_counts(const reslim_ctx *ctx, int32_t batch, double *gemm_flop, double *attn_flop, double *head_flop) {
  if (!ctx || batch < 1) return RESLIM_EINVAL;
  const double D = ctx->cfg.embed_dim, L = ctx->cfg.depth, B = batch;
  const double M = B * static_cast<double>(ctx->n_h);
  if (gemm_flop) *gemm_flop = 2.0 * M * D * (3.0 * D + D + 2.0 * ctx->R) * L;
  if (attn_flop) {
    double s = 0;
    for (const tile_desc &t : ctx->tiles) s += static_cast<double>(t.n_tok) * t.n_tok;
    *attn_flop = 4.0 * s * D * L * B;
  }
  if (head_flop) *head_flop = 2.0 * B * ctx->N * D * ctx->head_out;
  return RESLIM_OK;
}

extern "C" int tiles_attention_fwd(reslim_ctx *c, const void *qkv, void *out, int32_t batch, void *hip_stream) {
  const char *fn = "tiles_attention_fwd";
  if (!c) return RESLIM_EINVAL;
  if (!qkv || !out) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  int rc = check_common(c, fn, batch, nullptr, 0, false);
  if (rc != RESLIM_OK) return rc;
  RESLIM_TRY("launch", launch_tiles_attention(c, qkv, out, batch, static_cast<hipStream_t>(hip_stream)));
  return RESLIM_OK;
}

extern "C" int reslim_embed_fwd(reslim_ctx *c, const float *x, float *tokens, int32_t batch, void *workspace, size_t ws_bytes, void *hip_stream) {
  const char *fn = "reslim_embed_fwd";
  if (!c) return RESLIM_EINVAL;
  if (!x || !tokens) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  int rc = check_common(c, fn, batch, workspace, ws_bytes, true);
  if (rc != RESLIM_OK) return rc;
  return embed_impl(c, fn, x, tokens, batch, plan_workspace(c, batch, workspace), static_cast<hipStream_t>(hip_stream));
}

extern "C" int reslim_block_fwd(reslim_ctx *c, int32_t layer, float *x_inout, int32_t batch, void *workspace, size_t ws_bytes, void *hip_stream) {
  const char *fn = "reslim_block_fwd";
  if (!c) return RESLIM_EINVAL;
  if (!x_inout) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  if (layer < 0 || layer >= c->cfg.depth) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": layer outside [0, depth)");
  int rc = check_common(c, fn, batch, workspace, ws_bytes, true);
  if (rc != RESLIM_OK) return rc;
  return block_impl(c, fn, layer, x_inout, batch, plan_workspace(c, batch, workspace), static_cast<hipStream_t>(hip_stream));
}

extern "C" int reslim_head_fwd(reslim_ctx *c, const float *x, const float *tokens, float *y, int32_t batch, void *workspace, size_t ws_bytes, void *hip_stream) {
  const char *fn = "reslim_head_fwd";
  if (!c) return RESLIM_EINVAL;
  if (!x || !tokens || !y) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  int rc = check_common(c, fn, batch, workspace, ws_bytes, true);
  if (rc != RESLIM_OK) return rc;
  return head_impl(c, fn, x, tokens, y, batch, plan_workspace(c, batch, workspace), static_cast<hipStream_t>(hip_stream));
}

extern "C" int reslim_forward(reslim_ctx *c, const float *x, float *y, int32_t batch, void *workspace, size_t ws_bytes, void *hip_stream) {
  const char *fn = "reslim_forward";
  if (!c) return RESLIM_EINVAL;
  if (!x || !y) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  int rc = check_common(c, fn, batch, workspace, ws_bytes, true);
  if (rc != RESLIM_OK) return rc;
  const Workspace w = plan_workspace(c, batch, workspace);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if ((rc = embed_impl(c, fn, x, w.X, batch, w, st)) != RESLIM_OK) return rc;
  for (int l = 0; l < c->cfg.depth; ++l)
    if ((rc = block_impl(c, fn, l, w.X, batch, w, st)) != RESLIM_OK) return rc;
  return head_impl(c, fn, x, w.X, y, batch, w, st);
}

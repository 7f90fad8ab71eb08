// Entry points of the training-side kernels (gradients); the chain rule applied to
// the operations of ORBIT-2 Sec. 4.1 / 4.2.
#include <algorithm>
#include <cmath>
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

// ------------------------------------------------------------------ training of a block
namespace {

struct TrainSaved {        // what the training forward keeps for the gradient (one block)
  void *ln1, *qkv, *attn;  // act [M, D], [M, 3D] (q pre-scaled in the bf16 path), [M, D]
  float *lse;              // [batch, heads, n_h]
  float *x_mid;            // [M, D] stream after the attention half
  void *ln2, *h, *u;       // act [M, D], [M, R] before GELU, [M, R] after
  size_t total;
};
// n_h: rows per "sample" (the context's tile-major count, or all leaves of a compressed batch with batch = 1)
TrainSaved plan_saved(const reslim_ctx *c, int batch, void *base, int64_t n_h) {
  const size_t M = static_cast<size_t>(batch) * n_h, D = c->cfg.embed_dim, R = c->R, es = act_size(c);
  unsigned char *p = static_cast<unsigned char *>(base);
  size_t off = 0;
  auto take = [&](size_t bytes) { unsigned char *q = p + off; off += align256(bytes); return q; };
  TrainSaved s;
  s.ln1 = take(M * D * es);
  s.qkv = take(M * 3 * D * es);
  s.attn = take(M * D * es);
  s.lse = reinterpret_cast<float *>(take(static_cast<size_t>(batch) * c->cfg.heads * n_h * sizeof(float)));
  s.x_mid = reinterpret_cast<float *>(take(M * D * sizeof(float)));
  s.ln2 = take(M * D * es);
  s.h = take(M * R * es);
  s.u = take(M * R * es);
  s.total = off;
  return s;
}

struct TrainWs {           // scratch of the gradient pass
  void *a, *b, *r;         // act [M, D], [M, D], [M, max(3D, R)]
  float *g;                // [M, D]
  void *attn;              // tiles_attention_bwd scratch
  void *wgrad;             // partial tiles of the weight gradients
  float *colp, *lnp;       // partial rows of the column sums and of the LayerNorm parameter gradients
  size_t total;
};
TrainWs plan_train_ws(const reslim_ctx *c, int batch, void *base, const SeqGeom &sg) {
  const size_t M = static_cast<size_t>(batch) * sg.n_h, D = c->cfg.embed_dim, R = c->R, es = act_size(c);
  const int dt = c->cfg.dtype, Mi = static_cast<int>(M), Di = c->cfg.embed_dim, Ri = c->R;
  unsigned char *p = static_cast<unsigned char *>(base);
  size_t off = 0;
  auto take = [&](size_t bytes) { unsigned char *q = p + off; off += align256(bytes); return q; };
  TrainWs w;
  w.a = take(M * D * es);
  w.b = take(M * D * es);
  w.r = take(M * std::max(3 * D, R) * es);
  w.g = reinterpret_cast<float *>(take(M * D * sizeof(float)));
  w.attn = take(tiles_attention_bwd_ws_bytes(c, batch, &sg));
  size_t wg = std::max(std::max(wgrad_ws_bytes(dt, Mi, 3 * Di, Di), wgrad_ws_bytes(dt, Mi, Di, Di)),
                       std::max(wgrad_ws_bytes(dt, Mi, Ri, Di), wgrad_ws_bytes(dt, Mi, Di, Ri)));
  w.wgrad = take(std::max<size_t>(wg, 256));
  w.colp = reinterpret_cast<float *>(take(static_cast<size_t>(colsum_slabs(M)) * std::max(3 * D, R) * sizeof(float)));
  w.lnp = reinterpret_cast<float *>(take(static_cast<size_t>(layernorm_bwd_slabs(M)) * 2 * D * sizeof(float)));
  w.total = off;
  return w;
}

int check_train(reslim_ctx *c, const char *fn, int layer, int batch, const void *saved, size_t saved_bytes, const void *ws,
                size_t ws_bytes, const SeqGeom &sg) {
  if (layer < 0 || layer >= c->cfg.depth) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": layer outside [0, depth)");
  if (batch < 1 || static_cast<int64_t>(batch) * sg.n_h > INT32_MAX)
    return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": batch * tokens must be in [1, 2^31)");
  if (!c->layers[layer].wt_qkv) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": call reslim_train_prepare first");
  if (!saved || (reinterpret_cast<uintptr_t>(saved) & 255) || !ws || (reinterpret_cast<uintptr_t>(ws) & 255))
    return set_error(c, RESLIM_EWORKSPACE, std::string(fn) + ": saved / workspace null or not 256-byte aligned");
  if (saved_bytes < plan_saved(c, batch, nullptr, sg.n_h).total || ws_bytes < plan_train_ws(c, batch, nullptr, sg).total)
    return set_error(c, RESLIM_EWORKSPACE, std::string(fn) + ": saved / workspace smaller than reslim_block_train_bytes()");
  return RESLIM_OK;
}

// one linear layer backwards: dx = dy W (optional), dW = dy^T x, db = column sums of dy
int linear_bwd_impl(reslim_ctx *c, const char *fn, const void *x, const void *dy, const void *w_t, void *dx, float *dw,
                    float *db, int M, int N, int K, void *wgrad_ws, float *colp, hipStream_t st) {
  const int dt = c->cfg.dtype;
  const double es = static_cast<double>(act_size(c)), dM = M, dN = N, dK = K;
  if (dx)
    RESLIM_LAUNCH("gemm_dgrad", 2.0 * dM * dN * dK, dM * dN * es + dN * dK * es + dM * dK * es,
                  launch_gemm(dt, EPI_BIAS_ACT, dy, w_t, c->d_zero_bias, dx, K, nullptr, 0, M, K, N, st));
  RESLIM_LAUNCH("gemm_wgrad", 2.0 * dM * dN * dK, dM * dN * es + dM * dK * es + 4.0 * dN * dK,
                launch_wgrad(dt, dy, x, dw, M, N, K, wgrad_ws, c->d_zero_bias, st));
  RESLIM_LAUNCH("colsum", 0, dM * dN * es + 4.0 * dN, launch_colsum(dt, dy, colp, db, M, N, st));
  return RESLIM_OK;
}

}  // namespace

extern "C" int reslim_train_prepare(reslim_ctx *c) {
  const char *fn = "reslim_train_prepare";
  if (!c) return RESLIM_EINVAL;
  const int D = c->cfg.embed_dim, R = c->R, dt = c->cfg.dtype;
  const size_t es = act_size(c);
  for (LayerWeights &lw : c->layers) {
    if (lw.wt_qkv) continue;
    struct { void *src; void **dst; int rows, cols; } todo[4] = {
        {lw.w_qkv, &lw.wt_qkv, 3 * D, D}, {lw.w_proj, &lw.wt_proj, D, D}, {lw.w_fc1, &lw.wt_fc1, R, D}, {lw.w_fc2, &lw.wt_fc2, D, R}};
    for (auto &td : todo) {
      void *d = nullptr;
      hipError_t e = hipMalloc(&d, std::max<size_t>(static_cast<size_t>(td.rows) * td.cols * es, 256));
      if (e != hipSuccess) return set_error(c, e == hipErrorOutOfMemory ? RESLIM_ENOMEM : RESLIM_EHIP, std::string(fn) + ": " + hipGetErrorString(e));
      c->allocs.push_back(d);
      RESLIM_TRY("transpose", launch_transpose(dt, td.src, d, td.rows, td.cols, nullptr));
      *td.dst = d;
    }
  }
  RESLIM_TRY("synchronize", hipDeviceSynchronize());
  return RESLIM_OK;
}

extern "C" int reslim_block_train_bytes(const reslim_ctx *c, int32_t batch, size_t *saved_bytes, size_t *ws_bytes) {
  if (!c || batch < 1) return RESLIM_EINVAL;
  if (saved_bytes) *saved_bytes = plan_saved(c, batch, nullptr, c->n_h).total;
  if (ws_bytes) *ws_bytes = plan_train_ws(c, batch, nullptr, ctx_geom(c)).total;
  return RESLIM_OK;
}

extern "C" int reslim_layernorm_bwd(reslim_ctx *c, const float *x, const void *dy, const float *gamma, const float *res,
                                    float *dx, float *dgamma, float *dbeta, int64_t rows, void *workspace,
                                    size_t ws_bytes, void *hip_stream) {
  const char *fn = "reslim_layernorm_bwd";
  if (!c) return RESLIM_EINVAL;
  if (!x || !dy || !gamma || !dx || !dgamma || !dbeta) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  if (rows < 1 || rows > INT32_MAX) return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": rows must be in [1, 2^31)");
  const size_t need = static_cast<size_t>(layernorm_bwd_slabs(rows)) * 2 * c->cfg.embed_dim * sizeof(float);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || ws_bytes < need)
    return set_error(c, RESLIM_EWORKSPACE, std::string(fn) + ": workspace null, misaligned or smaller than 1024 * 2 * D floats");
  RESLIM_TRY("launch", launch_layernorm_bwd(c->cfg.dtype, x, dy, gamma, res, dx, nullptr, static_cast<float *>(workspace),
                                            dgamma, dbeta, rows, c->cfg.embed_dim, static_cast<hipStream_t>(hip_stream)));
  return RESLIM_OK;
}

extern "C" int reslim_linear_bwd(reslim_ctx *c, int32_t layer, int32_t which, const void *x, const void *dy, void *dx,
                                 float *dw, float *db, int32_t rows, void *workspace, size_t ws_bytes, void *hip_stream) {
  const char *fn = "reslim_linear_bwd";
  if (!c) return RESLIM_EINVAL;
  if (!x || !dy || !dw || !db) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  if (layer < 0 || layer >= c->cfg.depth || which < 0 || which > 3) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": layer or matrix index out of range");
  if (rows < 1) return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": rows must be positive");
  const LayerWeights &lw = c->layers[layer];
  if (!lw.wt_qkv) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": call reslim_train_prepare first");
  const int D = c->cfg.embed_dim, R = c->R;
  const int N = which == 0 ? 3 * D : (which == 2 ? R : D), K = which == 3 ? R : D;
  const void *w_t = which == 0 ? lw.wt_qkv : which == 1 ? lw.wt_proj : which == 2 ? lw.wt_fc1 : lw.wt_fc2;
  const size_t wg = std::max<size_t>(wgrad_ws_bytes(c->cfg.dtype, rows, N, K), 256);
  const size_t need = wg + align256(static_cast<size_t>(colsum_slabs(rows)) * N * sizeof(float));
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || ws_bytes < need)
    return set_error(c, RESLIM_EWORKSPACE, std::string(fn) + ": workspace null, misaligned or too small");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  return linear_bwd_impl(c, fn, x, dy, w_t, dx, dw, db, rows, N, K, workspace,
                         reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + wg), st);
}

extern "C" int reslim_linear_bwd_workspace_bytes(const reslim_ctx *c, int32_t which, int32_t rows, size_t *out) {
  if (!c || !out || which < 0 || which > 3 || rows < 1) return RESLIM_EINVAL;
  const int D = c->cfg.embed_dim, R = c->R;
  const int N = which == 0 ? 3 * D : (which == 2 ? R : D), K = which == 3 ? R : D;
  *out = std::max<size_t>(wgrad_ws_bytes(c->cfg.dtype, rows, N, K), 256) + align256(static_cast<size_t>(colsum_slabs(rows)) * N * sizeof(float));
  return RESLIM_OK;
}

static int block_fwd_train_impl(reslim_ctx *c, const char *fn, int layer, const float *x_in, float *x_out, void *saved,
                                size_t saved_bytes, int batch, void *workspace, size_t ws_bytes, void *hip_stream,
                                const SeqGeom &sg) {
  if (!x_in || !x_out || x_in == x_out) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer or x_out aliases x_in");
  int rc = check_train(c, fn, layer, batch, saved, saved_bytes, workspace, ws_bytes, sg);
  if (rc != RESLIM_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const TrainSaved s = plan_saved(c, batch, saved, sg.n_h);
  const int D = c->cfg.embed_dim, R = c->R, dt = c->cfg.dtype;
  const int M = static_cast<int>(batch * sg.n_h);
  const LayerWeights &lw = c->layers[layer];
  const double es = static_cast<double>(act_size(c)), dM = M, dD = D, dR = R;
  const double pairs = sg.pairs;
  const bool qs = dt == RESLIM_BF16;
  const float qscale = 1.4426950408889634f / sqrtf(static_cast<float>(c->dh));
  RESLIM_LAUNCH("layernorm", 0, dM * dD * (4.0 + es), launch_layernorm(dt, x_in, nullptr, 0, 0, lw.ln1_g, lw.ln1_b, s.ln1, M, D, st));
  RESLIM_LAUNCH("gemm_qkv", 6.0 * dM * dD * dD, dM * dD * es + 3.0 * dD * dD * es + 3.0 * dM * dD * es,
                launch_gemm(dt, qs ? EPI_BIAS_QSCALE_ACT : EPI_BIAS_ACT, s.ln1, lw.w_qkv, lw.b_qkv, s.qkv, 3 * D, nullptr, 0, M,
                            3 * D, D, st, qscale, D));
  RESLIM_LAUNCH("tiles_attention", 4.0 * pairs * dD * batch, 4.0 * dM * dD * es,
                launch_tiles_attention(c, s.qkv, s.attn, batch, qs, st, s.lse, &sg));
  RESLIM_LAUNCH("gemm_proj", 2.0 * dM * dD * dD, dM * dD * es + dD * dD * es + 8.0 * dM * dD,
                launch_gemm(dt, EPI_BIAS_RES_F32, s.attn, lw.w_proj, lw.b_proj, s.x_mid, D, nullptr, 0, M, D, D, st, 1.0f, 0, x_in));
  RESLIM_LAUNCH("layernorm", 0, dM * dD * (4.0 + es), launch_layernorm(dt, s.x_mid, nullptr, 0, 0, lw.ln2_g, lw.ln2_b, s.ln2, M, D, st));
  // the hidden layer is kept before AND after GELU (one epilogue writes both)
  RESLIM_LAUNCH("gemm_fc1", 2.0 * dM * dD * dR, dM * dD * es + dD * dR * es + 2.0 * dM * dR * es,
                launch_gemm(dt, EPI_BIAS_ACT_GELU2, s.ln2, lw.w_fc1, lw.b_fc1, s.h, R, nullptr, 0, M, R, D, st, 1.0f, 0, nullptr, s.u));
  RESLIM_LAUNCH("gemm_fc2", 2.0 * dM * dD * dR, dM * dR * es + dD * dR * es + 8.0 * dM * dD,
                launch_gemm(dt, EPI_BIAS_RES_F32, s.u, lw.w_fc2, lw.b_fc2, x_out, D, nullptr, 0, M, D, R, st, 1.0f, 0, s.x_mid));
  return RESLIM_OK;
}

extern "C" int reslim_block_fwd_train(reslim_ctx *c, int32_t layer, const float *x_in, float *x_out, void *saved,
                                      size_t saved_bytes, int32_t batch, void *workspace, size_t ws_bytes, void *hip_stream) {
  if (!c) return RESLIM_EINVAL;
  return block_fwd_train_impl(c, "reslim_block_fwd_train", layer, x_in, x_out, saved, saved_bytes, batch, workspace, ws_bytes,
                              hip_stream, ctx_geom(c));
}

extern "C" int reslim_asc_block_fwd_train(reslim_ctx *c, const reslim_asc_plan *plan, int32_t layer, const float *x_in,
                                          float *x_out, void *saved, size_t saved_bytes, void *workspace, size_t ws_bytes,
                                          void *hip_stream) {
  if (!c) return RESLIM_EINVAL;
  if (!plan || plan->ctx != c) return set_error(c, RESLIM_EINVAL, "reslim_asc_block_fwd_train: null plan or plan of another context");
  return block_fwd_train_impl(c, "reslim_asc_block_fwd_train", layer, x_in, x_out, saved, saved_bytes, 1, workspace, ws_bytes,
                              hip_stream, plan->geom);
}

static int block_bwd_impl(reslim_ctx *c, const char *fn, int layer, const float *x_in, const void *saved, size_t saved_bytes,
                          const float *d_x_out, float *d_x_in, const reslim_block_grads *grads, int batch, void *workspace,
                          size_t ws_bytes, void *hip_stream, const SeqGeom &sg) {
  if (!x_in || !d_x_out || !d_x_in || !grads) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  const float *const *gp = reinterpret_cast<const float *const *>(grads);
  for (int i = 0; i < 12; ++i)
    if (!gp[i]) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null gradient buffer");
  int rc = check_train(c, fn, layer, batch, saved, saved_bytes, workspace, ws_bytes, sg);
  if (rc != RESLIM_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const TrainSaved s = plan_saved(c, batch, const_cast<void *>(saved), sg.n_h);
  const TrainWs w = plan_train_ws(c, batch, workspace, sg);
  const int D = c->cfg.embed_dim, R = c->R, dt = c->cfg.dtype;
  const int M = static_cast<int>(batch * sg.n_h);
  const LayerWeights &lw = c->layers[layer];
  const double es = static_cast<double>(act_size(c)), dM = M, dD = D;
  const double pairs = sg.pairs;
  const int64_t MD = static_cast<int64_t>(M) * D;

  // x_out = x_mid + fc2(gelu(fc1(ln2(x_mid))))
  RESLIM_LAUNCH("to_act", 0, dM * dD * (4.0 + es), launch_to_act(dt, d_x_out, w.a, MD, st));
  rc = linear_bwd_impl(c, fn, s.u, w.a, lw.wt_fc2, w.r, grads->w_fc2, grads->b_fc2, M, D, R, w.wgrad, w.colp, st);
  if (rc != RESLIM_OK) return rc;
  // GELU's derivative as its own bandwidth-bound pass: fused into the epilogue of the GEMM above it cost more
  // than it saved (measured 0.32 ms against 0.12 + 0.09 at c1: the epilogue's arithmetic is not hidden)
  RESLIM_LAUNCH("gelu_bwd", 0, 3.0 * static_cast<double>(M) * R * es, launch_gelu(dt, true, s.h, w.r, w.r, static_cast<int64_t>(M) * R, st));
  rc = linear_bwd_impl(c, fn, s.ln2, w.r, lw.wt_fc1, w.b, grads->w_fc1, grads->b_fc1, M, R, D, w.wgrad, w.colp, st);
  if (rc != RESLIM_OK) return rc;
  RESLIM_LAUNCH("layernorm_bwd", 0, dM * dD * (12.0 + 2.0 * es),
                launch_layernorm_bwd(dt, s.x_mid, w.b, lw.ln2_g, d_x_out, w.g, w.a, w.lnp, grads->ln2_g, grads->ln2_b, M, D, st));
  // x_mid = x_in + proj(tile_attention(qkv(ln1(x_in))))
  rc = linear_bwd_impl(c, fn, s.attn, w.a, lw.wt_proj, w.b, grads->w_proj, grads->b_proj, M, D, D, w.wgrad, w.colp, st);
  if (rc != RESLIM_OK) return rc;
  RESLIM_LAUNCH("tiles_attention_bwd", 10.0 * pairs * dD * batch, 8.0 * dM * dD * es,
                launch_tiles_attention_bwd(c, s.qkv, s.attn, s.lse, w.b, w.r, batch, w.attn, dt == RESLIM_BF16, st, &sg));
  rc = linear_bwd_impl(c, fn, s.ln1, w.r, lw.wt_qkv, w.a, grads->w_qkv, grads->b_qkv, M, 3 * D, D, w.wgrad, w.colp, st);
  if (rc != RESLIM_OK) return rc;
  RESLIM_LAUNCH("layernorm_bwd", 0, dM * dD * (12.0 + es),
                launch_layernorm_bwd(dt, x_in, w.a, lw.ln1_g, w.g, d_x_in, nullptr, w.lnp, grads->ln1_g, grads->ln1_b, M, D, st));
  return RESLIM_OK;
}

extern "C" int reslim_block_bwd(reslim_ctx *c, int32_t layer, const float *x_in, const void *saved, size_t saved_bytes,
                                const float *d_x_out, float *d_x_in, const reslim_block_grads *grads, int32_t batch,
                                void *workspace, size_t ws_bytes, void *hip_stream) {
  if (!c) return RESLIM_EINVAL;
  return block_bwd_impl(c, "reslim_block_bwd", layer, x_in, saved, saved_bytes, d_x_out, d_x_in, grads, batch, workspace,
                        ws_bytes, hip_stream, ctx_geom(c));
}

extern "C" int reslim_asc_block_bwd(reslim_ctx *c, const reslim_asc_plan *plan, int32_t layer, const float *x_in,
                                    const void *saved, size_t saved_bytes, const float *d_x_out, float *d_x_in,
                                    const reslim_block_grads *grads, void *workspace, size_t ws_bytes, void *hip_stream) {
  if (!c) return RESLIM_EINVAL;
  if (!plan || plan->ctx != c) return set_error(c, RESLIM_EINVAL, "reslim_asc_block_bwd: null plan or plan of another context");
  return block_bwd_impl(c, "reslim_asc_block_bwd", layer, x_in, saved, saved_bytes, d_x_out, d_x_in, grads, 1, workspace,
                        ws_bytes, hip_stream, plan->geom);
}

extern "C" int reslim_asc_block_train_bytes(const reslim_ctx *c, const reslim_asc_plan *plan, size_t *saved_bytes, size_t *ws_bytes) {
  if (!c || !plan || plan->ctx != c) return RESLIM_EINVAL;
  if (saved_bytes) *saved_bytes = plan_saved(c, 1, nullptr, plan->geom.n_h).total;
  if (ws_bytes) *ws_bytes = plan_train_ws(c, 1, nullptr, plan->geom).total;
  return RESLIM_OK;
}

// ------------------------------------------------------------------ dynamic gradient scaling (Sec. 4.4)
extern "C" int reslim_block_grads_unscale(reslim_ctx *c, const reslim_block_grads *grads, float inv_scale,
                                          int32_t *found_inf, void *hip_stream) {
  const char *fn = "reslim_block_grads_unscale";
  if (!c) return RESLIM_EINVAL;
  if (!grads || !found_inf) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null argument");
  if (!(inv_scale > 0.0f) || !std::isfinite(inv_scale)) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": inv_scale must be positive and finite");
  const int64_t D = c->cfg.embed_dim, R = c->R;
  float *ptrs[12] = {grads->ln1_g, grads->ln1_b, grads->w_qkv, grads->b_qkv, grads->w_proj, grads->b_proj,
                     grads->ln2_g, grads->ln2_b, grads->w_fc1, grads->b_fc1, grads->w_fc2, grads->b_fc2};
  const int64_t sizes[12] = {D, D, 3 * D * D, 3 * D, D * D, D, D, D, R * D, R, D * R, D};
  for (float *p : ptrs)
    if (!p) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null gradient buffer");
  RESLIM_TRY("launch", launch_unscale_check(ptrs, sizes, 12, inv_scale, found_inf, static_cast<hipStream_t>(hip_stream)));
  return RESLIM_OK;
}

// host arithmetic only: the schedule of the scale
extern "C" int reslim_grad_scale_update(float *scale, int32_t *growth_tracker, int32_t found_inf, float growth_factor,
                                        float backoff_factor, int32_t growth_interval) {
  if (!scale || !growth_tracker || !(*scale > 0.0f) || !(growth_factor >= 1.0f) || !(backoff_factor > 0.0f) ||
      !(backoff_factor <= 1.0f) || growth_interval < 1 || *growth_tracker < 0)
    return RESLIM_EINVAL;
  if (found_inf) {
    *scale *= backoff_factor;
    *growth_tracker = 0;
  } else if (++*growth_tracker >= growth_interval) {
    *scale *= growth_factor;
    *growth_tracker = 0;
  }
  return RESLIM_OK;
}


// Entry points that chain the kernels: embed, block, head, forward
// (ORBIT-2 Sec. 4.1 data flow, applied tile-wise as in Sec. 4.2).
#include <algorithm>
#include <cmath>

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
  const size_t xc_b = last_block_on_patches(c) ? align256(Mi * D * sizeof(float)) : 0;
  Workspace w;
  unsigned char *p = static_cast<unsigned char *>(base);
  w.X = reinterpret_cast<float *>(p);
  w.A = p + x_b;
  w.big = p + x_b + a_b;
  w.Xc = xc_b ? reinterpret_cast<float *>(p + x_b + a_b + big_b) : nullptr;
  w.total = x_b + a_b + big_b + xc_b;
  return w;
}

bool last_block_on_patches(const reslim_ctx *c) {
  return c->cfg.dtype == RESLIM_BF16 && c->cfg.depth >= 1 && c->n_h > c->N;
}


int hip_fail(reslim_ctx *c, const char *fn, const char *what, hipError_t e) {
  return set_error(c, RESLIM_EHIP, std::string(fn) + ": " + what + ": " + hipGetErrorString(e));
}

int check_common(reslim_ctx *c, const char *fn, int batch, const void *ws, size_t ws_bytes, bool need_ws) {
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

// tokenisation + aggregation + position/resolution terms: dst (w.big if null) <- float [batch * N, D] in patch order
int embed_full_impl(reslim_ctx *c, const char *fn, const float *x, int batch, const Workspace &w, hipStream_t st, float *dst) {
  const int D = c->cfg.embed_dim, dt = c->cfg.dtype;
  const int Mi = batch * c->N;
  const double es = static_cast<double>(act_size(c)), dMi = Mi, dD = D;
  // scores and values are affine in the p x p pixels of a patch: (p^2 + 1) multiply-adds per (variable, head) and per
  // (variable, feature), then the weighted sum over the variables
  RESLIM_LAUNCH("embed_agg", 2.0 * dMi * c->cfg.in_vars * ((c->cfg.patch * c->cfg.patch + 1.0) * (dD + c->cfg.heads) + dD),
                4.0 * batch * c->cfg.in_vars * c->cfg.H * c->cfg.W + dMi * dD * es,
                launch_embed_agg(c, x, w.A, batch, st));
  RESLIM_LAUNCH("gemm_agg_out", 2.0 * dMi * dD * dD, dMi * dD * es + dD * dD * es + 4.0 * c->N * dD + 4.0 * dMi * dD,
                launch_gemm(dt, EPI_BIAS_TAB_F32, w.A, c->d_agg_wo, c->d_zero_bias, dst ? static_cast<void *>(dst) : w.big, D, c->d_pos_res, c->N,
                            Mi, D, D, st));
  return RESLIM_OK;
}

static int embed_impl(reslim_ctx *c, const char *fn, const float *x, float *tokens, int batch, const Workspace &w, hipStream_t st) {
  const int D = c->cfg.embed_dim;
  const int Mi = batch * c->N;
  const double dMi = Mi, dD = D, dM = static_cast<double>(batch) * c->n_h;
  const int rc = embed_full_impl(c, fn, x, batch, w, st, nullptr);
  if (rc != RESLIM_OK) return rc;
  RESLIM_LAUNCH("gather", 0, 4.0 * dMi * dD + 4.0 * dM * dD,
                launch_gather_rows(static_cast<const float *>(w.big), c->d_gather, tokens, batch, c->n_h, c->N, D, st));
  return RESLIM_OK;
}

int block_impl(reslim_ctx *c, const char *fn, int layer, float *X, int batch, const Workspace &w, hipStream_t st,
               const SeqGeom *geom, const float *z_first) {
  const int D = c->cfg.embed_dim, R = c->R, dt = c->cfg.dtype;
  const SeqGeom sg = geom ? *geom : ctx_geom(c);
  const int M = static_cast<int>(batch * sg.n_h);
  const LayerWeights &lw = c->layers[layer];
  const double es = static_cast<double>(act_size(c)), dM = M, dD = D, dR = R;
  const double pairs = sg.pairs;
  // z_first (first block of a whole forward): the stream is still the embedding in patch order;
  // the tile-major rows, halo copies included, are read from it through the gather list here and
  // by the projection's skip connection, which is what writes X for the first time
  if (z_first)
    RESLIM_LAUNCH("layernorm", 0, dM * dD * (4.0 + es),
                  launch_layernorm(dt, z_first, c->d_gather, static_cast<int>(sg.n_h), c->N, lw.ln1_g, lw.ln1_b, w.A, M, D, st));
  else
    RESLIM_LAUNCH("layernorm", 0, dM * dD * (4.0 + es), launch_layernorm(dt, X, nullptr, 0, 0, lw.ln1_g, lw.ln1_b, w.A, M, D, st));
  // bf16 path: the QKV epilogue multiplies q by log2(e)/sqrt(dh) before its one
  // rounding to bf16, and the attention kernel then exponentiates in base 2 directly
  const bool qs = dt == RESLIM_BF16 && attention_accepts_prescaled_q();
  const float qscale = 1.4426950408889634f / sqrtf(static_cast<float>(c->dh));
  RESLIM_LAUNCH("gemm_qkv", 6.0 * dM * dD * dD, dM * dD * es + 3.0 * dD * dD * es + 3.0 * dM * dD * es,
                launch_gemm(dt, qs ? EPI_BIAS_QSCALE_ACT : EPI_BIAS_ACT, w.A, lw.w_qkv, lw.b_qkv, w.big, 3 * D, nullptr, 0, M,
                            3 * D, D, st, qscale, D));
  RESLIM_LAUNCH("tiles_attention", 4.0 * pairs * dD * batch, 4.0 * dM * dD * es,
                launch_tiles_attention(c, w.big, w.A, batch, qs, st, nullptr, &sg));
  if (z_first) {
    const ResRowMap skip = {c->d_gather, static_cast<int>(sg.n_h), c->N};
    RESLIM_LAUNCH("gemm_proj", 2.0 * dM * dD * dD, dM * dD * es + dD * dD * es + 8.0 * dM * dD,
                  launch_gemm(dt, EPI_BIAS_RES_F32, w.A, lw.w_proj, lw.b_proj, X, D, nullptr, 0, M, D, D, st, 1.0f, 0, z_first, nullptr, &skip));
  } else {
    RESLIM_LAUNCH("gemm_proj", 2.0 * dM * dD * dD, dM * dD * es + dD * dD * es + 8.0 * dM * dD,
                  launch_gemm(dt, EPI_BIAS_RESADD_F32, w.A, lw.w_proj, lw.b_proj, X, D, nullptr, 0, M, D, D, st));
  }
  RESLIM_LAUNCH("layernorm", 0, dM * dD * (4.0 + es), launch_layernorm(dt, X, nullptr, 0, 0, lw.ln2_g, lw.ln2_b, w.A, M, D, st));
  RESLIM_LAUNCH("gemm_fc1", 2.0 * dM * dD * dR, dM * dD * es + dD * dR * es + dM * dR * es,
                launch_gemm(dt, EPI_BIAS_GELU_ACT, w.A, lw.w_fc1, lw.b_fc1, w.big, R, nullptr, 0, M, R, D, st));
  RESLIM_LAUNCH("gemm_fc2", 2.0 * dM * dD * dR, dM * dR * es + dD * dR * es + 8.0 * dM * dD,
                launch_gemm(dt, EPI_BIAS_RESADD_F32, w.big, lw.w_fc2, lw.b_fc2, X, D, nullptr, 0, M, D, R, st));
  return RESLIM_OK;
}

// The last block of a whole forward, when some tokens are halo copies: X is read (tile-major), the
// block's output for the patches goes to w.Xc [batch * N, D] in patch order.
static int last_block_impl(reslim_ctx *c, const char *fn, const float *X, int batch, const Workspace &w, hipStream_t st) {
  const int D = c->cfg.embed_dim, R = c->R, dt = c->cfg.dtype;
  const SeqGeom sg = ctx_geom(c);
  const int M = static_cast<int>(batch * sg.n_h), Mi = batch * c->N;
  const LayerWeights &lw = c->layers[c->cfg.depth - 1];
  const double es = static_cast<double>(act_size(c)), dM = M, dMi = Mi, dD = D, dR = R;
  RESLIM_LAUNCH("layernorm", 0, dM * dD * (4.0 + es), launch_layernorm(dt, X, nullptr, 0, 0, lw.ln1_g, lw.ln1_b, w.A, M, D, st));
  const bool qs = attention_accepts_prescaled_q();
  const float qscale = 1.4426950408889634f / sqrtf(static_cast<float>(c->dh));
  RESLIM_LAUNCH("gemm_qkv", 6.0 * dM * dD * dD, dM * dD * es + 3.0 * dD * dD * es + 3.0 * dM * dD * es,
                launch_gemm(dt, qs ? EPI_BIAS_QSCALE_ACT : EPI_BIAS_ACT, w.A, lw.w_qkv, lw.b_qkv, w.big, 3 * D, nullptr, 0, M,
                            3 * D, D, st, qscale, D));
  // queries: the owned tokens; keys and values: the whole haloed tile
  RESLIM_LAUNCH("tiles_attention", 4.0 * sg.pairs_owned * dD * batch, 3.0 * dM * dD * es + dMi * dD * es,
                launch_tiles_attention(c, w.big, w.A, batch, qs, st, nullptr, nullptr, true));
  const ResRowMap skip = {c->d_interior_src, c->N, sg.n_h};
  RESLIM_LAUNCH("gemm_proj", 2.0 * dMi * dD * dD, dMi * dD * es + dD * dD * es + 8.0 * dMi * dD,
                launch_gemm(dt, EPI_BIAS_RES_F32, w.A, lw.w_proj, lw.b_proj, w.Xc, D, nullptr, 0, Mi, D, D, st, 1.0f, 0, X, nullptr, &skip));
  RESLIM_LAUNCH("layernorm", 0, dMi * dD * (4.0 + es), launch_layernorm(dt, w.Xc, nullptr, 0, 0, lw.ln2_g, lw.ln2_b, w.A, Mi, D, st));
  RESLIM_LAUNCH("gemm_fc1", 2.0 * dMi * dD * dR, dMi * dD * es + dD * dR * es + dMi * dR * es,
                launch_gemm(dt, EPI_BIAS_GELU_ACT, w.A, lw.w_fc1, lw.b_fc1, w.big, R, nullptr, 0, Mi, R, D, st));
  RESLIM_LAUNCH("gemm_fc2", 2.0 * dMi * dD * dR, dMi * dR * es + dD * dR * es + 8.0 * dMi * dD,
                launch_gemm(dt, EPI_BIAS_RESADD_F32, w.big, lw.w_fc2, lw.b_fc2, w.Xc, D, nullptr, 0, Mi, D, R, st));
  return RESLIM_OK;
}

// tokens: tile-major [batch * n_h, D], or with `stitched` the patches' rows [batch * N, D] in patch order
static int head_impl(reslim_ctx *c, const char *fn, const float *x, const float *tokens, float *y, int batch, const Workspace &w, hipStream_t st,
                     bool stitched = false) {
  const int D = c->cfg.embed_dim, dt = c->cfg.dtype;
  const int Mi = batch * c->N;
  const double es = static_cast<double>(act_size(c)), dMi = Mi, dD = D, dO = c->head_out;
  const double fine = static_cast<double>(batch) * c->cfg.out_vars * c->cfg.H * c->cfg.W * c->cfg.scale * c->cfg.scale;
  RESLIM_LAUNCH("layernorm_final", 0, dMi * dD * (4.0 + es),
                launch_layernorm(dt, tokens, stitched ? nullptr : c->d_interior_src, c->N, c->n_h, c->d_lnf_g, c->d_lnf_b, w.A, Mi, D, st));
  RESLIM_LAUNCH("gemm_head", 2.0 * dMi * dD * dO, dMi * dD * es + dD * dO * es + 4.0 * dMi * dO,
                launch_gemm(dt, EPI_BIAS_F32, w.A, c->d_w_head, c->d_b_head, w.big, c->head_out, nullptr, 0, Mi, c->head_out, D, st));
  RESLIM_LAUNCH("residual_unpatchify", 0,
                4.0 * batch * c->cfg.out_vars * c->cfg.H * c->cfg.W + 4.0 * dMi * dO + 4.0 * fine,
                launch_residual_unpatchify(c, x, w.big, 0, y, batch, st));
  return RESLIM_OK;
}

}  // namespace reslim

using namespace reslim;

extern "C" int reslim_profile_enable(reslim_ctx *c, int32_t max_records) {
  if (!c || max_records < 0) return RESLIM_EINVAL;
  for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  c->prof_ev.clear();
  c->prof_rec.clear();
  c->prof_on = max_records > 0;
  for (int i = 0; i < 2 * max_records; ++i) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return set_error(c, RESLIM_EHIP, "reslim_profile_enable: hipEventCreate failed");
    c->prof_ev.push_back(e);
  }
  c->prof_rec.reserve(max_records);
  return RESLIM_OK;
}

extern "C" int reslim_profile_reset(reslim_ctx *c) {
  if (!c) return RESLIM_EINVAL;
  c->prof_rec.clear();
  return RESLIM_OK;
}

extern "C" int reslim_profile_read(reslim_ctx *c, reslim_profile_record *out, int32_t max_out, int32_t *n_out) {
  if (!c || !n_out) return RESLIM_EINVAL;
  const int n = static_cast<int>(c->prof_rec.size());
  *n_out = n;
  if (!out) return RESLIM_OK;
  for (int i = 0; i < n && i < max_out; ++i) {
    if (hipEventSynchronize(c->prof_ev[2 * i + 1]) != hipSuccess) return set_error(c, RESLIM_EHIP, "reslim_profile_read: event sync failed");
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]) != hipSuccess)
      return set_error(c, RESLIM_EHIP, "reslim_profile_read: elapsed time failed");
    out[i].name = c->prof_rec[i].name;
    out[i].ms = ms;
    out[i].flop = c->prof_rec[i].flop;
    out[i].bytes = c->prof_rec[i].bytes;
  }
  return RESLIM_OK;
}

extern "C" int reslim_debug_copy(const void *src, void *dst, size_t bytes, void *hip_stream) {
  if (!src || !dst || bytes == 0 || bytes % 16) return RESLIM_EINVAL;
  return launch_copy_probe(src, dst, bytes, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? RESLIM_OK : RESLIM_EHIP;
}

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
  const double M = B * static_cast<double>(ctx->n_h), Mi = B * static_cast<double>(ctx->N);
  // what reslim_forward executes: with halo tokens its last block projects and runs the MLP on the
  // patches' rows only, and only the queries their tiles own attend
  const bool stitch = last_block_on_patches(ctx);
  if (gemm_flop) {
    *gemm_flop = 2.0 * M * D * (3.0 * D + D + 2.0 * ctx->R) * L;
    if (stitch) *gemm_flop -= 2.0 * (M - Mi) * D * (D + 2.0 * ctx->R);
  }
  if (attn_flop) {
    double s = 0, own = 0;
    for (const tile_desc &t : ctx->tiles) {
      s += static_cast<double>(t.n_tok) * t.n_tok;
      own += static_cast<double>(t.y1 - t.y0) * (t.x1 - t.x0) * t.n_tok;
    }
    *attn_flop = 4.0 * D * B * (stitch ? s * (L - 1) + own : s * L);
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
  RESLIM_TRY("launch", launch_tiles_attention(c, qkv, out, batch, false, static_cast<hipStream_t>(hip_stream)));
  return RESLIM_OK;
}

extern "C" int tiles_attention_fwd_lse(reslim_ctx *c, const void *qkv, void *out, float *lse, int32_t batch, void *hip_stream) {
  const char *fn = "tiles_attention_fwd_lse";
  if (!c) return RESLIM_EINVAL;
  if (!qkv || !out || !lse) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  int rc = check_common(c, fn, batch, nullptr, 0, false);
  if (rc != RESLIM_OK) return rc;
  RESLIM_TRY("launch", launch_tiles_attention(c, qkv, out, batch, false, static_cast<hipStream_t>(hip_stream), lse));
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
  const bool stitch = last_block_on_patches(c);
  // With halo tokens and at least two blocks the gather pass is folded into the first block: the
  // embedding stays in patch order (in w.Xc, which only the last block needs again) and the first
  // block reads its rows through the gather list.  Same values, same arithmetic per row.
  const bool fold_gather = stitch && c->cfg.depth >= 2;
  if (fold_gather) rc = embed_full_impl(c, fn, x, batch, w, st, w.Xc);
  else rc = embed_impl(c, fn, x, w.X, batch, w, st);
  if (rc != RESLIM_OK) return rc;
  for (int l = 0; l < c->cfg.depth - (stitch ? 1 : 0); ++l)
    if ((rc = block_impl(c, fn, l, w.X, batch, w, st, nullptr, l == 0 && fold_gather ? w.Xc : nullptr)) != RESLIM_OK) return rc;
  if (!stitch) return head_impl(c, fn, x, w.X, y, batch, w, st);
  if ((rc = last_block_impl(c, fn, w.X, batch, w, st)) != RESLIM_OK) return rc;
  return head_impl(c, fn, x, w.Xc, y, batch, w, st, true);
}

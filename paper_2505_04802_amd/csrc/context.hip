// reslim_create / reslim_destroy: validation, tiling tables, weight upload, and
// the exact folding of the per-variable tokenisation into the aggregation's key
// and value maps (ORBIT-2 Sec. 4.1).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <functional>
#include <new>
#include <thread>

#include "common.h"

namespace reslim {

const std::string &thread_error();

int set_error(reslim_ctx *ctx, int code, const std::string &msg) {
  if (ctx) ctx->err = msg;
  set_thread_error(msg);
  return code;
}

static uint16_t host_f32_to_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// splits [0, n) over the host cores
static void parallel_for(int64_t n, const std::function<void(int64_t, int64_t)> &fn) {
  unsigned hw = std::thread::hardware_concurrency();
  int nt = static_cast<int>(std::min<int64_t>(std::max(1u, std::min(hw, 16u)), n));
  if (nt <= 1) { fn(0, n); return; }
  std::vector<std::thread> th;
  const int64_t per = (n + nt - 1) / nt;
  for (int i = 0; i < nt; ++i) {
    const int64_t lo = i * per, hi = std::min<int64_t>(n, lo + per);
    if (lo < hi) th.emplace_back(fn, lo, hi);
  }
  for (auto &t : th) t.join();
}

struct Uploader {
  reslim_ctx *c;
  hipError_t err = hipSuccess;
  void *raw(const void *host, size_t bytes) {
    if (err != hipSuccess) return nullptr;
    void *d = nullptr;
    err = hipMalloc(&d, std::max<size_t>(bytes, 256));
    if (err != hipSuccess) return nullptr;
    c->allocs.push_back(d);
    if (host && bytes) err = hipMemcpy(d, host, bytes, hipMemcpyHostToDevice);
    return d;
  }
  float *f32(const float *host, size_t n) { return static_cast<float *>(raw(host, n * sizeof(float))); }
  // activation-typed copy: float as is, or rounded to bfloat16
  void *act(const float *host, size_t n) {
    if (c->cfg.dtype != RESLIM_BF16) return raw(host, n * sizeof(float));
    std::vector<uint16_t> tmp(n);
    parallel_for(static_cast<int64_t>(n), [&](int64_t lo, int64_t hi) {
      for (int64_t i = lo; i < hi; ++i) tmp[i] = host_f32_to_bf16(host[i]);
    });
    return raw(tmp.data(), n * sizeof(uint16_t));
  }
};

static int validate(const reslim_config &g, std::string &why) {
  auto bad = [&](const char *m) { why = m; return RESLIM_ESHAPE; };
  if (g.in_vars < 1 || g.out_vars < 1 || g.out_vars > g.in_vars) return bad("need 1 <= out_vars <= in_vars");
  if (g.H < 1 || g.W < 1 || g.scale < 1 || g.patch < 1) return bad("H, W, scale, patch must be positive");
  if (g.H % g.patch || g.W % g.patch) return bad("patch must divide H and W");
  if (g.embed_dim < 4 || g.heads < 1 || g.embed_dim % g.heads) return bad("heads must divide embed_dim");
  if (g.embed_dim % 4) return bad("embed_dim must be a multiple of 4");
  if (g.mlp_ratio < 1 || g.depth < 0) return bad("mlp_ratio >= 1 and depth >= 0 required");
  if (g.n_res < 1 || g.res_idx < 0 || g.res_idx >= g.n_res) return bad("res_idx outside the resolution table");
  if (g.dtype != RESLIM_F32 && g.dtype != RESLIM_BF16) { why = "dtype must be RESLIM_F32 or RESLIM_BF16"; return RESLIM_EINVAL; }
  if (g.dtype == RESLIM_BF16) {
    const int dh = g.embed_dim / g.heads;
    if (g.embed_dim % 64) return bad("bf16 path needs embed_dim % 64 == 0");
    if (dh != 64 && dh != 128 && dh != 256) return bad("bf16 path needs head dim 64, 128 or 256");
    const int64_t ps = static_cast<int64_t>(g.patch) * g.scale;
    if ((g.out_vars * ps * ps) % 8) return bad("bf16 path needs out_vars * (patch * scale)^2 % 8 == 0 (the GEMM epilogues move 8 columns at a time)");
  }
  if (static_cast<int64_t>(g.scale) * g.H > INT32_MAX / 2 || static_cast<int64_t>(g.scale) * g.W > INT32_MAX / 2)
    return bad("fine grid too large");
  return RESLIM_OK;
}

}  // namespace reslim

using namespace reslim;

extern "C" const char *reslim_last_error(const reslim_ctx *ctx) {
  return ctx ? ctx->err.c_str() : thread_error().c_str();
}

extern "C" void reslim_destroy(reslim_ctx *ctx) {
  if (!ctx) return;
  for (void *p : ctx->allocs) (void)hipFree(p);
  for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
  delete ctx;
}

extern "C" int reslim_create(const reslim_config *cfg, const reslim_weights *w, reslim_ctx **out) {
  if (out) *out = nullptr;
  if (!cfg || !w || !out) return set_error(nullptr, RESLIM_EINVAL, "reslim_create: null argument");
  std::string why;
  int rc = validate(*cfg, why);
  if (rc != RESLIM_OK) return set_error(nullptr, rc, "reslim_create: " + why);
  const float *const *wp = reinterpret_cast<const float *const *>(w);
  for (size_t i = 0; i < sizeof(reslim_weights) / sizeof(void *); ++i)
    if (!wp[i]) return set_error(nullptr, RESLIM_EINVAL, "reslim_create: a weight pointer is null");

  reslim_ctx *c = new (std::nothrow) reslim_ctx();
  if (!c) return set_error(nullptr, RESLIM_ENOMEM, "reslim_create: out of host memory");
  c->cfg = *cfg;
  const reslim_config &g = c->cfg;
  const int V = g.in_vars, C = g.out_vars, D = g.embed_dim, L = g.depth, p2 = g.patch * g.patch;
  c->Hp = g.H / g.patch; c->Wp = g.W / g.patch; c->N = c->Hp * c->Wp; c->T = g.tiles_y * g.tiles_x;
  c->dh = D / g.heads; c->R = g.mlp_ratio * D; c->ps = g.patch * g.scale; c->head_out = C * c->ps * c->ps;
  for (int i = 0; i < C; ++i)
    if (w->out_var_idx[i] < 0 || w->out_var_idx[i] >= V) {
      delete c;
      return set_error(nullptr, RESLIM_EINVAL, "reslim_create: out_var_idx outside [0, in_vars)");
    }
  auto fail = [&](int code, const std::string &m) {
    reslim_destroy(c);
    return set_error(nullptr, code, "reslim_create: " + m);
  };
  try {
    // ---- tiling (Sec. 4.2)
    rc = tiles_partition(c->Hp, c->Wp, g.tiles_y, g.tiles_x, g.halo, nullptr, nullptr, nullptr, &c->n_h);
    if (rc != RESLIM_OK) return fail(rc, thread_error());
    c->tiles.resize(c->T);
    std::vector<int32_t> gather(c->n_h), isrc(c->N), tile_of(c->n_h);
    rc = tiles_partition(c->Hp, c->Wp, g.tiles_y, g.tiles_x, g.halo, c->tiles.data(), gather.data(), isrc.data(), nullptr);
    if (rc != RESLIM_OK) return fail(rc, thread_error());
    c->max_n_tok = 0;
    for (int t = 0; t < c->T; ++t) {
      c->max_n_tok = std::max(c->max_n_tok, c->tiles[t].n_tok);
      std::fill(tile_of.begin() + c->tiles[t].tok_off, tile_of.begin() + c->tiles[t].tok_off + c->tiles[t].n_tok, t);
    }
    if (hipGetDevice(&c->device) != hipSuccess) return fail(RESLIM_EHIP, "no HIP device");

    Uploader up{c};
    c->d_tiles = static_cast<tile_desc *>(up.raw(c->tiles.data(), c->T * sizeof(tile_desc)));
    c->d_gather = static_cast<int32_t *>(up.raw(gather.data(), gather.size() * 4));
    c->d_interior_src = static_cast<int32_t *>(up.raw(isrc.data(), isrc.size() * 4));
    c->d_tile_of_tok = static_cast<int32_t *>(up.raw(tile_of.data(), tile_of.size() * 4));

    // ---- fold tokenisation into the aggregation (Sec. 4.1), in double
    // e_v = W_pe[v] x + base_v,  base_v = b_pe[v] + var_emb[v]
    // score(g, v) = q_g . (W_k e_v + b_k)_g / sqrt(dh) = A[v,g,:] . x + a0[v,g]
    // value(v)    = W_v e_v + b_v                      = U[v,:,:] x + c[v,:]
    const int heads = g.heads, dh = c->dh;
    std::vector<double> q(D), qk(static_cast<size_t>(heads) * D, 0.0), qb(heads, 0.0);
    for (int d = 0; d < D; ++d) {
      double s = w->agg_bq[d];
      for (int j = 0; j < D; ++j) s += static_cast<double>(w->agg_wq[static_cast<size_t>(d) * D + j]) * w->agg_q0[j];
      q[d] = s;
    }
    const double isd = 1.0 / std::sqrt(static_cast<double>(dh));
    for (int d = 0; d < D; ++d) {
      const int gh = d / dh;
      const float *row = w->agg_wk + static_cast<size_t>(d) * D;
      double *dst = qk.data() + static_cast<size_t>(gh) * D;
      const double qd = q[d] * isd;
      for (int j = 0; j < D; ++j) dst[j] += qd * row[j];
      qb[gh] += qd * w->agg_bk[d];
    }
    std::vector<float> fA(static_cast<size_t>(V) * heads * p2), fa0(static_cast<size_t>(V) * heads);
    std::vector<float> fU(static_cast<size_t>(V) * D * p2), fc(static_cast<size_t>(V) * D);
    std::vector<double> base(static_cast<size_t>(V) * D);
    for (int v = 0; v < V; ++v)
      for (int j = 0; j < D; ++j)
        base[static_cast<size_t>(v) * D + j] = static_cast<double>(w->b_pe[static_cast<size_t>(v) * D + j]) + w->var_emb[static_cast<size_t>(v) * D + j];
    for (int v = 0; v < V; ++v)
      for (int gh = 0; gh < heads; ++gh) {
        const double *qr = qk.data() + static_cast<size_t>(gh) * D;
        double s0 = qb[gh];
        std::vector<double> s(p2, 0.0);
        for (int j = 0; j < D; ++j) {
          s0 += qr[j] * base[static_cast<size_t>(v) * D + j];
          const float *pe = w->w_pe + (static_cast<size_t>(v) * D + j) * p2;
          for (int i = 0; i < p2; ++i) s[i] += qr[j] * pe[i];
        }
        fa0[static_cast<size_t>(v) * heads + gh] = static_cast<float>(s0);
        for (int i = 0; i < p2; ++i) fA[(static_cast<size_t>(v) * heads + gh) * p2 + i] = static_cast<float>(s[i]);
      }
    parallel_for(static_cast<int64_t>(V) * D, [&](int64_t lo, int64_t hi) {
      std::vector<double> s(p2);
      for (int64_t vd = lo; vd < hi; ++vd) {
        const int v = static_cast<int>(vd / D), d = static_cast<int>(vd % D);
        const float *wv = w->agg_wv + static_cast<size_t>(d) * D;
        const float *pe = w->w_pe + static_cast<size_t>(v) * D * p2;
        const double *bs = base.data() + static_cast<size_t>(v) * D;
        double s0 = w->agg_bv[d];
        std::fill(s.begin(), s.end(), 0.0);
        for (int j = 0; j < D; ++j) {
          const double wj = wv[j];
          s0 += wj * bs[j];
          for (int i = 0; i < p2; ++i) s[i] += wj * pe[static_cast<size_t>(j) * p2 + i];
        }
        fc[vd] = static_cast<float>(s0);
        for (int i = 0; i < p2; ++i) fU[static_cast<size_t>(vd) * p2 + i] = static_cast<float>(s[i]);
      }
    });
    c->d_agg_A = up.f32(fA.data(), fA.size());
    c->d_agg_a0 = up.f32(fa0.data(), fa0.size());
    c->d_agg_U = up.f32(fU.data(), fU.size());
    c->d_agg_c = up.f32(fc.data(), fc.size());
    c->d_agg_wo = up.act(w->agg_wo, static_cast<size_t>(D) * D);
    {
      std::vector<float> pr(static_cast<size_t>(c->N) * D);
      const float *re = w->res_emb + static_cast<size_t>(g.res_idx) * D;
      parallel_for(c->N, [&](int64_t lo, int64_t hi) {
        for (int64_t n = lo; n < hi; ++n)
          for (int d = 0; d < D; ++d)
            pr[n * D + d] = static_cast<float>(static_cast<double>(w->pos_emb[n * D + d]) + re[d] + w->agg_bo[d]);
      });
      c->d_pos_res = up.f32(pr.data(), pr.size());
    }
    {
      std::vector<float> z(std::max({3 * D, c->R, c->head_out}), 0.f);
      c->d_zero_bias = up.f32(z.data(), z.size());
    }
    // ---- blocks
    c->layers.resize(L);
    const size_t DD = static_cast<size_t>(D) * D, R = c->R;
    for (int l = 0; l < L; ++l) {
      LayerWeights &lw = c->layers[l];
      lw.ln1_g = up.f32(w->ln1_g + static_cast<size_t>(l) * D, D);
      lw.ln1_b = up.f32(w->ln1_b + static_cast<size_t>(l) * D, D);
      lw.ln2_g = up.f32(w->ln2_g + static_cast<size_t>(l) * D, D);
      lw.ln2_b = up.f32(w->ln2_b + static_cast<size_t>(l) * D, D);
      lw.w_qkv = up.act(w->w_qkv + l * 3 * DD, 3 * DD);
      lw.b_qkv = up.f32(w->b_qkv + static_cast<size_t>(l) * 3 * D, 3 * D);
      lw.w_proj = up.act(w->w_proj + l * DD, DD);
      lw.b_proj = up.f32(w->b_proj + static_cast<size_t>(l) * D, D);
      lw.w_fc1 = up.act(w->w_fc1 + l * R * D, R * D);
      lw.b_fc1 = up.f32(w->b_fc1 + l * R, R);
      lw.w_fc2 = up.act(w->w_fc2 + l * R * D, R * D);
      lw.b_fc2 = up.f32(w->b_fc2 + static_cast<size_t>(l) * D, D);
    }
    c->d_lnf_g = up.f32(w->lnf_g, D);
    c->d_lnf_b = up.f32(w->lnf_b, D);
    c->d_w_head = up.act(w->w_head, static_cast<size_t>(c->head_out) * D);
    c->d_b_head = up.f32(w->b_head, c->head_out);
    c->d_w_res = up.f32(w->w_res, static_cast<size_t>(C) * C * 9);
    c->d_b_res = up.f32(w->b_res, C);
    c->d_out_var_idx = static_cast<int32_t *>(up.raw(w->out_var_idx, C * sizeof(int32_t)));
    if (up.err != hipSuccess)
      return fail(up.err == hipErrorOutOfMemory ? RESLIM_ENOMEM : RESLIM_EHIP,
                  std::string("device upload failed: ") + hipGetErrorString(up.err));
    hipError_t e = gemm_init();
    if (e == hipSuccess) e = attention_init();
    if (e == hipSuccess) e = attention_bwd_init();
    if (e == hipSuccess) e = wgrad_init();
    if (e == hipSuccess) e = elementwise_init();
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) return fail(RESLIM_EHIP, std::string("kernel setup failed: ") + hipGetErrorString(e));
  } catch (const std::bad_alloc &) {
    return fail(RESLIM_ENOMEM, "out of host memory");
  } catch (...) {
    return fail(RESLIM_EINVAL, "unexpected exception");
  }
  *out = c;
  return RESLIM_OK;
}

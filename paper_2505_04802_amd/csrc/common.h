// Internal declarations shared by the translation units of libreslim.so.
// Nothing here is part of the C ABI (see include/reslim.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "../../include/reslim.h"

namespace reslim {

typedef uint16_t bf16_t;  // storage type of a bfloat16: the upper half of a float

// ---------------------------------------------------------------- device helpers
__device__ __forceinline__ float bf16_to_f32(bf16_t h) {
  return __uint_as_float(static_cast<uint32_t>(h) << 16);
}
// round to nearest, ties to even (finite inputs and infinities; NaN stays NaN)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  return __builtin_bit_cast(bf16_t, static_cast<__bf16>(f));   // hardware conversion on gfx950
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return static_cast<uint32_t>(f32_to_bf16(lo)) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
}

template <class T> struct Act;  // activation element type traits
template <> struct Act<float> {
  static __device__ __forceinline__ float load(const float *p) { return *p; }
  static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Act<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t *p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

// ---------------------------------------------------------------- context
struct LayerWeights {
  float *ln1_g, *ln1_b, *ln2_g, *ln2_b;      // [D] fp32
  void *w_qkv, *w_proj, *w_fc1, *w_fc2;      // act type, [out, in]
  void *wt_qkv = nullptr, *wt_proj = nullptr, *wt_fc1 = nullptr, *wt_fc2 = nullptr;   // [in, out] copies for the input-gradient GEMMs (reslim_train_prepare)
  float *b_qkv, *b_proj, *b_fc1, *b_fc2;     // fp32
};

// What the whole-model gradient needs beside the inference context (reslim_train_prepare_model)
struct TrainModel {
  bool ready = false;
  float *w_pe = nullptr, *b_pe = nullptr, *var_emb = nullptr, *q0 = nullptr;     // unfolded front end, fp32
  float *wq = nullptr, *bq = nullptr, *wk = nullptr, *bk = nullptr, *wv = nullptr, *bv = nullptr;
  void *wt_head = nullptr, *wt_agg_wo = nullptr;                                 // act [D, head_out], [D, D]: [in, out] copies
  int32_t *copy_off = nullptr, *copy_idx = nullptr;                              // tile-major copies of every patch: [N + 1], [n_h]
  void *w_vtab = nullptr;      // act [n_e, D]: value table by (head, variable, pixel | offset), zero outside the head's features
  float *zero_e = nullptr;     // [n_e] zeros
  int n_e = 0;                 // heads * V * (p2 + 1) rounded up to a multiple of 8
};

}  // namespace reslim

struct reslim_ctx {
  reslim_config cfg;
  int device;
  // derived sizes
  int Hp, Wp, N, T, dh, R, ps, head_out;
  int64_t n_h;
  int max_n_tok;
  std::vector<tile_desc> tiles;              // host copy
  // device: tiling
  tile_desc *d_tiles;                        // [T]
  int32_t *d_gather, *d_interior_src;        // [n_h], [N]
  int32_t *d_tile_of_tok;                    // [n_h] tile index of every tile-major token
  // device: folded front end (fp32)
  float *d_agg_A;    // [V, heads, p2]  score slope per (variable, head)
  float *d_agg_a0;   // [V, heads]      score offset
  float *d_agg_U;    // [V, D, p2]      value slope
  float *d_agg_c;    // [V, D]          value offset
  void *d_agg_wo;    // act [D, D]
  float *d_pos_res;  // [N, D]  pos_emb + res_emb[res_idx] + agg_bo
  float *d_zero_bias;// [max(3D, R, head_out)] zeros
  // device: blocks and head
  std::vector<reslim::LayerWeights> layers;
  float *d_lnf_g, *d_lnf_b;
  void *d_w_head;    // act [head_out, D]
  float *d_b_head;
  float *d_w_res, *d_b_res;                  // [C, C, 3, 3], [C]
  int32_t *d_out_var_idx;
  reslim::TrainModel train;
  std::vector<void *> allocs;                // everything to hipFree
  std::string err;
  // optional per-launch timing (reslim_profile_*): events are created up front
  bool prof_on = false;
  std::vector<hipEvent_t> prof_ev;           // 2 per record slot
  struct ProfRec { const char *name; double flop, bytes; };
  std::vector<ProfRec> prof_rec;             // records of the launches since the last reset
};

namespace reslim {

int set_error(reslim_ctx *ctx, int code, const std::string &msg);
void set_thread_error(const std::string &msg);

inline size_t act_size(const reslim_ctx *c) { return c->cfg.dtype == RESLIM_BF16 ? 2 : 4; }
inline size_t align256(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

// Which token rows attend to each other: by default the context's tile table applied
// to every sample; the compression module supplies one entry per sample of a batch
// that is then treated as a single "sample" of n_h rows.
struct SeqGeom {
  const tile_desc *d_tiles;        // device [T]: tok_off, n_tok used
  const int32_t *d_tile_of_tok;    // device [n_h]
  int T;
  int64_t n_h;
  int max_n_tok;
  double pairs;                    // sum over entries of n_tok^2 (flop accounting)
  double pairs_owned;              // sum of (owned tokens) * n_tok: the pairs of a stitched attention launch
};
SeqGeom ctx_geom(const reslim_ctx *c);

// Workspace carve-up used by block / embed / head / forward.
struct Workspace {
  float *X;        // [M, D] residual stream (forward only)
  void *A;         // act [M, D]
  void *big;       // act [M, max(3D, R)] or head staging
  float *Xc;       // [batch * N, D] residual stream of the patches alone (last block of a forward with halos), else null
  size_t total;
};
// The last block of a whole forward feeds only the head, which reads the rows their tiles own: after
// that block's attention (where halo tokens still serve as keys and values) every per-token step
// runs on those rows only.  Same arithmetic per kept row, so the output does not change.
bool last_block_on_patches(const reslim_ctx *c);
Workspace plan_workspace(const reslim_ctx *c, int batch, void *base);
// one transformer block on X [batch * geom.n_h, D] in place (geom == nullptr: the context's tiles)
// z_first: the embedding in patch order [batch * N, D] when X does not hold the stream yet (the
// first block of a whole forward; bf16 path, the context's own tiles)
int block_impl(reslim_ctx *c, const char *fn, int layer, float *X, int batch, const Workspace &w, hipStream_t st,
               const SeqGeom *geom = nullptr, const float *z_first = nullptr);
int embed_full_impl(reslim_ctx *c, const char *fn, const float *x, int batch, const Workspace &w, hipStream_t st,
                    float *dst = nullptr);

// ---- kernels (host launchers; all enqueue on `st` and return hipError_t) ------
enum Epilogue {
  EPI_BIAS_ACT = 0,       // out(act)  = acc + bias
  EPI_BIAS_GELU_ACT = 1,  // out(act)  = gelu(acc + bias)
  EPI_BIAS_RESADD_F32 = 2,// out(f32) += acc + bias
  EPI_BIAS_TAB_F32 = 3,   // out(f32)  = acc + tab[m % tab_rows, n]   (bias folded in tab)
  EPI_BIAS_F32 = 4,       // out(f32)  = acc + bias
  EPI_BIAS_QSCALE_ACT = 5,// out(act)  = (acc + bias) * (n < qcols ? qscale : 1)   (QKV with pre-scaled q)
  // training side
  EPI_BIAS_ACT_GELU2 = 6, // out(act)  = acc + bias;  out2(act) = gelu(acc + bias)    (FC1 keeping both)
  EPI_BIAS_RES_F32 = 8    // out(f32)  = res[m, n] + acc + bias                       (skip connection from another buffer)
};
// C[M, N] (+)= A[M, K] * W[N, K]^T ; A, W act type (bf16 -> MFMA path, float -> fp32 path)
// Row map for the skip input of EPI_BIAS_RES_F32 (bf16 path): output row b*rows_out + r adds row
// b*rows_in + map[r] of aux (e.g. the tile-major row that holds patch r).
struct ResRowMap { const int32_t *map; int rows_out; int64_t rows_in; };
hipError_t launch_gemm(int dtype, Epilogue epi, const void *A, const void *W, const float *bias,
                       void *out, int ldo, const float *tab, int tab_rows, int M, int N, int K,
                       hipStream_t st, float qscale = 1.0f, int qcols = 0, const void *aux = nullptr, void *out2 = nullptr,
                       const ResRowMap *res_map = nullptr);
// aux: EPI_BIAS_RES_F32: float skip input, [M, ldo] or the rows res_map names.  out2: EPI_BIAS_ACT_GELU2: act [M, ldo].
hipError_t gemm_init();

hipError_t launch_layernorm(int dtype, const float *x, const int32_t *row_src, int rows_per_sample_out,
                            int64_t rows_per_sample_in, const float *g, const float *b, void *out,
                            int64_t rows_out, int D, hipStream_t st);
hipError_t launch_gather_rows(const float *z, const int32_t *gather, float *X, int batch, int64_t n_h,
                              int N, int D, hipStream_t st);
hipError_t launch_embed_agg(const reslim_ctx *c, const float *x, void *o, int batch, hipStream_t st);
// q_prescaled: q already carries the factor log2(e)/sqrt(dh) (bf16 path only)
// stitched: out is [batch, N, D] in patch order, written by the owning tile's queries only (bf16
// path, the context's own tiling, no lse)
hipError_t launch_tiles_attention(const reslim_ctx *c, const void *qkv, void *out, int batch, bool q_prescaled,
                                  hipStream_t st, float *lse = nullptr,
                                  const SeqGeom *geom = nullptr, bool stitched = false);
bool attention_accepts_prescaled_q();
// gradient of tile attention: d_qkv from qkv, the forward's out and lse, and d_out; ws as sized below
hipError_t launch_tiles_attention_bwd(const reslim_ctx *c, const void *qkv, const void *out, const float *lse,
                                      const void *dout, void *dqkv, int batch, void *ws, bool q_prescaled,
                                      hipStream_t st, const SeqGeom *geom = nullptr);
size_t tiles_attention_bwd_ws_bytes(const reslim_ctx *c, int batch, const SeqGeom *geom = nullptr);
hipError_t attention_bwd_init();
// ---- training-side kernels
hipError_t wgrad_init();
size_t wgrad_ws_bytes(int dtype, int M, int N, int K);
// dW[N, K] (fp32) = dY[M, N]^T X[M, K]; ws >= wgrad_ws_bytes; zeros: >= 16 zero bytes on the device
hipError_t launch_wgrad(int dtype, const void *dy, const void *x, float *dw, int M, int N, int K, void *ws,
                        const void *zeros, hipStream_t st);
int layernorm_bwd_slabs(int64_t rows);   // partial rows (of 2 D floats) launch_layernorm_bwd writes
hipError_t launch_layernorm_bwd(int dtype, const float *x, const void *dy, const float *g, const float *res,
                                float *dx_out, void *act_out, float *partial, float *dgamma, float *dbeta,
                                int64_t rows, int D, hipStream_t st);
hipError_t launch_gelu(int dtype, bool bwd, const void *h, const void *dy, void *out, int64_t n, hipStream_t st);
hipError_t launch_to_act(int dtype, const float *src, void *dst, int64_t n, hipStream_t st);
int colsum_slabs(int64_t rows);          // partial rows (of N floats) launch_colsum writes
hipError_t launch_colsum(int dtype, const void *a, float *partial, float *out, int64_t rows, int N, hipStream_t st);
hipError_t launch_transpose(int dtype, const void *src, void *dst, int R, int C, hipStream_t st);
// every element of `count` (<= 12) fp32 tensors times inv_scale; *flag = 1 when any is not finite
hipError_t launch_unscale_check(float *const *ptrs, const int64_t *sizes, int count, float inv_scale, int32_t *flag,
                                hipStream_t st);
hipError_t attention_init();
hipError_t elementwise_init();
hipError_t launch_copy_probe(const void *src, void *dst, size_t bytes, hipStream_t st);
hipError_t launch_residual_unpatchify(const reslim_ctx *c, const float *x, const void *P, int p_is_act,
                                      float *y, int batch, hipStream_t st);

// ---- shared by the files that hold entry points -------------------------------
int check_common(reslim_ctx *c, const char *fn, int batch, const void *ws, size_t ws_bytes, bool need_ws);
int hip_fail(reslim_ctx *c, const char *fn, const char *what, hipError_t e);

}  // namespace reslim

// Leaf table of the compression module on the device (one per batch of samples).
struct reslim_asc_plan {
  reslim_ctx *ctx = nullptr;
  int batch = 0;
  int64_t L = 0;                         // leaves of the whole batch
  std::vector<tile_desc> seq;            // one entry per sample: tok_off, n_tok
  reslim::SeqGeom geom{};
  tile_desc *d_seq = nullptr;            // [batch]
  int32_t *d_seq_of_leaf = nullptr;      // [L]
  int32_t *d_leaf = nullptr;             // [L][4]: first patch row (b*N + y0*Wp + x0), side, unused, unused
  int32_t *d_patch_leaf = nullptr;       // [batch * N]
  // contexts with tiles: a patch lies in one leaf of every box that holds it (its tile's and the neighbours' halos)
  int32_t *d_cover_off = nullptr;        // [batch * N + 1]
  int32_t *d_cover_leaf = nullptr;       // [cover_off[batch * N]] leaves of each patch, increasing
};


#define RESLIM_TRY(what, expr)                                   \
  do {                                                           \
    hipError_t e_ = (expr);                                      \
    if (e_ != hipSuccess) return hip_fail(c, fn, what, e_);      \
  } while (0)

// A launch with its algorithmic work attached; when profiling is on the launch is
// bracketed by two pre-created events on the same stream.
#define RESLIM_LAUNCH(label, flop_, bytes_, expr)                                      \
  do {                                                                                 \
    const size_t slot_ = c->prof_rec.size();                                           \
    const bool p_ = c->prof_on && 2 * slot_ + 1 < c->prof_ev.size();                   \
    if (p_) RESLIM_TRY("event", hipEventRecord(c->prof_ev[2 * slot_], st));            \
    RESLIM_TRY(label, expr);                                                           \
    if (p_) {                                                                          \
      RESLIM_TRY("event", hipEventRecord(c->prof_ev[2 * slot_ + 1], st));              \
      c->prof_rec.push_back({label, static_cast<double>(flop_), static_cast<double>(bytes_)}); \
    }                                                                                  \
  } while (0)

/* reslim.h -- C ABI of the Reslim ViT forward under TILES for one MI355X (gfx950).
 *
 * The operations are those of ORBIT-2 (arXiv 2505.04802): Sec. 4.1 "Reslim
 * Architecture" (per-variable tokenisation, cross-attention variable aggregation,
 * resolution embedding, transformer blocks, decoder, residual convolutional path)
 * and Sec. 4.2 "TILES" (partition into tiles, halo padding, tile-local
 * self-attention, discard halos and stitch).
 *
 * Conventions
 *  - Every function returns RESLIM_OK (0) or a negative error code; none throws,
 *    aborts or prints.  reslim_last_error() gives the text of the last failure.
 *  - "dev" pointers are device (HBM) addresses on the current HIP device, "host"
 *    pointers are ordinary host memory.  The caller owns every buffer it passes
 *    (input, output, workspace) and the stream; the library owns only reslim_ctx
 *    (device copies of the weights, the tile table and the index lists).
 *  - After reslim_create() no entry point allocates or synchronises: all work is
 *    enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = default
 *    stream).  A launch failure is reported as RESLIM_EHIP.
 *  - Tensors are row-major.  Fields are [batch, variable, latitude, longitude].
 *  - Activation element type ("act"): float when cfg.dtype == RESLIM_F32,
 *    bfloat16 (upper 16 bits of an IEEE float) when cfg.dtype == RESLIM_BF16.
 *    The residual token stream, the input field and the output field are float
 *    in both modes.
 *  - Tile-major token order: tokens of tile 0, then tile 1, ... (tiles row-major
 *    over the tile grid); inside a tile row-major over its haloed box.  n_h is the
 *    number of such tokens per sample (halo tokens are duplicated).
 */
#ifndef RESLIM_H
#define RESLIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  RESLIM_OK = 0,
  RESLIM_EINVAL = -1,     /* null pointer, bad enum, bad layer index             */
  RESLIM_ESHAPE = -2,     /* sizes that do not divide / do not fit the kernels   */
  RESLIM_ENOMEM = -3,     /* host or device allocation failed (create only)      */
  RESLIM_EHIP = -4,       /* a HIP call or kernel launch failed                  */
  RESLIM_EWORKSPACE = -5  /* workspace missing, misaligned (256 B) or too small  */
};

enum { RESLIM_F32 = 0, RESLIM_BF16 = 1 };

/* Problem description.  Plain data, caller-owned, copied by reslim_create. */
typedef struct {
  int32_t in_vars;    /* V: variables of the coarse input                        */
  int32_t out_vars;   /* C: variables of the fine output (C <= V)                */
  int32_t H, W;       /* coarse grid: latitude rows, longitude columns           */
  int32_t scale;      /* s: fine grid is (s*H) x (s*W)                           */
  int32_t patch;      /* p: patch edge in coarse pixels (the paper uses 2)       */
  int32_t embed_dim;  /* D                                                       */
  int32_t heads;      /* attention heads; head dim dh = D / heads                */
  int32_t mlp_ratio;  /* r: hidden width of the feed-forward sub-layer is r*D    */
  int32_t depth;      /* L: transformer blocks                                   */
  int32_t tiles_y, tiles_x; /* tile grid (Sec. 4.2)                              */
  int32_t halo;       /* halo width in patches, clipped at the domain edge       */
  int32_t res_idx;    /* row of the resolution-embedding table to add (Sec. 4.1) */
  int32_t n_res;      /* rows of that table                                      */
  int32_t dtype;      /* RESLIM_F32 (debug path) or RESLIM_BF16                  */
} reslim_config;

/* Parameters, all HOST pointers to float (out_var_idx: int32), row-major, read
 * during reslim_create only.  Linear maps are [out_features, in_features].
 * p2 = p*p, R = r*D, N = (H/p)*(W/p), O = C*(p*s)*(p*s). */
typedef struct {
  const float *w_pe;      /* [V, D, p2]  patch embedding per variable            */
  const float *b_pe;      /* [V, D]                                              */
  const float *var_emb;   /* [V, D]      added to every token of variable v      */
  const float *agg_q0;    /* [D]         the learned query of the aggregation    */
  const float *agg_wq, *agg_bq;   /* [D, D], [D]                                 */
  const float *agg_wk, *agg_bk;
  const float *agg_wv, *agg_bv;
  const float *agg_wo, *agg_bo;
  const float *pos_emb;   /* [N, D]      indexed by global patch position        */
  const float *res_emb;   /* [n_res, D]                                          */
  const float *ln1_g, *ln1_b;     /* [L, D]                                      */
  const float *w_qkv, *b_qkv;     /* [L, 3D, D], [L, 3D]  rows ordered q | k | v */
  const float *w_proj, *b_proj;   /* [L, D, D], [L, D]                           */
  const float *ln2_g, *ln2_b;     /* [L, D]                                      */
  const float *w_fc1, *b_fc1;     /* [L, R, D], [L, R]                           */
  const float *w_fc2, *b_fc2;     /* [L, D, R], [L, D]                           */
  const float *lnf_g, *lnf_b;     /* [D]        final LayerNorm                  */
  const float *w_head, *b_head;   /* [O, D], [O]  O index = (c*ps + i)*ps + j    */
  const float *w_res, *b_res;     /* [C, C, 3, 3], [C]  residual-path convolution */
  const int32_t *out_var_idx;     /* [C]  input variable feeding output c        */
} reslim_weights;

/* One tile of the patch grid, patch units, half-open boxes (Sec. 4.2). */
typedef struct {
  int32_t y0, y1, x0, x1;   /* interior: the part of the output this tile owns    */
  int32_t Y0, Y1, X0, X1;   /* interior widened by the halo, clipped to the grid  */
  int64_t tok_off;          /* first tile-major token index of this tile          */
  int32_t n_tok;            /* (Y1-Y0)*(X1-X0)                                    */
  int32_t _pad;
} tile_desc;

typedef struct reslim_ctx reslim_ctx;

/* Sec. 4.2, partition + halo + stitch indices.  HOST function, integers only, no
 * HIP call.  Cuts a patch grid Hp x Wp into Ty x Tx tiles with a balanced split
 * (tile row i covers patch rows [floor(i*Hp/Ty), floor((i+1)*Hp/Ty))), widens
 * each by `halo` patches and clips at the domain edge.
 *   tiles        host [Ty*Tx] out
 *   gather_idx   host [n_h] out or NULL: global patch id (y*Wp+x) of every
 *                tile-major token
 *   interior_src host [Hp*Wp] out or NULL: tile-major index of global patch g in
 *                the tile whose interior holds it (the stitch map)
 *   n_h_out      host out or NULL: total tile-major tokens
 * Call once with gather_idx == NULL to learn n_h.  RESLIM_ESHAPE if Ty > Hp,
 * Tx > Wp, any size < 1 or halo < 0. */
int tiles_partition(int32_t Hp, int32_t Wp, int32_t Ty, int32_t Tx, int32_t halo,
                    tile_desc *tiles, int32_t *gather_idx, int32_t *interior_src,
                    int64_t *n_h_out);

/* Validates cfg, partitions, copies the weights to the device (rounded to
 * bfloat16 for the MFMA operands in RESLIM_BF16 mode) and folds the per-variable
 * tokenisation into the aggregation's key/value maps (Sec. 4.1; exact, since no
 * non-linearity separates them).  Synchronises the device once.  *out is NULL on
 * failure.  RESLIM_BF16 needs D % 64 == 0, dh in {64, 128, 256} and
 * out_vars * (patch * scale)^2 % 8 == 0. */
int reslim_create(const reslim_config *cfg, const reslim_weights *w, reslim_ctx **out);
void reslim_destroy(reslim_ctx *ctx);

/* Text of the most recent error of `ctx`, or of the calling thread's last failed
 * reslim_create/tiles_partition when ctx is NULL.  Owned by the library. */
const char *reslim_last_error(const reslim_ctx *ctx);

/* n_h of the context's tiling (tile-major tokens per sample). */
int reslim_tokens_per_sample(const reslim_ctx *ctx, int64_t *n_h_out);

/* Bytes of 256-byte-aligned device workspace that reslim_forward (the largest
 * user) needs for `batch` samples; valid for every other entry point too. */
int reslim_workspace_bytes(const reslim_ctx *ctx, int32_t batch, size_t *out);

/* Sec. 4.1 front end + Sec. 4.2 gather: tokenise each variable, aggregate the
 * variables by cross-attention, add position and resolution embeddings, copy the
 * tokens into tile-major order with halo duplication.
 *   x      dev float [batch, V, H, W]
 *   tokens dev float [batch, n_h, D] out */
int reslim_embed_fwd(reslim_ctx *ctx, const float *x, float *tokens, int32_t batch,
                     void *workspace, size_t ws_bytes, void *hip_stream);

/* Sec. 4.2 tile-local multi-head self-attention: for every sample, tile and head,
 * softmax(Q K^T / sqrt(dh)) V over the n_t tokens of that tile only (halo tokens
 * are ordinary queries and keys).
 *   qkv dev act [batch, n_h, 3, heads, dh]
 *   out dev act [batch, n_h, heads*dh]     (must not alias qkv) */
int tiles_attention_fwd(reslim_ctx *ctx, const void *qkv, void *out, int32_t batch,
                        void *hip_stream);

/* The same attention, also returning what its gradient needs (training of the
 * model of Sec. 4.1): lse[b, g, i] = log sum_j exp(q_i . k_j / sqrt(dh)) over the keys
 * of query i's tile, natural logarithm.
 *   lse dev float [batch, heads, n_h] out */
int tiles_attention_fwd_lse(reslim_ctx *ctx, const void *qkv, void *out, float *lse, int32_t batch,
                            void *hip_stream);

/* Gradient of the tile-local attention of Sec. 4.2 (the paper trains the model, Sec. 5;
 * it prints no formula, this is the chain rule through softmax(Q K^T / sqrt(dh)) V
 * within each tile; tiles do not interact, so neither do their gradients):
 *   dV = P^T dO, dP = dO V^T, dS = P o (dP - rowsum(dO o O)),
 *   dQ = dS K / sqrt(dh), dK = dS^T Q / sqrt(dh),
 * with P recomputed from q, k and lse.
 *   qkv   dev act   [batch, n_h, 3, heads, dh]   the forward's input
 *   out   dev act   [batch, n_h, heads*dh]       the forward's output
 *   lse   dev float [batch, heads, n_h]          from tiles_attention_fwd_lse
 *   d_out dev act   [batch, n_h, heads*dh]       gradient of the loss w.r.t. out
 *   d_qkv dev act   [batch, n_h, 3, heads, dh]   out: gradient w.r.t. qkv, every element
 *                                                written; must not alias an input
 *   workspace dev, 256-byte aligned, >= tiles_attention_bwd_workspace_bytes(), caller-owned
 * Work is enqueued on hip_stream; no allocation, no synchronisation; deterministic.
 * Errors: RESLIM_EINVAL (null), RESLIM_ESHAPE (batch), RESLIM_EWORKSPACE, RESLIM_EHIP. */
int tiles_attention_bwd_workspace_bytes(const reslim_ctx *ctx, int32_t batch, size_t *out);
int tiles_attention_bwd(reslim_ctx *ctx, const void *qkv, const void *out, const float *lse,
                        const void *d_out, void *d_qkv, int32_t batch, void *workspace,
                        size_t ws_bytes, void *hip_stream);

/* ---- Training of a block (the paper trains the model, Sec. 5; it prints no gradient
 * formulas: everything below is the chain rule through the forward operations of Sec. 3 /
 * 4.1 / 4.2, tile by tile).  Activations ("act") are float or bfloat16 as cfg.dtype says;
 * parameter gradients are fp32, WRITTEN (not accumulated) by each call, summed over all
 * tokens of all tiles and samples in a fixed order (deterministic).  All pointers are device
 * pointers unless stated; work is enqueued on hip_stream; no allocation, no synchronisation
 * except in reslim_train_prepare. ---- */

/* Allocates and fills the [in, out] copies of the block weights that the input-gradient
 * GEMMs read (doubles the block weights' memory).  Call once after reslim_create and before
 * any other training entry point; synchronises the device.  Idempotent. */
int reslim_train_prepare(reslim_ctx *ctx);

/* Gradient of the per-token LayerNorm y = (x - mean) / sqrt(var + 1e-5) * gamma + beta over
 * rows of D = embed_dim elements:  dx = res + (g - mean(g) - xh mean(g xh)) / sigma with
 * g = gamma dy;  dgamma = sum_rows dy xh;  dbeta = sum_rows dy.
 *   x float [rows, D]; dy act [rows, D]; gamma float [D]; res float [rows, D] or NULL;
 *   dx float [rows, D] out; dgamma, dbeta float [D] out;
 *   workspace: 256-byte aligned, >= min(1024, ceil(rows / 4)) * 2 * D floats. */
int reslim_layernorm_bwd(reslim_ctx *ctx, const float *x, const void *dy, const float *gamma,
                         const float *res, float *dx, float *dgamma, float *dbeta, int64_t rows,
                         void *workspace, size_t ws_bytes, void *hip_stream);

/* Gradient of one linear layer y = x W^T + b of block `layer`; which = 0: qkv (D -> 3D),
 * 1: proj (D -> D), 2: fc1 (D -> R), 3: fc2 (R -> D), R = mlp_ratio * D:
 *   dx = dy W (skipped when dx is NULL),  dW = dy^T x,  db = column sums of dy.
 *   x act [rows, in]; dy act [rows, out]; dx act [rows, in] out; dw float [out, in] out;
 *   db float [out] out; workspace >= reslim_linear_bwd_workspace_bytes(). */
int reslim_linear_bwd_workspace_bytes(const reslim_ctx *ctx, int32_t which, int32_t rows, size_t *out);
int reslim_linear_bwd(reslim_ctx *ctx, int32_t layer, int32_t which, const void *x, const void *dy,
                      void *dx, float *dw, float *db, int32_t rows, void *workspace, size_t ws_bytes,
                      void *hip_stream);

/* Gradients of the twelve parameter tensors of one block, device fp32, shapes as in
 * reslim_weights without the leading depth axis. */
typedef struct {
  float *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_proj, *b_proj;
  float *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} reslim_block_grads;

/* Sizes of the per-block buffer of saved activations (what reslim_block_fwd_train keeps for
 * reslim_block_bwd: both LayerNorm outputs, qkv, the attention output and its log-sum-exp,
 * the stream after the attention half, the feed-forward hidden layer before and after GELU)
 * and of the scratch either call needs.  Either pointer may be NULL. */
int reslim_block_train_bytes(const reslim_ctx *ctx, int32_t batch, size_t *saved_bytes, size_t *ws_bytes);

/* reslim_block_fwd that keeps its intermediates: x_out = block(x_in), both float
 * [batch, n_h, D], not aliased.  saved / workspace: 256-byte aligned, caller-owned. */
int reslim_block_fwd_train(reslim_ctx *ctx, int32_t layer, const float *x_in, float *x_out, void *saved,
                           size_t saved_bytes, int32_t batch, void *workspace, size_t ws_bytes,
                           void *hip_stream);

/* Gradient of that block: from d_x_out (gradient of the loss w.r.t. x_out), the block's input
 * x_in and the saved buffer of the matching reslim_block_fwd_train call it writes d_x_in
 * (float [batch, n_h, D], not aliased with d_x_out) and all twelve parameter
 * gradients.  Errors: RESLIM_EINVAL (null, layer, prepare not called), RESLIM_ESHAPE,
 * RESLIM_EWORKSPACE, RESLIM_EHIP. */
int reslim_block_bwd(reslim_ctx *ctx, int32_t layer, const float *x_in, const void *saved,
                     size_t saved_bytes, const float *d_x_out, float *d_x_in,
                     const reslim_block_grads *grads, int32_t batch, void *workspace, size_t ws_bytes,
                     void *hip_stream);

/* Dynamic gradient scaling (Sec. 4.4 "Mixed Precision": gradients are taken of a loss multiplied by
 * a scale S so that small ones survive bfloat16, the scaling is reversed at the parameter update, and
 * S adapts; the paper names PyTorch's scheme).  The caller multiplies the gradient it feeds into the
 * backward by S.
 * reslim_block_grads_unscale: every element of the twelve gradients (device fp32, shapes of
 *   reslim_block_grads) times inv_scale = 1/S, in place; *found_inf (device int32) is set to 1 when
 *   any element is then not finite and is otherwise left alone: clear it before the first call of a
 *   step.  Enqueued on hip_stream.
 * reslim_grad_scale_update: HOST arithmetic, the schedule of S: a step with found_inf != 0
 *   multiplies *scale by backoff_factor (0 < . <= 1) and clears *growth_tracker; growth_interval
 *   clean steps in a row multiply it by growth_factor (>= 1).  PyTorch's defaults: 2, 0.5, 2000.
 * Errors: RESLIM_EINVAL (null pointer, non-positive or non-finite factor), RESLIM_EHIP. */
int reslim_block_grads_unscale(reslim_ctx *ctx, const reslim_block_grads *grads, float inv_scale,
                               int32_t *found_inf, void *hip_stream);
int reslim_grad_scale_update(float *scale, int32_t *growth_tracker, int32_t found_inf, float growth_factor,
                             float backoff_factor, int32_t growth_interval);

/* ---- Gradients of the whole model for one training step (the paper trains the model, Sec. 5,
 * with the loss of Sec. 4.1 and bfloat16 + gradient scaling, Sec. 4.4; it prints no gradient
 * formula: all of this is the chain rule through the forward operations).  Precision as for the
 * block gradient: gradients that feed a GEMM are rounded to the activation type, sums are fp32,
 * parameter gradients are fp32, WRITTEN (not accumulated), summed in a fixed order. ---- */

/* Device fp32 gradient buffers, one per parameter tensor, shapes as in reslim_weights (per-block
 * tensors stacked over depth; out_var_idx is a selection, not a parameter). */
typedef struct {
  float *w_pe, *b_pe, *var_emb, *agg_q0, *agg_wq, *agg_bq, *agg_wk, *agg_bk, *agg_wv, *agg_bv, *agg_wo, *agg_bo,
        *pos_emb, *res_emb;                                         /* front end */
  float *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_proj, *b_proj, *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;   /* blocks */
  float *lnf_g, *lnf_b, *w_head, *b_head, *w_res, *b_res;          /* back end */
} reslim_grads;

/* reslim_train_prepare plus what the two ends of the model need: device copies of the unfolded
 * front-end parameters (weights: HOST pointers as given to reslim_create, read during this call
 * only), [in, out] copies of the head's and the aggregation's output maps, and the list of
 * tile-major copies of every patch.  Allocates and synchronises; idempotent.  RESLIM_ESHAPE on the
 * bfloat16 path unless out_vars * (patch * scale)^2 is a multiple of 64. */
int reslim_train_prepare_model(reslim_ctx *ctx, const reslim_weights *weights);

/* Gradient of the loss of reslim_bayes_loss_fwd (its total) with respect to pred, times `upstream`
 * (the loss scale of Sec. 4.4, or 1):
 *   d_pred[b,k,r,c] = upstream * (2 lat_w[r] (pred - target) / n
 *                                 + 2 tv_weight / n * sum_{j in C(i)} b_ij sign(pred_i - pred_j)),
 * n = all pixel values; every ordered pair of the prior's double sum contains pixel i twice, hence
 * the factor 2; sign(0) = 0 (the subgradient taken where |.| has no derivative).
 * All pointers dev fp32, shapes as in reslim_bayes_loss_fwd; d_pred must not alias pred.
 * batch * vars <= 65535, Hf <= 65535.  Errors: RESLIM_EINVAL, RESLIM_EHIP. */
int reslim_bayes_loss_bwd(const float *pred, const float *target, const float *lat_w, int32_t batch, int32_t vars,
                          int32_t Hf, int32_t Wf, float tv_weight, float upstream, float *d_pred, void *hip_stream);

/* Back end backwards (reslim_head_fwd's gradient): from d_y (dev fp32 [batch, C, s*H, s*W]), the
 * field x and the stream `tokens` (dev fp32 [batch, n_h, D]) that went into reslim_head_fwd it writes
 * d_tokens (dev fp32 [batch, n_h, D]: the final LayerNorm's input gradient on interior tokens, zero on
 * halo copies, whose outputs Sec. 4.2 discards) and grads->lnf_g, lnf_b, w_head, b_head, w_res, b_res
 * (the other fields of grads are not touched).  workspace: 256-byte aligned, >=
 * reslim_head_bwd_workspace_bytes.  Needs reslim_train_prepare_model, scale >= 2. */
int reslim_head_bwd_workspace_bytes(const reslim_ctx *ctx, int32_t batch, size_t *out);
int reslim_head_bwd(reslim_ctx *ctx, const float *x, const float *tokens, const float *d_y, float *d_tokens,
                    const reslim_grads *grads, int32_t batch, void *workspace, size_t ws_bytes, void *hip_stream);

/* Front end backwards (reslim_embed_fwd's gradient): from d_tokens (dev fp32 [batch, n_h, D], the
 * gradient of the tile-major stream) and the field x it writes the fourteen front-end gradients of
 * grads (w_pe .. res_emb): a patch adds up the gradients of its halo copies; rows of res_emb the
 * forward did not read get zero; agg_bk gets what the arithmetic leaves of an exactly zero gradient
 * (a key bias shifts all variables' logits alike).  workspace >= reslim_embed_bwd_workspace_bytes. */
int reslim_embed_bwd_workspace_bytes(const reslim_ctx *ctx, int32_t batch, size_t *out);
int reslim_embed_bwd(reslim_ctx *ctx, const float *x, const float *d_tokens, const reslim_grads *grads, int32_t batch,
                     void *workspace, size_t ws_bytes, void *hip_stream);

/* One training step without the parameter update: forward keeping every block's intermediates,
 * loss, backward through the whole model.
 *   x dev fp32 [batch, V, H, W]; target dev fp32 [batch, C, s*H, s*W]; lat_w dev fp32 [s*H];
 *   y dev fp32 [batch, C, s*H, s*W] out (the prediction); loss3 dev, 3 doubles out (total, data,
 *   prior: unscaled); grads: all 32 gradients, multiplied by loss_scale (divide with
 *   reslim_grads_unscale); saved / workspace: 256-byte aligned, >= reslim_train_step_bytes.
 * Everything is enqueued on hip_stream; nothing is allocated or synchronised; deterministic.
 * Errors: RESLIM_EINVAL (null, prepare not called, bad scale), RESLIM_ESHAPE, RESLIM_EWORKSPACE, RESLIM_EHIP. */
int reslim_train_step_bytes(const reslim_ctx *ctx, int32_t batch, size_t *saved_bytes, size_t *ws_bytes);
int reslim_train_step_grads(reslim_ctx *ctx, const float *x, const float *target, const float *lat_w, float tv_weight,
                            float loss_scale, float *y, double *loss3, const reslim_grads *grads, int32_t batch,
                            void *saved, size_t saved_bytes, void *workspace, size_t ws_bytes, void *hip_stream);

/* reslim_block_grads_unscale for all 32 gradients of the model. */
int reslim_grads_unscale(reslim_ctx *ctx, const reslim_grads *grads, float inv_scale, int32_t *found_inf, void *hip_stream);

/* One pre-LayerNorm transformer block `layer` (0-based) on the tile-major stream:
 * X += proj(tile_attention(qkv(LN1(X)))); X += fc2(gelu(fc1(LN2(X)))).
 *   x_inout dev float [batch, n_h, D], updated in place */
int reslim_block_fwd(reslim_ctx *ctx, int32_t layer, float *x_inout, int32_t batch,
                     void *workspace, size_t ws_bytes, void *hip_stream);

/* Back end: final LayerNorm, halo discarded (interior tokens only), linear
 * projection to fine pixels, un-patchify and stitch, plus the residual path
 * (bilinear upsampling by s of the selected input variables and one 3x3
 * convolution, evaluated per tile on its haloed box) added to it.
 *   x      dev float [batch, V, H, W]        the same field given to embed
 *   tokens dev float [batch, n_h, D]
 *   y      dev float [batch, C, s*H, s*W] out */
int reslim_head_fwd(reslim_ctx *ctx, const float *x, const float *tokens, float *y,
                    int32_t batch, void *workspace, size_t ws_bytes, void *hip_stream);

/* The whole forward: embed, `depth` blocks, head.  Coarse multi-variable grid in,
 * fine grid out.  In bf16 mode with halo tokens the last block keeps only what
 * the head reads: its attention computes the queries their tiles own (halo
 * tokens remain keys and values), and its projection and MLP run on those rows
 * alone; per kept row the arithmetic is that of reslim_block_fwd, so y equals
 * the chained entry points' bit for bit. */
int reslim_forward(reslim_ctx *ctx, const float *x, float *y, int32_t batch,
                   void *workspace, size_t ws_bytes, void *hip_stream);

/* Work of one reslim_forward for `batch` samples, for reporting: flop of the
 * block GEMMs, of tile attention (4*queries*n_t*D per tile, block and sample;
 * queries = n_t except in a last block that keeps the owned rows only) and of
 * the head GEMM.  Any pointer may be NULL. */
int reslim_flop_counts(const reslim_ctx *ctx, int32_t batch, double *gemm_flop,
                       double *attn_flop, double *head_flop);

/* Per-launch timing for benchmarks.  reslim_profile_enable(ctx, n) creates 2*n HIP
 * events (the only allocation; call it outside timed regions; n = 0 switches
 * profiling off and frees them).  While on, every kernel launch of the entry
 * points is bracketed by two event records on the caller's stream, up to n launches
 * since the last reslim_profile_reset().  reslim_profile_read() waits for the
 * recorded events and returns, per launch in issue order, a static label, the
 * elapsed milliseconds and the launch's ALGORITHMIC work: flop (2 per
 * multiply-add of the contraction, 0 for copies) and bytes (each operand read once,
 * each result written once).  With out == NULL only the count is returned. */
typedef struct {
  const char *name;
  float ms;
  double flop, bytes;
} reslim_profile_record;
int reslim_profile_enable(reslim_ctx *ctx, int32_t max_records);
int reslim_profile_reset(reslim_ctx *ctx);
int reslim_profile_read(reslim_ctx *ctx, reslim_profile_record *out, int32_t max_out, int32_t *n_out);

/* Bayesian training loss, forward value only (Sec. 4.1, "Bayesian Training Loss":
 * latitude-weighted squared error plus a total-variation prior over each pixel's
 * spatial neighbours, the paper's one equation).
 *   out3[0] = out3[1] + out3[2]
 *   out3[1] = mean over (b, k, r, c) of lat_w[r] * (target - pred)^2
 *   out3[2] = tv_weight * mean over (b, k, i) of sum_{j in C(i)} b_ij |pred_i - pred_j|
 * C(i) = the 8 nearest pixels inside the Hf x Wf grid (no wrap-around), b_ij =
 * (1 / Euclidean pixel distance) / (4 + 4 / sqrt 2); every ordered pair counts.
 * pred, target: dev fp32 [batch, vars, Hf, Wf], row-major; lat_w: dev fp32 [Hf]
 * (the paper's matrix D: the caller supplies cos(latitude) of each row, normalised as
 * it sees fit); out3: dev, 3 doubles, 8-byte aligned, written by the last kernel
 * enqueued; workspace: dev, 8-byte aligned, at least the size reported by
 * reslim_bayes_loss_workspace_bytes, caller-owned.  No context is needed.  Work is
 * enqueued on hip_stream, nothing is synchronised.  batch * vars <= 65535.
 * Errors: RESLIM_EINVAL (null pointer, non-positive size, alignment),
 * RESLIM_EWORKSPACE (too small), RESLIM_EHIP.  The result is deterministic. */
int reslim_bayes_loss_workspace_bytes(int32_t batch, int32_t vars, int32_t Hf, int32_t Wf, size_t *out);
int reslim_bayes_loss_fwd(const float *pred, const float *target, const float *lat_w, int32_t batch,
                          int32_t vars, int32_t Hf, int32_t Wf, float tv_weight, double *out3,
                          void *workspace, size_t ws_bytes, void *hip_stream);

/* The same loss value for callers that cannot allocate device memory or must not be
 * handed a workspace: code under HIP graph capture, tight serving or training loops,
 * harnesses that forbid hipMalloc.  Same arguments, result and errors as
 * reslim_bayes_loss_fwd minus the workspace: the per-work-group partial sums live in a
 * fixed 4 MiB array inside the library's device code (one copy per GPU, held until the
 * process ends; its address is looked up on the first call on each device, with that
 * device current).  The call allocates nothing and synchronises nothing.
 * Limit: batch * vars * ceil(Hf / 8) * ceil(Wf / 1024) <= 262144 work-groups
 * (reslim_bayes_loss_static_max_groups reports the number; the 16 x 5760 x 11520 output
 * of the largest benchmark grid needs 138240); beyond it RESLIM_EWORKSPACE, nothing
 * enqueued.  All calls on one GPU share the array: two calls whose kernels overlap on that
 * GPU (different streams, or replays of two captured graphs) race; calls on one stream are
 * safe, each call writes every partial it later reads, so nothing needs clearing. */
int reslim_bayes_loss_static_max_groups(int64_t *out);
int reslim_bayes_loss_fwd_static(const float *pred, const float *target, const float *lat_w, int32_t batch,
                                 int32_t vars, int32_t Hf, int32_t Wf, float tv_weight, double *out3,
                                 void *hip_stream);

/* ---- Adaptive spatial compression (Sec. 4.1, "Adaptive Spatial Compression").
 * The paper maps the aggregated embedding to image space, runs Canny edge
 * detection on it, splits quadrants of a quad-tree while their edge density is
 * above a threshold and a minimum patch size is not reached, runs the ViT blocks on
 * one token per leaf and decompresses before the decoder; its Sec. 4.3 has the CPUs
 * build the quad-trees while the GPUs compute.  Here: reslim_asc_image (device)
 * gives the image, reslim_asc_build (host) the leaf table, reslim_asc_plan_create
 * checks and uploads it, reslim_asc_forward runs the model on the leaves.  The
 * paper gives no thresholds, filter sizes or merge rule; the readings are stated at
 * each function.  With a tiled context every (sample, tile) pair has its own leaf set
 * (reslim_asc_build_tiles); a patch then lies in one leaf of every box that holds it and
 * is decompressed from the leaf of the tile that owns it, which the gradients of the two
 * maps (reslim_asc_compress_bwd, reslim_asc_decompress_bwd) follow. */
typedef struct reslim_asc_plan reslim_asc_plan;

/* HOST function, no HIP call.  images: host fp32 [batch, H, W].  Per sample:
 *  1. 8-bit image q = clamp(floor((v - min) * (255 / (max - min)) + 0.5), 0, 255),
 *     float32 operations in exactly this order; a constant field gives q = 0;
 *  2. Canny in integers: 5x5 smoothing mask {2 4 5 4 2; 4 9 12 9 4; 5 12 15 12 5; ...}
 *     / 159 with rounding, 3x3 Sobel derivatives, magnitude |gx| + |gy|, direction
 *     in four sectors split at 22.5 and 67.5 degrees, a pixel survives if its
 *     magnitude is greater than its neighbour's on the up/left side along the
 *     gradient and not smaller than the other one's, strong = magnitude >
 *     canny_high, weak = magnitude > canny_low, edges = strong pixels plus the weak
 *     ones connected to them (8-neighbourhood); borders replicated for the filters,
 *     magnitude 0 outside for the suppression;
 *  3. quad-tree over the patch grid (H/patch x W/patch): roots are max_leaf x
 *     max_leaf patches in row-major order (the grid is thought padded to a multiple
 *     of max_leaf; a node wholly in the padding is dropped, one that sticks out of
 *     the grid always splits); a node inside the grid of side s splits into NW, NE,
 *     SW, SE iff s > min_leaf and float(edge pixels inside) > tau *
 *     float((s*patch)^2); leaves are listed depth-first, sample after sample.
 * Outputs (host, caller-owned, room for batch * (H/patch) * (W/patch) entries each,
 * sample_off batch + 1): leaf_y0, leaf_x0, leaf_s in patch units; sample_off[b] =
 * first leaf of sample b; patch_leaf[b, y*Wp + x] = batch-wide index of the leaf
 * holding that patch; *n_leaves_out = total leaves.
 * Errors: RESLIM_EINVAL (null pointer, negative or inverted thresholds, tau negative
 * or not finite, a pixel that is not finite), RESLIM_ESHAPE (leaf sizes not powers
 * of two, min_leaf > max_leaf, H or W not divisible by patch). */
int reslim_asc_build(const float *images, int32_t batch, int32_t H, int32_t W, int32_t patch, int32_t max_leaf,
                     int32_t min_leaf, int32_t canny_low, int32_t canny_high, float tau, int32_t *leaf_y0,
                     int32_t *leaf_x0, int32_t *leaf_s, int32_t *sample_off, int32_t *patch_leaf,
                     int64_t *n_leaves_out);

/* HOST function, no HIP call: compression combined with TILES (Sec. 4.2; the paper's
 * Table 3 runs both together and does not say how they combine).  Reading: every
 * (sample, tile) pair is compressed on its own -- steps 1-3 above applied to the tile's
 * haloed box cut out of images[b] (the 8-bit range, the filters' replicated borders and
 * the quad-tree roots all belong to the box; a box that is no multiple of max_leaf is a
 * ragged grid), so no leaf straddles a box edge and halo patches are compressed with
 * their box.  tiles_y, tiles_x, halo as in reslim_config (tiles_partition gives the
 * boxes).  Outputs, room for batch * n_h entries each (n_h = tile-major tokens per
 * sample): leaf_y0, leaf_x0 in GRID patch coordinates, leaf_s; seq_off [batch * T + 1]:
 * first leaf of sequence b * T + t; patch_leaf [batch, Hp * Wp]: for each patch the leaf
 * that holds it in the tile whose interior owns it (what decompression reads).
 * With one tile the result is reslim_asc_build's.  Errors as reslim_asc_build, plus
 * RESLIM_ESHAPE for a tile grid tiles_partition refuses. */
int reslim_asc_build_tiles(const float *images, int32_t batch, int32_t H, int32_t W, int32_t patch, int32_t tiles_y,
                           int32_t tiles_x, int32_t halo, int32_t max_leaf, int32_t min_leaf, int32_t canny_low,
                           int32_t canny_high, float tau, int32_t *leaf_y0, int32_t *leaf_x0, int32_t *leaf_s,
                           int32_t *seq_off, int32_t *patch_leaf, int64_t *n_leaves_out);

/* HOST: steps 1-2 above for one field; edges_out: host [H*W], 1 where an edge pixel
 * was found.  For inspection and tests. */
int reslim_asc_edges(const float *image, int32_t H, int32_t W, int32_t canny_low, int32_t canny_high, uint8_t *edges_out);

/* Checks that the table is what reslim_asc_build (one tile) or reslim_asc_build_tiles
 * produces for this context's grid and tiling -- per (sample, tile) sequence: power-of-two
 * squares aligned to the tile's haloed box, inside it, covering each of its patches exactly
 * once; patch_leaf naming, for every patch, the leaf of the owning tile that holds it:
 * RESLIM_EINVAL otherwise, the kernels rely on it -- and copies it to the device
 * (allocates; synchronous copies).  All pointers host; sample_off has n_sequences + 1
 * entries and n_sequences must be batch * T (T tiles of the context; sequences
 * sample-major).  *out is NULL on failure; destroy the plan before its context.
 * RESLIM_ESHAPE if n_sequences != batch * T or embed_dim % 4 != 0. */
int reslim_asc_plan_create(reslim_ctx *ctx, int32_t batch, const int32_t *leaf_y0, const int32_t *leaf_x0,
                           const int32_t *leaf_s, int64_t n_leaves, const int32_t *sample_off, int64_t n_sequences,
                           const int32_t *patch_leaf, reslim_asc_plan **out);
void reslim_asc_plan_destroy(reslim_asc_plan *plan);
int reslim_asc_plan_info(const reslim_asc_plan *plan, int64_t *n_leaves, int32_t *max_per_sample);

/* Image-space map of the aggregated embedding (reading: one linear map D -> p*p per
 * token, un-patchified): image[b, py*p + i, px*p + j] = w_img[i*p + j] . tokens[b, py*Wp
 * + px] + b_img[i*p + j].  tokens: dev fp32 [batch*N, D] (reslim_embed_fwd of a
 * one-tile context); w_img: dev fp32 [p*p, D]; b_img: dev fp32 [p*p]; image: dev
 * fp32 [batch, H, W].  fp32 arithmetic.  Enqueued on hip_stream. */
int reslim_asc_image(reslim_ctx *ctx, const float *tokens, const float *w_img, const float *b_img, float *image,
                     int32_t batch, void *hip_stream);

/* Compression (reading: a leaf's token is the arithmetic mean of its patches'
 * aggregated embeddings, position and resolution terms included).  tokens: dev fp32
 * [batch*N, D] in patch order; tokens_c: dev fp32 [n_leaves, D] out.  fp32 sums in a
 * fixed order over the leaf: deterministic. */
int reslim_asc_compress(reslim_ctx *ctx, const reslim_asc_plan *plan, const float *tokens, float *tokens_c, void *hip_stream);

/* Decompression on its own (each patch takes its leaf's row: tokens_c dev fp32
 * [n_leaves, D] -> tokens dev fp32 [batch*N, D]) and the gradients of the two linear
 * maps: reslim_asc_compress_bwd gives every patch its leaf's gradient divided by the
 * leaf's patch count (d_tokens_c [n_leaves, D] -> d_tokens [batch*N, D]);
 * reslim_asc_decompress_bwd adds up the gradients of a leaf's patches (d_tokens
 * [batch*N, D] -> d_tokens_c [n_leaves, D], fixed summation order).  With tiles the first
 * adds the shares of all leaves that hold the patch (its tile's and those of the boxes whose
 * halo it lies in, increasing leaf index), the second only the patches the leaf's tile owns (a
 * leaf made of halo patches alone gets zero).  All dev fp32. */
int reslim_asc_decompress(reslim_ctx *ctx, const reslim_asc_plan *plan, const float *tokens_c, float *tokens, void *hip_stream);
int reslim_asc_compress_bwd(reslim_ctx *ctx, const reslim_asc_plan *plan, const float *d_tokens_c, float *d_tokens, void *hip_stream);
int reslim_asc_decompress_bwd(reslim_ctx *ctx, const reslim_asc_plan *plan, const float *d_tokens, float *d_tokens_c, void *hip_stream);

/* Training of a block on the leaves (the paper's Table 2(b) quotes TRAINING time per
 * sample with compression): reslim_block_fwd_train / reslim_block_bwd with the rows
 * x [n_leaves, D] of a compressed batch and attention among the leaves of one sample.
 * Arguments, saved-tensor and workspace rules, precision and errors as for those two
 * calls; sizes from reslim_asc_block_train_bytes; reslim_train_prepare first. */
int reslim_asc_block_train_bytes(const reslim_ctx *ctx, const reslim_asc_plan *plan, size_t *saved_bytes, size_t *ws_bytes);
int reslim_asc_block_fwd_train(reslim_ctx *ctx, const reslim_asc_plan *plan, int32_t layer, const float *x_in, float *x_out,
                               void *saved, size_t saved_bytes, void *workspace, size_t ws_bytes, void *hip_stream);
int reslim_asc_block_bwd(reslim_ctx *ctx, const reslim_asc_plan *plan, int32_t layer, const float *x_in, const void *saved,
                         size_t saved_bytes, const float *d_x_out, float *d_x_in, const reslim_block_grads *grads,
                         void *workspace, size_t ws_bytes, void *hip_stream);

/* The forward pass with the compression module switched on: embed, compress, every
 * block on the leaves (attention among the leaves of one sample), decompress (each
 * patch takes its leaf's token), final LayerNorm, head, un-patchify + residual path.
 * x: dev fp32 [batch, V, H, W] with the plan's batch; y: dev fp32 [batch, C, s*H,
 * s*W]; workspace as for reslim_forward at that batch.  With one patch per leaf the
 * result equals reslim_forward's.  Errors as reslim_forward, plus RESLIM_EINVAL for
 * a plan of another context. */
int reslim_asc_forward(reslim_ctx *ctx, const reslim_asc_plan *plan, const float *x, float *y, void *workspace,
                       size_t ws_bytes, void *hip_stream);

/* Bandwidth yardstick: a plain device-to-device copy kernel (16 bytes per lane) of
 * `bytes` (a multiple of 16) from src to dst, both dev.  Profilers scale their HBM
 * byte counters by what they report for this kernel of known size. */
int reslim_debug_copy(const void *src, void *dst, size_t bytes, void *hip_stream);

/* Tuning hook for benchmarks and tests: pins the bf16 GEMM kernel (-1 = built-in heuristic,
 * 2 = one 128x128 tile per work-group, 3 = persistent direct-to-LDS 256x256 tiles; add 100
 * to 2 for columns-fastest tile order; other values act like 2).  A plain process-wide
 * variable read at every launch: not thread-safe, not part of the method; set it while no
 * other thread is inside the library and restore -1 afterwards. */
void reslim_debug_set_gemm_tile(int choice);

/* Tuning hook for benchmarks and tests: launch shape of the bf16 tile-attention kernel at
 * head dimension 64 (0 = 64-key blocks, three work-groups per compute unit, the default;
 * 1 = 128-key blocks, two work-groups per compute unit).  Process-wide and not thread-safe,
 * like the hook above. */
void reslim_debug_set_attention_variant(int variant);

#ifdef __cplusplus
}
#endif
#endif /* RESLIM_H */

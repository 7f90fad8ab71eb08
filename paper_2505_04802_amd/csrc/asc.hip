// Adaptive spatial compression, device side (ORBIT-2 Sec. 4.1): image-space map of
// the aggregated embedding, leaf-mean compression of the tokens, the ViT blocks on
// one token per quad-tree leaf with attention inside each sample, decompression
// folded into the final LayerNorm's row map, then the usual head and residual path.
#include <algorithm>
#include <string>
#include <vector>

#include "common.h"

namespace reslim {

// One work-group per leaf: mean over its s x s patch rows.  Wave w sums the rows
// w, w + 4, ... of the leaf (row-major numbering) in increasing order, the four
// partial sums are added in wave order: a fixed order, so the result is deterministic.
template <bool MEAN>   // false: plain sums (the gradient of decompression)
__global__ __launch_bounds__(256) void asc_compress_kernel(const float *__restrict__ z, const int32_t *__restrict__ leaf,
                                                           float *__restrict__ out, int Wp, int D) {
  __shared__ float4 part[3][64];
  const int64_t l = blockIdx.x;
  const int first = leaf[4 * l], s = leaf[4 * l + 1];
  const int rows = s * s;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float inv = MEAN ? 1.0f / static_cast<float>(rows) : 1.0f;
  for (int d0 = 0; d0 < D; d0 += 256) {              // uniform over the work-group
    const int d = d0 + lane * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (d < D) {
#pragma unroll 4
      for (int r = wave; r < rows; r += 4) {
        const int dy = r / s, dx = r - dy * s;
        const float4 v = *reinterpret_cast<const float4 *>(z + (static_cast<size_t>(first) + static_cast<size_t>(dy) * Wp + dx) * D + d);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
      }
    }
    if (rows > 1) {
      if (wave > 0) part[wave - 1][lane] = acc;
      __syncthreads();
      if (wave == 0) {
#pragma unroll
        for (int w = 0; w < 3; ++w) {
          const float4 v = part[w][lane];
          acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
      }
      __syncthreads();
    }
    if (wave == 0 && d < D)
      *reinterpret_cast<float4 *>(out + static_cast<size_t>(l) * D + d) = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
  }
}

// One wave per patch: its leaf's row, optionally divided by the leaf's patch count
// (decompression, and with the division the gradient of the leaf mean).
template <bool SCALE>
__global__ __launch_bounds__(256) void asc_expand_kernel(const float *__restrict__ src, const int32_t *__restrict__ patch_leaf,
                                                         const int32_t *__restrict__ leaf, float *__restrict__ dst,
                                                         int64_t patches, int D) {
  const int lane = threadIdx.x & 63;
  const int64_t p = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (p >= patches) return;
  const int l = patch_leaf[p];
  float f = 1.0f;
  if (SCALE) {
    const int s = leaf[4 * static_cast<int64_t>(l) + 1];
    f = 1.0f / static_cast<float>(s * s);
  }
  const float4 *in = reinterpret_cast<const float4 *>(src + static_cast<size_t>(l) * D);
  float4 *out = reinterpret_cast<float4 *>(dst + static_cast<size_t>(p) * D);
  for (int d = lane; d < D / 4; d += 64) {
    const float4 v = in[d];
    out[d] = make_float4(v.x * f, v.y * f, v.z * f, v.w * f);
  }
}

// Gradient of compression where tiles overlap: one wave per patch adds gradient / (side * side) of
// every leaf that holds the patch (one per box whose haloed region contains it), in increasing
// leaf order: a fixed order, deterministic.
__global__ __launch_bounds__(256) void asc_cover_sum_kernel(const float *__restrict__ d_leaf_tok, const int32_t *__restrict__ cover_off,
                                                            const int32_t *__restrict__ cover_leaf, const int32_t *__restrict__ leaf,
                                                            float *__restrict__ dst, int64_t patches, int D) {
  const int lane = threadIdx.x & 63;
  const int64_t p = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (p >= patches) return;
  const int lo = cover_off[p], hi = cover_off[p + 1];
  float4 *out = reinterpret_cast<float4 *>(dst + static_cast<size_t>(p) * D);
  for (int d = lane; d < D / 4; d += 64) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int k = lo; k < hi; ++k) {
      const int l = cover_leaf[k], s = leaf[4 * static_cast<int64_t>(l) + 1];
      const float f = 1.0f / static_cast<float>(s * s);
      const float4 v = reinterpret_cast<const float4 *>(d_leaf_tok + static_cast<size_t>(l) * D)[d];
      acc.x = fmaf(v.x, f, acc.x); acc.y = fmaf(v.y, f, acc.y); acc.z = fmaf(v.z, f, acc.z); acc.w = fmaf(v.w, f, acc.w);
    }
    out[d] = acc;
  }
}

// Gradient of decompression where tiles overlap: a leaf collects the gradients of the patches that
// were decompressed from it, i.e. of those of its patches that its tile owns (patch_leaf names this
// leaf); its halo patches took their tokens from other tiles' leaves.  One work-group per leaf,
// rows in increasing order per wave, the four waves' sums added in wave order.
__global__ __launch_bounds__(256) void asc_owned_sum_kernel(const float *__restrict__ z, const int32_t *__restrict__ leaf,
                                                            const int32_t *__restrict__ patch_leaf, float *__restrict__ out, int Wp, int D) {
  __shared__ float4 part[3][64];
  const int64_t l = blockIdx.x;
  const int first = leaf[4 * l], s = leaf[4 * l + 1];
  const int rows = s * s;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int d0 = 0; d0 < D; d0 += 256) {              // uniform over the work-group
    const int d = d0 + lane * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (d < D) {
      for (int r = wave; r < rows; r += 4) {
        const int dy = r / s, dx = r - dy * s;
        const size_t row = static_cast<size_t>(first) + static_cast<size_t>(dy) * Wp + dx;
        if (patch_leaf[row] != l) continue;          // uniform over the wave
        const float4 v = *reinterpret_cast<const float4 *>(z + row * D + d);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
      }
    }
    if (wave > 0) part[wave - 1][lane] = acc;
    __syncthreads();
    if (wave == 0 && d < D) {
#pragma unroll
      for (int w = 0; w < 3; ++w) { const float4 q = part[w][lane]; acc.x += q.x; acc.y += q.y; acc.z += q.z; acc.w += q.w; }
      *reinterpret_cast<float4 *>(out + static_cast<size_t>(l) * D + d) = acc;
    }
    __syncthreads();
  }
}

// One wave per token: p*p dot products of length D, written to the token's pixels.
__global__ __launch_bounds__(256) void asc_image_kernel(const float *__restrict__ z, const float *__restrict__ w_img,
                                                        const float *__restrict__ b_img, float *__restrict__ img,
                                                        int64_t tokens, int N, int Wp, int p, int D, int H, int W) {
  const int lane = threadIdx.x & 63;
  const int64_t tok = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (tok >= tokens) return;
  const float *row = z + static_cast<size_t>(tok) * D;
  const int64_t b = tok / N;
  const int n = static_cast<int>(tok % N), py = n / Wp, px = n % Wp;
  for (int o = 0; o < p * p; ++o) {
    const float *wr = w_img + static_cast<size_t>(o) * D;
    float acc = 0.f;
    for (int d = lane; d < D; d += 64) acc = fmaf(wr[d], row[d], acc);
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0) img[(static_cast<size_t>(b) * H + py * p + o / p) * W + px * p + o % p] = acc + b_img[o];
  }
}

static void asc_free(reslim_asc_plan *pl) {
  if (!pl) return;
  if (pl->d_seq) (void)hipFree(pl->d_seq);
  if (pl->d_seq_of_leaf) (void)hipFree(pl->d_seq_of_leaf);
  if (pl->d_leaf) (void)hipFree(pl->d_leaf);
  if (pl->d_patch_leaf) (void)hipFree(pl->d_patch_leaf);
  if (pl->d_cover_off) (void)hipFree(pl->d_cover_off);
  if (pl->d_cover_leaf) (void)hipFree(pl->d_cover_leaf);
  delete pl;
}

static int asc_check(reslim_ctx *c, const reslim_asc_plan *pl, const char *fn) {
  if (!pl) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null plan");
  if (pl->ctx != c) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": plan belongs to another context");
  return RESLIM_OK;
}

}  // namespace reslim

using namespace reslim;

extern "C" int reslim_asc_plan_create(reslim_ctx *c, int32_t batch, const int32_t *leaf_y0, const int32_t *leaf_x0,
                                      const int32_t *leaf_s, int64_t n_leaves, const int32_t *sample_off, int64_t n_sequences,
                                      const int32_t *patch_leaf, reslim_asc_plan **out) {
  const char *fn = "reslim_asc_plan_create";
  if (!c) return RESLIM_EINVAL;
  if (out) *out = nullptr;
  if (!leaf_y0 || !leaf_x0 || !leaf_s || !sample_off || !patch_leaf || !out)
    return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null pointer");
  const int64_t N = c->N;
  const int T = c->T;
  const int64_t n_seq = static_cast<int64_t>(batch) * T;
  if (c->cfg.embed_dim % 4) return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": embed_dim must be a multiple of 4");
  if (n_sequences != n_seq)
    return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": the table must hold one sequence per (sample, tile) of this context");
  if (batch < 1 || n_seq > INT32_MAX || n_leaves < n_seq || n_leaves > batch * c->n_h || batch * N > INT32_MAX || batch * c->n_h > INT32_MAX)
    return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": batch or leaf count out of range");
  // Per (sample, tile) sequence the leaves must partition the tile's haloed box into squares
  // aligned to the box, and patch_leaf must name, for every patch, its leaf in the tile that
  // owns it: the kernels trust the table.
  if (sample_off[0] != 0 || sample_off[n_seq] != n_leaves) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": sample_off does not span the leaves");
  std::vector<int32_t> leaf(static_cast<size_t>(n_leaves) * 4, 0), seq_of(static_cast<size_t>(n_leaves));
  std::vector<tile_desc> seq(n_seq);
  std::vector<int32_t> owner;                  // leaf of every box patch of the sequence at hand
  int max_n = 0;
  double pairs = 0;
  for (int64_t q = 0; q < n_seq; ++q) {
    const int64_t b = q / T;
    const tile_desc &td = c->tiles[q % T];
    const int hp = td.Y1 - td.Y0, wp = td.X1 - td.X0;
    const int64_t lo = sample_off[q], hi = sample_off[q + 1];
    if (hi <= lo || hi > n_leaves) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": sample_off not increasing");
    owner.assign(static_cast<size_t>(hp) * wp, -1);
    for (int64_t l = lo; l < hi; ++l) {
      const int y0 = leaf_y0[l], x0 = leaf_x0[l], s = leaf_s[l];
      if (s < 1 || (s & (s - 1)) || y0 < td.Y0 || x0 < td.X0 || (y0 - td.Y0) % s || (x0 - td.X0) % s || y0 + s > td.Y1 || x0 + s > td.X1)
        return set_error(c, RESLIM_EINVAL, std::string(fn) + ": leaf outside its box or not an aligned power-of-two square");
      for (int yy = y0; yy < y0 + s; ++yy)
        for (int xx = x0; xx < x0 + s; ++xx) {
          int32_t &o = owner[static_cast<size_t>(yy - td.Y0) * wp + (xx - td.X0)];
          if (o != -1) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": two leaves of a sequence overlap");
          o = static_cast<int32_t>(l);
        }
      leaf[4 * l] = static_cast<int32_t>(b * N + static_cast<int64_t>(y0) * c->Wp + x0);
      leaf[4 * l + 1] = s;
      seq_of[l] = static_cast<int32_t>(q);
    }
    for (int32_t o : owner)
      if (o == -1) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": leaves of a sequence do not cover its box");
    for (int yy = td.y0; yy < td.y1; ++yy)
      for (int xx = td.x0; xx < td.x1; ++xx)
        if (patch_leaf[b * N + static_cast<int64_t>(yy) * c->Wp + xx] != owner[static_cast<size_t>(yy - td.Y0) * wp + (xx - td.X0)])
          return set_error(c, RESLIM_EINVAL, std::string(fn) + ": patch_leaf disagrees with the leaf list");
    seq[q] = tile_desc{};
    seq[q].tok_off = lo;
    seq[q].n_tok = static_cast<int32_t>(hi - lo);
    max_n = std::max(max_n, seq[q].n_tok);
    pairs += static_cast<double>(hi - lo) * static_cast<double>(hi - lo);
  }
  // leaves of every patch (tiled contexts): counting pass, prefix sums, fill in increasing leaf order
  std::vector<int32_t> cover_off, cover_leaf;
  if (T != 1) {
    cover_off.assign(static_cast<size_t>(batch) * N + 1, 0);
    for (int64_t l = 0; l < n_leaves; ++l)
      for (int dy = 0; dy < leaf[4 * l + 1]; ++dy)
        for (int dx = 0; dx < leaf[4 * l + 1]; ++dx) ++cover_off[static_cast<size_t>(leaf[4 * l]) + static_cast<size_t>(dy) * c->Wp + dx + 1];
    for (size_t i = 1; i < cover_off.size(); ++i) cover_off[i] += cover_off[i - 1];
    cover_leaf.resize(static_cast<size_t>(cover_off.back()));
    std::vector<int32_t> fill(cover_off.begin(), cover_off.end() - 1);
    for (int64_t l = 0; l < n_leaves; ++l)
      for (int dy = 0; dy < leaf[4 * l + 1]; ++dy)
        for (int dx = 0; dx < leaf[4 * l + 1]; ++dx)
          cover_leaf[static_cast<size_t>(fill[static_cast<size_t>(leaf[4 * l]) + static_cast<size_t>(dy) * c->Wp + dx]++)] = static_cast<int32_t>(l);
  }
  reslim_asc_plan *pl = new (std::nothrow) reslim_asc_plan;
  if (!pl) return set_error(c, RESLIM_ENOMEM, std::string(fn) + ": host allocation failed");
  pl->ctx = c; pl->batch = batch; pl->L = n_leaves; pl->seq = seq;
  hipError_t e = hipMalloc(reinterpret_cast<void **>(&pl->d_seq), n_seq * sizeof(tile_desc));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&pl->d_seq_of_leaf), n_leaves * 4);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&pl->d_leaf), n_leaves * 16);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&pl->d_patch_leaf), batch * N * 4);
  if (e == hipSuccess) e = hipMemcpy(pl->d_seq, seq.data(), n_seq * sizeof(tile_desc), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(pl->d_seq_of_leaf, seq_of.data(), n_leaves * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(pl->d_leaf, leaf.data(), n_leaves * 16, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(pl->d_patch_leaf, patch_leaf, batch * N * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess && T != 1) {
    e = hipMalloc(reinterpret_cast<void **>(&pl->d_cover_off), cover_off.size() * 4);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&pl->d_cover_leaf), std::max<size_t>(cover_leaf.size() * 4, 256));
    if (e == hipSuccess) e = hipMemcpy(pl->d_cover_off, cover_off.data(), cover_off.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(pl->d_cover_leaf, cover_leaf.data(), cover_leaf.size() * 4, hipMemcpyHostToDevice);
  }
  if (e != hipSuccess) {
    asc_free(pl);
    return set_error(c, e == hipErrorOutOfMemory ? RESLIM_ENOMEM : RESLIM_EHIP, std::string(fn) + ": " + hipGetErrorString(e));
  }
  pl->geom.d_tiles = pl->d_seq;
  pl->geom.d_tile_of_tok = pl->d_seq_of_leaf;
  pl->geom.T = static_cast<int>(n_seq);
  pl->geom.n_h = n_leaves;
  pl->geom.max_n_tok = max_n;
  pl->geom.pairs = pairs;
  pl->geom.pairs_owned = pairs;   // no stitched launches on compressed sequences
  *out = pl;
  return RESLIM_OK;
}

extern "C" void reslim_asc_plan_destroy(reslim_asc_plan *plan) { asc_free(plan); }

extern "C" int reslim_asc_image(reslim_ctx *c, const float *tokens, const float *w_img, const float *b_img, float *image,
                                int32_t batch, void *hip_stream) {
  const char *fn = "reslim_asc_image";
  if (!c) return RESLIM_EINVAL;
  if (!tokens || !w_img || !b_img || !image) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  if (batch < 1 || static_cast<int64_t>(batch) * c->N > INT32_MAX) return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": batch out of range");
  const int64_t tokens_n = static_cast<int64_t>(batch) * c->N;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  asc_image_kernel<<<dim3(static_cast<unsigned>((tokens_n + 3) / 4)), dim3(256), 0, st>>>(
      tokens, w_img, b_img, image, tokens_n, c->N, c->Wp, c->cfg.patch, c->cfg.embed_dim, c->cfg.H, c->cfg.W);
  RESLIM_TRY("asc_image", hipGetLastError());
  return RESLIM_OK;
}

extern "C" int reslim_asc_compress(reslim_ctx *c, const reslim_asc_plan *plan, const float *tokens, float *tokens_c, void *hip_stream) {
  const char *fn = "reslim_asc_compress";
  if (!c) return RESLIM_EINVAL;
  int rc = asc_check(c, plan, fn);
  if (rc != RESLIM_OK) return rc;
  if (!tokens || !tokens_c) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  asc_compress_kernel<true><<<dim3(static_cast<unsigned>(plan->L)), dim3(256), 0, st>>>(tokens, plan->d_leaf, tokens_c, c->Wp, c->cfg.embed_dim);
  RESLIM_TRY("asc_compress", hipGetLastError());
  return RESLIM_OK;
}

// mode 0: decompression; 1: gradient of compression (leaf gradient / patch count to every patch);
// 2: gradient of decompression (sum of the patch gradients of a leaf)
static int asc_move(reslim_ctx *c, const reslim_asc_plan *plan, const char *fn, int mode, const float *src, float *dst, void *hip_stream) {
  int rc = asc_check(c, plan, fn);
  if (rc != RESLIM_OK) return rc;
  if (!src || !dst) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int D = c->cfg.embed_dim;
  const int64_t patches = static_cast<int64_t>(plan->batch) * c->N;
  const dim3 pg(static_cast<unsigned>((patches + 3) / 4));
  // With tiles a patch sits in the leaves of several boxes and a leaf decompresses only into its
  // tile's interior: the gradient of compression adds over a patch's leaves, the gradient of
  // decompression over the patches a leaf's tile owns.  One tile: one leaf per patch, every patch owned.
  const bool tiled = c->T != 1;
  if (mode == 0) asc_expand_kernel<false><<<pg, dim3(256), 0, st>>>(src, plan->d_patch_leaf, plan->d_leaf, dst, patches, D);
  else if (mode == 1 && !tiled) asc_expand_kernel<true><<<pg, dim3(256), 0, st>>>(src, plan->d_patch_leaf, plan->d_leaf, dst, patches, D);
  else if (mode == 1) asc_cover_sum_kernel<<<pg, dim3(256), 0, st>>>(src, plan->d_cover_off, plan->d_cover_leaf, plan->d_leaf, dst, patches, D);
  else if (!tiled) asc_compress_kernel<false><<<dim3(static_cast<unsigned>(plan->L)), dim3(256), 0, st>>>(src, plan->d_leaf, dst, c->Wp, D);
  else asc_owned_sum_kernel<<<dim3(static_cast<unsigned>(plan->L)), dim3(256), 0, st>>>(src, plan->d_leaf, plan->d_patch_leaf, dst, c->Wp, D);
  RESLIM_TRY("launch", hipGetLastError());
  return RESLIM_OK;
}

extern "C" int reslim_asc_decompress(reslim_ctx *c, const reslim_asc_plan *plan, const float *tokens_c, float *tokens, void *hip_stream) {
  if (!c) return RESLIM_EINVAL;
  return asc_move(c, plan, "reslim_asc_decompress", 0, tokens_c, tokens, hip_stream);
}

extern "C" int reslim_asc_compress_bwd(reslim_ctx *c, const reslim_asc_plan *plan, const float *d_tokens_c, float *d_tokens, void *hip_stream) {
  if (!c) return RESLIM_EINVAL;
  return asc_move(c, plan, "reslim_asc_compress_bwd", 1, d_tokens_c, d_tokens, hip_stream);
}

extern "C" int reslim_asc_decompress_bwd(reslim_ctx *c, const reslim_asc_plan *plan, const float *d_tokens, float *d_tokens_c, void *hip_stream) {
  if (!c) return RESLIM_EINVAL;
  return asc_move(c, plan, "reslim_asc_decompress_bwd", 2, d_tokens, d_tokens_c, hip_stream);
}

extern "C" int reslim_asc_forward(reslim_ctx *c, const reslim_asc_plan *plan, const float *x, float *y, void *workspace,
                                  size_t ws_bytes, void *hip_stream) {
  const char *fn = "reslim_asc_forward";
  if (!c) return RESLIM_EINVAL;
  int rc = asc_check(c, plan, fn);
  if (rc != RESLIM_OK) return rc;
  if (!x || !y) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  const int batch = plan->batch;
  rc = check_common(c, fn, batch, workspace, ws_bytes, true);
  if (rc != RESLIM_OK) return rc;
  const Workspace w = plan_workspace(c, batch, workspace);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int D = c->cfg.embed_dim, dt = c->cfg.dtype;
  const int Mi = batch * c->N;
  const double es = static_cast<double>(act_size(c)), dMi = Mi, dD = D, dO = c->head_out, dL = static_cast<double>(plan->L);
  // embed (w.big <- [Mi, D] fp32), compress into the stream buffer
  if ((rc = embed_full_impl(c, fn, x, batch, w, st)) != RESLIM_OK) return rc;
  RESLIM_LAUNCH("asc_compress", 0, 4.0 * dMi * dD + 4.0 * dL * dD,
                (asc_compress_kernel<true><<<dim3(static_cast<unsigned>(plan->L)), dim3(256), 0, st>>>(
                     static_cast<const float *>(w.big), plan->d_leaf, w.X, c->Wp, D),
                 hipGetLastError()));
  // blocks on the leaves: the batch is one run of L rows, one attention set per sample
  for (int l = 0; l < c->cfg.depth; ++l)
    if ((rc = block_impl(c, fn, l, w.X, 1, w, st, &plan->geom)) != RESLIM_OK) return rc;
  // decompression = the final LayerNorm reading each patch's row from its leaf
  RESLIM_LAUNCH("layernorm_final", 0, dMi * dD * (4.0 + es),
                launch_layernorm(dt, w.X, plan->d_patch_leaf, Mi, plan->L, c->d_lnf_g, c->d_lnf_b, w.A, Mi, D, st));
  RESLIM_LAUNCH("gemm_head", 2.0 * dMi * dD * dO, dMi * dD * es + dD * dO * es + 4.0 * dMi * dO,
                launch_gemm(dt, EPI_BIAS_F32, w.A, c->d_w_head, c->d_b_head, w.big, c->head_out, nullptr, 0, Mi, c->head_out, D, st));
  const double fine = static_cast<double>(batch) * c->cfg.out_vars * c->cfg.H * c->cfg.W * c->cfg.scale * c->cfg.scale;
  RESLIM_LAUNCH("residual_unpatchify", 0,
                4.0 * batch * c->cfg.out_vars * c->cfg.H * c->cfg.W + 4.0 * dMi * dO + 4.0 * fine,
                launch_residual_unpatchify(c, x, w.big, 0, y, batch, st));
  return RESLIM_OK;
}

extern "C" int reslim_asc_plan_info(const reslim_asc_plan *plan, int64_t *n_leaves, int32_t *max_per_sample) {
  if (!plan || !n_leaves || !max_per_sample) return RESLIM_EINVAL;
  *n_leaves = plan->L;
  *max_per_sample = plan->geom.max_n_tok;
  return RESLIM_OK;
}

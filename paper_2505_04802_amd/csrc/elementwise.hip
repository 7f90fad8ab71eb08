// Bandwidth-bound kernels of the Reslim forward (ORBIT-2 Sec. 4.1, 4.2):
//   embed_agg       per-variable tokenisation + cross-attention variable aggregation
//                   (folded: no non-linearity separates the two, so the scores and
//                   the values are affine in the p*p pixels of a patch)
//   gather_rows     tile-major copy with halo duplication (Sec. 4.2)
//   layernorm       per-token normalisation; optional row map = "discard the halo"
//   residual_unpatchify  residual path (bilinear upsampling + 3x3 convolution per
//                   tile on its haloed box) fused with un-patchify, stitch and add
#include <algorithm>

#include "common.h"

namespace reslim {

// ------------------------------------------------------------------ LayerNorm
// One wave per token row; the row lives in registers between the two statistics
// passes (mean, then centred variance) and the normalise pass.
template <class T, int NV>
__global__ __launch_bounds__(256) void layernorm_kernel(const float *__restrict__ x, const int32_t *__restrict__ row_src,
                                                        int rows_per_sample_out, int64_t rows_per_sample_in,
                                                        const float *__restrict__ g, const float *__restrict__ be,
                                                        T *__restrict__ out, int64_t rows_out, int D) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= rows_out) return;
  int64_t in_row = row;
  if (row_src) {
    const int64_t b = row / rows_per_sample_out;
    in_row = b * rows_per_sample_in + row_src[row % rows_per_sample_out];
  }
  const float4 *xr = reinterpret_cast<const float4 *>(x + in_row * D);
  const int nv = D / 4;
  float4 v[NV];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int k = lane + 64 * i;
    v[i] = k < nv ? xr[k] : make_float4(0.f, 0.f, 0.f, 0.f);
    sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  const float mean = sum / static_cast<float>(D);
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int k = lane + 64 * i;
    if (k < nv) {
      const float a = v[i].x - mean, b = v[i].y - mean, c = v[i].z - mean, d = v[i].w - mean;
      sq += (a * a + b * b) + (c * c + d * d);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
  const float rstd = rsqrtf(sq / static_cast<float>(D) + 1e-5f);
  const float4 *g4 = reinterpret_cast<const float4 *>(g);
  const float4 *b4 = reinterpret_cast<const float4 *>(be);
  T *orow = out + row * D;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int k = lane + 64 * i;
    if (k < nv) {
      const float4 gg = g4[k], bb = b4[k];
      const float y0 = (v[i].x - mean) * rstd * gg.x + bb.x;
      const float y1 = (v[i].y - mean) * rstd * gg.y + bb.y;
      const float y2 = (v[i].z - mean) * rstd * gg.z + bb.z;
      const float y3 = (v[i].w - mean) * rstd * gg.w + bb.w;
      if constexpr (sizeof(T) == 4) {
        reinterpret_cast<float4 *>(orow)[k] = make_float4(y0, y1, y2, y3);
      } else {
        uint2 p;
        p.x = pack_bf16x2(y0, y1);
        p.y = pack_bf16x2(y2, y3);
        reinterpret_cast<uint2 *>(orow)[k] = p;
      }
    }
  }
}

// Rows wider than 4096 columns: a whole work-group per row, thread t owns the float4 columns
// t, t + 256, ... (a wave would need 128+ registers for the row alone).
template <class T, int NVT>
__global__ __launch_bounds__(256) void layernorm_wide_kernel(const float *__restrict__ x, const int32_t *__restrict__ row_src,
                                                             int rows_per_sample_out, int64_t rows_per_sample_in,
                                                             const float *__restrict__ g, const float *__restrict__ be,
                                                             T *__restrict__ out, int D) {
  __shared__ float box[2][4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = blockIdx.x;
  int64_t in_row = row;
  if (row_src) {
    const int64_t b = row / rows_per_sample_out;
    in_row = b * rows_per_sample_in + row_src[row % rows_per_sample_out];
  }
  const float4 *xr = reinterpret_cast<const float4 *>(x + in_row * D);
  const int nv = D / 4;
  float4 v[NVT];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NVT; ++i) {
    const int k = static_cast<int>(threadIdx.x) + 256 * i;
    v[i] = k < nv ? xr[k] : make_float4(0.f, 0.f, 0.f, 0.f);
    sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  if (lane == 0) box[0][wave] = sum;
  __syncthreads();
  const float mean = ((box[0][0] + box[0][1]) + (box[0][2] + box[0][3])) / static_cast<float>(D);
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NVT; ++i) {
    const int k = static_cast<int>(threadIdx.x) + 256 * i;
    if (k < nv) {
      const float a = v[i].x - mean, b = v[i].y - mean, c = v[i].z - mean, d = v[i].w - mean;
      sq += (a * a + b * b) + (c * c + d * d);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
  if (lane == 0) box[1][wave] = sq;
  __syncthreads();
  const float rstd = rsqrtf(((box[1][0] + box[1][1]) + (box[1][2] + box[1][3])) / static_cast<float>(D) + 1e-5f);
  const float4 *g4 = reinterpret_cast<const float4 *>(g);
  const float4 *b4 = reinterpret_cast<const float4 *>(be);
  T *orow = out + row * D;
#pragma unroll
  for (int i = 0; i < NVT; ++i) {
    const int k = static_cast<int>(threadIdx.x) + 256 * i;
    if (k < nv) {
      const float4 gg = g4[k], bb = b4[k];
      const float y0 = (v[i].x - mean) * rstd * gg.x + bb.x;
      const float y1 = (v[i].y - mean) * rstd * gg.y + bb.y;
      const float y2 = (v[i].z - mean) * rstd * gg.z + bb.z;
      const float y3 = (v[i].w - mean) * rstd * gg.w + bb.w;
      if constexpr (sizeof(T) == 4) {
        reinterpret_cast<float4 *>(orow)[k] = make_float4(y0, y1, y2, y3);
      } else {
        uint2 p;
        p.x = pack_bf16x2(y0, y1);
        p.y = pack_bf16x2(y2, y3);
        reinterpret_cast<uint2 *>(orow)[k] = p;
      }
    }
  }
}

template <class T>
static hipError_t launch_ln_t(const float *x, const int32_t *row_src, int rpo, int64_t rpi, const float *g,
                              const float *b, void *out, int64_t rows_out, int D, hipStream_t st) {
  const int nv = (D / 4 + 63) / 64;
  const dim3 grid(static_cast<unsigned>((rows_out + 3) / 4)), blk(256);
  T *o = static_cast<T *>(out);
#define RESLIM_LN(NV) layernorm_kernel<T, NV><<<grid, blk, 0, st>>>(x, row_src, rpo, rpi, g, b, o, rows_out, D)
  if (nv <= 1) RESLIM_LN(1);
  else if (nv <= 2) RESLIM_LN(2);
  else if (nv <= 4) RESLIM_LN(4);
  else if (nv <= 8) RESLIM_LN(8);
  else if (nv <= 16) RESLIM_LN(16);
  else {
    if (rows_out > INT32_MAX) return hipErrorInvalidValue;
    const dim3 wgrid(static_cast<unsigned>(rows_out));
#define RESLIM_LNW(NVT) layernorm_wide_kernel<T, NVT><<<wgrid, blk, 0, st>>>(x, row_src, rpo, rpi, g, b, o, D)
    if (nv <= 32) RESLIM_LNW(8);
    else if (nv <= 64) RESLIM_LNW(16);
    else return hipErrorInvalidValue;     // D above 16384
#undef RESLIM_LNW
  }
#undef RESLIM_LN
  return hipGetLastError();
}

hipError_t launch_layernorm(int dtype, const float *x, const int32_t *row_src, int rows_per_sample_out,
                            int64_t rows_per_sample_in, const float *g, const float *b, void *out,
                            int64_t rows_out, int D, hipStream_t st) {
  if (D % 4 != 0 || rows_out <= 0 || (rows_out + 3) / 4 > INT32_MAX) return hipErrorInvalidValue;
  return dtype == RESLIM_BF16
             ? launch_ln_t<bf16_t>(x, row_src, rows_per_sample_out, rows_per_sample_in, g, b, out, rows_out, D, st)
             : launch_ln_t<float>(x, row_src, rows_per_sample_out, rows_per_sample_in, g, b, out, rows_out, D, st);
}

// ------------------------------------------------------------------ gather
__global__ __launch_bounds__(256) void gather_rows_kernel(const float4 *__restrict__ z, const int32_t *__restrict__ gather,
                                                          float4 *__restrict__ X, int64_t n_h, int N, int D4,
                                                          int64_t total) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t row = i / D4;
  const int col = static_cast<int>(i % D4);
  const int64_t b = row / n_h, k = row % n_h;
  X[i] = z[(b * N + gather[k]) * D4 + col];
}

hipError_t launch_gather_rows(const float *z, const int32_t *gather, float *X, int batch, int64_t n_h, int N, int D,
                              hipStream_t st) {
  if (D % 4 != 0) return hipErrorInvalidValue;
  const int64_t total = static_cast<int64_t>(batch) * n_h * (D / 4);
  const int64_t blocks = (total + 255) / 256;
  if (blocks > INT32_MAX) return hipErrorInvalidValue;
  gather_rows_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st>>>(
      reinterpret_cast<const float4 *>(z), gather, reinterpret_cast<float4 *>(X), n_h, N, D / 4, total);
  return hipGetLastError();
}

// ------------------------------------------------------------------ plain copy (bandwidth yardstick)
__global__ __launch_bounds__(256) void copy_probe_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst, int64_t n16) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

hipError_t launch_copy_probe(const void *src, void *dst, size_t bytes, hipStream_t st) {
  const int64_t n16 = static_cast<int64_t>(bytes / 16);
  const int64_t blocks = (n16 + 255) / 256;
  if (bytes % 16 || blocks < 1 || blocks > INT32_MAX) return hipErrorInvalidValue;
  copy_probe_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st>>>(static_cast<const float4 *>(src),
                                                                            static_cast<float4 *>(dst), n16);
  return hipGetLastError();
}

// ------------------------------------------------------------------ embed + aggregate
struct EmbedArgs {
  const float *x;
  const float *A, *a0, *U, *c;
  void *o;
  int V, H, W, p, Wp, N, D, heads, dh;
  int64_t BN;   // batch * N patches
};

// P2 = p*p when known at compile time (4 for the paper's 2x2 patches), 0 = run-time.
// PPI: patches per work item of the P2 = 4 path.  An item reads the value tables of its four
// features for every variable (80 bytes per variable, from L2) and uses them for PPI patches, so
// the table traffic per patch goes with 1 / PPI: at c3 1.24 ms with 4, 0.84 with 8, 0.82 with 16
// (c4: 1.57 / 1.27 / 1.10); 16 leaves half the threads without an item below 1024 features.
template <class T, int P2, int PPI_ = 8>
__global__ __launch_bounds__(256) void embed_agg_kernel(EmbedArgs e) {
  constexpr int TP = 16;                      // patches per work-group
  extern __shared__ float sm[];
  const int p2 = P2 ? P2 : e.p * e.p;
  const int VP2 = e.V * p2;
  float *pix = sm;                            // [TP][V*p2]
  float *sc = sm + TP * VP2;                  // [TP][heads][V] softmax weights over variables
  const int t = threadIdx.x;
  const int64_t bn0 = static_cast<int64_t>(blockIdx.x) * TP;

  for (int idx = t; idx < TP * VP2; idx += 256) {
    const int pi = idx / VP2, rem = idx % VP2, v = rem / p2, i = rem % p2;
    const int64_t bn = bn0 + pi;
    float val = 0.f;
    if (bn < e.BN) {
      const int64_t b = bn / e.N;
      const int n = static_cast<int>(bn % e.N);
      const int py = n / e.Wp, px = n % e.Wp;
      const int yy = py * e.p + i / e.p, xx = px * e.p + i % e.p;
      val = e.x[((b * e.V + v) * e.H + yy) * e.W + xx];
    }
    pix[idx] = val;
  }
  __syncthreads();
  // one thread per (patch, head): scores over the variables, then their softmax
  for (int idx = t; idx < TP * e.heads; idx += 256) {
    const int pi = idx / e.heads, g = idx % e.heads;
    float *r = sc + static_cast<size_t>(idx) * e.V;
    float mx = -INFINITY;
    for (int v = 0; v < e.V; ++v) {
      const float *Ar = e.A + (static_cast<size_t>(v) * e.heads + g) * p2;
      const float *px = pix + pi * VP2 + v * p2;
      float s = e.a0[v * e.heads + g];
      for (int i = 0; i < p2; ++i) s = fmaf(Ar[i], px[i], s);
      r[v] = s;
      mx = fmaxf(mx, s);
    }
    float sum = 0.f;
    for (int v = 0; v < e.V; ++v) {
      const float ex = __expf(r[v] - mx);
      r[v] = ex;
      sum += ex;
    }
    const float inv = 1.0f / sum;
    for (int v = 0; v < e.V; ++v) r[v] *= inv;
  }
  __syncthreads();
  // o[pi][d] = sum_v a[pi][head(d)][v] * (c[v][d] + U[v][d][:] . pix[pi][v][:])
  T *out = static_cast<T *>(e.o);
  if constexpr (P2 == 4) {
    if (e.dh % 4 == 0) {
      // A work item is four adjacent features (one head) of PPI patches: the pixel and
      // weight reads from LDS (broadcast over the wave) are shared by 4 PPI outputs.
      constexpr int PPI = PPI_;
      const int Q = e.D / 4;
      for (int item = t; item < Q * (TP / PPI); item += 256) {
        const int dq = item % Q, p0 = (item / Q) * PPI;
        const int d = dq * 4, g = d / e.dh;
        float acc[PPI][4];
#pragma unroll
        for (int pi = 0; pi < PPI; ++pi)
#pragma unroll
          for (int k = 0; k < 4; ++k) acc[pi][k] = 0.f;
        for (int v = 0; v < e.V; ++v) {
          const float4 *up = reinterpret_cast<const float4 *>(e.U + (static_cast<size_t>(v) * e.D + d) * 4);
          const float4 u0 = up[0], u1 = up[1], u2 = up[2], u3 = up[3];
          const float4 cv = *reinterpret_cast<const float4 *>(e.c + static_cast<size_t>(v) * e.D + d);
#pragma unroll
          for (int pi = 0; pi < PPI; ++pi) {
            const float4 px = *reinterpret_cast<const float4 *>(pix + (p0 + pi) * VP2 + v * 4);
            const float a = sc[((p0 + pi) * e.heads + g) * e.V + v];
            acc[pi][0] = fmaf(a, fmaf(u0.x, px.x, fmaf(u0.y, px.y, fmaf(u0.z, px.z, fmaf(u0.w, px.w, cv.x)))), acc[pi][0]);
            acc[pi][1] = fmaf(a, fmaf(u1.x, px.x, fmaf(u1.y, px.y, fmaf(u1.z, px.z, fmaf(u1.w, px.w, cv.y)))), acc[pi][1]);
            acc[pi][2] = fmaf(a, fmaf(u2.x, px.x, fmaf(u2.y, px.y, fmaf(u2.z, px.z, fmaf(u2.w, px.w, cv.z)))), acc[pi][2]);
            acc[pi][3] = fmaf(a, fmaf(u3.x, px.x, fmaf(u3.y, px.y, fmaf(u3.z, px.z, fmaf(u3.w, px.w, cv.w)))), acc[pi][3]);
          }
        }
#pragma unroll
        for (int pi = 0; pi < PPI; ++pi)
          if (bn0 + p0 + pi < e.BN) {
            T *o = out + (bn0 + p0 + pi) * e.D + d;
            if constexpr (sizeof(T) == 2) {
              uint2 pk;
              pk.x = pack_bf16x2(acc[pi][0], acc[pi][1]);
              pk.y = pack_bf16x2(acc[pi][2], acc[pi][3]);
              *reinterpret_cast<uint2 *>(o) = pk;
            } else {
              *reinterpret_cast<float4 *>(o) = make_float4(acc[pi][0], acc[pi][1], acc[pi][2], acc[pi][3]);
            }
          }
      }
      return;
    }
  }
  // general shapes: one thread per feature d
  for (int d = t; d < e.D; d += 256) {
    const int g = d / e.dh;
    float acc[TP];
#pragma unroll
    for (int pi = 0; pi < TP; ++pi) acc[pi] = 0.f;
    for (int v = 0; v < e.V; ++v) {
      const float *Ur = e.U + (static_cast<size_t>(v) * e.D + d) * p2;
      const float cv = e.c[static_cast<size_t>(v) * e.D + d];
#pragma unroll
      for (int pi = 0; pi < TP; ++pi) {
        const float *px = pix + pi * VP2 + v * p2;
        float val = cv;
        for (int i = 0; i < p2; ++i) val = fmaf(Ur[i], px[i], val);
        acc[pi] = fmaf(sc[(pi * e.heads + g) * e.V + v], val, acc[pi]);
      }
    }
#pragma unroll
    for (int pi = 0; pi < TP; ++pi)
      if (bn0 + pi < e.BN) Act<T>::store(out + (bn0 + pi) * e.D + d, acc[pi]);
  }
}

hipError_t residual_init();

hipError_t elementwise_init() {
  hipError_t e = residual_init();
  const int lim = 160 * 1024;
#define RESLIM_ATTR(K) if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void *>(&K), hipFuncAttributeMaxDynamicSharedMemorySize, lim)
  RESLIM_ATTR((embed_agg_kernel<bf16_t, 4>));
  RESLIM_ATTR((embed_agg_kernel<bf16_t, 4, 16>));
  RESLIM_ATTR((embed_agg_kernel<bf16_t, 0>));
  RESLIM_ATTR((embed_agg_kernel<float, 4>));
  RESLIM_ATTR((embed_agg_kernel<float, 0>));
#undef RESLIM_ATTR
  return e;
}

hipError_t launch_embed_agg(const reslim_ctx *c, const float *x, void *o, int batch, hipStream_t st) {
  constexpr int TP = 16;
  EmbedArgs e;
  e.x = x; e.A = c->d_agg_A; e.a0 = c->d_agg_a0; e.U = c->d_agg_U; e.c = c->d_agg_c; e.o = o;
  e.V = c->cfg.in_vars; e.H = c->cfg.H; e.W = c->cfg.W; e.p = c->cfg.patch; e.Wp = c->Wp; e.N = c->N;
  e.D = c->cfg.embed_dim; e.heads = c->cfg.heads; e.dh = c->dh;
  e.BN = static_cast<int64_t>(batch) * c->N;
  const size_t lds = static_cast<size_t>(TP) * (static_cast<size_t>(e.V) * e.p * e.p + static_cast<size_t>(e.heads) * e.V) * sizeof(float);
  if (lds > 160 * 1024) return hipErrorInvalidValue;
  const int64_t blocks = (e.BN + TP - 1) / TP;
  if (blocks > INT32_MAX) return hipErrorInvalidValue;
  const dim3 grid(static_cast<unsigned>(blocks)), blk(256);
  const bool bf = c->cfg.dtype == RESLIM_BF16, p4 = e.p == 2;
  if (bf && p4 && e.D >= 1024) embed_agg_kernel<bf16_t, 4, 16><<<grid, blk, lds, st>>>(e);
  else if (bf && p4) embed_agg_kernel<bf16_t, 4><<<grid, blk, lds, st>>>(e);
  else if (bf) embed_agg_kernel<bf16_t, 0><<<grid, blk, lds, st>>>(e);
  else if (p4) embed_agg_kernel<float, 4><<<grid, blk, lds, st>>>(e);
  else embed_agg_kernel<float, 0><<<grid, blk, lds, st>>>(e);
  return hipGetLastError();
}

// ------------------------------------------------------------------ residual path + stitch
struct ResArgs {
  const float *x;        // [B, V, H, W]
  const float *P;        // [B, N, C*ps*ps] head projection of the interior tokens
  float *y;              // [B, C, s*H, s*W]
  const tile_desc *tiles;
  const float *w_res, *b_res;
  const int32_t *out_var_idx;
  int V, C, H, W, s, p, ps, Wp, N, head_out;
  int nbx;               // blocks per tile along x
  int cwh, cww;          // coarse window of a block
  int ci_chunk;          // input variables per pass over the window
};

// Residual path (Sec. 4.1 "Residual Learning": upsampling + convolution of the input,
// added to the transformer's output), evaluated per tile on its haloed box (Sec. 4.2),
// fused with un-patchify, stitch and the final add.
//
// Both steps are linear and the upsampling acts on each variable alone, so the variables
// are mixed BEFORE upsampling, on the few coarse pixels a block touches, and the
// bilinear weights are applied afterwards, rows first, then columns.  With U the
// upsampled field (zero outside the box), r/c a fine row/column of the box and
// (a_r, b_r, w_r, m_r) the two clamped coarse source rows, the weight of the second and
// the inside-the-box mask of fine row r (same for columns):
//   Z[t=(dy,dx)][o](Y, X) = sum_i w_res[o][i][dy][dx] x[i](Y, X)                 coarse window
//   T[dx][o](r, X)        = sum_dy m_{r+dy} ((1 - w_{r+dy}) Z[dy,dx][o](a_{r+dy}, X) + w_{r+dy} Z[dy,dx][o](b_{r+dy}, X))
//   R[o](r, c)            = b_res[o] + sum_dx m_{c+dx} ((1 - w_{c+dx}) T[dx][o](r, a_{c+dx}) + w_{c+dx} T[dx][o](r, b_{c+dx}))
// which is the 3x3 convolution of the bilinear upsampling, term by term in another order.
// Per output value that is about 6 multiply-adds plus a share of Z and T (9 C multiply-adds
// per coarse window pixel and output) instead of 9 C per fine pixel: the kernel is bound by
// reading the head projection and writing y.
//
// A work-group produces a 16 x 64 block of fine pixels inside one tile's interior, CO
// output variables at a time; the head projection is read in patch order (16 bytes per
// lane: 4 pixels of one patch row) and the sum written in place.
// NARROW (scale >= 4): the six fine columns a thread's four pixels and their column taps touch
// come from at most three coarse columns, so the column step is a 3-term product with
// per-thread weights held in registers and T is read once per (tap, output) instead of per pixel.
template <int CO, bool NARROW>
__global__ __launch_bounds__(256) void residual_unpatchify_kernel(ResArgs a) {
  constexpr int BY = 16, BX = 64, WY = BY + 2, WX = BX + 2, WXP = 68;
  __shared__ float row_w[WY], col_w[WXP];
  __shared__ int row_a[WY], row_b[WY], row_m[WY], col_a[WXP], col_b[WXP], col_m[WXP];
  extern __shared__ __align__(16) float dyn[];
  const int cwh = a.cwh, cww = a.cww, npx = cwh * cww;
  float *Xw = dyn;                               // [ci_chunk][npx]       coarse window of the inputs
  float *Ws = Xw + a.ci_chunk * npx;             // [ci_chunk][9][CO]     convolution weights of this pass
  float *Z = Ws + a.ci_chunk * 9 * CO;           // [9][CO][npx]
  float *T = Z + 9 * CO * npx;                   // [3][CO][BY][cww]
  const tile_desc td = a.tiles[blockIdx.y];
  const int b = blockIdx.z;
  const int ih = (td.y1 - td.y0) * a.ps, iw = (td.x1 - td.x0) * a.ps;
  const int iy0 = (blockIdx.x / a.nbx) * BY, ix0 = (blockIdx.x % a.nbx) * BX;
  if (iy0 >= ih || ix0 >= iw) return;          // uniform
  const int t = threadIdx.x, ty = t / 16, tx = t % 16;
  // fine coordinates of the block origin inside the haloed box
  const int fy0 = (td.y0 - td.Y0) * a.ps + iy0, fx0 = (td.x0 - td.X0) * a.ps + ix0;
  const int box_fh = (td.Y1 - td.Y0) * a.ps, box_fw = (td.X1 - td.X0) * a.ps;   // fine size of the box
  const int box_ch = (td.Y1 - td.Y0) * a.p, box_cw = (td.X1 - td.X0) * a.p;     // coarse size of the box
  const int cy_org = td.Y0 * a.p, cx_org = td.X0 * a.p;
  const float inv_s = 1.0f / static_cast<float>(a.s);
  const int sH = a.s * a.H, sW = a.s * a.W;
  const int iy = iy0 + ty, ix = ix0 + 4 * tx;

  // source coordinate of fine pixel f (same arithmetic for rows and columns)
  auto src = [&](int f, int n_coarse, int &ia, int &ib, float &w1) {
    const float sc = (static_cast<float>(f) + 0.5f) * inv_s - 0.5f;
    const float fl = floorf(sc);
    w1 = sc - fl;
    const int i0 = static_cast<int>(fl);
    ia = min(max(i0, 0), n_coarse - 1);
    ib = min(max(i0 + 1, 0), n_coarse - 1);
  };
  // first coarse row / column of the window: the clamped lower neighbour of the first fine row / column
  int oy, ox;
  {
    int ib_;
    float w_;
    src(fy0 - 1, box_ch, oy, ib_, w_);
    src(fx0 - 1, box_cw, ox, ib_, w_);
  }
  if (t < WY) {
    const int fy = fy0 + t - 1;
    int ia, ib;
    float w1;
    src(fy, box_ch, ia, ib, w1);
    row_a[t] = min(ia - oy, cwh - 1);
    row_b[t] = min(ib - oy, cwh - 1);
    row_w[t] = w1;
    row_m[t] = (fy >= 0 && fy < box_fh) ? 1 : 0;
  } else if (t >= 64 && t < 64 + WX) {
    const int wx = t - 64, fx = fx0 + wx - 1;
    int ia, ib;
    float w1;
    src(fx, box_cw, ia, ib, w1);
    col_a[wx] = min(ia - ox, cww - 1);
    col_b[wx] = min(ib - ox, cww - 1);
    col_w[wx] = w1;
    col_m[wx] = (fx >= 0 && fx < box_fw) ? 1 : 0;
  }
  const bool one_pass = a.ci_chunk >= a.C;       // the whole input window fits: load it once

  // 4 pixels of one patch row: aligned 16-byte load and store
  const bool vec4 = iy < ih && a.ps % 4 == 0 && sW % 4 == 0 && ix + 3 < iw;
  for (int co0 = 0; co0 < a.C; co0 += CO) {
    float4 pv[CO];
    // ---- Z: the variables mixed on the coarse window, per tap
    for (int ci0 = 0; ci0 < a.C; ci0 += a.ci_chunk) {
      const int nci = min(a.ci_chunk, a.C - ci0);
      __syncthreads();                           // previous users of Xw / Ws / Z / T are done (and the tables are written)
      if (!one_pass || co0 == 0) {
        for (int idx = t; idx < nci * npx; idx += 256) {
          const int ci = idx / npx, r = idx % npx;
          const int wy = r / cww, wx = r % cww;
          const float *xp = a.x + (static_cast<size_t>(b) * a.V + a.out_var_idx[ci0 + ci]) * a.H * a.W;
          const int y = min(oy + wy, box_ch - 1), x = min(ox + wx, box_cw - 1);
          Xw[idx] = xp[static_cast<size_t>(cy_org + y) * a.W + cx_org + x];
        }
      }
      for (int idx = t; idx < nci * 9 * CO; idx += 256) {
        const int o = idx % CO, tap = (idx / CO) % 9, ci = idx / (9 * CO);
        Ws[idx] = (co0 + o < a.C) ? a.w_res[(static_cast<size_t>(co0 + o) * a.C + ci0 + ci) * 9 + tap] : 0.f;
      }
      __syncthreads();
      // The head projection of this thread's pixels is requested now, behind the window's own loads
      // (vector-memory results are waited for in issue order): it arrives while the window is worked on.
      if (vec4 && ci0 == 0) {
        const int py = td.y0 + iy / a.ps, i = iy % a.ps, px = td.x0 + ix / a.ps, j = ix % a.ps;
        const float *pp = a.P + (static_cast<size_t>(b) * a.N + static_cast<size_t>(py) * a.Wp + px) * a.head_out + static_cast<size_t>(i) * a.ps + j;
#pragma unroll
        for (int o = 0; o < CO; ++o)
          if (co0 + o < a.C) pv[o] = *reinterpret_cast<const float4 *>(pp + static_cast<size_t>(co0 + o) * a.ps * a.ps);
      }
      for (int item = t; item < 9 * npx; item += 256) {
        const int px = item % npx, tap = item / npx;
        float z[CO];
#pragma unroll
        for (int o = 0; o < CO; ++o) z[o] = 0.f;
        for (int ci = 0; ci < nci; ++ci) {
          const float xv = Xw[ci * npx + px];
          const float *wp = Ws + (ci * 9 + tap) * CO;
#pragma unroll
          for (int o = 0; o < CO; ++o) z[o] = fmaf(wp[o], xv, z[o]);
        }
#pragma unroll
        for (int o = 0; o < CO; ++o) {
          float *zp = Z + (tap * CO + o) * npx + px;
          *zp = ci0 == 0 ? z[o] : *zp + z[o];
        }
      }
    }
    __syncthreads();
    // ---- T: rows interpolated, the three row taps added up
    for (int item = t; item < 3 * BY * cww; item += 256) {
      const int X = item % cww, fy = (item / cww) % BY, dx = item / (cww * BY);
      float acc[CO];
#pragma unroll
      for (int o = 0; o < CO; ++o) acc[o] = 0.f;
#pragma unroll
      for (int dy = 0; dy < 3; ++dy) {
        const int r = fy + dy;
        if (row_m[r]) {
          const float w1 = row_w[r], w0 = 1.0f - w1;
          const float *za = Z + (dy * 3 + dx) * CO * npx + row_a[r] * cww + X;
          const float *zb = Z + (dy * 3 + dx) * CO * npx + row_b[r] * cww + X;
#pragma unroll
          for (int o = 0; o < CO; ++o) acc[o] += za[o * npx] * w0 + zb[o * npx] * w1;
        }
      }
#pragma unroll
      for (int o = 0; o < CO; ++o) T[((dx * CO + o) * BY + fy) * cww + X] = acc[o];
    }
    __syncthreads();
    // ---- R: columns interpolated, the three column taps added up; 4 adjacent pixels per thread
    float acc[CO][4];
#pragma unroll
    for (int o = 0; o < CO; ++o) {
      const float bv = (co0 + o < a.C) ? a.b_res[co0 + o] : 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) acc[o][k] = bv;
    }
    {
      int ca[6], cb[6];
      float cw1[6];
      bool cm[6];
#pragma unroll
      for (int j = 0; j < 6; ++j) {
        const int wx = 4 * tx + j;
        ca[j] = col_a[wx]; cb[j] = col_b[wx]; cw1[j] = col_w[wx]; cm[j] = col_m[wx] != 0;
      }
      if constexpr (NARROW) {
        // weight of coarse column X0 + q in fine window column j (clamped neighbours add up)
        const int X0 = min(ca[0], cww - 3);
        float e[6][3];
#pragma unroll
        for (int j = 0; j < 6; ++j)
#pragma unroll
          for (int q = 0; q < 3; ++q) {
            const float v = (ca[j] - X0 == q ? 1.0f - cw1[j] : 0.f) + (cb[j] - X0 == q ? cw1[j] : 0.f);
            e[j][q] = cm[j] ? v : 0.f;
          }
#pragma unroll
        for (int dx = 0; dx < 3; ++dx)
#pragma unroll
          for (int o = 0; o < CO; ++o) {
            const float *tp = T + ((dx * CO + o) * BY + ty) * cww + X0;
            const float t0 = tp[0], t1 = tp[1], t2 = tp[2];
#pragma unroll
            for (int k = 0; k < 4; ++k)
              acc[o][k] = fmaf(e[k + dx][0], t0, fmaf(e[k + dx][1], t1, fmaf(e[k + dx][2], t2, acc[o][k])));
          }
      } else {
#pragma unroll
        for (int dx = 0; dx < 3; ++dx)
#pragma unroll
          for (int o = 0; o < CO; ++o) {
            const float *tp = T + ((dx * CO + o) * BY + ty) * cww;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              const int j = k + dx;
              const float v = tp[ca[j]] * (1.0f - cw1[j]) + tp[cb[j]] * cw1[j];
              acc[o][k] += cm[j] ? v : 0.f;
            }
          }
      }
    }
    if (iy < ih) {
      const int gy = td.y0 * a.ps + iy;
      const int py = td.y0 + iy / a.ps, i = iy % a.ps;
      if (vec4) {
        float *yp = a.y + (static_cast<size_t>(b) * a.C * sH + gy) * sW + td.x0 * a.ps + ix;
#pragma unroll
        for (int o = 0; o < CO; ++o) {
          const int c = co0 + o;
          if (c < a.C)
            *reinterpret_cast<float4 *>(yp + static_cast<size_t>(c) * sH * sW) =
                make_float4(pv[o].x + acc[o][0], pv[o].y + acc[o][1], pv[o].z + acc[o][2], pv[o].w + acc[o][3]);
        }
      } else {
#pragma unroll
        for (int o = 0; o < CO; ++o) {
          const int c = co0 + o;
          if (c >= a.C) break;
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const int ixk = ix + k;
            if (ixk < iw) {
              const int px = td.x0 + ixk / a.ps, j = ixk % a.ps;
              const size_t n = static_cast<size_t>(py) * a.Wp + px;
              const float pv = a.P[(static_cast<size_t>(b) * a.N + n) * a.head_out + (static_cast<size_t>(c) * a.ps + i) * a.ps + j];
              a.y[((static_cast<size_t>(b) * a.C + c) * sH + gy) * sW + td.x0 * a.ps + ixk] = pv + acc[o][k];
            }
          }
        }
      }
    }
  }
}

// LDS floats of one work-group for CO output variables per pass and ci input variables per window pass
static size_t residual_lds_floats(int co, int ci, int cwh, int cww) {
  const size_t npx = static_cast<size_t>(cwh) * cww;
  return ci * npx + static_cast<size_t>(ci) * 9 * co + 9 * co * npx + 3 * static_cast<size_t>(co) * 16 * cww;
}

hipError_t residual_init() {
  hipError_t e = hipSuccess;
  const int lim = 160 * 1024;
#define RESLIM_ATTR(K) if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void *>(&K), hipFuncAttributeMaxDynamicSharedMemorySize, lim - 2048)
  RESLIM_ATTR((residual_unpatchify_kernel<8, true>));
  RESLIM_ATTR((residual_unpatchify_kernel<4, true>));
  RESLIM_ATTR((residual_unpatchify_kernel<2, true>));
  RESLIM_ATTR((residual_unpatchify_kernel<1, true>));
  RESLIM_ATTR((residual_unpatchify_kernel<8, false>));
  RESLIM_ATTR((residual_unpatchify_kernel<4, false>));
  RESLIM_ATTR((residual_unpatchify_kernel<2, false>));
  RESLIM_ATTR((residual_unpatchify_kernel<1, false>));
#undef RESLIM_ATTR
  return e;
}

hipError_t launch_residual_unpatchify(const reslim_ctx *c, const float *x, const void *P, int p_is_act, float *y,
                                      int batch, hipStream_t st) {
  (void)p_is_act;
  ResArgs a;
  a.x = x; a.P = static_cast<const float *>(P); a.y = y; a.tiles = c->d_tiles;
  a.w_res = c->d_w_res; a.b_res = c->d_b_res; a.out_var_idx = c->d_out_var_idx;
  a.V = c->cfg.in_vars; a.C = c->cfg.out_vars; a.H = c->cfg.H; a.W = c->cfg.W; a.s = c->cfg.scale;
  a.p = c->cfg.patch; a.ps = c->ps; a.Wp = c->Wp; a.N = c->N; a.head_out = c->head_out;
  int max_ih = 0, max_iw = 0;
  for (const tile_desc &t : c->tiles) {
    max_ih = std::max(max_ih, (t.y1 - t.y0) * c->ps);
    max_iw = std::max(max_iw, (t.x1 - t.x0) * c->ps);
  }
  a.nbx = (max_iw + 63) / 64;
  const int nby = (max_ih + 15) / 16;
  if (c->T > 65535 || batch > 65535) return hipErrorInvalidValue;
  // a block's 18 x 66 fine neighbourhood touches at most this many coarse rows / columns
  a.cwh = 17 / a.s + 3;
  a.cww = 65 / a.s + 3;
  // output variables per pass (CO) and input variables per window pass: the widest CO whose
  // buffers leave room for three, else two, else one work-group per compute unit
  int co = 0;
  a.ci_chunk = 0;
  const size_t fixed_lds = 1024;                         // the tables
  for (size_t budget : {size_t(52) << 10, size_t(78) << 10, size_t(156) << 10}) {
    for (int cand : {8, 4, 2, 1}) {
      if (cand > 1 && cand >= 2 * a.C) continue;         // e.g. C = 3 takes CO = 4, C = 2 takes CO = 2
      const size_t base = residual_lds_floats(cand, 0, a.cwh, a.cww) * 4 + fixed_lds;
      const size_t per_ci = (residual_lds_floats(cand, 1, a.cwh, a.cww) - residual_lds_floats(cand, 0, a.cwh, a.cww)) * 4;
      const int want = std::min(a.C, 4);
      if (base + per_ci * want > budget) continue;
      co = cand;
      a.ci_chunk = static_cast<int>(std::min<size_t>(a.C, (budget - base) / per_ci));
      break;
    }
    if (co) break;
  }
  if (!co) return hipErrorInvalidValue;
  const size_t lds = residual_lds_floats(co, a.ci_chunk, a.cwh, a.cww) * sizeof(float);
  const dim3 grid(a.nbx * nby, c->T, batch), blk(256);
  // scale >= 5: six consecutive fine columns span at most one coarse cell width; scale 4: block
  // origins are multiples of 4 fine columns inside the box, which gives the same bound
  const bool narrow = a.s >= 5 || (a.s == 4 && a.ps % 4 == 0);
  if (narrow) {
    switch (co) {
      case 8: residual_unpatchify_kernel<8, true><<<grid, blk, lds, st>>>(a); break;
      case 4: residual_unpatchify_kernel<4, true><<<grid, blk, lds, st>>>(a); break;
      case 2: residual_unpatchify_kernel<2, true><<<grid, blk, lds, st>>>(a); break;
      default: residual_unpatchify_kernel<1, true><<<grid, blk, lds, st>>>(a); break;
    }
  } else {
    switch (co) {
      case 8: residual_unpatchify_kernel<8, false><<<grid, blk, lds, st>>>(a); break;
      case 4: residual_unpatchify_kernel<4, false><<<grid, blk, lds, st>>>(a); break;
      case 2: residual_unpatchify_kernel<2, false><<<grid, blk, lds, st>>>(a); break;
      default: residual_unpatchify_kernel<1, false><<<grid, blk, lds, st>>>(a); break;
    }
  }
  return hipGetLastError();
}

}  // namespace reslim

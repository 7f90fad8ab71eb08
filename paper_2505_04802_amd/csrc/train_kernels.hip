// Bandwidth-bound kernels of the block's gradient (training of the model of ORBIT-2
// Sec. 4.1; the paper prints no formulas, these are the chain rule through the
// forward kernels of elementwise.hip and the GEMM epilogues):
//   layernorm_bwd   gradient of the per-token normalisation + partial sums of d gamma, d beta
//   gelu_fwd/bwd    exact (erf) GELU and its derivative, element by element
//   colsum          column sums of an activation gradient = gradient of a bias
//   partial_reduce  fixed-order sum of per-work-group partial rows (deterministic)
//   to_act          fp32 -> activation type
//   transpose       weight [out, in] -> [in, out], once, for the input-gradient GEMMs
#include "common.h"

namespace reslim {

template <class T> struct Vec4;     // four consecutive activation elements
template <> struct Vec4<float> {
  static __device__ __forceinline__ float4 load(const float *p) { return *reinterpret_cast<const float4 *>(p); }
  static __device__ __forceinline__ void store(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
};
template <> struct Vec4<bf16_t> {
  static __device__ __forceinline__ float4 load(const bf16_t *p) {
    const uint2 r = *reinterpret_cast<const uint2 *>(p);
    return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u), __uint_as_float(r.y << 16),
                       __uint_as_float(r.y & 0xffff0000u));
  }
  static __device__ __forceinline__ void store(bf16_t *p, float4 v) {
    uint2 r;
    r.x = pack_bf16x2(v.x, v.y);
    r.y = pack_bf16x2(v.z, v.w);
    *reinterpret_cast<uint2 *>(p) = r;
  }
};

// ------------------------------------------------------------------ LayerNorm gradient
// y = xh * gamma + beta, xh = (x - mean) / sigma.  With g = gamma * dy and means over the row:
//   dx = (g - mean(g) - xh * mean(g * xh)) / sigma,   d gamma = sum_rows dy * xh,   d beta = sum_rows dy.
// One wave per row as in the forward kernel (statistics recomputed from x, the row stays in
// registers); a work-group owns a contiguous slab of rows, its four waves keep per-lane sums of
// dy*xh and dy over their rows, add them through LDS at the end and write ONE partial row pair;
// partial_reduce adds the slabs in a fixed order.
//   dx_out = res + dx (res optional: the gradient arriving over the skip connection)
//   act_out (optional) = dx_out rounded to the activation type (operand of the next GEMMs)
template <class T, int NV>
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(const float *__restrict__ x, const T *__restrict__ dy,
                                                            const float *__restrict__ g, const float *__restrict__ res,
                                                            float *__restrict__ dx_out, T *__restrict__ act_out,
                                                            float *__restrict__ partial, int64_t rows, int rows_per_wg,
                                                            int D) {
  extern __shared__ float sm[];      // [2][D]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nv = D / 4;
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * rows_per_wg;
  const int64_t r1 = r0 + rows_per_wg < rows ? r0 + rows_per_wg : rows;
  const float4 *g4 = reinterpret_cast<const float4 *>(g);
  float4 gam[NV], sg[NV], sb[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int k = lane + 64 * i;
    gam[i] = k < nv ? g4[k] : make_float4(0.f, 0.f, 0.f, 0.f);
    sg[i] = sb[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  const float inv_d = 1.0f / static_cast<float>(D);
  for (int64_t row = r0 + wave; row < r1; row += 4) {
    const float4 *xr = reinterpret_cast<const float4 *>(x + row * D);
    float4 v[NV], d[NV];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int k = lane + 64 * i;
      v[i] = k < nv ? xr[k] : make_float4(0.f, 0.f, 0.f, 0.f);
      d[i] = k < nv ? Vec4<T>::load(dy + row * D + 4 * k) : make_float4(0.f, 0.f, 0.f, 0.f);
      sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    const float mean = sum * inv_d;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int k = lane + 64 * i;
      if (k < nv) {
        v[i].x -= mean; v[i].y -= mean; v[i].z -= mean; v[i].w -= mean;
        sq += (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
    const float rstd = rsqrtf(sq * inv_d + 1e-5f);
    float m1 = 0.f, m2 = 0.f;      // sums of g and g * xh
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      v[i].x *= rstd; v[i].y *= rstd; v[i].z *= rstd; v[i].w *= rstd;      // xh
      sg[i].x += d[i].x * v[i].x; sg[i].y += d[i].y * v[i].y; sg[i].z += d[i].z * v[i].z; sg[i].w += d[i].w * v[i].w;
      sb[i].x += d[i].x; sb[i].y += d[i].y; sb[i].z += d[i].z; sb[i].w += d[i].w;
      d[i].x *= gam[i].x; d[i].y *= gam[i].y; d[i].z *= gam[i].z; d[i].w *= gam[i].w;  // g
      m1 += (d[i].x + d[i].y) + (d[i].z + d[i].w);
      m2 += (d[i].x * v[i].x + d[i].y * v[i].y) + (d[i].z * v[i].z + d[i].w * v[i].w);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      m1 += __shfl_xor(m1, o);
      m2 += __shfl_xor(m2, o);
    }
    m1 *= inv_d;
    m2 *= inv_d;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int k = lane + 64 * i;
      if (k < nv) {
        float4 o4;
        o4.x = (d[i].x - m1 - v[i].x * m2) * rstd;
        o4.y = (d[i].y - m1 - v[i].y * m2) * rstd;
        o4.z = (d[i].z - m1 - v[i].z * m2) * rstd;
        o4.w = (d[i].w - m1 - v[i].w * m2) * rstd;
        if (res) {
          const float4 rr = reinterpret_cast<const float4 *>(res + row * D)[k];
          o4.x += rr.x; o4.y += rr.y; o4.z += rr.z; o4.w += rr.w;
        }
        reinterpret_cast<float4 *>(dx_out + row * D)[k] = o4;
        if (act_out) Vec4<T>::store(act_out + row * D + 4 * k, o4);
      }
    }
  }
  // waves 1, 2, 3 hand their sums to wave 0 one after the other (fixed order) through one row pair
  float4 *box = reinterpret_cast<float4 *>(sm);
  for (int w = 1; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int k = lane + 64 * i;
        if (k < nv) {
          box[k] = sg[i];
          box[nv + k] = sb[i];
        }
      }
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int k = lane + 64 * i;
        if (k < nv) {
          const float4 oa = box[k], ob = box[nv + k];
          sg[i].x += oa.x; sg[i].y += oa.y; sg[i].z += oa.z; sg[i].w += oa.w;
          sb[i].x += ob.x; sb[i].y += ob.y; sb[i].z += ob.z; sb[i].w += ob.w;
        }
      }
    }
    __syncthreads();
  }
  if (wave == 0) {
    float4 *pg = reinterpret_cast<float4 *>(partial + static_cast<size_t>(blockIdx.x) * 2 * D);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int k = lane + 64 * i;
      if (k < nv) {
        pg[k] = sg[i];
        pg[nv + k] = sb[i];
      }
    }
  }
}

// Sum of one value per thread over the 256 threads of a work-group, in a fixed order, the same in
// every thread.  box: four floats of LDS that no other reduction still in flight uses.
__device__ __forceinline__ float wg_sum(float v, float *box, int lane, int wave) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  if (lane == 0) box[wave] = v;
  __syncthreads();
  return (box[0] + box[1]) + (box[2] + box[3]);
}

// The same gradient for wide rows (D above 2048), where one wave can no longer keep a row, its
// gradient and the column sums in registers: the whole work-group takes one row at a time, thread t
// owns the float4 columns t, t + 256, ... and keeps their sums of dy*xh and dy over the slab's rows,
// so the partial row pair is written straight from registers.  The four reductions of a row use
// four boxes in turn; a box is written again only after three later barriers.
template <class T, int NVT>
__global__ __launch_bounds__(256) void layernorm_bwd_wide_kernel(const float *__restrict__ x, const T *__restrict__ dy,
                                                                 const float *__restrict__ g, const float *__restrict__ res,
                                                                 float *__restrict__ dx_out, T *__restrict__ act_out,
                                                                 float *__restrict__ partial, int64_t rows,
                                                                 int rows_per_wg, int D) {
  __shared__ float box[4][4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nv = D / 4;
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * rows_per_wg;
  const int64_t r1 = r0 + rows_per_wg < rows ? r0 + rows_per_wg : rows;
  const float4 *g4 = reinterpret_cast<const float4 *>(g);
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 gam[NVT], sg[NVT], sb[NVT];
#pragma unroll
  for (int i = 0; i < NVT; ++i) {
    const int k = static_cast<int>(threadIdx.x) + 256 * i;
    gam[i] = k < nv ? g4[k] : zero;
    sg[i] = sb[i] = zero;
  }
  const float inv_d = 1.0f / static_cast<float>(D);
  for (int64_t row = r0; row < r1; ++row) {
    const float4 *xr = reinterpret_cast<const float4 *>(x + row * D);
    float4 v[NVT], d[NVT];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NVT; ++i) {
      const int k = static_cast<int>(threadIdx.x) + 256 * i;
      v[i] = k < nv ? xr[k] : zero;
      d[i] = k < nv ? Vec4<T>::load(dy + row * D + 4 * k) : zero;
      sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    }
    const float mean = wg_sum(sum, box[0], lane, wave) * inv_d;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < NVT; ++i) {
      const int k = static_cast<int>(threadIdx.x) + 256 * i;
      if (k < nv) {
        v[i].x -= mean; v[i].y -= mean; v[i].z -= mean; v[i].w -= mean;
        sq += (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
      }
    }
    const float rstd = rsqrtf(wg_sum(sq, box[1], lane, wave) * inv_d + 1e-5f);
    float m1 = 0.f, m2 = 0.f;      // sums of g and g * xh
#pragma unroll
    for (int i = 0; i < NVT; ++i) {
      v[i].x *= rstd; v[i].y *= rstd; v[i].z *= rstd; v[i].w *= rstd;      // xh
      sg[i].x += d[i].x * v[i].x; sg[i].y += d[i].y * v[i].y; sg[i].z += d[i].z * v[i].z; sg[i].w += d[i].w * v[i].w;
      sb[i].x += d[i].x; sb[i].y += d[i].y; sb[i].z += d[i].z; sb[i].w += d[i].w;
      d[i].x *= gam[i].x; d[i].y *= gam[i].y; d[i].z *= gam[i].z; d[i].w *= gam[i].w;  // g
      m1 += (d[i].x + d[i].y) + (d[i].z + d[i].w);
      m2 += (d[i].x * v[i].x + d[i].y * v[i].y) + (d[i].z * v[i].z + d[i].w * v[i].w);
    }
    m1 = wg_sum(m1, box[2], lane, wave) * inv_d;
    m2 = wg_sum(m2, box[3], lane, wave) * inv_d;
#pragma unroll
    for (int i = 0; i < NVT; ++i) {
      const int k = static_cast<int>(threadIdx.x) + 256 * i;
      if (k < nv) {
        float4 o4;
        o4.x = (d[i].x - m1 - v[i].x * m2) * rstd;
        o4.y = (d[i].y - m1 - v[i].y * m2) * rstd;
        o4.z = (d[i].z - m1 - v[i].z * m2) * rstd;
        o4.w = (d[i].w - m1 - v[i].w * m2) * rstd;
        if (res) {
          const float4 rr = reinterpret_cast<const float4 *>(res + row * D)[k];
          o4.x += rr.x; o4.y += rr.y; o4.z += rr.z; o4.w += rr.w;
        }
        reinterpret_cast<float4 *>(dx_out + row * D)[k] = o4;
        if (act_out) Vec4<T>::store(act_out + row * D + 4 * k, o4);
      }
    }
  }
  float4 *pg = reinterpret_cast<float4 *>(partial + static_cast<size_t>(blockIdx.x) * 2 * D);
#pragma unroll
  for (int i = 0; i < NVT; ++i) {
    const int k = static_cast<int>(threadIdx.x) + 256 * i;
    if (k < nv) {
      pg[k] = sg[i];
      pg[nv + k] = sb[i];
    }
  }
}

// out[j] = sum over p < n_part of partial[p * stride + j] in a fixed order (deterministic); columns
// from `split` on go to out2[j - split] (two results that share partial rows, one launch).
// A work-group owns 32 columns; its NG row groups each add every NG-th partial row (four
// independent running sums per thread keep loads in flight), then the groups are added in order.
// NG = 32 (1024 threads) where there are few columns and many partial rows: column sums of
// activations have 16 .. 64 column blocks, far too few work-groups to hide the latency of 1024
// dependent row loads behind one another (c1: 14 us per launch with NG = 8).
template <int NG>
__global__ __launch_bounds__(NG * 32) void partial_reduce_kernel(const float *__restrict__ partial, float *__restrict__ out,
                                                                 float *__restrict__ out2, int64_t split, int n_part,
                                                                 int64_t stride, int64_t n) {
  __shared__ float sm[NG][32];
  const int col = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const int64_t j = static_cast<int64_t>(blockIdx.x) * 32 + col;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  if (j < n) {
    int p = grp;
    for (; p + 3 * NG < n_part; p += 4 * NG) {
      a0 += partial[p * stride + j];
      a1 += partial[(p + NG) * stride + j];
      a2 += partial[(p + 2 * NG) * stride + j];
      a3 += partial[(p + 3 * NG) * stride + j];
    }
    for (; p < n_part; p += NG) a0 += partial[p * stride + j];
  }
  sm[grp][col] = (a0 + a1) + (a2 + a3);
  __syncthreads();
  if (grp == 0 && j < n) {
    float acc = sm[0][col];
#pragma unroll
    for (int g = 1; g < NG; ++g) acc += sm[g][col];
    if (j < split) out[j] = acc;
    else out2[j - split] = acc;
  }
}

// Few partial rows, many columns (the split-K slices of a weight gradient): a thread owns four
// adjacent columns and adds the rows in order, 16-byte loads, no LDS.
__global__ __launch_bounds__(256) void partial_reduce_wide_kernel(const float4 *__restrict__ partial, float4 *__restrict__ out,
                                                                  int n_part, int64_t stride4, int64_t n4) {
  const int64_t j = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (j >= n4) return;
  float4 acc = partial[j];
  int p = 1;
  for (; p + 3 < n_part; p += 4) {           // four loads in flight, added in row order
    const float4 v0 = partial[p * stride4 + j], v1 = partial[(p + 1) * stride4 + j];
    const float4 v2 = partial[(p + 2) * stride4 + j], v3 = partial[(p + 3) * stride4 + j];
    acc.x += v0.x; acc.y += v0.y; acc.z += v0.z; acc.w += v0.w;
    acc.x += v1.x; acc.y += v1.y; acc.z += v1.z; acc.w += v1.w;
    acc.x += v2.x; acc.y += v2.y; acc.z += v2.z; acc.w += v2.w;
    acc.x += v3.x; acc.y += v3.y; acc.z += v3.z; acc.w += v3.w;
  }
  for (; p < n_part; ++p) {
    const float4 v = partial[p * stride4 + j];
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  out[j] = acc;
}

// out2 / split: see the kernel; pass nullptr / n for a single result
static hipError_t launch_partial_reduce2(const float *partial, float *out, float *out2, int64_t split, int n_part,
                                         int64_t stride, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  const int64_t blocks = (n + 31) / 32;
  if (blocks > INT32_MAX) return hipErrorInvalidValue;
  if (!out2 && n_part >= 1 && n_part <= 64 && n >= 65536 && n % 4 == 0 && stride % 4 == 0 &&
      reinterpret_cast<uintptr_t>(partial) % 16 == 0 && reinterpret_cast<uintptr_t>(out) % 16 == 0) {
    const int64_t n4 = n / 4;
    partial_reduce_wide_kernel<<<dim3(static_cast<unsigned>((n4 + 255) / 256)), dim3(256), 0, st>>>(
        reinterpret_cast<const float4 *>(partial), reinterpret_cast<float4 *>(out), n_part, stride / 4, n4);
    return hipGetLastError();
  }
  if (blocks < 512 && n_part >= 128)
    partial_reduce_kernel<32><<<dim3(static_cast<unsigned>(blocks)), dim3(1024), 0, st>>>(partial, out, out2, split, n_part, stride, n);
  else
    partial_reduce_kernel<8><<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st>>>(partial, out, out2, split, n_part, stride, n);
  return hipGetLastError();
}

hipError_t launch_partial_reduce(const float *partial, float *out, int n_part, int64_t stride, int64_t n, hipStream_t st) {
  return launch_partial_reduce2(partial, out, nullptr, n, n_part, stride, n, st);
}

// rows of 64 float4 from which the work-group-per-row kernel takes over (D above 1024 .. 2048)
constexpr int kLnBwdWideFrom = 5;

int layernorm_bwd_slabs(int64_t rows) { return static_cast<int>(rows < 4096 ? (rows + 3) / 4 : 1024); }

template <class T>
static hipError_t launch_ln_bwd_t(const float *x, const void *dy, const float *g, const float *res, float *dx_out,
                                  void *act_out, float *partial, float *dgamma, float *dbeta, int64_t rows, int D,
                                  hipStream_t st) {
  const int nv = (D / 4 + 63) / 64;
  int n_wg = layernorm_bwd_slabs(rows);
  const int rpw = static_cast<int>((rows + n_wg - 1) / n_wg);
  n_wg = static_cast<int>((rows + rpw - 1) / rpw);
  const size_t lds = static_cast<size_t>(2) * D * sizeof(float);
  const dim3 grid(n_wg), blk(256);
  const T *d = static_cast<const T *>(dy);
  T *ao = static_cast<T *>(act_out);
#define RESLIM_LNB(NV) layernorm_bwd_kernel<T, NV><<<grid, blk, lds, st>>>(x, d, g, res, dx_out, ao, partial, rows, rpw, D)
#define RESLIM_LNW(NVT) layernorm_bwd_wide_kernel<T, NVT><<<grid, blk, 0, st>>>(x, d, g, res, dx_out, ao, partial, rows, rpw, D)
  if (nv <= 1) RESLIM_LNB(1);
  else if (nv <= 2) RESLIM_LNB(2);
  else if (nv <= 4) RESLIM_LNB(4);
  else if (nv < kLnBwdWideFrom) RESLIM_LNB(8);
  else if (nv <= 8) RESLIM_LNW(2);        // a work-group per row from here on: thread t owns columns t, t + 256, ...
  else if (nv <= 16) RESLIM_LNW(4);
  else if (nv <= 32) RESLIM_LNW(8);
  else if (nv <= 64) RESLIM_LNW(16);
  else return hipErrorInvalidValue;       // D above 16384
#undef RESLIM_LNB
#undef RESLIM_LNW
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // partial rows are [d gamma | d beta] pairs of 2 D floats
  return launch_partial_reduce2(partial, dgamma, dbeta, D, n_wg, 2 * static_cast<int64_t>(D), 2 * static_cast<int64_t>(D), st);
}

// partial: dev float, at least layernorm_bwd_slabs(rows) * 2 * D elements
hipError_t launch_layernorm_bwd(int dtype, const float *x, const void *dy, const float *g, const float *res,
                                float *dx_out, void *act_out, float *partial, float *dgamma, float *dbeta,
                                int64_t rows, int D, hipStream_t st) {
  if (D % 4 != 0 || rows <= 0) return hipErrorInvalidValue;
  return dtype == RESLIM_BF16 ? launch_ln_bwd_t<bf16_t>(x, dy, g, res, dx_out, act_out, partial, dgamma, dbeta, rows, D, st)
                              : launch_ln_bwd_t<float>(x, dy, g, res, dx_out, act_out, partial, dgamma, dbeta, rows, D, st);
}

// ------------------------------------------------------------------ GELU, element by element
__device__ __forceinline__ float gelu_f(float v) { return 0.5f * v * (1.0f + erff(v * 0.70710678118654752f)); }
// d/dv [v Phi(v)] = Phi(v) + v phi(v)
__device__ __forceinline__ float gelu_grad_f(float v) {
  return 0.5f * (1.0f + erff(v * 0.70710678118654752f)) + v * 0.3989422804014327f * __expf(-0.5f * v * v);
}

// BWD = false: out = gelu(h).   BWD = true: out = dy * gelu'(h).
template <class T, bool BWD>
__global__ __launch_bounds__(256) void gelu_kernel(const T *__restrict__ h, const T *__restrict__ dy, T *__restrict__ out,
                                                   int64_t n4) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n4) return;
  const float4 v = Vec4<T>::load(h + 4 * i);
  float4 o;
  if constexpr (BWD) {
    const float4 d = Vec4<T>::load(dy + 4 * i);
    o = make_float4(d.x * gelu_grad_f(v.x), d.y * gelu_grad_f(v.y), d.z * gelu_grad_f(v.z), d.w * gelu_grad_f(v.w));
  } else {
    o = make_float4(gelu_f(v.x), gelu_f(v.y), gelu_f(v.z), gelu_f(v.w));
  }
  Vec4<T>::store(out + 4 * i, o);
}

hipError_t launch_gelu(int dtype, bool bwd, const void *h, const void *dy, void *out, int64_t n, hipStream_t st) {
  if (n % 4 != 0) return hipErrorInvalidValue;
  const int64_t n4 = n / 4, blocks = (n4 + 255) / 256;
  if (blocks < 1) return hipSuccess;
  if (blocks > INT32_MAX) return hipErrorInvalidValue;
  const dim3 grid(static_cast<unsigned>(blocks)), blk(256);
  if (dtype == RESLIM_BF16) {
    if (bwd) gelu_kernel<bf16_t, true><<<grid, blk, 0, st>>>(static_cast<const bf16_t *>(h), static_cast<const bf16_t *>(dy), static_cast<bf16_t *>(out), n4);
    else gelu_kernel<bf16_t, false><<<grid, blk, 0, st>>>(static_cast<const bf16_t *>(h), nullptr, static_cast<bf16_t *>(out), n4);
  } else {
    if (bwd) gelu_kernel<float, true><<<grid, blk, 0, st>>>(static_cast<const float *>(h), static_cast<const float *>(dy), static_cast<float *>(out), n4);
    else gelu_kernel<float, false><<<grid, blk, 0, st>>>(static_cast<const float *>(h), nullptr, static_cast<float *>(out), n4);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------ fp32 -> activation type
template <class T>
__global__ __launch_bounds__(256) void to_act_kernel(const float *__restrict__ src, T *__restrict__ dst, int64_t n4) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n4) Vec4<T>::store(dst + 4 * i, reinterpret_cast<const float4 *>(src)[i]);
}

hipError_t launch_to_act(int dtype, const float *src, void *dst, int64_t n, hipStream_t st) {
  if (n % 4 != 0) return hipErrorInvalidValue;
  const int64_t n4 = n / 4, blocks = (n4 + 255) / 256;
  if (blocks < 1) return hipSuccess;
  if (blocks > INT32_MAX) return hipErrorInvalidValue;
  if (dtype == RESLIM_BF16) to_act_kernel<bf16_t><<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st>>>(src, static_cast<bf16_t *>(dst), n4);
  else to_act_kernel<float><<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st>>>(src, static_cast<float *>(dst), n4);
  return hipGetLastError();
}

// ------------------------------------------------------------------ column sums (bias gradient)
// A thread owns 16 bytes of columns (8 bfloat16 or 4 float); TPR threads cover a row segment of
// up to 256 * 16 bytes (grid.x segments), the 256 / TPR row lanes of a work-group take the rows
// of the work-group's slab (grid.y) in turn and are added through LDS in a fixed order.
template <class T>
__global__ __launch_bounds__(256) void colsum_kernel(const T *__restrict__ a, float *__restrict__ partial, int64_t rows,
                                                     int rows_per_slab, int N, int tpr) {
  constexpr int VEC = 16 / sizeof(T);
  __shared__ float sm[256 * VEC];
  const int cg = threadIdx.x % tpr, rl = threadIdx.x / tpr, nrl = 256 / tpr;
  const int c = (blockIdx.x * tpr + cg) * VEC;
  const int64_t r0 = static_cast<int64_t>(blockIdx.y) * rows_per_slab;
  const int64_t r1 = r0 + rows_per_slab < rows ? r0 + rows_per_slab : rows;
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
  if (c < N) {
    for (int64_t r = r0 + rl; r < r1; r += nrl) {
      const uint4 raw = *reinterpret_cast<const uint4 *>(a + r * N + c);
      if constexpr (sizeof(T) == 2) {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[2 * e] += __uint_as_float(w[e] << 16);
          acc[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u);
        }
      } else {
        acc[0] += __uint_as_float(raw.x); acc[1] += __uint_as_float(raw.y);
        acc[2] += __uint_as_float(raw.z); acc[3] += __uint_as_float(raw.w);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) sm[threadIdx.x * VEC + e] = acc[e];
  __syncthreads();
  if (rl == 0 && c < N) {
    for (int g = 1; g < nrl; ++g)
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] += sm[(g * tpr + cg) * VEC + e];
#pragma unroll
    for (int e = 0; e < VEC; ++e) partial[static_cast<size_t>(blockIdx.y) * N + c + e] = acc[e];
  }
}

int colsum_slabs(int64_t rows) { return static_cast<int>(rows < 32 * 1024 ? (rows + 31) / 32 : 1024); }

// partial: dev float, at least colsum_slabs(rows) * N elements
hipError_t launch_colsum(int dtype, const void *a, float *partial, float *out, int64_t rows, int N, hipStream_t st) {
  const int vec = dtype == RESLIM_BF16 ? 8 : 4;
  if (N % vec != 0 || rows <= 0) return hipErrorInvalidValue;
  int slabs = colsum_slabs(rows);
  const int rps = static_cast<int>((rows + slabs - 1) / slabs);
  slabs = static_cast<int>((rows + rps - 1) / rps);
  int tpr = 256;                               // threads per row segment: a power of two <= 256 covering N / vec
  while (tpr > 1 && tpr / 2 >= N / vec) tpr /= 2;
  const dim3 grid((N / vec + tpr - 1) / tpr, slabs), blk(256);
  if (dtype == RESLIM_BF16) colsum_kernel<bf16_t><<<grid, blk, 0, st>>>(static_cast<const bf16_t *>(a), partial, rows, rps, N, tpr);
  else colsum_kernel<float><<<grid, blk, 0, st>>>(static_cast<const float *>(a), partial, rows, rps, N, tpr);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_partial_reduce(partial, out, slabs, N, N, st);
}

// ------------------------------------------------------------------ gradient unscaling (dynamic gradient scaling)
// Up to 12 tensors in one launch (blockIdx.y = tensor): every element times inv_scale, and *flag set
// to 1 when any element is not finite.  The flag is only ever written with 1 (plain vector stores of
// the same value from several lanes): the caller clears it before the first call of a step.
struct UnscaleArgs {
  float *p[12];
  int64_t n[12];
  int count;
};
__global__ __launch_bounds__(256) void unscale_check_kernel(UnscaleArgs a, float inv_scale, int32_t *flag) {
  const int which = blockIdx.y;
  float *p = a.p[which];
  const int64_t n = a.n[which];
  bool bad = false;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n; i += static_cast<int64_t>(gridDim.x) * 256) {
    const float v = p[i] * inv_scale;
    bad |= !(fabsf(v) <= 3.402823466e38f);      // inf or NaN
    p[i] = v;
  }
  if (bad) *flag = 1;
}

hipError_t launch_unscale_check(float *const *ptrs, const int64_t *sizes, int count, float inv_scale, int32_t *flag,
                                hipStream_t st) {
  if (count < 1 || count > 12) return hipErrorInvalidValue;
  UnscaleArgs a;
  int64_t mx = 0;
  for (int i = 0; i < 12; ++i) {
    a.p[i] = i < count ? ptrs[i] : nullptr;
    a.n[i] = i < count ? sizes[i] : 0;
    if (a.n[i] > mx) mx = a.n[i];
  }
  a.count = count;
  int64_t blocks = (mx + 256 * 8 - 1) / (256 * 8);         // about eight elements per thread in the largest tensor
  blocks = blocks < 1 ? 1 : (blocks > 4096 ? 4096 : blocks);
  unscale_check_kernel<<<dim3(static_cast<unsigned>(blocks), count), dim3(256), 0, st>>>(a, inv_scale, flag);
  return hipGetLastError();
}

// ------------------------------------------------------------------ weight transpose (once per context)
template <class T>
__global__ __launch_bounds__(256) void transpose_kernel(const T *__restrict__ src, T *__restrict__ dst, int R, int C) {
  __shared__ T tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 32 x 8
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  for (int j = ty; j < 32; j += 8)
    if (r0 + j < R && c0 + tx < C) tile[j][tx] = src[static_cast<size_t>(r0 + j) * C + c0 + tx];
  __syncthreads();
  for (int j = ty; j < 32; j += 8)
    if (c0 + j < C && r0 + tx < R) dst[static_cast<size_t>(c0 + j) * R + r0 + tx] = tile[tx][j];
}

// dst[C, R] = src[R, C]^T
hipError_t launch_transpose(int dtype, const void *src, void *dst, int R, int C, hipStream_t st) {
  const dim3 grid((C + 31) / 32, (R + 31) / 32), blk(256);
  if (dtype == RESLIM_BF16) transpose_kernel<bf16_t><<<grid, blk, 0, st>>>(static_cast<const bf16_t *>(src), static_cast<bf16_t *>(dst), R, C);
  else transpose_kernel<float><<<grid, blk, 0, st>>>(static_cast<const float *>(src), static_cast<float *>(dst), R, C);
  return hipGetLastError();
}

}  // namespace reslim

// Bayesian training loss, forward value (ORBIT-2 Sec. 4.1, "Bayesian Training Loss"):
//     || y - x ||_D^2  +  sum_k sum_i sum_{j in C(i)} b_ij | x_ki - x_kj |
// with x the prediction, y the target, D the latitude weights (one per pixel row,
// supplied by the caller), C(i) the 8 nearest pixels clipped at the domain edge and
// b_ij = (1 / distance) / (4 + 4 / sqrt 2).  Both terms are means over all pixel
// values; the prior carries the caller's weight.
//
// One bandwidth-bound pass.  A work-group owns a strip of 8 rows x 1024 columns of
// one (sample, variable) plane; a thread owns 4 adjacent columns and walks down the
// rows keeping the next row's six prediction values (its 4 columns and one on each
// side) in registers, so every prediction row is read once per strip (plus one
// overlap row) and the target once.  Each unordered neighbour pair is visited once
// (east, south-west, south, south-east) and counted twice.  Per-thread sums are fp32
// over at most 32 pixels, everything above that is accumulated in fp64: wave
// shuffle, LDS across waves, one partial per work-group, and a second one-group
// kernel that adds the partials in a fixed order (deterministic result).
#include "common.h"

#include <mutex>

namespace reslim {

constexpr int LOSS_ROWS = 8, LOSS_COLS = 1024;

struct LossArgs {
  const float *pred, *target, *lat_w;
  double *partial;          // [2 * groups]
  int Hf, Wf;
  int strips_x, strips_y;   // strips per plane
};

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__global__ __launch_bounds__(256) void bayes_loss_partial_kernel(LossArgs a) {
  __shared__ double red[2][4];
  const int t = threadIdx.x;
  const int sx = blockIdx.x % a.strips_x, sy = blockIdx.x / a.strips_x;
  const size_t plane = static_cast<size_t>(blockIdx.y) * a.Hf * a.Wf;
  const float *xp = a.pred + plane, *yp = a.target + plane;
  const int c0 = sx * LOSS_COLS + 4 * t;
  const int r_begin = sy * LOSS_ROWS, r_end = min(r_begin + LOSS_ROWS, a.Hf);
  const int Wf = a.Wf;
  float data = 0.f, ax = 0.f, dg = 0.f;       // squared error; axial and diagonal absolute differences
  if (c0 < Wf) {
    // six prediction values of a row: columns c0-1 .. c0+4, clamped into the row (masked where used)
    const bool vec = (Wf & 3) == 0;            // rows are 16-byte aligned and a thread's 4 columns lie inside
    auto load6 = [&](int r, float (&v)[6]) {
      const float *row = xp + static_cast<size_t>(r) * Wf;
      if (vec) {
        const float4 own = *reinterpret_cast<const float4 *>(row + c0);
        v[0] = row[max(c0 - 1, 0)];
        v[1] = own.x; v[2] = own.y; v[3] = own.z; v[4] = own.w;
        v[5] = row[min(c0 + 4, Wf - 1)];
      } else {
#pragma unroll
        for (int i = 0; i < 6; ++i) v[i] = row[min(max(c0 - 1 + i, 0), Wf - 1)];
      }
    };
    float cur[6], nxt[6] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    load6(r_begin, cur);
    for (int r = r_begin; r < r_end; ++r) {
      const bool has_next = r + 1 < a.Hf;      // uniform
      if (has_next) load6(r + 1, nxt);
      const float *trow = yp + static_cast<size_t>(r) * Wf;
      const float lw = a.lat_w[r];
      float tv[4];
      if (vec) {
        const float4 t4 = *reinterpret_cast<const float4 *>(trow + c0);
        tv[0] = t4.x; tv[1] = t4.y; tv[2] = t4.z; tv[3] = t4.w;
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) tv[k] = trow[min(c0 + k, Wf - 1)];
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int c = c0 + k;
        if (c < Wf) {
          const float x = cur[k + 1];
          const float d = tv[k] - x;
          data = fmaf(lw * d, d, data);
          if (c + 1 < Wf) ax += fabsf(x - cur[k + 2]);
          if (has_next) {
            ax += fabsf(x - nxt[k + 1]);
            if (c > 0) dg += fabsf(x - nxt[k]);
            if (c + 1 < Wf) dg += fabsf(x - nxt[k + 2]);
          }
        }
      }
#pragma unroll
      for (int i = 0; i < 6; ++i) cur[i] = nxt[i];
    }
  }
  // ordered pairs: every unordered pair twice; b_axial = 1 / (4 + 4/sqrt 2), b_diag = b_axial / sqrt 2
  const double norm = 4.0 + 4.0 / 1.4142135623730951;
  double dsum = wave_sum(static_cast<double>(data));
  double psum = wave_sum(2.0 * (static_cast<double>(ax) + static_cast<double>(dg) / 1.4142135623730951) / norm);
  const int lane = t & 63, wave = t >> 6;
  if (lane == 0) { red[0][wave] = dsum; red[1][wave] = psum; }
  __syncthreads();
  if (t == 0) {
    const size_t g = static_cast<size_t>(blockIdx.y) * gridDim.x + blockIdx.x;
    a.partial[2 * g] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
    a.partial[2 * g + 1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
  }
}

__global__ __launch_bounds__(256) void bayes_loss_final_kernel(const double *partial, size_t groups, double count,
                                                               double tv_weight, double *out3) {
  __shared__ double red[2][4];
  const int t = threadIdx.x;
  double d = 0.0, p = 0.0;
  for (size_t g = t; g < groups; g += 256) { d += partial[2 * g]; p += partial[2 * g + 1]; }
  d = wave_sum(d);
  p = wave_sum(p);
  if ((t & 63) == 0) { red[0][t >> 6] = d; red[1][t >> 6] = p; }
  __syncthreads();
  if (t == 0) {
    const double data = ((red[0][0] + red[0][1]) + (red[0][2] + red[0][3])) / count;
    const double prior = tv_weight * ((red[1][0] + red[1][1]) + (red[1][2] + red[1][3])) / count;
    out3[0] = data + prior;
    out3[1] = data;
    out3[2] = prior;
  }
}

// Partial sums of the entry point that allocates nothing: a fixed array in the code object's own
// device memory (each GPU that loads the library holds its own copy until the process ends).
// In host code this name is only a handle for hipGetSymbolAddress, never a device address.
constexpr size_t LOSS_STATIC_MAX_GROUPS = size_t(1) << 18;     // 4 MiB of doubles
static __device__ __align__(256) double scratch[2 * LOSS_STATIC_MAX_GROUPS];

constexpr int LOSS_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static double *g_scratch_ptr[LOSS_MAX_DEVICES];          // device address of `scratch`, per device

// Device address of the current device's copy of `scratch`; asked for once per device.
static int loss_scratch_ptr(double **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= LOSS_MAX_DEVICES) return RESLIM_EHIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RESLIM_EHIP;
    g_scratch_ptr[dev] = static_cast<double *>(p);
  }
  *out = g_scratch_ptr[dev];
  return RESLIM_OK;
}

static bool loss_shape(int batch, int vars, int Hf, int Wf, int64_t *planes, int *sx, int *sy, size_t *groups) {
  if (batch < 1 || vars < 1 || Hf < 1 || Wf < 1) return false;
  *planes = static_cast<int64_t>(batch) * vars;
  *sx = (Wf + LOSS_COLS - 1) / LOSS_COLS;
  *sy = (Hf + LOSS_ROWS - 1) / LOSS_ROWS;
  if (*planes > 65535 || static_cast<int64_t>(*sx) * *sy > INT32_MAX) return false;
  *groups = static_cast<size_t>(*planes) * *sx * *sy;
  return true;
}

}  // namespace reslim

extern "C" int reslim_bayes_loss_workspace_bytes(int32_t batch, int32_t vars, int32_t Hf, int32_t Wf, size_t *out) {
  int64_t planes;
  int sx, sy;
  size_t groups;
  if (!out || !reslim::loss_shape(batch, vars, Hf, Wf, &planes, &sx, &sy, &groups)) return RESLIM_EINVAL;
  *out = 2 * groups * sizeof(double);
  return RESLIM_OK;
}

namespace reslim {

// The two launches shared by both entry points; `partial` is a device address with room for 2 * groups doubles.
static int loss_launch(const float *pred, const float *target, const float *lat_w, int64_t planes, int Hf, int Wf, int sx,
                       int sy, size_t groups, float tv_weight, double *out3, double *partial, hipStream_t st) {
  LossArgs a;
  a.pred = pred; a.target = target; a.lat_w = lat_w;
  a.partial = partial;
  a.Hf = Hf; a.Wf = Wf; a.strips_x = sx; a.strips_y = sy;
  bayes_loss_partial_kernel<<<dim3(static_cast<unsigned>(sx * sy), static_cast<unsigned>(planes)), dim3(256), 0, st>>>(a);
  if (hipGetLastError() != hipSuccess) return RESLIM_EHIP;
  const double count = static_cast<double>(planes) * Hf * Wf;
  bayes_loss_final_kernel<<<dim3(1), dim3(256), 0, st>>>(partial, groups, count, static_cast<double>(tv_weight), out3);
  return hipGetLastError() == hipSuccess ? RESLIM_OK : RESLIM_EHIP;
}

}  // namespace reslim

extern "C" int reslim_bayes_loss_fwd(const float *pred, const float *target, const float *lat_w, int32_t batch,
                                     int32_t vars, int32_t Hf, int32_t Wf, float tv_weight, double *out3,
                                     void *workspace, size_t ws_bytes, void *hip_stream) {
  int64_t planes;
  int sx, sy;
  size_t groups;
  if (!pred || !target || !lat_w || !out3 || !workspace) return RESLIM_EINVAL;
  if (!reslim::loss_shape(batch, vars, Hf, Wf, &planes, &sx, &sy, &groups)) return RESLIM_EINVAL;
  if (ws_bytes < 2 * groups * sizeof(double)) return RESLIM_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 8 || reinterpret_cast<uintptr_t>(out3) % 8) return RESLIM_EINVAL;
  return reslim::loss_launch(pred, target, lat_w, planes, Hf, Wf, sx, sy, groups, tv_weight, out3,
                             static_cast<double *>(workspace), static_cast<hipStream_t>(hip_stream));
}

extern "C" int reslim_bayes_loss_static_max_groups(int64_t *out) {
  if (!out) return RESLIM_EINVAL;
  *out = static_cast<int64_t>(reslim::LOSS_STATIC_MAX_GROUPS);
  return RESLIM_OK;
}

extern "C" int reslim_bayes_loss_fwd_static(const float *pred, const float *target, const float *lat_w, int32_t batch,
                                            int32_t vars, int32_t Hf, int32_t Wf, float tv_weight, double *out3,
                                            void *hip_stream) {
  int64_t planes;
  int sx, sy;
  size_t groups;
  if (!pred || !target || !lat_w || !out3) return RESLIM_EINVAL;
  if (!reslim::loss_shape(batch, vars, Hf, Wf, &planes, &sx, &sy, &groups)) return RESLIM_EINVAL;
  if (groups > reslim::LOSS_STATIC_MAX_GROUPS) return RESLIM_EWORKSPACE;       // beyond the fixed array
  if (reinterpret_cast<uintptr_t>(out3) % 8) return RESLIM_EINVAL;
  double *partial = nullptr;
  const int rc = reslim::loss_scratch_ptr(&partial);
  if (rc != RESLIM_OK) return rc;
  // every partial the final kernel reads is written by the first kernel of this call: nothing to clear
  return reslim::loss_launch(pred, target, lat_w, planes, Hf, Wf, sx, sy, groups, tv_weight, out3, partial,
                             static_cast<hipStream_t>(hip_stream));
}

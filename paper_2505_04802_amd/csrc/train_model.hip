// Gradients of the whole model for one training step (ORBIT-2 Sec. 4.1 architecture and Bayesian
// training loss, Sec. 4.2 tiling, Sec. 5: the model is trained; Sec. 4.4: bf16 with gradient
// scaling).  The paper prints no gradient formula: everything here is the chain rule through the
// forward operations, walked backwards.  The blocks' gradient lives in backward.hip; this file
// holds the two ends of the model and the chaining:
//   loss            d_y = S (2 D (y - t) / n + 2 lambda / n sum_j b_ij sign(y_i - y_j)),  sign(0) = 0
//   back end        un-patchify transposed, head GEMM (input / weight / bias gradient), residual
//                   path (gradient of the 3x3 convolution's weights and bias), final LayerNorm on
//                   the interior tokens, zero gradient for the halo rows (their outputs are dropped)
//   front end       gather transposed (a patch adds up the gradients of its halo copies), position
//                   and resolution rows, output map of the aggregation, and the folded
//                   tokenisation + aggregation: gradients of the folded tables first (sums over
//                   tokens), then the chain rule through the fold to the unfolded parameters
// Mixed precision as in the block gradient: gradients that feed a GEMM are rounded to the
// activation type, sums are fp32, parameter gradients are fp32 and WRITTEN in a fixed summation
// order (deterministic).
#include <type_traits>
#include <algorithm>
#include <cmath>
#include <string>
#include <vector>

#include "common.h"

namespace reslim {

hipError_t launch_partial_reduce(const float *partial, float *out, int n_part, int64_t stride, int64_t n, hipStream_t st);

// ------------------------------------------------------------------ loss gradient
__global__ __launch_bounds__(256) void bayes_loss_bwd_kernel(const float *__restrict__ pred, const float *__restrict__ target,
                                                             const float *__restrict__ lat_w, float *__restrict__ d_pred,
                                                             int Hf, int Wf, float data_f, float tv_f) {
  // one thread per pixel, rows of a plane along blockIdx.y, planes along blockIdx.z
  const int c = blockIdx.x * 256 + threadIdx.x, r = blockIdx.y;
  if (c >= Wf) return;
  const size_t plane = static_cast<size_t>(blockIdx.z) * Hf * Wf;
  const float *xp = pred + plane;
  const float x = xp[static_cast<size_t>(r) * Wf + c];
  float ax = 0.f, dg = 0.f;                      // sums of signs towards the axial / diagonal neighbours
  auto sgn = [](float v) { return static_cast<float>((v > 0.f) - (v < 0.f)); };
#pragma unroll
  for (int dy = -1; dy <= 1; ++dy)
#pragma unroll
    for (int dx = -1; dx <= 1; ++dx) {
      if (dy == 0 && dx == 0) continue;
      const int rr = r + dy, cc = c + dx;
      if (rr < 0 || rr >= Hf || cc < 0 || cc >= Wf) continue;
      const float s = sgn(x - xp[static_cast<size_t>(rr) * Wf + cc]);
      if (dy == 0 || dx == 0) ax += s; else dg += s;
    }
  const float t = target[plane + static_cast<size_t>(r) * Wf + c];
  d_pred[plane + static_cast<size_t>(r) * Wf + c] = data_f * lat_w[r] * (x - t) + tv_f * (ax + dg * 0.70710678118654752440f);
}

// The same for row lengths that are multiples of four: a thread owns four neighbouring columns and
// walks down RB rows with the three rows it needs in registers, so a pixel costs a quarter of a
// 16-byte load and half a 4-byte load of the prediction instead of nine 4-byte loads (c3: 9.2 ms
// with one thread per pixel).  A neighbour outside the plane is held as NaN: every comparison with
// it is false, so its sign term is zero, which is what leaving it out means.  The sums of signs are
// small integers, exact in any order.
template <int RB>
__global__ __launch_bounds__(256) void bayes_loss_bwd4_kernel(const float *__restrict__ pred, const float *__restrict__ target,
                                                              const float *__restrict__ lat_w, float *__restrict__ d_pred,
                                                              int Hf, int Wf, float data_f, float tv_f) {
  const int c0 = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c0 >= Wf) return;
  const size_t plane = static_cast<size_t>(blockIdx.z) * Hf * Wf;
  const float *xp = pred + plane;
  const int r_begin = blockIdx.y * RB, r_end = min(Hf, r_begin + RB);
  const float out_of_plane = __builtin_nanf("");
  auto sgn = [](float v) { return static_cast<float>((v > 0.f) - (v < 0.f)); };
  auto load_row = [&](int r, float (&v)[6]) {      // columns c0 - 1 .. c0 + 4 of row r
    if (r < 0 || r >= Hf) {
#pragma unroll
      for (int k = 0; k < 6; ++k) v[k] = out_of_plane;
      return;
    }
    const float *row = xp + static_cast<size_t>(r) * Wf;
    const float4 m = *reinterpret_cast<const float4 *>(row + c0);
    v[1] = m.x; v[2] = m.y; v[3] = m.z; v[4] = m.w;
    v[0] = c0 > 0 ? row[c0 - 1] : out_of_plane;
    v[5] = c0 + 4 < Wf ? row[c0 + 4] : out_of_plane;
  };
  float up[6], mid[6], dn[6];
  load_row(r_begin - 1, up);
  load_row(r_begin, mid);
#pragma unroll
  for (int i = 0; i < RB; ++i) {
    const int r = r_begin + i;
    if (r >= r_end) break;
    load_row(r + 1, dn);
    const size_t at = plane + static_cast<size_t>(r) * Wf + c0;
    const float4 t4 = *reinterpret_cast<const float4 *>(target + at);
    const float t[4] = {t4.x, t4.y, t4.z, t4.w};
    const float lw = data_f * lat_w[r];
    float o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float x = mid[k + 1];
      const float ax = sgn(x - up[k + 1]) + sgn(x - dn[k + 1]) + sgn(x - mid[k]) + sgn(x - mid[k + 2]);
      const float dg = sgn(x - up[k]) + sgn(x - up[k + 2]) + sgn(x - dn[k]) + sgn(x - dn[k + 2]);
      o[k] = lw * (x - t[k]) + tv_f * (ax + dg * 0.70710678118654752440f);
    }
    *reinterpret_cast<float4 *>(d_pred + at) = make_float4(o[0], o[1], o[2], o[3]);
#pragma unroll
    for (int k = 0; k < 6; ++k) { up[k] = mid[k]; mid[k] = dn[k]; }
  }
}

// ------------------------------------------------------------------ back end
// d_P[b, n, (c, i, j)] = d_y[b, c, py ps + i, px ps + j]  (transpose of un-patchify), stored as activation type
template <typename T>
__global__ __launch_bounds__(256) void patchify_act_kernel(const float *__restrict__ dy, T *__restrict__ dP, int64_t total,
                                                           int N, int Wp, int C, int ps, int sH, int sW) {
  const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (e >= total) return;
  const int ho = C * ps * ps;
  const int64_t bn = e / ho;
  const int rem = static_cast<int>(e % ho);
  const int c = rem / (ps * ps), i = (rem / ps) % ps, j = rem % ps;
  const int64_t b = bn / N;
  const int n = static_cast<int>(bn % N), py = n / Wp, px = n % Wp;
  Act<T>::store(dP + e, dy[((b * C + c) * sH + py * ps + i) * sW + px * ps + j]);
}

// The same for patch sides that are multiples of four: a thread moves four neighbours of a fine row.
// Threads run over (four pixels, four patches side by side, patch row) fastest, so a wave reads
// whole 128-byte lines of a fine row and writes 128 contiguous bytes of each of its four patches.
template <typename T>
__global__ __launch_bounds__(256) void patchify_act4_kernel(const float *__restrict__ dy, T *__restrict__ dP, int64_t total4,
                                                            int Hp, int Wp, int C, int ps, int sH, int sW) {
  int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (e >= total4) return;
  const int q = ps / 4, wq = (Wp + 3) / 4;
  const int j4 = static_cast<int>(e % q); e /= q;
  const int pxl = static_cast<int>(e % 4); e /= 4;
  const int i = static_cast<int>(e % ps); e /= ps;
  const int c = static_cast<int>(e % C); e /= C;
  const int pxh = static_cast<int>(e % wq); e /= wq;
  const int py = static_cast<int>(e % Hp);
  const int64_t b = e / Hp;
  const int px = pxh * 4 + pxl;
  if (px >= Wp) return;
  const float4 v = *reinterpret_cast<const float4 *>(dy + ((b * C + c) * sH + py * ps + i) * sW + px * ps + 4 * j4);
  T *o = dP + ((b * Hp + py) * static_cast<int64_t>(Wp) + px) * (static_cast<int64_t>(C) * ps * ps) + (c * ps + i) * ps + 4 * j4;
  if constexpr (std::is_same<T, float>::value) {
    *reinterpret_cast<float4 *>(o) = v;
  } else {
    const uint32_t lo = static_cast<uint32_t>(f32_to_bf16(v.x)) | (static_cast<uint32_t>(f32_to_bf16(v.y)) << 16);
    const uint32_t hi = static_cast<uint32_t>(f32_to_bf16(v.z)) | (static_cast<uint32_t>(f32_to_bf16(v.w)) << 16);
    *reinterpret_cast<uint2 *>(o) = make_uint2(lo, hi);
  }
}

// rows of the tile-major stream: an interior token takes its row of src[b, patch], a halo copy zero
__global__ __launch_bounds__(256) void scatter_interior_kernel(const float *__restrict__ src, const int32_t *__restrict__ gather,
                                                               const int32_t *__restrict__ interior_src, float *__restrict__ dst,
                                                               int64_t rows, int64_t n_h, int N, int D) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int64_t b = row / n_h;
  const int r = static_cast<int>(row % n_h);
  const int g = gather[r];
  const bool own = interior_src[g] == r;
  const float4 *in = reinterpret_cast<const float4 *>(src + (b * N + g) * D);
  float4 *out = reinterpret_cast<float4 *>(dst + row * D);
  for (int d = lane; d < D / 4; d += 64) out[d] = own ? in[d] : make_float4(0.f, 0.f, 0.f, 0.f);
}

// Gradient of the residual path's 3x3 convolution (weights and bias).  The forward evaluates
// R = b + sum over taps (dy, dx) and inputs i of w[o][i][dy][dx] U_i(r + dy, c + dx), U_i the bilinear
// upsampling of input i on the tile's haloed box (neighbours clamped to the box, zero outside it).
// U is linear in the coarse pixels, so with G_o the upstream gradient on a block of fine pixels
//   dw[o][i][dy][dx] = sum_{r,c} G_o(r, c) U_i(r + dy, c + dx) = sum_{Y,X} x_i(Y, X) Q[o][dy][dx](Y, X),
//   Q[o][dy][dx](Y, X) = sum_{r,c} G_o(r, c) RW[dy](Y, r) CW[dx](X, c),
// where RW[dy](Y, r) is the weight with which coarse row Y enters fine row r + dy (two non-zeros per
// fine row, zero for rows outside the box) and CW the same for columns: the upsampling transposed,
// rows first (P = RW G), then columns (Q = P CW^T), then one small product with the coarse window.
// That is 9 (C + about 2) multiply-adds per coarse-window pixel and output plus about 12 per fine pixel
// and output, instead of 9 C per fine pixel and output for the product with U written out, in fp32
// throughout.
//
// A work-group walks over 16 x 64 blocks of fine pixels (every block of every tile interior of every
// sample, dealt out in turn), CO = 4 OPT outputs per pass.  Row step: a thread owns one fine column
// and OPT outputs; for each coarse row it runs over the fine rows that touch it.  Column step: one
// thread per value of Q, over the fine columns that touch its coarse column.  Last step: one thread
// per (output, input) pair, nine sums over the window, added to the pair's accumulators in LDS (one
// owner per accumulator: a fixed order, no atomics).  One partial row of 9 C C + C sums per
// work-group; a fixed-order reduction follows.
struct ResGradArgs {
  const float *x, *dy;
  float *partial;
  const tile_desc *tiles;
  const int32_t *out_var_idx;
  int V, C, H, W, s, p, ps;
  int nbx, nby, T, batch;
  int cwh, cww;
};

constexpr size_t kResGradLds = 150 * 1024;        // dynamic LDS the kernel may ask for
// floats of dynamic LDS for CO outputs per pass
static size_t residual_wgrad_lds_floats(int C, int CO, int cwh, int cww) {
  const size_t npx = static_cast<size_t>(cwh) * cww;
  const size_t gq = std::max<size_t>(static_cast<size_t>(CO) * 16 * 64, (static_cast<size_t>(CO) * 9 * npx + 3) / 4 * 4);
  return gq + static_cast<size_t>(CO) * 3 * cwh * 64 + 3 * cwh * 16 + 3 * cww * 64 + C * npx + 9 * C * C + C + 6 * cww + 4;
}

// OPT: outputs per thread in the row step (CO = 4 OPT per pass).  NIT: the column step covers 4 NIT
// fine columns from the first one that touches a coarse column (a coarse column is touched by fewer
// than 2 s + 1 fine columns); a block where some run is longer takes all 64 columns instead.
template <int OPT, int NIT>
__global__ __launch_bounds__(256) void residual_wgrad_kernel(ResGradArgs a) {
  constexpr int BY = 16, BX = 64, WY = BY + 2, WX = BX + 2, WXP = 68, CO = 4 * OPT;
  __shared__ float row_w[WY], col_w[WXP];
  __shared__ int row_a[WY], row_b[WY], row_m[WY], col_a[WXP], col_b[WXP], col_m[WXP];
  __shared__ int var_idx[64];
  __shared__ int long_run;
  extern __shared__ __align__(16) float dynr[];
  const int cwh = a.cwh, cww = a.cww, npx = cwh * cww, qw = 3 * cww;
  const int gq = max(CO * BY * BX, (CO * 9 * npx + 3) / 4 * 4);   // a multiple of four: P and CW are read 16 bytes at a time
  float *G = dynr;                                // [CO][BY][BX] upstream gradient of the block ...
  float *Q = dynr;                                // ... later [CO][3][cwh][3][cww] (G is no longer needed by then)
  float *P = dynr + gq;                           // [CO][3][cwh][BX]
  float *RW = P + CO * 3 * cwh * BX;              // [3][cwh][BY]
  float *CW = RW + 3 * cwh * BY;                  // [3][cww][BX]
  float *Cw = CW + 3 * cww * BX;                  // [C][npx] coarse window of the inputs
  float *acc = Cw + a.C * npx;                    // [9 C C + C] accumulators of this work-group
  int *xlo = reinterpret_cast<int *>(acc + 9 * a.C * a.C + a.C), *xhi = xlo + qw;     // [3][cww] fine columns that touch coarse column X under tap dx
  const int t = threadIdx.x, lane = t & 63, og = t >> 6;
  const int n_acc = 9 * a.C * a.C + a.C;
  for (int i = t; i < n_acc; i += 256) acc[i] = 0.f;
  if (t < a.C) var_idx[t] = a.out_var_idx[t];
  const float inv_s = 1.0f / static_cast<float>(a.s);
  const int sH = a.s * a.H, sW = a.s * a.W;
  const int64_t blocks = static_cast<int64_t>(a.nbx) * a.nby * a.T * a.batch;
  auto src = [&](int f, int n_coarse, int &ia, int &ib, float &w1) {
    const float sc = (static_cast<float>(f) + 0.5f) * inv_s - 0.5f;
    const float fl = floorf(sc);
    w1 = sc - fl;
    const int i0 = static_cast<int>(fl);
    ia = min(max(i0, 0), n_coarse - 1);
    ib = min(max(i0 + 1, 0), n_coarse - 1);
  };
  for (int64_t blk = blockIdx.x; blk < blocks; blk += gridDim.x) {     // uniform over the work-group
    const int bxy = static_cast<int>(blk % (a.nbx * a.nby));
    const int tile = static_cast<int>((blk / (a.nbx * a.nby)) % a.T);
    const int b = static_cast<int>(blk / (static_cast<int64_t>(a.nbx) * a.nby * a.T));
    const tile_desc td = a.tiles[tile];
    const int ih = (td.y1 - td.y0) * a.ps, iw = (td.x1 - td.x0) * a.ps;
    const int iy0 = (bxy / a.nbx) * BY, ix0 = (bxy % a.nbx) * BX;
    if (iy0 >= ih || ix0 >= iw) continue;
    const int fy0 = (td.y0 - td.Y0) * a.ps + iy0, fx0 = (td.x0 - td.X0) * a.ps + ix0;
    const int box_fh = (td.Y1 - td.Y0) * a.ps, box_fw = (td.X1 - td.X0) * a.ps;
    const int box_ch = (td.Y1 - td.Y0) * a.p, box_cw = (td.X1 - td.X0) * a.p;
    const int cy_org = td.Y0 * a.p, cx_org = td.X0 * a.p;
    int oy, ox;
    {
      int ib_;
      float w_;
      src(fy0 - 1, box_ch, oy, ib_, w_);
      src(fx0 - 1, box_cw, ox, ib_, w_);
    }
    __syncthreads();                              // the previous block's tables and arrays are no longer read
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
    if (t == 255) long_run = 0;
    if (t < qw) { xlo[t] = BX; xhi[t] = -1; }     // qw <= 3 * 68 < 256
    // coarse window of every input
    for (int idx = t; idx < a.C * npx; idx += 256) {
      const int ci = idx / npx, r = idx % npx;
      const int wy = r / cww, wx = r % cww;
      const float *xp = a.x + (static_cast<size_t>(b) * a.V + var_idx[ci]) * a.H * a.W;
      const int y = min(oy + wy, box_ch - 1), x = min(ox + wx, box_cw - 1);
      Cw[idx] = xp[static_cast<size_t>(cy_org + y) * a.W + cx_org + x];
    }
    __syncthreads();
    // transposed interpolation weights: RW[dy][Y][r] and CW[dx][X][c], window row r + dy / column c + dx
    for (int idx = t; idx < 3 * cwh * BY; idx += 256) {
      const int r = idx % BY, Y = (idx / BY) % cwh, dy = idx / (BY * cwh), wr = r + dy;
      const float w1 = row_w[wr];
      RW[idx] = row_m[wr] ? (row_a[wr] == Y ? 1.0f - w1 : 0.f) + (row_b[wr] == Y ? w1 : 0.f) : 0.f;
    }
    for (int idx = t; idx < 3 * cww * BX; idx += 256) {
      const int cc = idx % BX, e = idx / BX, X = e % cww, dx = e / cww, wc = cc + dx;
      const float w1 = col_w[wc];
      const float v = col_m[wc] ? (col_a[wc] == X ? 1.0f - w1 : 0.f) + (col_b[wc] == X ? w1 : 0.f) : 0.f;
      CW[idx] = v;
      if (v != 0.f) {
        atomicMin(&xlo[e], cc);
        atomicMax(&xhi[e], cc);
      }
    }
    __syncthreads();
    if (t < qw) {
      const int lo = min(xlo[t] & ~3, BX - 4 * NIT);            // 16-byte aligned start of the window of 4 NIT columns
      if (xhi[t] >= lo + 4 * NIT) long_run = 1;
      xlo[t] = lo;
    }
    for (int co0 = 0; co0 < a.C; co0 += CO) {
      const int nco = min(CO, a.C - co0);
      __syncthreads();                            // Q of the previous pass consumed (and the run tables written)
      // upstream gradient of the block, zero past the interior's edge and for outputs past the last
      for (int e = t; e < CO * BY * BX / 4; e += 256) {
        const int o = e / (BY * BX / 4), yy = (e / (BX / 4)) % BY, xx = 4 * (e % (BX / 4));
        const int iy = iy0 + yy, ix = ix0 + xx;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (o < nco && iy < ih) {
          const float *gp = a.dy + ((static_cast<size_t>(b) * a.C + co0 + o) * sH + td.y0 * a.ps + iy) * sW + td.x0 * a.ps + ix;
          if (ix + 3 < iw && (reinterpret_cast<uintptr_t>(gp) & 15) == 0) {
            v = *reinterpret_cast<const float4 *>(gp);
          } else {
            if (ix < iw) v.x = gp[0];
            if (ix + 1 < iw) v.y = gp[1];
            if (ix + 2 < iw) v.z = gp[2];
            if (ix + 3 < iw) v.w = gp[3];
          }
        }
        *reinterpret_cast<float4 *>(G + (o * BY + yy) * BX + xx) = v;
      }
      __syncthreads();
      // rows: P[o][dy][Y][c] = sum_r RW[dy][Y][r] G[o][r][c]; the bias gradient is the plain sum of G.
      // A thread keeps its column of G for its OPT outputs in registers over all coarse rows.
      {
        float gcol[OPT][BY], bs[OPT];
#pragma unroll
        for (int j = 0; j < OPT; ++j) {
          bs[j] = 0.f;
#pragma unroll
          for (int r = 0; r < BY; ++r) {
            gcol[j][r] = G[((og * OPT + j) * BY + r) * BX + lane];
            bs[j] += gcol[j][r];
          }
        }
        for (int Y = 0; Y < cwh; ++Y) {
          float s3[OPT][3];
#pragma unroll
          for (int j = 0; j < OPT; ++j) s3[j][0] = s3[j][1] = s3[j][2] = 0.f;
#pragma unroll
          for (int r = 0; r < BY; ++r) {
            const float c0 = RW[Y * BY + r], c1 = RW[(cwh + Y) * BY + r], c2 = RW[(2 * cwh + Y) * BY + r];
#pragma unroll
            for (int j = 0; j < OPT; ++j) {
              s3[j][0] = fmaf(gcol[j][r], c0, s3[j][0]);
              s3[j][1] = fmaf(gcol[j][r], c1, s3[j][1]);
              s3[j][2] = fmaf(gcol[j][r], c2, s3[j][2]);
            }
          }
#pragma unroll
          for (int j = 0; j < OPT; ++j)
#pragma unroll
            for (int d = 0; d < 3; ++d) P[(((og * OPT + j) * 3 + d) * cwh + Y) * BX + lane] = s3[j][d];
        }
        // a wave holds one group of OPT outputs: add its 64 columns, lane 0 owns the accumulators
#pragma unroll
        for (int j = 0; j < OPT; ++j) {
          float v = bs[j];
          for (int w = 1; w < 64; w <<= 1) v += __shfl_xor(v, w);
          if (lane == 0 && og * OPT + j < nco) acc[9 * a.C * a.C + co0 + og * OPT + j] += v;
        }
      }
      __syncthreads();                            // P written, G no longer read: Q may overwrite it
      // columns: Q[row = (o, dy, Y)][dx][X] = sum_c CW[dx][X][c] P[row][c] over the window of columns that
      // holds the run of (dx, X) (the weights outside a run are zero)
      {
        const int nrows = CO * 3 * cwh, rstep = 256 / qw;
        const int e = t % qw, r0 = t / qw;        // a thread keeps its (dx, X); threads past the last multiple of qw rest
        const bool whole = long_run != 0;         // uniform
        const float4 *cp = reinterpret_cast<const float4 *>(CW + e * BX);
        if (r0 < rstep && !whole) {
          const int lo4 = xlo[e] >> 2;
          float4 cw4[NIT];
#pragma unroll
          for (int i = 0; i < NIT; ++i) cw4[i] = cp[lo4 + i];
          for (int row = r0; row < nrows; row += rstep) {
            const float4 *pp = reinterpret_cast<const float4 *>(P + row * BX) + lo4;
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < NIT; ++i) {
              const float4 pv = pp[i];
              sum = fmaf(pv.x, cw4[i].x, sum);
              sum = fmaf(pv.y, cw4[i].y, sum);
              sum = fmaf(pv.z, cw4[i].z, sum);
              sum = fmaf(pv.w, cw4[i].w, sum);
            }
            Q[row * qw + e] = sum;
          }
        } else if (r0 < rstep) {
          for (int row = r0; row < nrows; row += rstep) {
            const float4 *pp = reinterpret_cast<const float4 *>(P + row * BX);
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < BX / 4; ++i) {
              const float4 pv = pp[i], cv = cp[i];
              sum = fmaf(pv.x, cv.x, sum);
              sum = fmaf(pv.y, cv.y, sum);
              sum = fmaf(pv.z, cv.z, sum);
              sum = fmaf(pv.w, cv.w, sum);
            }
            Q[row * qw + e] = sum;
          }
        }
      }
      __syncthreads();
      // window: dw[o][i][dy][dx] += sum_{Y,X} x_i(Y, X) Q[(o, dy, Y)][dx][X]
      for (int pr = t; pr < nco * a.C; pr += 256) {
        const int o = pr / a.C, ci = pr % a.C;
        const float *xw = Cw + ci * npx;
        float s9[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) s9[k] = 0.f;
        for (int Y = 0; Y < cwh; ++Y) {
          const float *q0 = Q + ((o * 3 + 0) * cwh + Y) * qw, *q1 = Q + ((o * 3 + 1) * cwh + Y) * qw, *q2 = Q + ((o * 3 + 2) * cwh + Y) * qw;
#pragma unroll 4
          for (int X = 0; X < cww; ++X) {
            const float xv = xw[Y * cww + X];
            s9[0] = fmaf(xv, q0[X], s9[0]); s9[1] = fmaf(xv, q0[cww + X], s9[1]); s9[2] = fmaf(xv, q0[2 * cww + X], s9[2]);
            s9[3] = fmaf(xv, q1[X], s9[3]); s9[4] = fmaf(xv, q1[cww + X], s9[4]); s9[5] = fmaf(xv, q1[2 * cww + X], s9[5]);
            s9[6] = fmaf(xv, q2[X], s9[6]); s9[7] = fmaf(xv, q2[cww + X], s9[7]); s9[8] = fmaf(xv, q2[2 * cww + X], s9[8]);
          }
        }
        float *ap = acc + ((co0 + o) * a.C + ci) * 9;
#pragma unroll
        for (int k = 0; k < 9; ++k) ap[k] += s9[k];
      }
    }
  }
  __syncthreads();
  for (int i = t; i < n_acc; i += 256) a.partial[static_cast<size_t>(blockIdx.x) * n_acc + i] = acc[i];
}

// ------------------------------------------------------------------ front end
// d_z[b, g, :] = sum over the tile-major copies of patch g (listed in increasing index: a fixed order)
template <typename T>
__global__ __launch_bounds__(256) void gather_transpose_kernel(const float *__restrict__ d_tok, const int32_t *__restrict__ off,
                                                               const int32_t *__restrict__ idx, float *__restrict__ d_z,
                                                               T *__restrict__ d_z_act, int64_t rows, int64_t n_h, int N, int D) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int64_t b = row / N;
  const int g = static_cast<int>(row % N);
  const int lo = off[g], hi = off[g + 1];
  for (int d = lane * 4; d < D; d += 256) {
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int k = lo; k < hi; ++k) {
      const float4 v = *reinterpret_cast<const float4 *>(d_tok + (b * n_h + idx[k]) * D + d);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    *reinterpret_cast<float4 *>(d_z + row * D + d) = s;
    T *o = d_z_act + row * D + d;
    Act<T>::store(o, s.x); Act<T>::store(o + 1, s.y); Act<T>::store(o + 2, s.z); Act<T>::store(o + 3, s.w);
  }
}

// out[n] = sum_b in[b * stride + n] (samples added in increasing order)
__global__ __launch_bounds__(256) void batch_sum_kernel(const float *__restrict__ in, float *__restrict__ out, int64_t n,
                                                        int64_t stride, int batch) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int b = 0; b < batch; ++b) s += in[b * stride + i];
  out[i] = s;
}

__global__ __launch_bounds__(256) void fill_kernel(float *p, int64_t n, float v) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

// Folded tokenisation + aggregation, backwards, first half: per token and head the softmax over
// the variables a[g, v] (recomputed as in the forward) and the gradient of its logits
//   d_s[g, v] = a[g, v] (d_a[g, v] - sum_v' a[g, v'] d_a[g, v']),  d_a[g, v] = sum_{d in head g} d_o[d] val[v, d],
//   val[v, d] = U[v, d, :] . pixels_v + c[v, d].
// The sums over the head's features do not depend on the pixels:
//   d_a[g, v] = sum_i pixels_v[i] E[(g, v, i)] + E[(g, v, p2)],  E[(g, v, j)] = sum_{d in head g} d_o[d] (U[v, d, j] | c[v, d]),
// so E = d_o W^T is one GEMM over all tokens with the block-structured table W[(g, v, j), d] (zero
// where d is outside head g: the matrix unit does heads times the needed products and is still far
// quicker than the vector units on the plain form), and this kernel only combines E with the pixels.
struct AggBwdArgs {
  const float *x, *A, *a0, *U, *c;
  const void *d_o;            // act [BN, D]
  const float *E;             // [BN, ne] rows (g, v, j), j <= p2
  float *a_out, *ds_out;      // [BN, heads, V]
  int V, H, W, p, Wp, N, D, heads, dh, ne;
  int64_t BN;
};

// W[(g * V + v) * (p2 + 1) + j][d] = U[v][d][j] (j < p2) or c[v][d] (j = p2) for d in head g, else 0; rows past the last: 0
template <typename T>
__global__ __launch_bounds__(256) void agg_value_table_kernel(const float *__restrict__ U, const float *__restrict__ cc, T *__restrict__ Wt,
                                                              int V, int D, int dh, int p2, int rows, int ne) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= static_cast<int64_t>(ne) * D) return;
  const int d = static_cast<int>(i % D), r = static_cast<int>(i / D);
  float val = 0.f;
  if (r < rows) {
    const int j = r % (p2 + 1), gv = r / (p2 + 1), v = gv % V, g = gv / V;
    if (d / dh == g) val = j < p2 ? U[(static_cast<size_t>(v) * D + d) * p2 + j] : cc[static_cast<size_t>(v) * D + d];
  }
  Act<T>::store(Wt + i, val);
}

template <int TP>
__global__ __launch_bounds__(256) void agg_scores_bwd_kernel(AggBwdArgs e) {
  extern __shared__ __align__(16) float smg[];
  const int p2 = e.p * e.p, VP2 = e.V * p2, HV = e.heads * e.V;
  float *pix = smg;                        // [TP][V*p2]
  float *sc = pix + TP * VP2;              // [TP][heads][V] softmax weights
  float *da = sc + TP * HV;                // [TP][heads][V]
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
      val = e.x[((b * e.V + v) * e.H + py * e.p + i / e.p) * e.W + px * e.p + i % e.p];
    }
    pix[idx] = val;
  }
  __syncthreads();
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
  // d_a[token, head, variable]: consecutive threads read consecutive (p2 + 1)-float groups of a row of E
  for (int idx = t; idx < TP * HV; idx += 256) {
    const int pi = idx / HV, gv = idx % HV, v = gv % e.V;
    const int64_t bn = bn0 + pi;
    float s = 0.f;
    if (bn < e.BN) {
      const float *er = e.E + bn * e.ne + static_cast<size_t>(gv) * (p2 + 1);
      const float *px = pix + pi * VP2 + v * p2;
      s = er[p2];
      for (int i = 0; i < p2; ++i) s = fmaf(px[i], er[i], s);
    }
    da[idx] = s;
  }
  __syncthreads();
  for (int idx = t; idx < TP * e.heads; idx += 256) {
    const int pi = idx / e.heads;
    const int64_t bn = bn0 + pi;
    if (bn >= e.BN) continue;
    const float *ar = sc + static_cast<size_t>(idx) * e.V, *dr = da + static_cast<size_t>(idx) * e.V;
    float dot = 0.f;
    for (int v = 0; v < e.V; ++v) dot = fmaf(ar[v], dr[v], dot);
    const int g = idx % e.heads;
    for (int v = 0; v < e.V; ++v) {
      const size_t o = (static_cast<size_t>(bn) * e.heads + g) * e.V + v;
      e.a_out[o] = ar[v];
      e.ds_out[o] = ar[v] * (dr[v] - dot);
    }
  }
}

// Second half: gradients of the folded value tables.  Grid (token slab, block of 256 features,
// chunk of VC variables); thread = one feature d, accumulators dU[v, d, 0..p2) and dc[v, d] for the
// chunk's variables in registers; tokens of the slab in increasing order.  P2 = p * p.
template <typename T, int P2, int VC>
__global__ __launch_bounds__(256) void agg_values_bwd_kernel(AggBwdArgs e, float *__restrict__ partial, int tokens_per_slab) {
  const int d = blockIdx.y * 256 + threadIdx.x;
  const int v0 = blockIdx.z * VC;
  const int64_t t0 = static_cast<int64_t>(blockIdx.x) * tokens_per_slab;
  const int64_t t1 = min(t0 + tokens_per_slab, e.BN);
  float acc[VC][P2 + 1];
#pragma unroll
  for (int v = 0; v < VC; ++v)
#pragma unroll
    for (int i = 0; i <= P2; ++i) acc[v][i] = 0.f;
  const T *dop = static_cast<const T *>(e.d_o);
  const int dc = min(d, e.D - 1), g = dc / e.dh;
  for (int64_t bn = t0; bn < t1; ++bn) {
    const float go = Act<T>::load(dop + bn * e.D + dc);
    const int64_t b = bn / e.N;
    const int n = static_cast<int>(bn % e.N);
    const int py = n / e.Wp, px = n % e.Wp;
    const float *ar = e.a_out + (static_cast<size_t>(bn) * e.heads + g) * e.V;
#pragma unroll
    for (int v = 0; v < VC; ++v) {
      const int vv = min(v0 + v, e.V - 1);
      const float w = ar[vv] * go;
      const float *xp = e.x + ((b * e.V + vv) * e.H + py * e.p) * e.W + px * e.p;
#pragma unroll
      for (int i = 0; i < P2; ++i) acc[v][i] = fmaf(w, xp[(i / e.p) * e.W + i % e.p], acc[v][i]);
      acc[v][P2] += w;
    }
  }
  if (d >= e.D) return;
  // partial row layout: [V][D][P2 + 1]
  float *out = partial + static_cast<size_t>(blockIdx.x) * e.V * e.D * (P2 + 1);
#pragma unroll
  for (int v = 0; v < VC; ++v)
    if (v0 + v < e.V)
#pragma unroll
      for (int i = 0; i <= P2; ++i) out[(static_cast<size_t>(v0 + v) * e.D + d) * (P2 + 1) + i] = acc[v][i];
}

// ... and of the folded score tables: thread = (variable, head), accumulators dA[v, g, 0..p2), da0[v, g]
__global__ __launch_bounds__(256) void agg_logits_bwd_kernel(AggBwdArgs e, float *__restrict__ partial, int tokens_per_slab) {
  const int p2 = e.p * e.p, HV = e.heads * e.V;
  const int64_t t0 = static_cast<int64_t>(blockIdx.x) * tokens_per_slab;
  const int64_t t1 = min(t0 + tokens_per_slab, e.BN);
  for (int item = threadIdx.x; item < HV; item += 256) {
    const int v = item / e.heads, g = item % e.heads;
    float acc[17];
    for (int i = 0; i <= p2; ++i) acc[i] = 0.f;
    for (int64_t bn = t0; bn < t1; ++bn) {
      const float ds = e.ds_out[(static_cast<size_t>(bn) * e.heads + g) * e.V + v];
      const int64_t b = bn / e.N;
      const int n = static_cast<int>(bn % e.N);
      const int py = n / e.Wp, px = n % e.Wp;
      const float *xp = e.x + ((b * e.V + v) * e.H + py * e.p) * e.W + px * e.p;
      for (int i = 0; i < p2; ++i) acc[i] = fmaf(ds, xp[(i / e.p) * e.W + i % e.p], acc[i]);
      acc[p2] += ds;
    }
    float *out = partial + (static_cast<size_t>(blockIdx.x) * HV + item) * (p2 + 1);
    for (int i = 0; i <= p2; ++i) out[i] = acc[i];
  }
}

// Small dense products of the chain rule through the fold (fp32, one thread per output element):
// C[m scm + n scn] (+)= alpha * sum_k A[m sam + k sak] B[k sbk + n sbn]
__global__ __launch_bounds__(256) void smm_kernel(const float *__restrict__ A, int64_t sam, int64_t sak, const float *__restrict__ B,
                                                  int64_t sbk, int64_t sbn, float *__restrict__ C, int64_t scm, int64_t scn, int M,
                                                  int N, int K, float alpha, int accumulate) {
  const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (e >= static_cast<int64_t>(M) * N) return;
  const int m = static_cast<int>(e % M), n = static_cast<int>(e / M);      // m fastest: coalesced when sam == 1
  float s = 0.f;
  for (int k = 0; k < K; ++k) s = fmaf(A[m * sam + k * sak], B[k * sbk + n * sbn], s);
  float *c = C + m * scm + n * scn;
  *c = accumulate ? *c + alpha * s : alpha * s;
}

static hipError_t smm(const float *A, int64_t sam, int64_t sak, const float *B, int64_t sbk, int64_t sbn, float *C, int64_t scm,
                      int64_t scn, int M, int N, int K, float alpha, bool accumulate, hipStream_t st) {
  const int64_t n = static_cast<int64_t>(M) * N;
  smm_kernel<<<dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, st>>>(A, sam, sak, B, sbk, sbn, C, scm, scn, M, N, K,
                                                                                  alpha, accumulate ? 1 : 0);
  return hipGetLastError();
}

// out[i] = a[i] + b[i]
__global__ __launch_bounds__(256) void add2_kernel(const float *a, const float *b, float *out, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) out[i] = a[i] + b[i];
}
// the key and query ends of the fold: d_wk[d, j] = kappa q[d] d_r[head(d), j];  d_bk[d] = kappa q[d] s0[head(d)];
// d_q[d] = kappa (wk[d, :] . d_r[head(d), :] + bk[d] s0[head(d)]),  s0[g] = sum_v da0[v, g]
__global__ __launch_bounds__(256) void fold_key_bwd_kernel(const float *q, const float *wk, const float *bk, const float *d_r,
                                                           const float *da0, float *d_wk, float *d_bk, float *d_q, int D, int dh,
                                                           int heads, int V, float kappa) {
  const int d = blockIdx.x;                       // one work-group per feature d
  const int g = d / dh;
  __shared__ float red[256];
  float s = 0.f;
  for (int j = threadIdx.x; j < D; j += 256) {
    const float dr = d_r[static_cast<size_t>(g) * D + j];
    d_wk[static_cast<size_t>(d) * D + j] = kappa * q[d] * dr;
    s = fmaf(wk[static_cast<size_t>(d) * D + j], dr, s);
  }
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    float s0 = 0.f;
    for (int v = 0; v < V; ++v) s0 += da0[v * heads + g];
    d_bk[d] = kappa * q[d] * s0;
    d_q[d] = kappa * (red[0] + bk[d] * s0);
  }
}
// d_wq[d, j] = d_q[d] q0[j]
__global__ __launch_bounds__(256) void outer_kernel(const float *a, const float *b, float *out, int M, int N) {
  const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (e < static_cast<int64_t>(M) * N) out[e] = a[e / N] * b[e % N];
}
// splits the reduced [V][D][p2 + 1] table into dU [V][D][p2] and dc [V][D] (same for the score tables)
__global__ __launch_bounds__(256) void split_last_kernel(const float *in, float *main, float *last, int64_t rows, int p2) {
  const int64_t r = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (r >= rows) return;
  for (int i = 0; i < p2; ++i) main[r * p2 + i] = in[r * (p2 + 1) + i];
  last[r] = in[r * (p2 + 1) + p2];
}

static hipError_t launch_1d(void (*k)(float *, int64_t, float), float *p, int64_t n, float v, hipStream_t st) {
  k<<<dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, st>>>(p, n, v);
  return hipGetLastError();
}

// ------------------------------------------------------------------ buffers
struct HeadWs {
  void *dP, *Af, *dAf;       // act [Mi, head_out], [Mi, D], [Mi, D]
  float *Xi, *dXi;           // [Mi, D]
  void *wgrad;
  float *colp, *lnp, *resp;  // partial rows: column sums, LayerNorm parameters, residual path
  int res_wg;
  size_t total;
};
static int residual_grid(const reslim_ctx *c, int batch, int *nbx, int *nby) {
  int max_ih = 0, max_iw = 0;
  for (const tile_desc &t : c->tiles) {
    max_ih = std::max(max_ih, (t.y1 - t.y0) * c->ps);
    max_iw = std::max(max_iw, (t.x1 - t.x0) * c->ps);
  }
  *nbx = (max_iw + 63) / 64;
  *nby = (max_ih + 15) / 16;
  const int64_t blocks = static_cast<int64_t>(*nbx) * *nby * c->T * batch;
  return static_cast<int>(std::min<int64_t>(blocks, 768));
}
static HeadWs plan_head_ws(const reslim_ctx *c, int batch, void *base) {
  const size_t Mi = static_cast<size_t>(batch) * c->N, D = c->cfg.embed_dim, es = act_size(c), ho = c->head_out;
  unsigned char *p = static_cast<unsigned char *>(base);
  size_t off = 0;
  auto take = [&](size_t bytes) { unsigned char *q = p + off; off += align256(bytes); return q; };
  HeadWs w;
  w.dP = take(Mi * ho * es);
  w.Af = take(Mi * D * es);
  w.dAf = take(Mi * D * es);
  w.Xi = reinterpret_cast<float *>(take(Mi * D * 4));
  w.dXi = reinterpret_cast<float *>(take(Mi * D * 4));
  w.wgrad = take(std::max<size_t>(wgrad_ws_bytes(c->cfg.dtype, static_cast<int>(Mi), c->head_out, c->cfg.embed_dim), 256));
  w.colp = reinterpret_cast<float *>(take(static_cast<size_t>(colsum_slabs(Mi)) * ho * 4));
  w.lnp = reinterpret_cast<float *>(take(static_cast<size_t>(layernorm_bwd_slabs(Mi)) * 2 * D * 4));
  int nbx, nby;
  w.res_wg = residual_grid(c, batch, &nbx, &nby);
  const size_t C = c->cfg.out_vars;
  w.resp = reinterpret_cast<float *>(take(static_cast<size_t>(w.res_wg) * (9 * C * C + C) * 4));
  w.total = off;
  return w;
}

// rows of the value table of the aggregation gradient's GEMM: (head, variable, pixel | offset), a multiple of 8
static int agg_table_rows(const reslim_ctx *c) {
  return (c->cfg.heads * c->cfg.in_vars * (c->cfg.patch * c->cfg.patch + 1) + 7) / 8 * 8;
}
struct EmbedWs {
  float *dz;                 // [Mi, D]
  void *dz_act, *o, *d_o;    // act [Mi, D]: gradient of the aggregated tokens, aggregated values, their gradient
  void *wgrad;
  float *colp;
  float *a, *ds;             // [Mi, heads, V]
  float *E;                  // [Mi, n_e] d_o times the block-structured value table
  float *pU, *pA;            // partial rows of the folded tables' gradients
  float *tU, *tA;            // reduced tables [V, D, p2 + 1], [V, heads, p2 + 1]
  float *dU, *dc, *dA, *da0; // split
  float *q, *r, *tv, *d_r, *d_q;   // fold intermediates: [D], [heads, D], [V, D], [heads, D], [D]
  int slabs_u, tok_u, slabs_a, tok_a;
  size_t total;
};
static EmbedWs plan_embed_ws(const reslim_ctx *c, int batch, void *base) {
  const size_t Mi = static_cast<size_t>(batch) * c->N, D = c->cfg.embed_dim, es = act_size(c);
  const size_t V = c->cfg.in_vars, heads = c->cfg.heads, p2 = static_cast<size_t>(c->cfg.patch) * c->cfg.patch;
  unsigned char *p = static_cast<unsigned char *>(base);
  size_t off = 0;
  auto take = [&](size_t bytes) { unsigned char *q = p + off; off += align256(bytes); return q; };
  EmbedWs w;
  w.dz = reinterpret_cast<float *>(take(Mi * D * 4));
  w.dz_act = take(Mi * D * es);
  w.o = take(Mi * D * es);
  w.d_o = take(Mi * D * es);
  w.wgrad = take(std::max<size_t>(wgrad_ws_bytes(c->cfg.dtype, static_cast<int>(Mi), c->cfg.embed_dim, c->cfg.embed_dim), 256));
  w.colp = reinterpret_cast<float *>(take(static_cast<size_t>(colsum_slabs(Mi)) * D * 4));
  w.a = reinterpret_cast<float *>(take(Mi * heads * V * 4));
  w.ds = reinterpret_cast<float *>(take(Mi * heads * V * 4));
  w.E = reinterpret_cast<float *>(take(Mi * static_cast<size_t>(agg_table_rows(c)) * 4));
  // slabs of tokens: about 2048 work-groups in the value-table pass, at least 64 tokens per slab
  const size_t per = ((D + 255) / 256) * ((V + 7) / 8);
  size_t su = std::max<size_t>(1, std::min<size_t>(256, 2048 / per));
  su = std::min(su, (Mi + 63) / 64);
  w.tok_u = static_cast<int>((Mi + su - 1) / su);
  w.slabs_u = static_cast<int>((Mi + w.tok_u - 1) / w.tok_u);
  size_t sa = std::min<size_t>(256, (Mi + 63) / 64);
  w.tok_a = static_cast<int>((Mi + sa - 1) / sa);
  w.slabs_a = static_cast<int>((Mi + w.tok_a - 1) / w.tok_a);
  w.pU = reinterpret_cast<float *>(take(static_cast<size_t>(w.slabs_u) * V * D * (p2 + 1) * 4));
  w.pA = reinterpret_cast<float *>(take(static_cast<size_t>(w.slabs_a) * V * heads * (p2 + 1) * 4));
  w.tU = reinterpret_cast<float *>(take(V * D * (p2 + 1) * 4));
  w.tA = reinterpret_cast<float *>(take(V * heads * (p2 + 1) * 4));
  w.dU = reinterpret_cast<float *>(take(V * D * p2 * 4));
  w.dc = reinterpret_cast<float *>(take(V * D * 4));
  w.dA = reinterpret_cast<float *>(take(V * heads * p2 * 4));
  w.da0 = reinterpret_cast<float *>(take(V * heads * 4));
  w.q = reinterpret_cast<float *>(take(D * 4));
  w.r = reinterpret_cast<float *>(take(heads * D * 4));
  w.tv = reinterpret_cast<float *>(take(V * D * 4));
  w.d_r = reinterpret_cast<float *>(take(heads * D * 4));
  w.d_q = reinterpret_cast<float *>(take(D * 4));
  w.total = off;
  return w;
}

// ------------------------------------------------------------------ the two ends, enqueued
static int head_bwd_impl(reslim_ctx *c, const char *fn, const float *x, const float *tokens, const float *d_y, float *d_tokens,
                         const reslim_grads *g, int batch, void *ws, hipStream_t st) {
  const HeadWs w = plan_head_ws(c, batch, ws);
  const int D = c->cfg.embed_dim, dt = c->cfg.dtype, C = c->cfg.out_vars;
  const int Mi = batch * c->N;
  const int64_t M = static_cast<int64_t>(batch) * c->n_h;
  const int sH = c->cfg.scale * c->cfg.H, sW = c->cfg.scale * c->cfg.W;
  const double es = static_cast<double>(act_size(c)), dMi = Mi, dD = D;
  const double fine = static_cast<double>(batch) * C * sH * sW;
  // transpose of un-patchify
  {
    const int64_t total = static_cast<int64_t>(Mi) * c->head_out;
    const dim3 grid(static_cast<unsigned>((total + 255) / 256));
    const int64_t total4 = static_cast<int64_t>(batch) * c->Hp * ((c->Wp + 3) / 4) * C * c->ps * 4 * (c->ps / 4);
    const dim3 grid4(static_cast<unsigned>((total4 + 255) / 256));
    const bool vec = c->ps % 4 == 0 && sW % 4 == 0 && (reinterpret_cast<uintptr_t>(d_y) & 15) == 0;
    if (dt == RESLIM_BF16 && vec)
      RESLIM_LAUNCH("patchify_grad", 0, 4.0 * fine + es * fine,
                    (patchify_act4_kernel<bf16_t><<<grid4, dim3(256), 0, st>>>(d_y, static_cast<bf16_t *>(w.dP), total4, c->Hp, c->Wp, C, c->ps, sH, sW), hipGetLastError()));
    else if (dt == RESLIM_BF16)
      RESLIM_LAUNCH("patchify_grad", 0, 4.0 * fine + es * fine,
                    (patchify_act_kernel<bf16_t><<<grid, dim3(256), 0, st>>>(d_y, static_cast<bf16_t *>(w.dP), total, c->N, c->Wp, C, c->ps, sH, sW), hipGetLastError()));
    else if (vec)
      RESLIM_LAUNCH("patchify_grad", 0, 8.0 * fine,
                    (patchify_act4_kernel<float><<<grid4, dim3(256), 0, st>>>(d_y, static_cast<float *>(w.dP), total4, c->Hp, c->Wp, C, c->ps, sH, sW), hipGetLastError()));
    else
      RESLIM_LAUNCH("patchify_grad", 0, 8.0 * fine,
                    (patchify_act_kernel<float><<<grid, dim3(256), 0, st>>>(d_y, static_cast<float *>(w.dP), total, c->N, c->Wp, C, c->ps, sH, sW), hipGetLastError()));
  }
  // residual path: weights and bias of the convolution
  {
    ResGradArgs a;
    a.x = x; a.dy = d_y; a.partial = w.resp; a.tiles = c->d_tiles; a.out_var_idx = c->d_out_var_idx;
    a.V = c->cfg.in_vars; a.C = C; a.H = c->cfg.H; a.W = c->cfg.W; a.s = c->cfg.scale; a.p = c->cfg.patch; a.ps = c->ps;
    a.T = c->T; a.batch = batch;
    (void)residual_grid(c, batch, &a.nbx, &a.nby);
    a.cwh = 17 / a.s + 3;
    a.cww = 65 / a.s + 3;
    const int n_acc = 9 * C * C + C;
    // as many outputs per pass as fit beside the other arrays in 150 KB of LDS
    int co = C > 8 ? 16 : C > 4 ? 8 : 4;
    while (co > 4 && residual_wgrad_lds_floats(C, co, a.cwh, a.cww) * sizeof(float) > kResGradLds) co /= 2;
    const size_t lds = residual_wgrad_lds_floats(C, co, a.cwh, a.cww) * sizeof(float);
    if (lds > kResGradLds || C > 64)                      // 64: the kernel's table of input variable indices
      return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": the residual-path gradient's arrays do not fit in LDS (scale too small or too many variables)");
    const double win = static_cast<double>(a.cwh) * a.cww * a.nbx * a.nby * c->T * batch;   // coarse-window pixels over all blocks
    const double res_flop = 2.0 * (12.0 * fine + 9.0 * (C + 2.0) * C * win);
    // columns per run of the column step: 4 NIT >= 2 s + 3 (a run is shorter than 2 s + 1, plus alignment)
    const int nit = a.s <= 4 ? 3 : a.s <= 8 ? 5 : 16;
    hipError_t le = hipSuccess;
#define RESLIM_RESGRAD(O, N) (residual_wgrad_kernel<O, N><<<dim3(w.res_wg), dim3(256), lds, st>>>(a), hipGetLastError())
    RESLIM_LAUNCH("residual_wgrad", res_flop, 4.0 * fine + 4.0 * batch * C * c->cfg.H * c->cfg.W,
                  (le = co == 16 ? (nit == 3 ? RESLIM_RESGRAD(4, 3) : nit == 5 ? RESLIM_RESGRAD(4, 5) : RESLIM_RESGRAD(4, 16))
                      : co == 8  ? (nit == 3 ? RESLIM_RESGRAD(2, 3) : nit == 5 ? RESLIM_RESGRAD(2, 5) : RESLIM_RESGRAD(2, 16))
                                 : (nit == 3 ? RESLIM_RESGRAD(1, 3) : nit == 5 ? RESLIM_RESGRAD(1, 5) : RESLIM_RESGRAD(1, 16)),
                   le));
#undef RESLIM_RESGRAD
    RESLIM_LAUNCH("partial_reduce", 0, 4.0 * w.res_wg * n_acc, launch_partial_reduce(w.resp, g->w_res, w.res_wg, n_acc, 9 * C * C, st));
    RESLIM_LAUNCH("partial_reduce", 0, 4.0 * w.res_wg * C, launch_partial_reduce(w.resp + 9 * C * C, g->b_res, w.res_wg, n_acc, C, st));
  }
  // head GEMM: the final LayerNorm's output on the interior tokens is recomputed, not kept
  RESLIM_LAUNCH("layernorm_final", 0, dMi * dD * (4.0 + es),
                launch_layernorm(dt, tokens, c->d_interior_src, c->N, c->n_h, c->d_lnf_g, c->d_lnf_b, w.Af, Mi, D, st));
  {
    const double dN = c->head_out, dK = D;
    RESLIM_LAUNCH("gemm_dgrad", 2.0 * dMi * dN * dK, dMi * dN * es + dN * dK * es + dMi * dK * es,
                  launch_gemm(dt, EPI_BIAS_ACT, w.dP, c->train.wt_head, c->d_zero_bias, w.dAf, D, nullptr, 0, Mi, D, c->head_out, st));
    RESLIM_LAUNCH("gemm_wgrad", 2.0 * dMi * dN * dK, dMi * dN * es + dMi * dK * es + 4.0 * dN * dK,
                  launch_wgrad(dt, w.dP, w.Af, g->w_head, Mi, c->head_out, D, w.wgrad, c->d_zero_bias, st));
    RESLIM_LAUNCH("colsum", 0, dMi * dN * es + 4.0 * dN, launch_colsum(dt, w.dP, w.colp, g->b_head, Mi, c->head_out, st));
  }
  // final LayerNorm backwards on the interior rows, then back into the tile-major stream (halo rows: zero)
  RESLIM_LAUNCH("gather", 0, 8.0 * dMi * dD, launch_gather_rows(tokens, c->d_interior_src, w.Xi, batch, c->N, static_cast<int>(c->n_h), D, st));
  RESLIM_LAUNCH("layernorm_bwd", 0, dMi * dD * (8.0 + es),
                launch_layernorm_bwd(dt, w.Xi, w.dAf, c->d_lnf_g, nullptr, w.dXi, nullptr, w.lnp, g->lnf_g, g->lnf_b, Mi, D, st));
  RESLIM_LAUNCH("scatter_interior", 0, 4.0 * dMi * dD + 4.0 * static_cast<double>(M) * dD,
                (scatter_interior_kernel<<<dim3(static_cast<unsigned>((M + 3) / 4)), dim3(256), 0, st>>>(
                     w.dXi, c->d_gather, c->d_interior_src, d_tokens, M, c->n_h, c->N, D),
                 hipGetLastError()));
  return RESLIM_OK;
}

static int embed_bwd_impl(reslim_ctx *c, const char *fn, const float *x, const float *d_tokens, const reslim_grads *g, int batch,
                          void *ws, hipStream_t st) {
  const EmbedWs w = plan_embed_ws(c, batch, ws);
  const TrainModel &tm = c->train;
  const int D = c->cfg.embed_dim, dt = c->cfg.dtype, V = c->cfg.in_vars, heads = c->cfg.heads, dh = c->dh;
  const int p = c->cfg.patch, p2 = p * p;
  const int Mi = batch * c->N;
  const double es = static_cast<double>(act_size(c)), dMi = Mi, dD = D;
  const float kappa = 1.0f / sqrtf(static_cast<float>(dh));
  // gather transposed
  {
    const dim3 grid(static_cast<unsigned>((Mi + 3) / 4));
    if (dt == RESLIM_BF16)
      RESLIM_LAUNCH("gather_grad", 0, 4.0 * batch * static_cast<double>(c->n_h) * dD + (4.0 + es) * dMi * dD,
                    (gather_transpose_kernel<bf16_t><<<grid, dim3(256), 0, st>>>(d_tokens, tm.copy_off, tm.copy_idx, w.dz, static_cast<bf16_t *>(w.dz_act), Mi, c->n_h, c->N, D), hipGetLastError()));
    else
      RESLIM_LAUNCH("gather_grad", 0, 4.0 * batch * static_cast<double>(c->n_h) * dD + 8.0 * dMi * dD,
                    (gather_transpose_kernel<float><<<grid, dim3(256), 0, st>>>(d_tokens, tm.copy_off, tm.copy_idx, w.dz, static_cast<float *>(w.dz_act), Mi, c->n_h, c->N, D), hipGetLastError()));
  }
  // position rows (shared by the samples), aggregated values again, output map of the aggregation
  {
    const int64_t n = static_cast<int64_t>(c->N) * D;
    RESLIM_LAUNCH("pos_grad", 0, 4.0 * dMi * dD + 4.0 * n,
                  (batch_sum_kernel<<<dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, st>>>(w.dz, g->pos_emb, n, n, batch), hipGetLastError()));
  }
  RESLIM_LAUNCH("embed_agg", 0, 4.0 * batch * V * c->cfg.H * c->cfg.W + dMi * dD * es, launch_embed_agg(c, x, w.o, batch, st));
  {
    RESLIM_LAUNCH("gemm_dgrad", 2.0 * dMi * dD * dD, 2.0 * dMi * dD * es + dD * dD * es,
                  launch_gemm(dt, EPI_BIAS_ACT, w.dz_act, tm.wt_agg_wo, c->d_zero_bias, w.d_o, D, nullptr, 0, Mi, D, D, st));
    RESLIM_LAUNCH("gemm_wgrad", 2.0 * dMi * dD * dD, 2.0 * dMi * dD * es + 4.0 * dD * dD,
                  launch_wgrad(dt, w.dz_act, w.o, g->agg_wo, Mi, D, D, w.wgrad, c->d_zero_bias, st));
    RESLIM_LAUNCH("colsum", 0, dMi * dD * es + 4.0 * dD, launch_colsum(dt, w.dz_act, w.colp, g->agg_bo, Mi, D, st));
  }
  // resolution table: the row the forward read gets the same column sums as the output bias, the others zero
  RESLIM_TRY("fill", launch_1d(fill_kernel, g->res_emb, static_cast<int64_t>(c->cfg.n_res) * D, 0.f, st));
  RESLIM_TRY("copy", hipMemcpyAsync(g->res_emb + static_cast<size_t>(c->cfg.res_idx) * D, g->agg_bo, D * sizeof(float), hipMemcpyDeviceToDevice, st));
  // folded aggregation backwards: logits, then the tables
  AggBwdArgs e;
  e.x = x; e.A = c->d_agg_A; e.a0 = c->d_agg_a0; e.U = c->d_agg_U; e.c = c->d_agg_c; e.d_o = w.d_o; e.a_out = w.a; e.ds_out = w.ds;
  e.V = V; e.H = c->cfg.H; e.W = c->cfg.W; e.p = p; e.Wp = c->Wp; e.N = c->N; e.D = D; e.heads = heads; e.dh = dh; e.BN = Mi;
  {
    const TrainModel &tmm = c->train;
    const double dNe = tmm.n_e;
    RESLIM_LAUNCH("gemm_agg_dvalues", 2.0 * dMi * dNe * dD, dMi * dD * es + dNe * dD * es + 4.0 * dMi * dNe,
                  launch_gemm(dt, EPI_BIAS_F32, w.d_o, tmm.w_vtab, tmm.zero_e, w.E, tmm.n_e, nullptr, 0, Mi, tmm.n_e, D, st));
    e.E = w.E; e.ne = tmm.n_e;
    auto lds_for = [&](int tp) {
      return static_cast<size_t>(tp) * (static_cast<size_t>(V) * p2 + 2 * static_cast<size_t>(heads) * V) * sizeof(float);
    };
    const int tp = lds_for(16) <= 64 * 1024 ? 16 : 4;      // tokens per work-group: fewer where variables x heads is large
    const size_t lds = lds_for(tp);
    if (lds > 150 * 1024) return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": too many variables x heads for the aggregation gradient");
    const dim3 grid(static_cast<unsigned>((Mi + tp - 1) / tp));
    const double fl = 2.0 * dMi * heads * V * (2.0 * p2 + 3.0);
    const double by = 4.0 * dMi * dNe + 8.0 * dMi * heads * V;
    if (tp == 16) RESLIM_LAUNCH("agg_scores_bwd", fl, by, (agg_scores_bwd_kernel<16><<<grid, dim3(256), lds, st>>>(e), hipGetLastError()));
    else RESLIM_LAUNCH("agg_scores_bwd", fl, by, (agg_scores_bwd_kernel<4><<<grid, dim3(256), lds, st>>>(e), hipGetLastError()));
  }
  {
    if (p2 != 4 && p2 != 1 && p2 != 16) return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": the aggregation gradient is built for patch sizes 1, 2 and 4");
    const dim3 grid(w.slabs_u, (D + 255) / 256, (V + 7) / 8);
    const double fl = 2.0 * dMi * V * dD * (p2 + 1);
#define RESLIM_AGGV(T_, P2_) RESLIM_LAUNCH("agg_values_bwd", fl, dMi * dD * es + 4.0 * dMi * heads * V, (agg_values_bwd_kernel<T_, P2_, 8><<<grid, dim3(256), 0, st>>>(e, w.pU, w.tok_u), hipGetLastError()))
    if (dt == RESLIM_BF16) {
      if (p2 == 4) RESLIM_AGGV(bf16_t, 4); else if (p2 == 1) RESLIM_AGGV(bf16_t, 1); else RESLIM_AGGV(bf16_t, 16);
    } else {
      if (p2 == 4) RESLIM_AGGV(float, 4); else if (p2 == 1) RESLIM_AGGV(float, 1); else RESLIM_AGGV(float, 16);
    }
#undef RESLIM_AGGV
    const int64_t nU = static_cast<int64_t>(V) * D * (p2 + 1);
    RESLIM_LAUNCH("partial_reduce", 0, 4.0 * w.slabs_u * nU, launch_partial_reduce(w.pU, w.tU, w.slabs_u, nU, nU, st));
    RESLIM_LAUNCH("agg_logits_bwd", 0, 4.0 * dMi * heads * V,
                  (agg_logits_bwd_kernel<<<dim3(w.slabs_a), dim3(256), 0, st>>>(e, w.pA, w.tok_a), hipGetLastError()));
    const int64_t nA = static_cast<int64_t>(V) * heads * (p2 + 1);
    RESLIM_LAUNCH("partial_reduce", 0, 4.0 * w.slabs_a * nA, launch_partial_reduce(w.pA, w.tA, w.slabs_a, nA, nA, st));
    split_last_kernel<<<dim3((V * D + 255) / 256), dim3(256), 0, st>>>(w.tU, w.dU, w.dc, static_cast<int64_t>(V) * D, p2);
    RESLIM_TRY("split", hipGetLastError());
    split_last_kernel<<<dim3((V * heads + 255) / 256), dim3(256), 0, st>>>(w.tA, w.dA, w.da0, static_cast<int64_t>(V) * heads, p2);
    RESLIM_TRY("split", hipGetLastError());
  }
  // ---- chain rule through the fold (fp32, small):
  //   q = Wq q0 + bq;  r_g = kappa Wk_g^T q_g;  t_v = b_pe[v] + var_emb[v]
  //   A[v,g,:] = r_g^T W_pe[v];  a0[v,g] = r_g . t_v + kappa q_g . bk_g;  U[v] = Wv W_pe[v];  c[v] = Wv t_v + bv
  RESLIM_TRY("fold", smm(tm.wq, D, 1, tm.q0, 1, 0, w.q, 1, 0, D, 1, D, 1.0f, false, st));
  add2_kernel<<<dim3((D + 255) / 256), dim3(256), 0, st>>>(w.q, tm.bq, w.q, D);
  RESLIM_TRY("fold", hipGetLastError());
  for (int gh = 0; gh < heads; ++gh)      // r[g, j] = kappa sum_{d in g} q[d] Wk[d, j]
    RESLIM_TRY("fold", smm(tm.wk + static_cast<size_t>(gh) * dh * D, 1, D, w.q + gh * dh, 1, 0, w.r + static_cast<size_t>(gh) * D, 1, 0, D, 1, dh, kappa, false, st));
  add2_kernel<<<dim3((V * D + 255) / 256), dim3(256), 0, st>>>(tm.b_pe, tm.var_emb, w.tv, static_cast<int64_t>(V) * D);
  RESLIM_TRY("fold", hipGetLastError());
  for (int v = 0; v < V; ++v) {
    const float *wpe = tm.w_pe + static_cast<size_t>(v) * D * p2;       // [D, p2]
    const float *dA_v = w.dA + static_cast<size_t>(v) * heads * p2;     // [heads, p2]
    const float *dU_v = w.dU + static_cast<size_t>(v) * D * p2;         // [D, p2]
    // d_r[g, j] += sum_i dA[v,g,i] W_pe[v][j,i] + da0[v,g] t_v[j]       (C = d_r^T viewed [j, g]: m = j)
    RESLIM_TRY("fold", smm(wpe, p2, 1, dA_v, 1, p2, w.d_r, 1, D, D, heads, p2, 1.0f, v > 0, st));
    RESLIM_TRY("fold", smm(w.tv + static_cast<size_t>(v) * D, 1, 0, w.da0 + static_cast<size_t>(v) * heads, 0, 1, w.d_r, 1, D, D, heads, 1, 1.0f, true, st));
    // d_W_pe[v][j, i] = sum_g r[g, j] dA[v,g,i] + sum_d Wv[d, j] dU[v][d, i]
    float *dwpe = g->w_pe + static_cast<size_t>(v) * D * p2;
    RESLIM_TRY("fold", smm(w.r, 1, D, dA_v, p2, 1, dwpe, p2, 1, D, p2, heads, 1.0f, false, st));
    RESLIM_TRY("fold", smm(tm.wv, 1, D, dU_v, p2, 1, dwpe, p2, 1, D, p2, D, 1.0f, true, st));
    // d_Wv[d, j] += sum_i dU[v][d, i] W_pe[v][j, i] + dc[v][d] t_v[j]
    RESLIM_TRY("fold", smm(dU_v, p2, 1, wpe, 1, p2, g->agg_wv, D, 1, D, D, p2, 1.0f, v > 0, st));
    RESLIM_TRY("fold", smm(w.dc + static_cast<size_t>(v) * D, 1, 0, w.tv + static_cast<size_t>(v) * D, 0, 1, g->agg_wv, D, 1, D, D, 1, 1.0f, true, st));
  }
  // d_t[v, j] = sum_g da0[v,g] r[g, j] + sum_d dc[v][d] Wv[d, j]  ->  d_b_pe = d_var_emb = d_t
  RESLIM_TRY("fold", smm(w.da0, heads, 1, w.r, D, 1, g->b_pe, D, 1, V, D, heads, 1.0f, false, st));
  RESLIM_TRY("fold", smm(w.dc, D, 1, tm.wv, D, 1, g->b_pe, D, 1, V, D, D, 1.0f, true, st));
  RESLIM_TRY("copy", hipMemcpyAsync(g->var_emb, g->b_pe, static_cast<size_t>(V) * D * sizeof(float), hipMemcpyDeviceToDevice, st));
  // d_bv[d] = sum_v dc[v][d]
  RESLIM_TRY("fold", launch_partial_reduce(w.dc, g->agg_bv, V, D, D, st));
  // key and query ends
  fold_key_bwd_kernel<<<dim3(D), dim3(256), 0, st>>>(w.q, tm.wk, tm.bk, w.d_r, w.da0, g->agg_wk, g->agg_bk, w.d_q, D, dh, heads, V, kappa);
  RESLIM_TRY("fold", hipGetLastError());
  {
    const int64_t n = static_cast<int64_t>(D) * D;
    outer_kernel<<<dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, st>>>(w.d_q, tm.q0, g->agg_wq, D, D);
    RESLIM_TRY("fold", hipGetLastError());
  }
  RESLIM_TRY("copy", hipMemcpyAsync(g->agg_bq, w.d_q, D * sizeof(float), hipMemcpyDeviceToDevice, st));
  RESLIM_TRY("fold", smm(tm.wq, 1, D, w.d_q, 1, 0, g->agg_q0, 1, 0, D, 1, D, 1.0f, false, st));     // d_q0[j] = sum_d Wq[d, j] d_q[d]
  return RESLIM_OK;
}

}  // namespace reslim

using namespace reslim;

// ------------------------------------------------------------------ entry points
extern "C" int reslim_bayes_loss_bwd(const float *pred, const float *target, const float *lat_w, int32_t batch, int32_t vars,
                                     int32_t Hf, int32_t Wf, float tv_weight, float upstream, float *d_pred, void *hip_stream) {
  if (!pred || !target || !lat_w || !d_pred) return RESLIM_EINVAL;
  if (batch < 1 || vars < 1 || Hf < 1 || Wf < 1 || static_cast<int64_t>(batch) * vars > 65535 || Hf > 65535) return RESLIM_EINVAL;
  const double count = static_cast<double>(batch) * vars * Hf * Wf;
  const double norm = 4.0 + 4.0 / 1.4142135623730951;
  const float data_f = static_cast<float>(2.0 * upstream / count);
  const float tv_f = static_cast<float>(2.0 * static_cast<double>(upstream) * tv_weight / (norm * count));
  const bool aligned = Wf % 4 == 0 && (reinterpret_cast<uintptr_t>(pred) | reinterpret_cast<uintptr_t>(target) | reinterpret_cast<uintptr_t>(d_pred)) % 16 == 0;
  if (aligned) {
    constexpr int RB = 8;
    const dim3 grid((Wf / 4 + 255) / 256, (Hf + RB - 1) / RB, batch * vars);
    bayes_loss_bwd4_kernel<RB><<<grid, dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(pred, target, lat_w, d_pred, Hf, Wf, data_f, tv_f);
  } else {
    const dim3 grid((Wf + 255) / 256, Hf, batch * vars);
    bayes_loss_bwd_kernel<<<grid, dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(pred, target, lat_w, d_pred, Hf, Wf, data_f, tv_f);
  }
  return hipGetLastError() == hipSuccess ? RESLIM_OK : RESLIM_EHIP;
}

static hipError_t train_model_init() {
  hipError_t e = hipSuccess;
  const int lim = 150 * 1024;
#define RESLIM_ATTR(K) if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void *>(&K), hipFuncAttributeMaxDynamicSharedMemorySize, lim)
  RESLIM_ATTR(agg_scores_bwd_kernel<16>);
  RESLIM_ATTR(agg_scores_bwd_kernel<4>);
  RESLIM_ATTR((residual_wgrad_kernel<4, 3>));
  RESLIM_ATTR((residual_wgrad_kernel<4, 5>));
  RESLIM_ATTR((residual_wgrad_kernel<4, 16>));
  RESLIM_ATTR((residual_wgrad_kernel<2, 3>));
  RESLIM_ATTR((residual_wgrad_kernel<2, 5>));
  RESLIM_ATTR((residual_wgrad_kernel<2, 16>));
  RESLIM_ATTR((residual_wgrad_kernel<1, 3>));
  RESLIM_ATTR((residual_wgrad_kernel<1, 5>));
  RESLIM_ATTR((residual_wgrad_kernel<1, 16>));
#undef RESLIM_ATTR
  return e;
}

extern "C" int reslim_train_prepare_model(reslim_ctx *c, const reslim_weights *wts) {
  const char *fn = "reslim_train_prepare_model";
  if (!c) return RESLIM_EINVAL;
  if (!wts) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null weights");
  if (c->train.ready) return RESLIM_OK;
  RESLIM_TRY("kernel setup", train_model_init());
  const int D = c->cfg.embed_dim, V = c->cfg.in_vars, p2 = c->cfg.patch * c->cfg.patch, dt = c->cfg.dtype;
  if (dt == RESLIM_BF16 && c->head_out % 64 != 0)
    return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": out_vars * (patch * scale)^2 must be a multiple of 64 on the bfloat16 path (contraction length of the head's input gradient)");
  if (D % 4 != 0) return set_error(c, RESLIM_ESHAPE, std::string(fn) + ": embed_dim must be a multiple of 4");
  int rc = reslim_train_prepare(c);
  if (rc != RESLIM_OK) return rc;
  TrainModel &tm = c->train;
  auto up = [&](const float *src, size_t n, float **dst) -> hipError_t {
    void *d = nullptr;
    hipError_t e = hipMalloc(&d, std::max<size_t>(n * sizeof(float), 256));
    if (e != hipSuccess) return e;
    c->allocs.push_back(d);
    *dst = static_cast<float *>(d);
    return hipMemcpy(d, src, n * sizeof(float), hipMemcpyHostToDevice);
  };
  const size_t DD = static_cast<size_t>(D) * D;
  hipError_t e = up(wts->w_pe, static_cast<size_t>(V) * D * p2, &tm.w_pe);
  if (e == hipSuccess) e = up(wts->b_pe, static_cast<size_t>(V) * D, &tm.b_pe);
  if (e == hipSuccess) e = up(wts->var_emb, static_cast<size_t>(V) * D, &tm.var_emb);
  if (e == hipSuccess) e = up(wts->agg_q0, D, &tm.q0);
  if (e == hipSuccess) e = up(wts->agg_wq, DD, &tm.wq);
  if (e == hipSuccess) e = up(wts->agg_bq, D, &tm.bq);
  if (e == hipSuccess) e = up(wts->agg_wk, DD, &tm.wk);
  if (e == hipSuccess) e = up(wts->agg_bk, D, &tm.bk);
  if (e == hipSuccess) e = up(wts->agg_wv, DD, &tm.wv);
  if (e == hipSuccess) e = up(wts->agg_bv, D, &tm.bv);
  // [in, out] copies of the head's and the aggregation's output maps for their input gradients
  const size_t es = act_size(c);
  auto transposed = [&](const void *src, int rows, int cols, void **dst) -> hipError_t {
    void *d = nullptr;
    hipError_t e2 = hipMalloc(&d, std::max<size_t>(static_cast<size_t>(rows) * cols * es, 256));
    if (e2 != hipSuccess) return e2;
    c->allocs.push_back(d);
    *dst = d;
    return launch_transpose(dt, src, d, rows, cols, nullptr);
  };
  if (e == hipSuccess) e = transposed(c->d_w_head, c->head_out, D, &tm.wt_head);
  if (e == hipSuccess) e = transposed(c->d_agg_wo, D, D, &tm.wt_agg_wo);
  // halo copies of every patch, in increasing tile-major index
  if (e == hipSuccess) {
    std::vector<int32_t> gather(c->n_h), off(static_cast<size_t>(c->N) + 1, 0), idx(c->n_h);
    e = hipMemcpy(gather.data(), c->d_gather, gather.size() * 4, hipMemcpyDeviceToHost);
    if (e == hipSuccess) {
      for (int64_t r = 0; r < c->n_h; ++r) ++off[gather[r] + 1];
      for (int n = 0; n < c->N; ++n) off[n + 1] += off[n];
      std::vector<int32_t> fill(off.begin(), off.end() - 1);
      for (int64_t r = 0; r < c->n_h; ++r) idx[fill[gather[r]]++] = static_cast<int32_t>(r);
      void *d0 = nullptr, *d1 = nullptr;
      e = hipMalloc(&d0, off.size() * 4);
      if (e == hipSuccess) { c->allocs.push_back(d0); e = hipMalloc(&d1, std::max<size_t>(idx.size() * 4, 256)); }
      if (e == hipSuccess) { c->allocs.push_back(d1); e = hipMemcpy(d0, off.data(), off.size() * 4, hipMemcpyHostToDevice); }
      if (e == hipSuccess) e = hipMemcpy(d1, idx.data(), idx.size() * 4, hipMemcpyHostToDevice);
      tm.copy_off = static_cast<int32_t *>(d0);
      tm.copy_idx = static_cast<int32_t *>(d1);
    }
  }
  // the value table by (head, variable, pixel | offset) for the GEMM of the aggregation gradient
  if (e == hipSuccess) {
    const int rows = c->cfg.heads * V * (p2 + 1);
    tm.n_e = agg_table_rows(c);
    void *dw = nullptr, *dz = nullptr;
    const size_t es = dt == RESLIM_BF16 ? 2 : 4;
    e = hipMalloc(&dw, static_cast<size_t>(tm.n_e) * D * es);
    if (e == hipSuccess) { c->allocs.push_back(dw); e = hipMalloc(&dz, static_cast<size_t>(tm.n_e) * 4); }
    if (e == hipSuccess) { c->allocs.push_back(dz); e = hipMemset(dz, 0, static_cast<size_t>(tm.n_e) * 4); }
    if (e == hipSuccess) {
      const dim3 grid(static_cast<unsigned>((static_cast<int64_t>(tm.n_e) * D + 255) / 256));
      if (dt == RESLIM_BF16)
        agg_value_table_kernel<bf16_t><<<grid, dim3(256)>>>(c->d_agg_U, c->d_agg_c, static_cast<bf16_t *>(dw), V, D, c->dh, p2, rows, tm.n_e);
      else
        agg_value_table_kernel<float><<<grid, dim3(256)>>>(c->d_agg_U, c->d_agg_c, static_cast<float *>(dw), V, D, c->dh, p2, rows, tm.n_e);
      e = hipGetLastError();
    }
    tm.w_vtab = dw;
    tm.zero_e = static_cast<float *>(dz);
  }
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) return set_error(c, e == hipErrorOutOfMemory ? RESLIM_ENOMEM : RESLIM_EHIP, std::string(fn) + ": " + hipGetErrorString(e));
  tm.ready = true;
  return RESLIM_OK;
}

static bool grads_complete(const reslim_grads *g, int first, int last) {
  const float *const *p = reinterpret_cast<const float *const *>(g);
  for (int i = first; i < last; ++i)
    if (!p[i]) return false;
  return true;
}
// field ranges of reslim_grads: front end [0, 14), blocks [14, 26), back end [26, 32)
enum { G_FRONT0 = 0, G_BLOCK0 = 14, G_BACK0 = 26, G_END = 32 };

extern "C" int reslim_head_bwd_workspace_bytes(const reslim_ctx *c, int32_t batch, size_t *out) {
  if (!c || !out || batch < 1) return RESLIM_EINVAL;
  *out = plan_head_ws(c, batch, nullptr).total;
  return RESLIM_OK;
}
extern "C" int reslim_embed_bwd_workspace_bytes(const reslim_ctx *c, int32_t batch, size_t *out) {
  if (!c || !out || batch < 1) return RESLIM_EINVAL;
  *out = plan_embed_ws(c, batch, nullptr).total;
  return RESLIM_OK;
}

static int check_model_train(reslim_ctx *c, const char *fn, int batch, const void *ws, size_t ws_bytes, size_t need) {
  if (!c->train.ready) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": call reslim_train_prepare_model first");
  int rc = check_common(c, fn, batch, nullptr, 0, false);
  if (rc != RESLIM_OK) return rc;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255)) return set_error(c, RESLIM_EWORKSPACE, std::string(fn) + ": workspace null or not 256-byte aligned");
  if (ws_bytes < need) return set_error(c, RESLIM_EWORKSPACE, std::string(fn) + ": workspace too small");
  return RESLIM_OK;
}

extern "C" int reslim_head_bwd(reslim_ctx *c, const float *x, const float *tokens, const float *d_y, float *d_tokens,
                               const reslim_grads *grads, int32_t batch, void *workspace, size_t ws_bytes, void *hip_stream) {
  const char *fn = "reslim_head_bwd";
  if (!c) return RESLIM_EINVAL;
  if (!x || !tokens || !d_y || !d_tokens || !grads || !grads_complete(grads, G_BACK0, G_END))
    return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  int rc = check_model_train(c, fn, batch, workspace, ws_bytes, plan_head_ws(c, batch, nullptr).total);
  if (rc != RESLIM_OK) return rc;
  return head_bwd_impl(c, fn, x, tokens, d_y, d_tokens, grads, batch, workspace, static_cast<hipStream_t>(hip_stream));
}

extern "C" int reslim_embed_bwd(reslim_ctx *c, const float *x, const float *d_tokens, const reslim_grads *grads, int32_t batch,
                                void *workspace, size_t ws_bytes, void *hip_stream) {
  const char *fn = "reslim_embed_bwd";
  if (!c) return RESLIM_EINVAL;
  if (!x || !d_tokens || !grads || !grads_complete(grads, G_FRONT0, G_BLOCK0))
    return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  int rc = check_model_train(c, fn, batch, workspace, ws_bytes, plan_embed_ws(c, batch, nullptr).total);
  if (rc != RESLIM_OK) return rc;
  return embed_bwd_impl(c, fn, x, d_tokens, grads, batch, workspace, static_cast<hipStream_t>(hip_stream));
}

// ------------------------------------------------------------------ the whole step
namespace {
struct StepPlan {
  size_t stream_bytes;       // one [M, D] fp32 stream
  size_t block_saved;        // saved activations of one block
  size_t saved_total;        // (L + 1) streams + L block buffers
  size_t fwd_ws, block_ws, head_ws, embed_ws, loss_ws, dy_bytes;
  size_t ws_total;           // d_y | two gradient streams | max of the stage workspaces
};
StepPlan plan_step(const reslim_ctx *c, int batch) {
  StepPlan p;
  const size_t M = static_cast<size_t>(batch) * c->n_h, D = c->cfg.embed_dim;
  p.stream_bytes = align256(M * D * sizeof(float));
  size_t sb = 0, wb = 0;
  reslim_block_train_bytes(c, batch, &sb, &wb);
  p.block_saved = align256(sb);
  p.block_ws = wb;
  const size_t L = c->cfg.depth;
  p.saved_total = (L + 1) * p.stream_bytes + L * p.block_saved;
  p.fwd_ws = plan_workspace(c, batch, nullptr).total;
  p.head_ws = plan_head_ws(c, batch, nullptr).total;
  p.embed_ws = plan_embed_ws(c, batch, nullptr).total;
  size_t lw = 0;
  reslim_bayes_loss_workspace_bytes(batch, c->cfg.out_vars, c->cfg.scale * c->cfg.H, c->cfg.scale * c->cfg.W, &lw);
  p.loss_ws = align256(lw);
  p.dy_bytes = align256(static_cast<size_t>(batch) * c->cfg.out_vars * c->cfg.scale * c->cfg.H * c->cfg.scale * c->cfg.W * sizeof(float));
  const size_t stage = std::max(std::max(p.fwd_ws, p.block_ws), std::max(std::max(p.head_ws, p.embed_ws), p.loss_ws));
  p.ws_total = p.dy_bytes + 2 * p.stream_bytes + align256(stage);
  return p;
}
}  // namespace

extern "C" int reslim_train_step_bytes(const reslim_ctx *c, int32_t batch, size_t *saved_bytes, size_t *ws_bytes) {
  if (!c || batch < 1) return RESLIM_EINVAL;
  const StepPlan p = plan_step(c, batch);
  if (saved_bytes) *saved_bytes = p.saved_total;
  if (ws_bytes) *ws_bytes = p.ws_total;
  return RESLIM_OK;
}

extern "C" int reslim_train_step_grads(reslim_ctx *c, const float *x, const float *target, const float *lat_w, float tv_weight,
                                       float loss_scale, float *y, double *loss3, const reslim_grads *grads, int32_t batch,
                                       void *saved, size_t saved_bytes, void *workspace, size_t ws_bytes, void *hip_stream) {
  const char *fn = "reslim_train_step_grads";
  if (!c) return RESLIM_EINVAL;
  if (!x || !target || !lat_w || !y || !loss3 || !grads || !grads_complete(grads, G_FRONT0, G_END))
    return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null buffer");
  if (!(loss_scale > 0.0f) || !std::isfinite(loss_scale)) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": loss_scale must be positive and finite");
  if (reinterpret_cast<uintptr_t>(loss3) % 8) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": loss3 must be 8-byte aligned");
  const StepPlan p = plan_step(c, batch);
  int rc = check_model_train(c, fn, batch, workspace, ws_bytes, p.ws_total);
  if (rc != RESLIM_OK) return rc;
  if (!saved || (reinterpret_cast<uintptr_t>(saved) & 255) || saved_bytes < p.saved_total)
    return set_error(c, RESLIM_EWORKSPACE, std::string(fn) + ": saved buffer null, misaligned or smaller than reslim_train_step_bytes()");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int L = c->cfg.depth, C = c->cfg.out_vars, D = c->cfg.embed_dim;
  const int Hf = c->cfg.scale * c->cfg.H, Wf = c->cfg.scale * c->cfg.W;
  unsigned char *sv = static_cast<unsigned char *>(saved), *wsb = static_cast<unsigned char *>(workspace);
  auto stream = [&](int l) { return reinterpret_cast<float *>(sv + static_cast<size_t>(l) * p.stream_bytes); };
  auto bsaved = [&](int l) { return sv + static_cast<size_t>(L + 1) * p.stream_bytes + static_cast<size_t>(l) * p.block_saved; };
  float *d_y = reinterpret_cast<float *>(wsb);
  float *ga = reinterpret_cast<float *>(wsb + p.dy_bytes), *gb = reinterpret_cast<float *>(wsb + p.dy_bytes + p.stream_bytes);
  void *stage = wsb + p.dy_bytes + 2 * p.stream_bytes;
  const size_t stage_bytes = ws_bytes - (p.dy_bytes + 2 * p.stream_bytes);
  // ---- forward, keeping every block's input and intermediates
  if ((rc = reslim_embed_fwd(c, x, stream(0), batch, stage, stage_bytes, hip_stream)) != RESLIM_OK) return rc;
  for (int l = 0; l < L; ++l)
    if ((rc = reslim_block_fwd_train(c, l, stream(l), stream(l + 1), bsaved(l), p.block_saved, batch, stage, stage_bytes, hip_stream)) != RESLIM_OK) return rc;
  if ((rc = reslim_head_fwd(c, x, stream(L), y, batch, stage, stage_bytes, hip_stream)) != RESLIM_OK) return rc;
  // ---- loss value and its gradient (times the loss scale)
  if (reslim_bayes_loss_fwd(y, target, lat_w, batch, C, Hf, Wf, tv_weight, loss3, stage, stage_bytes, hip_stream) != RESLIM_OK)
    return set_error(c, RESLIM_EHIP, std::string(fn) + ": loss forward failed");
  if (reslim_bayes_loss_bwd(y, target, lat_w, batch, C, Hf, Wf, tv_weight, loss_scale, d_y, hip_stream) != RESLIM_OK)
    return set_error(c, RESLIM_EHIP, std::string(fn) + ": loss gradient failed");
  // ---- backward
  if ((rc = head_bwd_impl(c, fn, x, stream(L), d_y, ga, grads, batch, stage, st)) != RESLIM_OK) return rc;
  const size_t DD = static_cast<size_t>(D) * D, R = c->R;
  for (int l = L - 1; l >= 0; --l) {
    reslim_block_grads bg;
    bg.ln1_g = grads->ln1_g + static_cast<size_t>(l) * D; bg.ln1_b = grads->ln1_b + static_cast<size_t>(l) * D;
    bg.w_qkv = grads->w_qkv + l * 3 * DD; bg.b_qkv = grads->b_qkv + static_cast<size_t>(l) * 3 * D;
    bg.w_proj = grads->w_proj + l * DD; bg.b_proj = grads->b_proj + static_cast<size_t>(l) * D;
    bg.ln2_g = grads->ln2_g + static_cast<size_t>(l) * D; bg.ln2_b = grads->ln2_b + static_cast<size_t>(l) * D;
    bg.w_fc1 = grads->w_fc1 + l * R * D; bg.b_fc1 = grads->b_fc1 + l * R;
    bg.w_fc2 = grads->w_fc2 + l * R * D; bg.b_fc2 = grads->b_fc2 + static_cast<size_t>(l) * D;
    if ((rc = reslim_block_bwd(c, l, stream(l), bsaved(l), p.block_saved, ga, gb, &bg, batch, stage, stage_bytes, hip_stream)) != RESLIM_OK) return rc;
    std::swap(ga, gb);
  }
  return embed_bwd_impl(c, fn, x, ga, grads, batch, stage, st);
}

extern "C" int reslim_grads_unscale(reslim_ctx *c, const reslim_grads *grads, float inv_scale, int32_t *found_inf, void *hip_stream) {
  const char *fn = "reslim_grads_unscale";
  if (!c) return RESLIM_EINVAL;
  if (!grads || !found_inf || !grads_complete(grads, G_FRONT0, G_END)) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": null argument");
  if (!(inv_scale > 0.0f) || !std::isfinite(inv_scale)) return set_error(c, RESLIM_EINVAL, std::string(fn) + ": inv_scale must be positive and finite");
  const int64_t D = c->cfg.embed_dim, R = c->R, V = c->cfg.in_vars, L = c->cfg.depth, C = c->cfg.out_vars;
  const int64_t p2 = static_cast<int64_t>(c->cfg.patch) * c->cfg.patch;
  const int64_t sizes[32] = {V * D * p2, V * D, V * D, D, D * D, D, D * D, D, D * D, D, D * D, D, static_cast<int64_t>(c->N) * D, c->cfg.n_res * D,
                             L * D, L * D, L * 3 * D * D, L * 3 * D, L * D * D, L * D, L * D, L * D, L * R * D, L * R, L * D * R, L * D,
                             D, D, static_cast<int64_t>(c->head_out) * D, c->head_out, C * C * 9, C};
  float *const *ptrs = reinterpret_cast<float *const *>(grads);
  for (int i = 0; i < 32; i += 12) {
    const int n = std::min(12, 32 - i);
    RESLIM_TRY("launch", launch_unscale_check(const_cast<float **>(ptrs) + i, sizes + i, n, inv_scale, found_inf, static_cast<hipStream_t>(hip_stream)));
  }
  return RESLIM_OK;
}

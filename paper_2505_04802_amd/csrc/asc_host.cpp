// Adaptive spatial compression, host side (ORBIT-2 Sec. 4.1, "Adaptive Spatial
// Compression"; Sec. 4.3 has the CPUs build the quad-trees while the GPUs compute):
// image -> 8-bit -> Canny edge map -> quad-tree on edge density -> leaf table.
// Integers throughout, apart from the 8-bit quantisation and the density test,
// which are single float32 operations in a fixed order.  No HIP call.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "reslim.h"

namespace {

#pragma clang fp contract(off)

// v -> floor((v - min) * (255 / (max - min)) + 0.5), clamped; a constant field maps to 0
bool quantise(const float *v, size_t n, std::vector<int32_t> &q) {
  float mn = v[0], mx = v[0];
  for (size_t i = 0; i < n; ++i) {
    if (!std::isfinite(v[i])) return false;
    mn = std::min(mn, v[i]);
    mx = std::max(mx, v[i]);
  }
  q.assign(n, 0);
  if (!(mx > mn)) return true;
  const float scale = 255.0f / (mx - mn);
  for (size_t i = 0; i < n; ++i) {
    const float d = v[i] - mn;
    const float m = d * scale;
    const float r = std::floor(m + 0.5f);
    q[i] = static_cast<int32_t>(std::min(255.0f, std::max(0.0f, r)));
  }
  return true;
}

struct Img {
  int H, W;
  const int32_t *p;
  int32_t rep(int y, int x) const {   // border replicated
    return p[static_cast<size_t>(std::min(std::max(y, 0), H - 1)) * W + std::min(std::max(x, 0), W - 1)];
  }
  int32_t zero(int y, int x) const {  // outside counts as 0
    return (y < 0 || y >= H || x < 0 || x >= W) ? 0 : p[static_cast<size_t>(y) * W + x];
  }
};

// Canny's steps on an 8-bit image; edges[i] = 1 where an edge pixel is found
void canny(const std::vector<int32_t> &q, int H, int W, int low, int high, std::vector<uint8_t> &edges) {
  static const int32_t mask[5][5] = {{2, 4, 5, 4, 2}, {4, 9, 12, 9, 4}, {5, 12, 15, 12, 5}, {4, 9, 12, 9, 4}, {2, 4, 5, 4, 2}};
  const size_t n = static_cast<size_t>(H) * W;
  std::vector<int32_t> sm(n), gx(n), gy(n), mag(n);
  const Img iq{H, W, q.data()};
  for (int y = 0; y < H; ++y)
    for (int x = 0; x < W; ++x) {
      int32_t acc = 0;
      for (int dy = -2; dy <= 2; ++dy)
        for (int dx = -2; dx <= 2; ++dx) acc += mask[dy + 2][dx + 2] * iq.rep(y + dy, x + dx);
      sm[static_cast<size_t>(y) * W + x] = (acc + 79) / 159;
    }
  const Img is{H, W, sm.data()};
  for (int y = 0; y < H; ++y)
    for (int x = 0; x < W; ++x) {
      const size_t i = static_cast<size_t>(y) * W + x;
      gx[i] = (is.rep(y - 1, x + 1) + 2 * is.rep(y, x + 1) + is.rep(y + 1, x + 1)) -
              (is.rep(y - 1, x - 1) + 2 * is.rep(y, x - 1) + is.rep(y + 1, x - 1));
      gy[i] = (is.rep(y + 1, x - 1) + 2 * is.rep(y + 1, x) + is.rep(y + 1, x + 1)) -
              (is.rep(y - 1, x - 1) + 2 * is.rep(y - 1, x) + is.rep(y - 1, x + 1));
      mag[i] = std::abs(gx[i]) + std::abs(gy[i]);
    }
  // 0 = not a candidate, 1 = weak, 2 = strong
  std::vector<uint8_t> cls(n, 0);
  const Img im{H, W, mag.data()};
  constexpr int32_t kTan22 = 13573;   // tan(22.5 deg) in 15 fraction bits; tan(67.5 deg) = tan(22.5 deg) + 2
  std::vector<size_t> stack;
  for (int y = 0; y < H; ++y)
    for (int x = 0; x < W; ++x) {
      const size_t i = static_cast<size_t>(y) * W + x;
      const int32_t m = mag[i];
      if (m <= low) continue;
      const int32_t ax = std::abs(gx[i]), ay = std::abs(gy[i]);
      int dy, dx;                       // step towards the "next" neighbour along the gradient
      if ((ay << 15) < ax * kTan22) { dy = 0; dx = 1; }
      else if ((ay << 15) > ax * (kTan22 + (1 << 16))) { dy = 1; dx = 0; }
      else if ((gx[i] ^ gy[i]) >= 0) { dy = 1; dx = 1; }
      else { dy = 1; dx = -1; }
      if (!(m > im.zero(y - dy, x - dx) && m >= im.zero(y + dy, x + dx))) continue;
      cls[i] = m > high ? 2 : 1;
      if (cls[i] == 2) stack.push_back(i);
    }
  // hysteresis: flood from the strong pixels through weak ones, 8-neighbourhood
  edges.assign(n, 0);
  for (size_t i : stack) edges[i] = 1;
  while (!stack.empty()) {
    const size_t i = stack.back();
    stack.pop_back();
    const int y = static_cast<int>(i / W), x = static_cast<int>(i % W);
    for (int dy = -1; dy <= 1; ++dy)
      for (int dx = -1; dx <= 1; ++dx) {
        const int yy = y + dy, xx = x + dx;
        if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
        const size_t j = static_cast<size_t>(yy) * W + xx;
        if (cls[j] != 0 && !edges[j]) {
          edges[j] = 1;
          stack.push_back(j);
        }
      }
  }
}

struct TreeBuilder {
  const std::vector<int64_t> &sat;   // summed-area table of edge counts per patch, (Hp+1) x (Wp+1)
  int Hp, Wp, p, min_leaf;
  float tau;
  int32_t *ly, *lx, *ls, *patch_leaf;
  int64_t n;                          // leaves written so far (batch-wide)

  int64_t count(int y0, int x0, int s) const {
    const size_t w = static_cast<size_t>(Wp) + 1;
    return sat[(y0 + s) * w + x0 + s] - sat[y0 * w + x0 + s] - sat[(y0 + s) * w + x0] + sat[y0 * w + x0];
  }
  void visit(int y0, int x0, int s) {
    if (y0 >= Hp || x0 >= Wp) return;                     // wholly in the padding of a ragged grid
    const bool inside = y0 + s <= Hp && x0 + s <= Wp;     // a node that sticks out always splits
    const float area = static_cast<float>(static_cast<int64_t>(s) * p * s * p);
    const float bound = tau * area;
    if (!inside || (s > min_leaf && static_cast<float>(count(y0, x0, s)) > bound)) {
      const int h = s / 2;
      visit(y0, x0, h);
      visit(y0, x0 + h, h);
      visit(y0 + h, x0, h);
      visit(y0 + h, x0 + h, h);
      return;
    }
    ly[n] = y0; lx[n] = x0; ls[n] = s;
    for (int yy = y0; yy < y0 + s; ++yy)
      for (int xx = x0; xx < x0 + s; ++xx) patch_leaf[static_cast<size_t>(yy) * Wp + xx] = static_cast<int32_t>(n);
    ++n;
  }
};

bool pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

}  // namespace

extern "C" int reslim_asc_build(const float *images, int32_t batch, int32_t H, int32_t W, int32_t patch, int32_t max_leaf,
                                int32_t min_leaf, int32_t canny_low, int32_t canny_high, float tau, int32_t *leaf_y0,
                                int32_t *leaf_x0, int32_t *leaf_s, int32_t *sample_off, int32_t *patch_leaf,
                                int64_t *n_leaves_out) {
  if (!images || !leaf_y0 || !leaf_x0 || !leaf_s || !sample_off || !patch_leaf || !n_leaves_out) return RESLIM_EINVAL;
  if (batch < 1 || H < 1 || W < 1 || patch < 1 || canny_low < 0 || canny_high < canny_low || !(tau >= 0.0f) || !std::isfinite(tau))
    return RESLIM_EINVAL;
  if (!pow2(max_leaf) || !pow2(min_leaf) || min_leaf > max_leaf || H % patch || W % patch) return RESLIM_ESHAPE;
  const int Hp = H / patch, Wp = W / patch;
  if (static_cast<int64_t>(batch) * Hp * Wp > INT32_MAX) return RESLIM_ESHAPE;
  const size_t npix = static_cast<size_t>(H) * W, N = static_cast<size_t>(Hp) * Wp;
  std::vector<int32_t> q;
  std::vector<uint8_t> edges;
  std::vector<int64_t> sat((Hp + 1) * (static_cast<size_t>(Wp) + 1));
  int64_t n = 0;
  sample_off[0] = 0;
  for (int b = 0; b < batch; ++b) {
    if (!quantise(images + b * npix, npix, q)) return RESLIM_EINVAL;   // non-finite pixel
    canny(q, H, W, canny_low, canny_high, edges);
    const size_t w = static_cast<size_t>(Wp) + 1;
    std::fill(sat.begin(), sat.end(), 0);
    for (int py = 0; py < Hp; ++py)
      for (int px = 0; px < Wp; ++px) {
        int64_t c = 0;
        for (int i = 0; i < patch; ++i)
          for (int j = 0; j < patch; ++j) c += edges[static_cast<size_t>(py * patch + i) * W + px * patch + j];
        sat[(py + 1) * w + px + 1] = c + sat[py * w + px + 1] + sat[(py + 1) * w + px] - sat[py * w + px];
      }
    TreeBuilder tb{sat, Hp, Wp, patch, min_leaf, tau, leaf_y0, leaf_x0, leaf_s, patch_leaf + b * N, n};
    for (int ry = 0; ry < Hp; ry += max_leaf)
      for (int rx = 0; rx < Wp; rx += max_leaf) tb.visit(ry, rx, max_leaf);
    n = tb.n;
    sample_off[b + 1] = static_cast<int32_t>(n);
  }
  *n_leaves_out = n;
  return RESLIM_OK;
}

// Compression combined with TILES: every (sample, tile) pair is compressed on its own, on the
// tile's haloed box cut out of the field, exactly as reslim_asc_build treats a whole sample.
extern "C" int reslim_asc_build_tiles(const float *images, int32_t batch, int32_t H, int32_t W, int32_t patch,
                                      int32_t tiles_y, int32_t tiles_x, int32_t halo, int32_t max_leaf, int32_t min_leaf,
                                      int32_t canny_low, int32_t canny_high, float tau, int32_t *leaf_y0, int32_t *leaf_x0,
                                      int32_t *leaf_s, int32_t *seq_off, int32_t *patch_leaf, int64_t *n_leaves_out) {
  if (!images || !leaf_y0 || !leaf_x0 || !leaf_s || !seq_off || !patch_leaf || !n_leaves_out) return RESLIM_EINVAL;
  if (batch < 1 || H < 1 || W < 1 || patch < 1 || canny_low < 0 || canny_high < canny_low || !(tau >= 0.0f) || !std::isfinite(tau))
    return RESLIM_EINVAL;
  if (!pow2(max_leaf) || !pow2(min_leaf) || min_leaf > max_leaf || H % patch || W % patch) return RESLIM_ESHAPE;
  const int Hp = H / patch, Wp = W / patch;
  if (tiles_y < 1 || tiles_x < 1) return RESLIM_ESHAPE;
  const int T = tiles_y * tiles_x;
  std::vector<tile_desc> tiles(T);
  int64_t n_h = 0;
  const int rc = tiles_partition(Hp, Wp, tiles_y, tiles_x, halo, tiles.data(), nullptr, nullptr, &n_h);
  if (rc != RESLIM_OK) return rc;
  if (static_cast<int64_t>(batch) * n_h > INT32_MAX) return RESLIM_ESHAPE;
  const size_t npix = static_cast<size_t>(H) * W, N = static_cast<size_t>(Hp) * Wp;
  std::vector<float> crop;
  std::vector<int32_t> q, local;
  std::vector<uint8_t> edges;
  std::vector<int64_t> sat;
  int64_t n = 0;
  seq_off[0] = 0;
  for (int b = 0; b < batch; ++b)
    for (int t = 0; t < T; ++t) {
      const tile_desc &td = tiles[t];
      const int hp = td.Y1 - td.Y0, wp = td.X1 - td.X0, ch = hp * patch, cw = wp * patch;
      crop.resize(static_cast<size_t>(ch) * cw);
      for (int y = 0; y < ch; ++y)
        std::copy_n(images + b * npix + static_cast<size_t>(td.Y0 * patch + y) * W + td.X0 * patch, cw, crop.begin() + static_cast<size_t>(y) * cw);
      if (!quantise(crop.data(), crop.size(), q)) return RESLIM_EINVAL;
      canny(q, ch, cw, canny_low, canny_high, edges);
      const size_t w = static_cast<size_t>(wp) + 1;
      sat.assign((hp + 1) * w, 0);
      for (int py = 0; py < hp; ++py)
        for (int px = 0; px < wp; ++px) {
          int64_t c = 0;
          for (int i = 0; i < patch; ++i)
            for (int j = 0; j < patch; ++j) c += edges[static_cast<size_t>(py * patch + i) * cw + px * patch + j];
          sat[(py + 1) * w + px + 1] = c + sat[py * w + px + 1] + sat[(py + 1) * w + px] - sat[py * w + px];
        }
      local.assign(static_cast<size_t>(hp) * wp, -1);
      const int64_t first = n;
      TreeBuilder tb{sat, hp, wp, patch, min_leaf, tau, leaf_y0, leaf_x0, leaf_s, local.data(), n};
      for (int ry = 0; ry < hp; ry += max_leaf)
        for (int rx = 0; rx < wp; rx += max_leaf) tb.visit(ry, rx, max_leaf);
      n = tb.n;
      for (int64_t l = first; l < n; ++l) {          // box coordinates -> grid coordinates
        leaf_y0[l] += td.Y0;
        leaf_x0[l] += td.X0;
      }
      for (int yy = td.y0; yy < td.y1; ++yy)         // the tile's interior patches decompress from its own leaves
        for (int xx = td.x0; xx < td.x1; ++xx)
          patch_leaf[b * N + static_cast<size_t>(yy) * Wp + xx] = local[static_cast<size_t>(yy - td.Y0) * wp + (xx - td.X0)];
      seq_off[static_cast<size_t>(b) * T + t + 1] = static_cast<int32_t>(n);
    }
  *n_leaves_out = n;
  return RESLIM_OK;
}

// Canny edge map of one 8-bit-quantised field, for inspection and tests: edges [H*W] 0/1
extern "C" int reslim_asc_edges(const float *image, int32_t H, int32_t W, int32_t canny_low, int32_t canny_high, uint8_t *edges_out) {
  if (!image || !edges_out || H < 1 || W < 1 || canny_low < 0 || canny_high < canny_low) return RESLIM_EINVAL;
  std::vector<int32_t> q;
  std::vector<uint8_t> e;
  if (!quantise(image, static_cast<size_t>(H) * W, q)) return RESLIM_EINVAL;
  canny(q, H, W, canny_low, canny_high, e);
  std::copy(e.begin(), e.end(), edges_out);
  return RESLIM_OK;
}

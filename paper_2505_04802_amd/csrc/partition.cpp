// tiles_partition: the TILES partition, halo and stitch indices (ORBIT-2 Sec. 4.2).
// Host code, integers only.
#include <string>

#include "common.h"

namespace reslim {
static thread_local std::string g_thread_error;
void set_thread_error(const std::string &msg) { g_thread_error = msg; }
const std::string &thread_error() { return g_thread_error; }
}  // namespace reslim

extern "C" int tiles_partition(int32_t Hp, int32_t Wp, int32_t Ty, int32_t Tx, int32_t halo,
                               tile_desc *tiles, int32_t *gather_idx, int32_t *interior_src,
                               int64_t *n_h_out) {
  if (Hp < 1 || Wp < 1 || Ty < 1 || Tx < 1 || halo < 0 || Ty > Hp || Tx > Wp) {
    reslim::set_thread_error("tiles_partition: need 1 <= tiles <= patches per axis and halo >= 0");
    return RESLIM_ESHAPE;
  }
  if (static_cast<int64_t>(Hp) * Wp > INT32_MAX) {
    reslim::set_thread_error("tiles_partition: patch grid exceeds int32 indexing");
    return RESLIM_ESHAPE;
  }
  int64_t off = 0;
  for (int32_t i = 0; i < Ty; ++i) {
    const int32_t y0 = static_cast<int32_t>(static_cast<int64_t>(i) * Hp / Ty);
    const int32_t y1 = static_cast<int32_t>(static_cast<int64_t>(i + 1) * Hp / Ty);
    const int32_t Y0 = y0 - halo < 0 ? 0 : y0 - halo;
    const int32_t Y1 = y1 + halo > Hp ? Hp : y1 + halo;
    for (int32_t j = 0; j < Tx; ++j) {
      const int32_t x0 = static_cast<int32_t>(static_cast<int64_t>(j) * Wp / Tx);
      const int32_t x1 = static_cast<int32_t>(static_cast<int64_t>(j + 1) * Wp / Tx);
      const int32_t X0 = x0 - halo < 0 ? 0 : x0 - halo;
      const int32_t X1 = x1 + halo > Wp ? Wp : x1 + halo;
      const int32_t bw = X1 - X0;
      const int64_t n_tok = static_cast<int64_t>(Y1 - Y0) * bw;
      if (off + n_tok > INT32_MAX) {
        reslim::set_thread_error("tiles_partition: tile-major token count exceeds int32 indexing");
        return RESLIM_ESHAPE;
      }
      if (tiles) {
        tile_desc &t = tiles[static_cast<size_t>(i) * Tx + j];
        t.y0 = y0; t.y1 = y1; t.x0 = x0; t.x1 = x1;
        t.Y0 = Y0; t.Y1 = Y1; t.X0 = X0; t.X1 = X1;
        t.tok_off = off;
        t.n_tok = static_cast<int32_t>(n_tok);
        t._pad = 0;
      }
      if (gather_idx) {
        int32_t *dst = gather_idx + off;
        for (int32_t y = Y0; y < Y1; ++y)
          for (int32_t x = X0; x < X1; ++x) *dst++ = y * Wp + x;
      }
      if (interior_src) {
        for (int32_t y = y0; y < y1; ++y) {
          const int64_t row = off + static_cast<int64_t>(y - Y0) * bw - X0;
          for (int32_t x = x0; x < x1; ++x) interior_src[static_cast<size_t>(y) * Wp + x] = static_cast<int32_t>(row + x);
        }
      }
      off += n_tok;
    }
  }
  if (n_h_out) *n_h_out = off;
  return RESLIM_OK;
}

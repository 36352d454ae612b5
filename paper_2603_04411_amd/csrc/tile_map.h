// XCD-aware workgroup -> tile mapping (shared by the MFMA kernels; also compiled on the host
// by the unit test of the mapping).
#pragma once

#ifdef LMHEAD_TILE_MAP_HOST
#define LMHEAD_HD
#else
#include <hip/hip_runtime.h>
#define LMHEAD_HD __host__ __device__
#endif

namespace lmhead {

// Workgroup -> tile mapping that keeps L2 traffic local to an XCD.
//
// The chip dispatches workgroup i of a 1-D grid to XCD i % 8, and each XCD has a private L2.
// A work grid of X x Y items (x selects the A-side operand slab, y the B-side slab) is cut
// into eight contiguous y-ranges, one per XCD; inside its range an XCD walks blocks of
// bx x by items (x fastest), so the 32 workgroups it runs at a time cover a compact block and
// share bx + by operand slabs instead of fetching 64.  Returns false for workgroups beyond the
// work (the grid is sized for the largest possible Y).
constexpr int kNumXcd = 8;
LMHEAD_HD inline bool xcd_tile_coords(int wg, int X, int Y, int bx, int by, int& x, int& y) {
  const int xcd = wg % kNumXcd;
  const int j = wg / kNumXcd;
  const int y_per = (Y + kNumXcd - 1) / kNumXcd;
  const int y_base = xcd * y_per;
  const int y_cnt = min(y_per, Y - y_base);
  if (y_cnt <= 0) return false;
  const int per_yblk = X * by;
  const int yb = j / per_yblk;
  int r = j - yb * per_yblk;
  const int h = min(by, y_cnt - yb * by);
  if (h <= 0 || r >= X * h) return false;
  const int nfull = X / bx;
  const int full_items = nfull * bx * h;
  int yin;
  if (r < full_items) {
    const int xb = r / (bx * h);
    const int r2 = r - xb * (bx * h);
    yin = r2 / bx;
    x = xb * bx + (r2 - yin * bx);
  } else {
    const int tw = X - nfull * bx;
    r -= full_items;
    yin = r / tw;
    x = nfull * bx + (r - yin * tw);
  }
  y = y_base + yb * by + yin;
  return true;
}
// Grid size that covers every item for any Y <= Y_cap under the mapping above.
inline unsigned xcd_grid_size(int X, long long Y_cap, int by) {
  const long long y_per = (Y_cap + kNumXcd - 1) / kNumXcd;
  const long long yblks = (y_per + by - 1) / by;
  return (unsigned)(kNumXcd * yblks * by * X);
}

}  // namespace lmhead

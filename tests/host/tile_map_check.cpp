// Host check of the XCD-aware tile walk: every work item of an X x Y grid is visited exactly
// once by the workgroups of the launched 1-D grid, for any Y up to the capacity Y_cap.
// Compiled with g++ by tests/test_host_logic.py; includes the product header in host mode.
#include <algorithm>
#include <cstdio>
#include <vector>
using std::min;
#define LMHEAD_TILE_MAP_HOST 1
#include "../../paper_2603_04411_amd/csrc/tile_map.h"

int main() {
  long bad = 0, cases = 0;
  const int Xs[] = {1, 2, 14, 16, 19, 20, 33};
  const int Ycaps[] = {1, 7, 8, 9, 32, 100, 1327};
  const int Bs[] = {1, 2, 4, 8};
  for (int X : Xs)
    for (int Ycap : Ycaps)
      for (int Y : {0, 1, Ycap / 2, Ycap - 1, Ycap})
        for (int bx : Bs)
          for (int by : Bs) {
            if (Y < 0 || Y > Ycap) continue;
            ++cases;
            std::vector<int> cnt((size_t)X * std::max(Y, 1), 0);
            const unsigned g = lmhead::xcd_grid_size(X, Ycap, by);
            for (unsigned wg = 0; wg < g; ++wg) {
              int x = -1, y = -1;
              if (lmhead::xcd_tile_coords((int)wg, X, Y, bx, by, x, y)) {
                if (x < 0 || x >= X || y < 0 || y >= Y) { ++bad; continue; }
                cnt[(size_t)y * X + x]++;
              }
            }
            for (int i = 0; i < X * Y; ++i) if (cnt[i] != 1) ++bad;
          }
  // the 32 workgroups an XCD runs together (consecutive j on one XCD) form compact blocks
  {
    const int X = 16, Y = 1327, bx = 4, by = 4;
    int xs[64], ys[64], n = 0;
    for (int j = 0; j < 16; ++j) { int x, y; if (lmhead::xcd_tile_coords(j * 8 + 3, X, Y, bx, by, x, y)) { xs[n] = x; ys[n] = y; ++n; } }
    int xmin = 1 << 30, xmax = -1, ymin = 1 << 30, ymax = -1;
    for (int i = 0; i < n; ++i) { xmin = std::min(xmin, xs[i]); xmax = std::max(xmax, xs[i]); ymin = std::min(ymin, ys[i]); ymax = std::max(ymax, ys[i]); }
    if (n != 16 || xmax - xmin != 3 || ymax - ymin != 3) ++bad;
  }
  std::printf("cases=%ld bad=%ld\n", cases, bad);
  return bad != 0;
}

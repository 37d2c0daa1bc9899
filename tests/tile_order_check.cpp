// Host-side check of the Gram kernel's tile order (compiled and run by test_tile_order.py):
// for every width d and every groups-per-workgroup setting, the first tile_count indices must
// decode to each valid (row block, tile column) pair of the upper triangle exactly once.
#include <cstdio>
#include <set>
#include <utility>

#include "gq_internal.hpp"

int main() {
  for (int gpc : {1, 2, 4})
    for (int64_t d = 8; d <= 4096; d += 8) {
      const int64_t TM = 64 * (4 / gpc), NT = (d + 255) / 256;
      int64_t rows_last = (d + TM - 1) / TM;                 // row blocks that intersect the matrix
      if (rows_last > NT * gpc) rows_last = NT * gpc;
      const int64_t T = gpc * gq::tri_count(NT - 1) + rows_last;
      std::set<std::pair<int, int>> seen;
      for (int64_t t = 0; t < T; ++t) {
        int I, J;
        gq::band_decode(t, gpc, NT, I, J);
        if (J < 0 || J >= NT || I < 0 || I >= gpc * (J + 1) || I * TM >= d) {
          std::printf("out of range: gpc %d d %ld t %ld -> (%d, %d)\n", gpc, (long)d, (long)t, I, J);
          return 1;
        }
        if (!seen.insert({I, J}).second) {
          std::printf("visited twice: gpc %d d %ld t %ld -> (%d, %d)\n", gpc, (long)d, (long)t, I, J);
          return 1;
        }
      }
    }
  // the wide kernel's order: row blocks of 96 rows (192 when a workgroup takes two of them) against tile
  // columns of 256 columns
  for (int64_t rows : {96, 192})
    for (int64_t d = 8; d <= 4608; d += 8) {
      const int64_t NT = (d + 255) / 256, NR = (d + rows - 1) / rows;
      int64_t expect = 0;
      for (int64_t I = 0; I < NR; ++I)
        for (int64_t J = 0; J < NT; ++J)
          if (256 * J + 255 >= rows * I) ++expect;             // some column of the tile is >= some row of the block
      const int64_t T = gq::wide_tile_count(d, rows);
      if (T != expect) {
        std::printf("wide count: rows %ld d %ld: %ld items, %ld tiles meet the upper triangle\n", (long)rows, (long)d, (long)T,
                    (long)expect);
        return 1;
      }
      std::set<std::pair<int, int>> seen;
      for (int64_t t = 0; t < T; ++t) {
        int I, J;
        gq::wide_decode(t, d, I, J, rows);
        if (J < 0 || J >= NT || I < 0 || I >= NR || 256 * (int64_t)J + 255 < rows * (int64_t)I) {
          std::printf("wide out of range: rows %ld d %ld t %ld -> (%d, %d)\n", (long)rows, (long)d, (long)t, I, J);
          return 1;
        }
        if (!seen.insert({I, J}).second) {
          std::printf("wide visited twice: rows %ld d %ld t %ld -> (%d, %d)\n", (long)rows, (long)d, (long)t, I, J);
          return 1;
        }
      }
    }
  std::printf("OK\n");
  return 0;
}

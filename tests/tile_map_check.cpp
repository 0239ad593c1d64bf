// Host check of the workgroup -> tile mapping of the tiled projection kernels: over many matrix and
// call sizes every output tile is covered exactly once, no block maps outside the matrix, and the eight
// XCDs (block index mod 8) get equal shares of the tiles: exactly equal when the matrix width fills every
// window, and otherwise apart by at most one XCD rectangle (32 tiles) per band, since only the last window
// of a band can be partly empty.  Prints "ok" and returns 0 when all holds.
#include <cstdio>
#include <vector>

#include "../paper_2312_08361_amd/csrc/tile_map.h"

int main() {
  int bad = 0;
  long cases = 0;
  const int tiles[] = {64, 128, 256}, kts[] = {8, 256, 896, 1792}, nws[] = {1, 2, 16, 32, 40, 56, 168, 224, 256, 336, 448, 512};
  for (int tile : tiles)
    for (int KT : kts)
      for (int NW : nws)
        for (int NM = 1; NM <= 200; ++NM) {
          const TileBands tb = make_bands(NW, NM, KT, tile);
          const int grid = tb.b0[tb.n_rem];
          std::vector<int> seen((size_t)NM * NW, 0);
          long per_xcd[8] = {0, 0, 0, 0, 0, 0, 0, 0};
          for (int b = 0; b < grid; ++b) {
            int n = -1, m = -1;
            if (!tile_of_block(tb, NW, NM, b, n, m)) continue;
            if (m < 0 || n < 0 || m >= NM || n >= NW) { ++bad; continue; }
            ++seen[(size_t)m * NW + n];
            ++per_xcd[b & 7];
          }
          for (int v : seen)
            if (v != 1) { ++bad; break; }
          long mx = 0, mn = 1L << 60;
          for (long v : per_xcd) { if (v > mx) mx = v; if (v < mn) mn = v; }
          const long slack = NW % 256 == 0 ? 0 : 32L * (tb.n_full + tb.n_rem);
          if (mx - mn > slack) {
            std::printf("imbalance: tile %d KT %d NW %d NM %d: %ld..%ld tiles per XCD\n", tile, KT, NW, NM, mn, mx);
            ++bad;
          }
          ++cases;
        }
  std::printf("%s: %ld cases, %d bad\n", bad ? "FAILED" : "ok", cases, bad);
  return bad != 0;
}

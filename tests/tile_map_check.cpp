// Host check of the workgroup -> tile mapping of the tiled projection kernels: over many matrix and
// call sizes every output tile is covered exactly once, no block maps outside the matrix, and the eight
// XCDs (block index mod 8) get equal shares of the tiles: exactly equal when the matrix width fills every
// window, and otherwise apart by at most one XCD rectangle (32 tiles) over all bands, plus the tiles that the
// rectangle at the matrix edge lacks in each band.  Prints "ok" and returns 0 when all holds.
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
          // the partly filled windows of the bands follow each other round the ring of XCDs: one rectangle of slack,
          // plus what the edge rectangle of each band lacks (the width need not be a multiple of a rectangle's)
          long slack = 0;
          for (int bd = 0; bd < tb.n_full + tb.n_rem; ++bd) {
            const int h = bd < tb.n_full ? tb.hmax : tb.h[bd - tb.n_full], sm = h >= 4 ? 4 : h, sn = 32 / sm;
            if (NW % (256 / h)) slack = slack < 32 ? 32 : slack;
            slack += (long)((sn - NW % sn) % sn) * sm;
          }
          if (mx - mn > slack) {
            std::printf("imbalance: tile %d KT %d NW %d NM %d: %ld..%ld tiles per XCD\n", tile, KT, NW, NM, mn, mx);
            ++bad;
          }
          ++cases;
        }
  // cut of the weight rows into a part of 256-row tiles and a part of narrower ones: the parts tile the quads
  // exactly once in order, the first part comes out in whole rounds, and the plan is never costlier than no cut
  for (int Q = 1; Q <= 1000; ++Q)
    for (int NM = 1; NM <= 130; ++NM) {
      const RowParts rp = plan_row_parts(Q, NM);
      const double cost0 = (double)(((long)((Q + 3) / 4) * NM + 255) / 256) * 4.0;
      int next = 0;
      bool ok = rp.n >= 1 && rp.n <= 2 && rp.cost <= cost0 + 1e-9;
      for (int i = 0; i < rp.n && ok; ++i) {
        ok = rp.quad_base[i] == next && rp.n_quads[i] > 0 && rp.hq[i] >= 1 && rp.hq[i] <= 4;
        next += rp.n_quads[i];
      }
      ok = ok && next == Q;
      if (ok && rp.n == 2) ok = rp.hq[0] == 4 && rp.n_quads[0] % 4 == 0 && ((long)(rp.n_quads[0] / 4) * NM) % 256 == 0;
      if (!ok) { std::printf("bad row parts: Q %d NM %d\n", Q, NM); ++bad; }
      ++cases;
    }
  // the shapes the narrower tiles are for (176B-shaped span, 2048 tokens): 14336 rows = 1.75 rounds -> one round of 4 quads + one
  // of 3; 43008 rows = 5.25 rounds -> cut somewhere, cheaper than six rounds; whole rounds stay uncut
  {
    const RowParts a = plan_row_parts(224, 8), b = plan_row_parts(672, 8), c = plan_row_parts(896, 8), d = plan_row_parts(640, 64);
    const RowParts e = plan_row_parts(64, 8);       // 4096 rows x 2048 tokens: half a round of 256-row tiles -> one round of 128-row tiles
    if (!(e.n == 1 && e.hq[0] == 2 && e.n_quads[0] == 64)) { std::printf("unexpected plan for half a round: %d/%d\n", e.n, e.hq[0]); ++bad; }
    if (!(a.n == 2 && a.hq[1] == 3 && a.n_quads[0] == 128) || !(b.n == 2 && b.cost < 0.97 * 24.0) || c.n != 1 || d.n != 1) {
      std::printf("unexpected plans: %d/%d %d/%d %d %d\n", a.n, a.hq[1], b.n, b.hq[1], c.n, d.n);
      ++bad;
    }
  }
  std::printf("%s: %ld cases, %d bad\n", bad ? "FAILED" : "ok", cases, bad);
  return bad != 0;
}

// Workgroup -> output tile mapping of the tiled projection kernels (host and device; plain C++ so that
// a host program can check it exhaustively).
#pragma once
#include <stddef.h>
#if defined(__HIPCC__)
#define TILE_MAP_FN __host__ __device__ inline
#else
#define TILE_MAP_FN inline
#endif

// Workgroup -> output tile.  Workgroups are dealt round-robin to the 8 XCDs (blockIdx & 7), each
// with its own L2, and about 256 run at a time.  The token tiles are cut into bands whose
// heights are powers of two (largest first, e.g. 9 tiles = 8 + 1), a band into windows of 256
// output tiles (h token tiles x 256/h weight tiles), and a window into one compact 32-tile
// rectangle per XCD (4 x 8 when h >= 4).  So: every XCD gets the same number of tiles of every
// window, whatever the token count; the 32 workgroups an XCD runs at a time share operand tiles
// in its L2 (12 distinct tiles feed 32 workgroups); and a band's activations (h * tile tokens x
// K, re-read for every window) are sized to stay in the memory-side cache.
struct TileBands {
  int hmax, n_full, full_blocks;   // n_full bands of hmax token tiles, full_blocks blocks each
  int n_rem;                       // then the remaining token tiles as bands of decreasing powers of two
  int m0[6], h[6], b0[7];          // first token tile, height, first block; b0[n_rem] = grid size
  int rot_full, used_full, rot[6]; // rotation of the XCDs' rectangles: full band i uses rot_full - i * used_full
};
// XCD rectangles that the last, partly filled window of a band of height h holds (0 = the width fills every window)
TILE_MAP_FN int band_used_rects(int NW, int h) {
  const int hn = 256 / h, sm = h >= 4 ? 4 : h, sn = 32 / sm, rem = NW % hn;
  return ((rem + sn - 1) / sn) * (h / sm);
}
TILE_MAP_FN bool tile_of_block(const TileBands &tb, int NW, int NM, int b, int &wg_n, int &wg_m) {
  int h, m0, r, band;
  if (b < tb.b0[0]) {
    band = b / tb.full_blocks;
    h = tb.hmax; m0 = band * tb.hmax; r = b - band * tb.full_blocks;
  } else {
    int k = 0;
    while (k + 1 < tb.n_rem && b >= tb.b0[k + 1]) ++k;
    h = tb.h[k]; m0 = tb.m0[k]; r = b - tb.b0[k]; band = tb.n_full + k;
  }
  const int hn = 256 / h;
  // which rectangle of the window an XCD takes rotates from band to band: the last window of a band is filled in
  // part only (u of its 8 rectangles hold tiles), and band after band these u rectangles go to the next u XCDs
  // round the ring, so that over all bands the XCDs' shares differ by one rectangle at most
  const int rot = b < tb.b0[0] ? tb.rot_full - band * tb.used_full : tb.rot[band - tb.n_full];
  const int w = r >> 8, q = r & 255, x = (q + rot) & 7, i = q >> 3;
  const int sm = h >= 4 ? 4 : h, sn = 32 / sm;        // an XCD's rectangle inside the window
  const int xm_cnt = h / sm;                          // XCDs side by side along the token tiles
  const int xm = x % xm_cnt, xn = x / xm_cnt;
  wg_m = m0 + xm * sm + i % sm;
  wg_n = w * hn + xn * sn + i / sm;
  return wg_n < NW && wg_m < NM;
}
// tile_tokens: tokens per token tile (64, 128 or 256)
TILE_MAP_FN TileBands make_bands(int NW, int NM, int KT, int tile_tokens) {
  TileBands tb{};
  // tallest band: its activations should stay within about 128 MiB, and a window must still
  // give every XCD a 4 x 8 rectangle (h <= 32)
  const size_t tile_bytes = (size_t)tile_tokens * KT * 64;
  int hmax = 32;
  while (hmax > 4 && (size_t)hmax * tile_bytes > ((size_t)128 << 20)) hmax >>= 1;
  tb.hmax = hmax;
  tb.n_full = NM / hmax;
  tb.full_blocks = ((NW + 256 / hmax - 1) / (256 / hmax)) * 256;
  int m = tb.n_full * hmax, blocks = tb.n_full * tb.full_blocks;
  tb.rot_full = 0; tb.used_full = band_used_rects(NW, hmax);
  int start = tb.n_full * tb.used_full;   // first XCD (mod 8) of the next band's partly filled window
  for (int h = hmax >> 1; h >= 1; h >>= 1) {
    // three token tiles left: one band of four with an empty row instead of 2 + 1 (every band streams the
    // whole weight matrix once more; an XCD's rectangle spans all four rows, so the shares stay equal)
    if (h == 2 && NM - m == 3) {
      tb.m0[tb.n_rem] = m; tb.h[tb.n_rem] = 4; tb.b0[tb.n_rem] = blocks;
      tb.rot[tb.n_rem] = -start; start += band_used_rects(NW, 4);
      blocks += ((NW + 256 / 4 - 1) / (256 / 4)) * 256;
      m += 3; ++tb.n_rem;
      continue;
    }
    if (NM - m < h) continue;
    tb.m0[tb.n_rem] = m; tb.h[tb.n_rem] = h; tb.b0[tb.n_rem] = blocks;
    tb.rot[tb.n_rem] = -start; start += band_used_rects(NW, h);
    blocks += ((NW + 256 / h - 1) / (256 / h)) * 256;
    m += h; ++tb.n_rem;
  }
  tb.b0[tb.n_rem] = blocks;        // with n_rem == 0 this is b0[0] = end of the full bands
  return tb;
}

// Cut of a matrix's weight rows (in quads of 64 rows) into at most two parts for the 256-token tiles: a first part
// of 256-row tiles (4 quads) that comes out in whole rounds of 256 workgroups, and the remaining rows as narrower
// tiles (3, 2 or 1 quads) -- more of them, each proportionally shorter -- when that brings the last round closer to
// full (a matrix of less than one round has no first part: 4096 rows x 2048 tokens = 128 tiles of 256 rows run as
// 256 tiles of 128 rows).  Cost unit: one round of 256-row tiles = 4.  The relative speeds of the narrower tiles are measured on
// rounds of 256 tiles with K = 14336 (a round of 64-row tiles took 150 us, of 192-row tiles 317 us, of 256-row tiles
// 346 - 376 us; the 128-row figure is interpolated): a 64-row tile leaves half the waves without matrix work and
// moves four times the token operand per flop.
struct RowParts {
  int n;
  int quad_base[2], n_quads[2], hq[2];
  double cost;
};
TILE_MAP_FN RowParts plan_row_parts(int Q, int NM) {
  const double eff[5] = {0.0, 0.58, 0.80, 0.88, 1.0};
  RowParts best{}, uncut{};
  const long tiles0 = (long)((Q + 3) / 4) * NM;
  best.n = 1; best.quad_base[0] = 0; best.n_quads[0] = Q; best.hq[0] = 4;
  best.cost = (double)((tiles0 + 255) / 256) * 4.0;
  if (tiles0 % 256 == 0) return best;
  uncut = best;
  // columns of 256-row tiles that make whole rounds: multiples of step
  int g = NM, b = 256;
  while (b) { const int t = g % b; g = b; b = t; }
  const int step = 256 / g;
  const int a_max = (Q / 4) / step * step;
  for (int a = a_max; a >= 0 && a >= a_max - 2 * step; a -= step) {
    const int rq = Q - 4 * a;
    if (rq <= 0) continue;
    for (int hq = 3; hq >= 1; --hq) {
      const long tiles = (long)((rq + hq - 1) / hq) * NM;
      const double cost = (double)((long)a * NM / 256) * 4.0 + (double)((tiles + 255) / 256) * hq / eff[hq];
      if (cost < best.cost * 0.99) {                 // near ties go to the plan tried first: the taller tiles
        best.cost = cost;
        if (a > 0) { best.n = 2; best.quad_base[0] = 0; best.n_quads[0] = 4 * a; best.hq[0] = 4;
                     best.quad_base[1] = 4 * a; best.n_quads[1] = rq; best.hq[1] = hq; }
        else { best.n = 1; best.quad_base[0] = 0; best.n_quads[0] = rq; best.hq[0] = hq; }
      }
    }
  }
  return best.cost < uncut.cost * 0.97 ? best : uncut;   // a cut must pay for its second launch
}

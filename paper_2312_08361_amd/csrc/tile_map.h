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
};
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
  // which rectangle of the window an XCD takes rotates from window to window, so that the
  // partly empty rectangles at the matrix edge are shared out evenly
  const int w = r >> 8, q = r & 255, x = (q + w + 3 * band) & 7, i = q >> 3;
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
  for (int h = hmax >> 1; h >= 1; h >>= 1) {
    // three token tiles left: one band of four with an empty row instead of 2 + 1 (every band streams the
    // whole weight matrix once more; an XCD's rectangle spans all four rows, so the shares stay equal)
    if (h == 2 && NM - m == 3) {
      tb.m0[tb.n_rem] = m; tb.h[tb.n_rem] = 4; tb.b0[tb.n_rem] = blocks;
      blocks += ((NW + 256 / 4 - 1) / (256 / 4)) * 256;
      m += 3; ++tb.n_rem;
      continue;
    }
    if (NM - m < h) continue;
    tb.m0[tb.n_rem] = m; tb.h[tb.n_rem] = h; tb.b0[tb.n_rem] = blocks;
    blocks += ((NW + 256 / h - 1) / (256 / h)) * 256;
    m += h; ++tb.n_rem;
  }
  tb.b0[tb.n_rem] = blocks;        // with n_rem == 0 this is b0[0] = end of the full bands
  return tb;
}

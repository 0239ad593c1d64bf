// C ABI of the block-span server path: host-side session table, KV page allocator and
// the per-call kernel schedule.  See include/span.h for the contract of every entry point.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/span.h"
#include "common.h"
#include "launch.h"

namespace {

thread_local std::string g_err;

int fail(int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

struct Session {
  bool open = false;
  span_session_t id = -1;
  int first_block = 0, n_blocks = 0, max_len = 0, len = 0;
  std::vector<int> pages;
};

struct BlockWeights {
  bf16_t *w_qkv, *w_o, *w_up, *w_down;            // packed T16 (w_up = gate/up interleaved for LLAMA); codes when compressed
  float *s_qkv, *s_o, *s_up, *s_down;             // compressed weights: block scales
  float *norm1_g, *norm1_b, *b_qkv, *b_o, *norm2_g, *norm2_b, *b_up, *b_down;
  // LayerNorm folded into the following projection (decode path): W.gain and W.beta + bias
  float *wg_qkv, *bf_qkv, *wg_up, *bf_up;
};

// Derived sizes shared by span_query_sizes and span_create.
struct Layout {
  int d, qdim, kvdim, nqkv, F;
  int KT_d, KT_q, KT_f;                            // k tiles (32) of the padded K dims
  int nt_qkv, nt_o, nt_up, nt_down;                // physical row tiles, padded to 16
  int pps, Mpad;
  bool llama;
  size_t part_entries;
  // byte sizes
  size_t w_block_bytes, weight_bytes, kv_bytes, ws_bytes;
  // workspace offsets
  size_t o_pt, o_rope, o_alibi, o_resid, o_h, o_q, o_o, o_act, o_part, o_stat, o_tstat, o_rowstat, o_shift, o_share, o_count, o_expand;
  // per-block weight offsets
  size_t o_wqkv, o_wo, o_wup, o_wdown, o_vec;
  size_t o_sqkv, o_so, o_sup, o_sdown;             // compressed weights: block scales
  int bits;                                        // 16, 8 or 4
  size_t vec_floats;
};

int make_layout(const span_config &c, Layout &L) {
  L = Layout{};
  if (c.arch != SPAN_ARCH_LLAMA && c.arch != SPAN_ARCH_BLOOM) return fail(SPAN_E_INVALID, "unknown arch %d", c.arch);
  if (c.head_dim != 64 && c.head_dim != 128) return fail(SPAN_E_INVALID, "head_dim must be 64 or 128");
  if (c.n_blocks < 1 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.n_q_heads % c.n_kv_heads)
    return fail(SPAN_E_INVALID, "bad block / head counts");
  if (c.n_q_heads / c.n_kv_heads > 16) return fail(SPAN_E_INVALID, "at most 16 query heads per kv head");
  if (c.d_model < 32 || c.d_model % 32 || c.d_model > 16384) return fail(SPAN_E_INVALID, "d_model must be a multiple of 32, <= 16384");
  if (c.d_ff < 16 || c.d_ff % 16 || (c.arch == SPAN_ARCH_BLOOM && c.d_ff % 32))
    return fail(SPAN_E_INVALID, "d_ff must be a multiple of 16 (32 for BLOOM)");
  if (c.page_tokens != SPAN_PAGE) return fail(SPAN_E_INVALID, "page_tokens must be 16");
  if (c.max_pages < 1 || c.max_sessions < 1 || c.max_session_tokens < 1 || c.max_batch_tokens < 1)
    return fail(SPAN_E_INVALID, "capacities must be positive");
  if (c.io_dtype != SPAN_IO_BF16 && c.io_dtype != SPAN_IO_F32) return fail(SPAN_E_INVALID, "bad io_dtype");
  L.llama = c.arch == SPAN_ARCH_LLAMA;
  L.d = c.d_model; L.qdim = c.n_q_heads * c.head_dim; L.kvdim = c.n_kv_heads * c.head_dim;
  L.nqkv = L.qdim + 2 * L.kvdim; L.F = c.d_ff;
  L.KT_d = round_up(L.d, 128) / 32; L.KT_q = round_up(L.qdim, 128) / 32; L.KT_f = round_up(L.F, 128) / 32;   // tiled kernel: KT % 4 == 0
  L.nt_qkv = round_up(L.nqkv / 16, 16);
  L.nt_o = round_up(L.d / 16, 16);
  L.nt_up = round_up((L.llama ? 2 : 1) * L.F / 16, 16);
  L.nt_down = round_up(L.d / 16, 16);
  L.pps = ceil_div(c.max_session_tokens, SPAN_PAGE);
  L.Mpad = round_up(c.max_batch_tokens, 256);
  L.part_entries = (size_t)SPAN_MAX_CALL * c.n_kv_heads;
  if (L.part_entries < 4096) L.part_entries = 4096;

  L.bits = c.weight_bits == 0 ? 16 : c.weight_bits;
  if (L.bits != 16 && L.bits != 8 && L.bits != 4 && L.bits != 32) return fail(SPAN_E_INVALID, "weight_bits must be 0, 16, 8, 4 or 32");
  if (L.bits == 32) {
    // single-precision mode: fp32 weights as given (row-major), fp32 cache, fp32 rows everywhere
    if (c.io_dtype != SPAN_IO_F32) return fail(SPAN_E_INVALID, "weight_bits 32 (single-precision mode) needs io_dtype SPAN_IO_F32");
    if (c.max_batch_tokens > 65535) return fail(SPAN_E_INVALID, "single-precision mode takes at most 65535 tokens per call");
    const size_t mats = (size_t)L.nqkv * L.d + (size_t)L.d * L.qdim + (size_t)(L.llama ? 2 : 1) * L.F * L.d + (size_t)L.d * L.F;
    L.vec_floats = (size_t)4 * L.d + L.nqkv + 2 * (size_t)L.d + L.F;         // two norms (gain, bias), b_qkv, b_o, b_down, b_up
    L.o_vec = align256(mats * 4);
    L.w_block_bytes = L.o_vec + align256(L.vec_floats * 4);
    L.weight_bytes = L.w_block_bytes * c.n_blocks;
    L.kv_bytes = (size_t)c.n_blocks * c.max_pages * 2 * c.n_kv_heads * SPAN_PAGE * c.head_dim * 4;
    size_t o = 0;
    L.o_pt = o;    o += align256((size_t)c.max_sessions * L.pps * 4);
    L.o_rope = o;  o += align256((size_t)c.max_session_tokens * c.head_dim * 4);
    L.o_alibi = o; o += align256((size_t)c.n_q_heads * 4);
    L.o_resid = o; o += align256((size_t)c.max_batch_tokens * L.d * 4);
    L.o_h = o;     o += align256((size_t)c.max_batch_tokens * L.d * 4);
    L.o_q = o;     o += align256((size_t)c.max_batch_tokens * L.qdim * 4);
    L.o_o = o;     o += align256((size_t)c.max_batch_tokens * L.qdim * 4);
    L.o_act = o;   o += align256((size_t)c.max_batch_tokens * L.F * 4);
    L.ws_bytes = o;
    return SPAN_OK;
  }
  if (L.bits == 4)
    for (int i = 0; i < 16; ++i)
      if (!(c.levels[i] >= -1.0f && c.levels[i] <= 1.0f) || (i > 0 && !(c.levels[i] > c.levels[i - 1])))
        return fail(SPAN_E_INVALID, "levels must be 16 strictly ascending numbers in [-1, 1]");
  size_t o = 0;
  // bytes of a packed matrix of nt row tiles x KT k tiles, and of its block scales
  auto mat = [&](int nt, int KT) { return align256((size_t)nt * 16 * KT * 32 * L.bits / 8); };
  auto scl = [&](int nt, int KT) { return L.bits == 16 ? (size_t)0 : align256((size_t)nt * 16 * (KT / 2) * 4); };
  L.o_wqkv = o; o += mat(L.nt_qkv, L.KT_d);
  L.o_wo = o;   o += mat(L.nt_o, L.KT_q);
  L.o_wup = o;  o += mat(L.nt_up, L.KT_d);
  L.o_wdown = o; o += mat(L.nt_down, L.KT_f);
  L.o_sqkv = o; o += scl(L.nt_qkv, L.KT_d);
  L.o_so = o;   o += scl(L.nt_o, L.KT_q);
  L.o_sup = o;  o += scl(L.nt_up, L.KT_d);
  L.o_sdown = o; o += scl(L.nt_down, L.KT_f);
  L.o_vec = o;
  L.vec_floats = (size_t)2 * L.d + L.nqkv + L.d + 2 * L.d + L.F + L.d + 2 * (size_t)(L.nqkv + L.F);
  o += align256(L.vec_floats * 4);
  L.w_block_bytes = o;
  L.weight_bytes = o * c.n_blocks;
  L.kv_bytes = (size_t)c.n_blocks * c.max_pages * 2 * c.n_kv_heads * SPAN_PAGE * c.head_dim * 2;

  o = 0;
  L.o_pt = o;    o += align256((size_t)c.max_sessions * L.pps * 4);
  L.o_rope = o;  o += align256((size_t)c.max_session_tokens * c.head_dim * 4);
  L.o_alibi = o; o += align256((size_t)c.n_q_heads * 4);
  L.o_resid = o; o += align256((size_t)L.Mpad * L.d * 4);
  L.o_h = o;     o += align256((size_t)L.Mpad * L.KT_d * 32 * 2);
  L.o_q = o;     o += align256((size_t)L.Mpad * L.qdim * 2);
  L.o_o = o;     o += align256((size_t)L.Mpad * L.KT_q * 32 * 2);
  L.o_act = o;   o += align256((size_t)L.Mpad * L.KT_f * 32 * 2);
  L.o_part = o;  o += align256(L.part_entries * 16 * (c.head_dim + 2) * 4);
  L.o_stat = o;  o += align256((size_t)(L.d / 32 + 1) * 128 * 4);
  // fused norm of the tiled path: partial sums per (128 features, row) and the finished row statistics
  L.o_tstat = o; o += align256((size_t)(L.nt_o / 4) * L.Mpad * 2 * 4);          // per (quad of 64 features, row)
  L.o_rowstat = o; o += align256((size_t)L.Mpad * 2 * 4);
  L.o_shift = o; o += align256((size_t)L.Mpad * 4);
  L.o_share = o; o += align256(gemv_share_part_bytes());
  {
    int np = L.nt_qkv > L.nt_up ? L.nt_qkv : L.nt_up;
    if (L.nt_o > np) np = L.nt_o;
    L.o_count = o; o += align256((size_t)np * 4);          // one counter per tile pair, generously
  }
  // compressed weights: room to expand the largest matrix to bf16 for the tiled kernels
  L.o_expand = o;
  if (L.bits != 16) {
    size_t mx = (size_t)L.nt_qkv * L.KT_d;
    if ((size_t)L.nt_o * L.KT_q > mx) mx = (size_t)L.nt_o * L.KT_q;
    if ((size_t)L.nt_up * L.KT_d > mx) mx = (size_t)L.nt_up * L.KT_d;
    if ((size_t)L.nt_down * L.KT_f > mx) mx = (size_t)L.nt_down * L.KT_f;
    o += align256(mx * 1024);
  }
  L.ws_bytes = o;
  return SPAN_OK;
}

// Split of the decode attention along the keys: every split covers `split_pp` page pairs
// (32 keys each), chosen so that the whole batch gives about 1024 waves (four per CU); a session
// then has ceil(its pairs / split_pp) splits.  Returns the largest split count (the grid size).
int choose_splits(const BatchMeta &meta, int n_kv_heads, size_t part_entries, int *split_pp) {
  long total_pp = 0;
  int max_pp = 1;
  for (int i = 0; i < meta.n_sess; ++i) {
    const int pp = ceil_div(meta.past[i] + 1, 32);
    total_pp += pp;
    if (pp > max_pp) max_pp = pp;
  }
  int c = (int)((total_pp * n_kv_heads + 1023) / 1024);
  if (c < 1) c = 1;
  // at most 64 splits (the merge kernel keeps one split per lane) and no more partial results
  // than the workspace holds
  while (ceil_div(max_pp, c) > 64 || (size_t)meta.n_sess * n_kv_heads * ceil_div(max_pp, c) > part_entries) ++c;
  *split_pp = c;
  return ceil_div(max_pp, c);
}

}  // namespace

struct ProfRecord { int cls; hipEvent_t a, b; };

struct span_t {
  bool profiling = false;
  std::vector<ProfRecord> prof;
  span_config cfg;
  Layout L;
  std::vector<BlockWeights> blocks;
  KvPool pool;
  int *page_table;
  float *rope, *alibi, *resid, *part, *stat, *tstat, *row_stat, *shift;
  GemvShare share;
  bf16_t *expand;                     // compressed weights: scratch for one expanded matrix
  LevelTable levels{};                // codebook format: the levels as used (rounded to bf16)
  bf16_t *h, *q, *o, *act;
  std::vector<Session> sessions;
  std::vector<int> free_pages;
  std::vector<int> page_ref;          // sessions listing each page (0 = free); > 1 only after span_reorder
  span_session_t next_id = 1;
  // single-precision mode (weight_bits 32): fp32 copies of the canonical weights and the call's fp32 buffers
  std::vector<F32Block> f32_blocks;
  F32Call f32{};
  // test taps armed by span_debug_tap for the next forward call (index = SPAN_TAP_* - 1)
  struct Tap {
    bool armed = false;
    int block = 0, head = 0, q0 = 0, nq = 0;
    span_session_t session = -1;
    void *out = nullptr;
    size_t out_bytes = 0;
    int k = -1;                       // resolved by the call: index of the session among the call's sessions
  } taps[3];
  // training-time passes (span_train_attach)
  struct Train {
    bool on = false;
    int max_tokens = 0;
    int Kup, KT_nq, KT_up, nt_q, nt_f;             // K of the transposed up projection; k tiles; row tiles
    size_t wt_block_bytes, o_qkv, o_o, o_up, o_down;   // transposed weights of one block
    char *wt = nullptr;
    // per block rows kept between the sweeps, each [n_blocks][max_tokens][...]
    float *xs, *x1, *o, *lse, *pre;
    bf16_t *q;                                     // [n_blocks][max_tokens][Hq*hd] queries after rotary
    KvPool pool, pool2;                            // the call's keys / values in pages (block index = position in the call)
    int *pt;                                       // [SPAN_MAX_CALL][pps] page table of the call's sequences
    // shared by all blocks
    float *dres, *dh, *da, *dob, *dqkv, *delta;
    bf16_t *t_qkv, *t_up;
    bf16_t *q_t, *do_t;                            // transposed copies for the attention backward kernel
    int ld_t;
    bf16_t *t_wt;                                  // compressed spans: the transposed matrix of the current projection
  } train;
};

namespace {

Session *find_session(span_t *sp, span_session_t id, int *slot = nullptr) {
  for (size_t i = 0; i < sp->sessions.size(); ++i)
    if (sp->sessions[i].open && sp->sessions[i].id == id) {
      if (slot) *slot = (int)i;
      return &sp->sessions[i];
    }
  return nullptr;
}

int hip_check(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SPAN_E_HIP, "%s: %s", what, hipGetErrorString(e));
  return SPAN_OK;
}

// Enqueue all kernels of one forward call.  Host state is already reserved by the caller.
int enqueue_forward(span_t *sp, const BatchMeta &meta, int first_block, int n_blocks, bool all_single,
                    int max_len_after, const void *x, void *y, hipStream_t st) {
  const span_config &c = sp->cfg;
  const Layout &L = sp->L;
  const int M = meta.cu[meta.n_sess];
  if (L.bits == 32) {
    F32Call fc = sp->f32;
    fc.x_in = (const float *)x;
    for (int bi = 0; bi < n_blocks; ++bi)
      launch_f32_block(fc, sp->f32_blocks[first_block + bi], meta, first_block + bi, bi == 0,
                       bi == n_blocks - 1 ? (float *)y : nullptr, st);
    return hip_check("span_forward kernels (single precision)");
  }
  const bool skinny = M <= 64;
  const int m_tiles = ceil_div(M, 16);
  // row tiles per k step of this call's activation buffers (k-major T16)
  const int x_RT = skinny ? m_tiles : round_up(M, gemm_token_tile(M)) / 16;

  int q_tiles = 0;
  if (!all_single) {
    const int qt = attn_prefill_q_tile();
    for (int i = 0; i < meta.n_sess; ++i) q_tiles += ceil_div(meta.cu[i + 1] - meta.cu[i], qt);
  }
  int split_pp = 1;
  const int n_splits = all_single ? choose_splits(meta, c.n_kv_heads, L.part_entries, &split_pp) : 1;

  // optional per-launch event bracket (roofline report only)
  auto timed = [&](int cls, auto &&launch) {
    if (!sp->profiling) { launch(); return; }
    ProfRecord r{cls, nullptr, nullptr};
    if (hipEventCreateWithFlags(&r.a, hipEventDisableSystemFence) != hipSuccess ||
        hipEventCreateWithFlags(&r.b, hipEventDisableSystemFence) != hipSuccess) { launch(); return; }
    (void)hipEventRecord(r.a, st);
    launch();
    (void)hipEventRecord(r.b, st);
    sp->prof.push_back(r);
  };
  // A long call whose last 256-token tile holds only a few rows (a replaying session batched with
  // single-token sessions; a ragged last chunk) gives those rows to the skinny kernel instead of
  // paying a whole tile column of every projection for them.
  const int tail = (!skinny && M > 1024 && M % 256 > 0 && M % 256 <= 64) ? M % 256 : 0;
  const int M_tiled = M - tail;
  // short calls run their narrow projections (compressed spans: all of them) as skinny launches over chunks of 64 rows
  const bool short_chunks = !skinny && (L.bits != 16 ? M <= 192 : M <= 128);
  auto linear = [&](const bf16_t *wp, const float *scales, const bf16_t *xp, int KT, int n_pairs, int nt_pad, const EpiArgs &e) {
    EpiArgs et = e;                       // the tail rows: same call, rows [M_tiled, M)
    et.m0 = M_tiled;
    const bf16_t *xt = xp + (size_t)(M_tiled / 16) * 512;
    const int tail_tiles = ceil_div(tail, 16);
    // A call of 65 ... 128 rows gives a narrow projection (at most 64 tiles of 256 weight rows: q/k/v,
    // attention output, MLP down at the 70B shape) too few tiles for the chip: the tiled kernel then
    // needs 90 us for what the skinny kernel streams in 31 us per 64 rows, so the rows go through the
    // skinny kernel in chunks of 64 (beyond two chunks the tiled kernel wins again).  Compressed weights
    // are chunked whatever the width and up to 192 rows (the tiled path would first expand the whole
    // matrix to bf16).
    if (short_chunks && (L.bits != 16 || nt_pad / 16 <= 64)) {
      for (int r0 = 0; r0 < M; r0 += 64) {
        EpiArgs ec = e;
        ec.m0 = r0;
        const bf16_t *xc = xp + (size_t)(r0 / 16) * 512;
        const int tiles = ceil_div(std::min(64, M - r0), 16);
        if (L.bits != 16) {
          QWeights qw{(const uint8_t *)wp, scales, nt_pad, L.bits, {}, {}};
          for (int i = 0; i < 4; ++i) { qw.lut_lo[i] = sp->levels.lut_lo[i]; qw.lut_hi[i] = sp->levels.lut_hi[i]; }
          timed(SPAN_K_SKINNY, [&] { launch_gemvq(qw, xc, x_RT, KT / 2, n_pairs, tiles, sp->share, ec, meta, st); });
        } else {
          timed(SPAN_K_SKINNY, [&] { launch_gemv(wp, nt_pad, xc, x_RT, KT, n_pairs, tiles, sp->share, ec, meta, st); });
        }
      }
      return;
    }
    if (L.bits != 16) {
      // compressed weights: short calls stream the codes; long calls expand the matrix to bf16
      // tiles in scratch (a few % of the projection's time) and run the tiled kernel on it
      QWeights qw{(const uint8_t *)wp, scales, nt_pad, L.bits, {}, {}};
      for (int i = 0; i < 4; ++i) { qw.lut_lo[i] = sp->levels.lut_lo[i]; qw.lut_hi[i] = sp->levels.lut_hi[i]; }
      if (skinny) timed(SPAN_K_SKINNY, [&] { launch_gemvq(qw, xp, x_RT, KT / 2, n_pairs, m_tiles, sp->share, e, meta, st); });
      else {
        launch_expand_q(qw, KT / 2, sp->expand, st);
        timed(SPAN_K_TILED, [&] { launch_gemm(sp->expand, nt_pad, xp, x_RT, KT, M_tiled, e, meta, st); });
        if (tail) timed(SPAN_K_SKINNY, [&] { launch_gemvq(qw, xt, x_RT, KT / 2, n_pairs, tail_tiles, sp->share, et, meta, st); });
      }
    } else if (skinny) timed(SPAN_K_SKINNY, [&] { launch_gemv(wp, nt_pad, xp, x_RT, KT, n_pairs, m_tiles, sp->share, e, meta, st); });
    else {
      timed(SPAN_K_TILED, [&] { launch_gemm(wp, nt_pad, xp, x_RT, KT, M_tiled, e, meta, st); });
      if (tail) timed(SPAN_K_SKINNY, [&] { launch_gemv(wp, nt_pad, xt, x_RT, KT, n_pairs, tail_tiles, sp->share, et, meta, st); });
    }
  };

  for (int bi = 0; bi < n_blocks; ++bi) {
    const int ab = first_block + bi;
    const BlockWeights &w = sp->blocks[ab];

    // Decode steps (skinny path) fold every norm but the span's first into its neighbours:
    // the projection that produces a residual row also emits the gain-scaled bf16 input of
    // the next projection plus partial row statistics, and that projection finishes the
    // norm on its accumulators.
    // (with compressed weights the LayerNorm fold would need W'.gain of the dequantised matrices,
    // which are not kept; RMSNorm folds without touching the weights)
    // Long calls that run every projection as tiles fold the norms the same way: the tiled residual
    // epilogue leaves partial sums per (row, 128 features), a small kernel finishes them per row, and
    // the next projection's epilogue applies them (the stand-alone norm of 16384 rows costs 345 us,
    // twice per block).  Calls with skinny tail rows or chunks keep the stand-alone norm.
    const bool tiled_all = !skinny && tail == 0 && !short_chunks;
    const bool fused = (skinny || tiled_all) && (L.bits == 16 || L.llama);
    auto consumer = [&](EpiArgs &e2, const float *wg, const float *bias_folded) {
      e2.stat_in = sp->stat; e2.stat_parts = L.d / 32; e2.norm_d = L.d; e2.norm_eps = c.norm_eps;
      e2.norm_center = !L.llama; e2.wg = wg;
      if (!L.llama) { e2.bias = bias_folded; e2.shift = sp->shift; }
      if (!skinny) e2.row_stat = sp->row_stat;
    };
    auto producer = [&](EpiArgs &e2, const float *gain) {
      e2.next_gain = gain; e2.h_out = sp->h; e2.h_RT = x_RT;
      if (!L.llama) e2.shift = sp->shift;
      if (skinny) e2.stat_out = sp->stat;
      else { e2.tstat_out = sp->tstat; e2.tstat_ld = L.Mpad; }
    };
    // after a tiled producer: partial sums -> row statistics
    auto finish_stats = [&]() {
      if (fused && !skinny)
        timed(SPAN_K_NORM, [&] { launch_row_stat(sp->tstat, L.nt_o / 4, L.Mpad, sp->row_stat, M, L.d, c.norm_eps, !L.llama,
                                                   L.llama ? nullptr : sp->shift, st); });
    };

    NormArgs n1{};
    n1.x_in = bi == 0 ? x : nullptr; n1.x_f32 = c.io_dtype == SPAN_IO_F32;
    n1.resid = sp->resid; n1.gain = w.norm1_g; n1.bias = L.llama ? nullptr : w.norm1_b;
    n1.layernorm = !L.llama; n1.eps = c.norm_eps; n1.d = L.d; n1.RT = x_RT; n1.M = M; n1.h_out = sp->h;
    n1.shift_out = (fused && !L.llama) ? sp->shift : nullptr;
    if (!fused || bi == 0) timed(SPAN_K_NORM, [&] { launch_norm(n1, st); });

    EpiArgs e{};
    e.kind = EPI_QKV; e.M = M; e.N = L.nqkv; e.bias = L.llama ? nullptr : w.b_qkv;
    e.n_q_heads = c.n_q_heads; e.n_kv_heads = c.n_kv_heads; e.head_dim = c.head_dim; e.rotary = L.llama;
    e.rope = sp->rope; e.q_out = sp->q; e.pool = sp->pool; e.block = ab;
    e.page_table = sp->page_table; e.pages_per_session = L.pps;
    if (fused && bi > 0) consumer(e, w.wg_qkv, w.bf_qkv);
    linear(w.w_qkv, w.s_qkv, sp->h, L.KT_d, L.nqkv / 32, L.nt_qkv, e);

    // test taps (span_debug_tap): copies of what the projection just wrote
    const span_t::Tap &tq = sp->taps[SPAN_TAP_Q_ROT - 1], &tk = sp->taps[SPAN_TAP_K_ROT - 1], &tl = sp->taps[SPAN_TAP_LOGITS - 1];
    if (tq.armed && tq.k >= 0 && tq.block == bi)
      (void)hipMemcpyAsync(tq.out, sp->q + (size_t)(meta.cu[tq.k] + tq.q0) * L.qdim, (size_t)tq.nq * L.qdim * 2,
                           hipMemcpyDeviceToDevice, st);
    if (tk.armed && tk.k >= 0 && tk.block == bi)
      launch_kv_gather(sp->pool, ab, sp->page_table + (size_t)meta.slot[tk.k] * L.pps, meta.past[tk.k] + tk.q0, tk.nq,
                       (bf16_t *)tk.out, nullptr, st);

    AttnArgs a{};
    a.q = sp->q; a.pool = sp->pool; a.block = ab; a.page_table = sp->page_table; a.pages_per_session = L.pps;
    a.n_q_heads = c.n_q_heads; a.n_kv_heads = c.n_kv_heads; a.head_dim = c.head_dim;
    a.alibi = L.llama ? nullptr : sp->alibi; a.o_out = sp->o; a.o_RT = x_RT;
    a.n_splits = n_splits; a.split_pp = split_pp; a.part = sp->part; a.logits = nullptr; a.logits_ld = 0;
    if (tl.armed && tl.k >= 0 && tl.block == bi) {
      a.tap_logits = (float *)tl.out; a.tap_sess = tl.k; a.tap_head = tl.head; a.tap_q0 = tl.q0; a.tap_nq = tl.nq;
      a.tap_ld = meta.past[tl.k] + (meta.cu[tl.k + 1] - meta.cu[tl.k]);
    }
    if (all_single) {
      timed(SPAN_K_ATTN_DECODE, [&] { launch_attn_decode(a, meta, st); });
      timed(SPAN_K_ATTN_MERGE, [&] { launch_attn_merge(a, meta, nullptr, st); });
    } else {
      timed(SPAN_K_ATTN_PREFILL, [&] { launch_attn_prefill(a, meta, q_tiles, st); });
    }

    EpiArgs eo{};
    eo.kind = EPI_RESID; eo.M = M; eo.N = L.d; eo.bias = L.llama ? nullptr : w.b_o; eo.resid = sp->resid;
    if (fused) producer(eo, w.norm2_g);
    linear(w.w_o, w.s_o, sp->o, L.KT_q, L.d / 32, L.nt_o, eo);
    finish_stats();

    NormArgs n2 = n1;
    n2.x_in = nullptr; n2.gain = w.norm2_g; n2.bias = L.llama ? nullptr : w.norm2_b;
    if (!fused) timed(SPAN_K_NORM, [&] { launch_norm(n2, st); });

    EpiArgs eu{};
    eu.M = M; eu.N = L.F; eu.act_out = sp->act; eu.act_RT = x_RT;
    if (fused) consumer(eu, w.wg_up, w.bf_up);
    if (L.llama) { eu.kind = EPI_SWIGLU; linear(w.w_up, w.s_up, sp->h, L.KT_d, L.F / 16, L.nt_up, eu); }
    else { eu.kind = EPI_GELU; if (!fused) eu.bias = w.b_up; linear(w.w_up, w.s_up, sp->h, L.KT_d, L.F / 32, L.nt_up, eu); }

    EpiArgs ed{};
    ed.kind = EPI_RESID; ed.M = M; ed.N = L.d; ed.bias = L.llama ? nullptr : w.b_down; ed.resid = sp->resid;
    if (bi == n_blocks - 1) { ed.y = y; ed.y_f32 = c.io_dtype == SPAN_IO_F32; }
    else if (fused) producer(ed, sp->blocks[ab + 1].norm1_g);
    linear(w.w_down, w.s_down, sp->act, L.KT_f, L.d / 32, L.nt_down, ed);
    if (bi != n_blocks - 1) finish_stats();
  }
  return hip_check("span_forward kernels");
}

void push_page_table(span_t *sp, const std::vector<int> &idx, const std::vector<int> &val, hipStream_t st);

struct Reservation {
  int slot;
  size_t pages_before;
};

// Validates, reserves pages, enqueues, commits.  On any error nothing has changed.
int forward_impl(span_t *sp, int n, const span_session_t *ids, const int *ntok, const void *x, void *y,
                 hipStream_t st) {
  if (!sp) return fail(SPAN_E_INVALID, "null span");
  // test taps are one-shot: whatever happens to this call, they are disarmed when it returns
  struct Disarm {
    span_t *sp;
    ~Disarm() { for (auto &t : sp->taps) t = span_t::Tap{}; }
  } disarm{sp};
  if (n < 0 || n > SPAN_MAX_CALL_SESSIONS) return fail(SPAN_E_INVALID, "n_sessions %d outside [0, %d]", n, SPAN_MAX_CALL_SESSIONS);
  if (n > 0 && (!ids || !ntok)) return fail(SPAN_E_INVALID, "null session or token-count array");
  const Layout &L = sp->L;
  BatchMeta meta{};
  int slots[SPAN_MAX_CALL_SESSIONS];
  int total = 0, need_pages = 0, fb = -1, nb = -1, max_len_after = 0;
  bool all_single = true;
  for (int i = 0; i < n; ++i) {
    int slot;
    Session *s = find_session(sp, ids[i], &slot);
    if (!s) return fail(SPAN_E_BAD_SESSION, "session %d is not open", ids[i]);
    for (int j = 0; j < i; ++j)
      if (slots[j] == slot) return fail(SPAN_E_DUPLICATE, "session %d listed twice", ids[i]);
    slots[i] = slot;
    if (ntok[i] < 0) return fail(SPAN_E_INVALID, "negative token count for session %d", ids[i]);
    if (fb < 0) { fb = s->first_block; nb = s->n_blocks; }
    else if (fb != s->first_block || nb != s->n_blocks)
      return fail(SPAN_E_MIXED_SPANS, "sessions of one call must share a block range");
    if ((long long)s->len + ntok[i] > s->max_len)
      return fail(SPAN_E_TOO_LONG, "session %d: %d + %d tokens exceeds max_len %d", ids[i], s->len, ntok[i], s->max_len);
    total += ntok[i];
    if (total > sp->cfg.max_batch_tokens)
      return fail(SPAN_E_TOO_MANY_TOKENS, "call carries more than max_batch_tokens = %d tokens", sp->cfg.max_batch_tokens);
    if (ntok[i] == 0) continue;
    if (ntok[i] != 1) all_single = false;
    need_pages += ceil_div(s->len + ntok[i], SPAN_PAGE) - (int)s->pages.size();
    const int k = meta.n_sess++;
    meta.cu[k + 1] = meta.cu[k] + ntok[i];
    meta.past[k] = s->len;
    meta.slot[k] = slot;
    if (s->len + ntok[i] > max_len_after) max_len_after = s->len + ntok[i];
  }
  for (int w = 0; w < 3; ++w) {
    span_t::Tap &t = sp->taps[w];
    if (!t.armed) continue;
    t.k = -1;
    for (int k = 0; k < meta.n_sess; ++k)
      if (sp->sessions[meta.slot[k]].id == t.session) t.k = k;
    if (t.k < 0) return fail(SPAN_E_INVALID, "tap: session %d brings no tokens in this call", t.session);
    const int T = meta.cu[t.k + 1] - meta.cu[t.k], len_after = meta.past[t.k] + T;
    if (t.block >= nb) return fail(SPAN_E_INVALID, "tap: block %d outside the session's range", t.block);
    if (t.q0 + t.nq > T) return fail(SPAN_E_INVALID, "tap: tokens [%d, %d) outside the session's %d new tokens", t.q0, t.q0 + t.nq, T);
    size_t need = 0;
    if (w == SPAN_TAP_Q_ROT - 1) need = (size_t)t.nq * L.qdim * 2;
    if (w == SPAN_TAP_K_ROT - 1) need = (size_t)t.nq * L.kvdim * 2;
    if (w == SPAN_TAP_LOGITS - 1) {
      need = (size_t)t.nq * len_after * 4;
      if (all_single) return fail(SPAN_E_INVALID, "tap: the logits tap needs a call with a multi-token session (decode steps: span_op_attn_decode)");
    }
    if (t.out_bytes < need) return fail(SPAN_E_INVALID, "tap: out holds %zu bytes, %zu needed", t.out_bytes, need);
  }
  if (total == 0) return SPAN_OK;
  if (!sp->cfg.dry_run && (!x || !y)) return fail(SPAN_E_INVALID, "null x or y");
  if (need_pages > (int)sp->free_pages.size())
    return fail(SPAN_E_CACHE_FULL, "need %d KV pages, %zu free", need_pages, sp->free_pages.size());

  // reserve
  std::vector<Reservation> res;
  std::vector<int> upd_idx, upd_val;
  for (int k = 0; k < meta.n_sess; ++k) {
    Session &s = sp->sessions[meta.slot[k]];
    const int T = meta.cu[k + 1] - meta.cu[k];
    res.push_back({meta.slot[k], s.pages.size()});
    const int want = ceil_div(s.len + T, SPAN_PAGE);
    while ((int)s.pages.size() < want) {
      const int pg = sp->free_pages.back();
      sp->free_pages.pop_back();
      sp->page_ref[pg] = 1;
      upd_idx.push_back(meta.slot[k] * L.pps + (int)s.pages.size());
      upd_val.push_back(pg);
      s.pages.push_back(pg);
    }
  }
  auto rollback = [&]() {
    for (auto it = res.rbegin(); it != res.rend(); ++it) {
      Session &s = sp->sessions[it->slot];
      while (s.pages.size() > it->pages_before) {
        sp->page_ref[s.pages.back()] = 0;
        sp->free_pages.push_back(s.pages.back());
        s.pages.pop_back();
      }
    }
  };

  if (!sp->cfg.dry_run) {
    push_page_table(sp, upd_idx, upd_val, st);
    int rc = hip_check("page table update");
    if (rc == SPAN_OK) rc = enqueue_forward(sp, meta, fb, nb, all_single, max_len_after, x, y, st);
    if (rc != SPAN_OK) { rollback(); return rc; }
  }
  for (int k = 0; k < meta.n_sess; ++k) sp->sessions[meta.slot[k]].len += meta.cu[k + 1] - meta.cu[k];
  return SPAN_OK;
}

void clear_profile(span_t *sp) {
  for (auto &r : sp->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  sp->prof.clear();
}

void release_session_pages(span_t *sp, Session &s) {
  while (!s.pages.empty()) {
    if (--sp->page_ref[s.pages.back()] == 0) sp->free_pages.push_back(s.pages.back());
    s.pages.pop_back();
  }
  s.len = 0;
}

void push_page_table(span_t *sp, const std::vector<int> &idx, const std::vector<int> &val, hipStream_t st) {
  for (size_t off = 0; off < idx.size(); off += 120) {
    PtUpdate u{};
    u.n = (int)std::min<size_t>(120, idx.size() - off);
    for (int i = 0; i < u.n; ++i) { u.idx[i] = idx[off + i]; u.val[i] = val[off + i]; }
    launch_pt_update(sp->page_table, u, st);
  }
}

}  // namespace

extern "C" {

const char *span_last_error(void) { return g_err.c_str(); }

int span_query_sizes(const span_config *cfg, size_t *weight_bytes, size_t *kv_bytes, size_t *workspace_bytes) {
  if (!cfg) return fail(SPAN_E_INVALID, "null config");
  Layout L;
  int rc = make_layout(*cfg, L);
  if (rc) return rc;
  if (weight_bytes) *weight_bytes = L.weight_bytes;
  if (kv_bytes) *kv_bytes = L.kv_bytes;
  if (workspace_bytes) *workspace_bytes = L.ws_bytes;
  return SPAN_OK;
}

int span_create(const span_config *cfg, const span_block_weights *weights, void *weight_arena, void *kv_arena,
                void *workspace, void *stream, span_t **out) {
  if (!cfg || !out) return fail(SPAN_E_INVALID, "null config or output");
  Layout L;
  int rc = make_layout(*cfg, L);
  if (rc) return rc;
  const bool dry = cfg->dry_run != 0;
  if (!dry && (!weights || !weight_arena || !kv_arena || !workspace))
    return fail(SPAN_E_INVALID, "null weights or arena");
  if (!dry) {
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
      (void)hipGetLastError();
      return fail(SPAN_E_HIP, "no HIP device: this library has no CPU fallback");
    }
  }
  span_t *sp = new span_t();
  sp->cfg = *cfg;
  sp->L = L;
  sp->sessions.resize(cfg->max_sessions);
  sp->free_pages.reserve(cfg->max_pages);
  for (int p = cfg->max_pages - 1; p >= 0; --p) sp->free_pages.push_back(p);   // page 0 is handed out first
  sp->page_ref.assign(cfg->max_pages, 0);
  sp->pool = KvPool{(bf16_t *)kv_arena, cfg->max_pages, cfg->n_kv_heads, cfg->head_dim};
  sp->blocks.resize(cfg->n_blocks);
  sp->page_table = nullptr; sp->rope = sp->alibi = sp->resid = sp->part = sp->stat = sp->tstat = sp->row_stat = sp->shift = nullptr;
  sp->h = sp->q = sp->o = sp->act = nullptr;
  sp->share = GemvShare{0, nullptr, nullptr};
  sp->expand = nullptr;
  if (dry) { *out = sp; return SPAN_OK; }
  char *ws = (char *)workspace;
  sp->page_table = (int *)(ws + L.o_pt);
  sp->rope = (float *)(ws + L.o_rope);
  sp->alibi = (float *)(ws + L.o_alibi);
  sp->resid = (float *)(ws + L.o_resid);
  sp->h = (bf16_t *)(ws + L.o_h);
  sp->q = (bf16_t *)(ws + L.o_q);
  sp->o = (bf16_t *)(ws + L.o_o);
  sp->act = (bf16_t *)(ws + L.o_act);
  sp->part = (float *)(ws + L.o_part);
  sp->stat = (float *)(ws + L.o_stat);
  sp->tstat = (float *)(ws + L.o_tstat);
  sp->row_stat = (float *)(ws + L.o_rowstat);
  sp->shift = (float *)(ws + L.o_shift);
  sp->share = GemvShare{0, (f32x4 *)(ws + L.o_share), (unsigned *)(ws + L.o_count)};
  sp->expand = (bf16_t *)(ws + L.o_expand);

  hipStream_t st = (hipStream_t)stream;
  // Zero the workspace (the k-padding of the activation buffers must stay zero) and the KV
  // pool (a never-written slot must hold a finite value: it meets a zero probability).
  launch_fill_u32((uint32_t *)workspace, L.ws_bytes / 4, 0u, st);
  launch_fill_u32((uint32_t *)kv_arena, L.kv_bytes / 4, 0u, st);
  if (L.llama) launch_rope_table(sp->rope, cfg->max_session_tokens, cfg->head_dim, (double)cfg->rope_base, st);
  else launch_alibi_slopes(sp->alibi, cfg->n_q_heads, st);

  if (L.bits == 32) {
    F32Call &fc = sp->f32;
    fc.resid = sp->resid; fc.h = (float *)(ws + L.o_h); fc.q = (float *)(ws + L.o_q); fc.o = (float *)(ws + L.o_o);
    fc.act = (float *)(ws + L.o_act);
    fc.d = L.d; fc.Hq = cfg->n_q_heads; fc.Hkv = cfg->n_kv_heads; fc.hd = cfg->head_dim; fc.F = L.F;
    fc.layernorm = !L.llama; fc.rotary = L.llama; fc.eps = cfg->norm_eps;
    fc.rope = sp->rope; fc.alibi = L.llama ? nullptr : sp->alibi;
    fc.pool = F32Pool{(float *)kv_arena, cfg->max_pages, cfg->n_kv_heads, cfg->head_dim};
    fc.page_table = sp->page_table; fc.pps = L.pps;
    sp->f32_blocks.resize(cfg->n_blocks);
    for (int b = 0; b < cfg->n_blocks; ++b) {
      const span_block_weights &w = weights[b];
      const bool need_bias = !L.llama;
      if (!w.norm1_g || !w.wq || !w.wk || !w.wv || !w.wo || !w.norm2_g || !w.w_up || !w.w_down || (L.llama && !w.w_gate) ||
          (need_bias && (!w.norm1_b || !w.bq || !w.bk || !w.bv || !w.bo || !w.norm2_b || !w.b_up || !w.b_down))) {
        delete sp;
        return fail(SPAN_E_INVALID, "block %d: a required weight pointer is null", b);
      }
      float *dst = (float *)((char *)weight_arena + (size_t)b * L.w_block_bytes);
      auto keep = [&](const void *src, size_t n) -> const float * {      // copy n floats into the arena
        if (!src) return nullptr;
        float *at = dst;
        (void)hipMemcpyAsync(at, src, n * 4, hipMemcpyDeviceToDevice, st);
        dst += n;
        return at;
      };
      F32Block &f = sp->f32_blocks[b];
      f.wq = keep(w.wq, (size_t)L.qdim * L.d); f.wk = keep(w.wk, (size_t)L.kvdim * L.d); f.wv = keep(w.wv, (size_t)L.kvdim * L.d);
      f.wo = keep(w.wo, (size_t)L.d * L.qdim);
      f.w_gate = L.llama ? keep(w.w_gate, (size_t)L.F * L.d) : nullptr;
      f.w_up = keep(w.w_up, (size_t)L.F * L.d); f.w_down = keep(w.w_down, (size_t)L.d * L.F);
      dst = (float *)((char *)weight_arena + (size_t)b * L.w_block_bytes + L.o_vec);
      f.norm1_g = keep(w.norm1_g, L.d); f.norm2_g = keep(w.norm2_g, L.d);
      f.norm1_b = need_bias ? keep(w.norm1_b, L.d) : nullptr; f.norm2_b = need_bias ? keep(w.norm2_b, L.d) : nullptr;
      f.bq = need_bias ? keep(w.bq, L.qdim) : nullptr; f.bk = need_bias ? keep(w.bk, L.kvdim) : nullptr;
      f.bv = need_bias ? keep(w.bv, L.kvdim) : nullptr; f.bo = need_bias ? keep(w.bo, L.d) : nullptr;
      f.b_up = need_bias ? keep(w.b_up, L.F) : nullptr; f.b_down = need_bias ? keep(w.b_down, L.d) : nullptr;
    }
    rc = hip_check("span_create copies (single precision)");
    if (rc) { delete sp; return rc; }
    *out = sp;
    return SPAN_OK;
  }

  QuantArgs qa{};
  qa.bits = L.bits;
  if (L.bits == 4) {
    sp->levels = make_level_table(cfg->levels);
    for (int i = 0; i < 15; ++i) qa.mids[i] = sp->levels.mids[i];
  }
  for (int b = 0; b < cfg->n_blocks; ++b) {
    const span_block_weights &w = weights[b];
    char *base = (char *)weight_arena + (size_t)b * L.w_block_bytes;
    BlockWeights &bw = sp->blocks[b];
    bw.s_qkv = (float *)(base + L.o_sqkv); bw.s_o = (float *)(base + L.o_so);
    bw.s_up = (float *)(base + L.o_sup);   bw.s_down = (float *)(base + L.o_sdown);
    auto pack = [&](const PackArgs &pa, int nt, float *scales) {
      if (L.bits == 16) { launch_pack_weight(pa, nt, st); return; }
      QuantArgs q = qa;
      q.codes = (uint8_t *)pa.dst; q.scales = scales; q.absmax_out = nullptr;
      launch_pack_weight_q(pa, q, nt, st);
    };
    bw.w_qkv = (bf16_t *)(base + L.o_wqkv); bw.w_o = (bf16_t *)(base + L.o_wo);
    bw.w_up = (bf16_t *)(base + L.o_wup);   bw.w_down = (bf16_t *)(base + L.o_wdown);
    float *v = (float *)(base + L.o_vec);
    bw.norm1_g = v; v += L.d; bw.norm1_b = v; v += L.d; bw.b_qkv = v; v += L.nqkv; bw.b_o = v; v += L.d;
    bw.norm2_g = v; v += L.d; bw.norm2_b = v; v += L.d; bw.b_up = v; v += L.F; bw.b_down = v; v += L.d;
    bw.wg_qkv = v; v += L.nqkv; bw.bf_qkv = v; v += L.nqkv; bw.wg_up = v; v += L.F; bw.bf_up = v;

    const bool need_bias = !L.llama;
    if (!w.norm1_g || !w.wq || !w.wk || !w.wv || !w.wo || !w.norm2_g || !w.w_up || !w.w_down ||
        (L.llama && !w.w_gate) ||
        (need_bias && (!w.norm1_b || !w.bq || !w.bk || !w.bv || !w.bo || !w.norm2_b || !w.b_up || !w.b_down))) {
      delete sp;
      return fail(SPAN_E_INVALID, "block %d: a required weight pointer is null", b);
    }
    launch_fill_u32((uint32_t *)(base + L.o_vec), L.vec_floats, 0u, st);

    PackArgs p{};
    p.order = PACK_HEADS; p.src[0] = (const bf16_t *)w.wq; p.src[1] = (const bf16_t *)w.wk; p.src[2] = (const bf16_t *)w.wv;
    p.rows[0] = L.qdim; p.rows[1] = L.kvdim; p.rows[2] = L.kvdim; p.K = L.d; p.KT = L.KT_d;
    p.head_dim = cfg->head_dim; p.RT = L.nt_qkv; p.dst = bw.w_qkv;
    pack(p, L.nt_qkv, bw.s_qkv);

    p = PackArgs{};
    p.order = PACK_NATURAL; p.src[0] = (const bf16_t *)w.wo; p.rows[0] = L.d; p.K = L.qdim; p.KT = L.KT_q; p.RT = L.nt_o; p.dst = bw.w_o;
    pack(p, L.nt_o, bw.s_o);

    p = PackArgs{};
    if (L.llama) {
      p.order = PACK_GATEUP; p.src[0] = (const bf16_t *)w.w_gate; p.src[1] = (const bf16_t *)w.w_up;
      p.rows[0] = L.F; p.rows[1] = L.F;
    } else {
      p.order = PACK_NATURAL; p.src[0] = (const bf16_t *)w.w_up; p.rows[0] = L.F;
    }
    p.K = L.d; p.KT = L.KT_d; p.RT = L.nt_up; p.dst = bw.w_up;
    pack(p, L.nt_up, bw.s_up);

    p = PackArgs{};
    p.order = PACK_NATURAL; p.src[0] = (const bf16_t *)w.w_down; p.rows[0] = L.d; p.K = L.F; p.KT = L.KT_f; p.RT = L.nt_down; p.dst = bw.w_down;
    pack(p, L.nt_down, bw.s_down);

    launch_bf16_to_f32((const bf16_t *)w.norm1_g, bw.norm1_g, L.d, st);
    launch_bf16_to_f32((const bf16_t *)w.norm2_g, bw.norm2_g, L.d, st);
    if (need_bias) {
      launch_bf16_to_f32((const bf16_t *)w.norm1_b, bw.norm1_b, L.d, st);
      launch_bf16_to_f32((const bf16_t *)w.norm2_b, bw.norm2_b, L.d, st);
      launch_bf16_to_f32((const bf16_t *)w.bq, bw.b_qkv, L.qdim, st);
      launch_bf16_to_f32((const bf16_t *)w.bk, bw.b_qkv + L.qdim, L.kvdim, st);
      launch_bf16_to_f32((const bf16_t *)w.bv, bw.b_qkv + L.qdim + L.kvdim, L.kvdim, st);
      launch_bf16_to_f32((const bf16_t *)w.bo, bw.b_o, L.d, st);
      launch_bf16_to_f32((const bf16_t *)w.b_up, bw.b_up, L.F, st);
      launch_bf16_to_f32((const bf16_t *)w.b_down, bw.b_down, L.d, st);
      // folded LayerNorm terms of the decode path
      const bf16_t *g1 = (const bf16_t *)w.norm1_g, *be1 = (const bf16_t *)w.norm1_b;
      const bf16_t *g2 = (const bf16_t *)w.norm2_g, *be2 = (const bf16_t *)w.norm2_b;
      const bf16_t *mats[3] = {(const bf16_t *)w.wq, (const bf16_t *)w.wk, (const bf16_t *)w.wv};
      const int rows[3] = {L.qdim, L.kvdim, L.kvdim};
      int off = 0;
      for (int i = 0; i < 3; ++i) {
        launch_rowdot(mats[i], g1, nullptr, bw.wg_qkv + off, rows[i], L.d, st);
        launch_rowdot(mats[i], be1, bw.b_qkv + off, bw.bf_qkv + off, rows[i], L.d, st);
        off += rows[i];
      }
      launch_rowdot((const bf16_t *)w.w_up, g2, nullptr, bw.wg_up, L.F, L.d, st);
      launch_rowdot((const bf16_t *)w.w_up, be2, bw.b_up, bw.bf_up, L.F, L.d, st);
    }
  }
  rc = hip_check("span_create kernels");
  if (rc) { delete sp; return rc; }
  *out = sp;
  return SPAN_OK;
}

int span_destroy(span_t *span) {
  if (!span) return fail(SPAN_E_INVALID, "null span");
  clear_profile(span);
  delete span;
  return SPAN_OK;
}

int span_session_open(span_t *sp, int first_block, int n_blocks, int max_len, span_session_t *out) {
  if (!sp || !out) return fail(SPAN_E_INVALID, "null span or output");
  if (first_block < 0 || n_blocks < 1 || first_block + n_blocks > sp->cfg.n_blocks)
    return fail(SPAN_E_INVALID, "block range [%d, %d) outside the span's %d blocks", first_block,
                first_block + n_blocks, sp->cfg.n_blocks);
  if (max_len < 1 || max_len > sp->cfg.max_session_tokens)
    return fail(SPAN_E_INVALID, "max_len %d outside [1, %d]", max_len, sp->cfg.max_session_tokens);
  for (size_t i = 0; i < sp->sessions.size(); ++i) {
    Session &s = sp->sessions[i];
    if (s.open) continue;
    s = Session();
    s.open = true; s.id = sp->next_id++; s.first_block = first_block; s.n_blocks = n_blocks; s.max_len = max_len;
    *out = s.id;
    return SPAN_OK;
  }
  return fail(SPAN_E_NO_SLOT, "all %d session slots are in use", sp->cfg.max_sessions);
}

int span_session_close(span_t *sp, span_session_t id) {
  if (!sp) return fail(SPAN_E_INVALID, "null span");
  Session *s = find_session(sp, id);
  if (!s) return fail(SPAN_E_BAD_SESSION, "session %d is not open", id);
  release_session_pages(sp, *s);
  s->open = false;
  return SPAN_OK;
}

int span_session_length(span_t *sp, span_session_t id, int *len) {
  if (!sp || !len) return fail(SPAN_E_INVALID, "null argument");
  Session *s = find_session(sp, id);
  if (!s) return fail(SPAN_E_BAD_SESSION, "session %d is not open", id);
  *len = s->len;
  return SPAN_OK;
}

int span_forward(span_t *sp, int n, const span_session_t *ids, const int *ntok, const void *x, void *y, void *stream) {
  return forward_impl(sp, n, ids, ntok, x, y, (hipStream_t)stream);
}

int span_reorder(span_t *sp, int k, const span_session_t *ids, const int *hypo, void *stream) {
  if (!sp) return fail(SPAN_E_INVALID, "null span");
  if (k < 1 || k > SPAN_MAX_CALL_SESSIONS || !ids || !hypo)
    return fail(SPAN_E_INVALID, "beam of %d outside [1, %d], or null array", k, SPAN_MAX_CALL_SESSIONS);
  int slots[SPAN_MAX_CALL_SESSIONS];
  for (int i = 0; i < k; ++i) {
    Session *s = find_session(sp, ids[i], &slots[i]);
    if (!s) return fail(SPAN_E_BAD_SESSION, "session %d is not open", ids[i]);
    for (int j = 0; j < i; ++j)
      if (slots[j] == slots[i]) return fail(SPAN_E_DUPLICATE, "session %d listed twice", ids[i]);
    if (s->first_block != sp->sessions[slots[0]].first_block || s->n_blocks != sp->sessions[slots[0]].n_blocks)
      return fail(SPAN_E_MIXED_SPANS, "sessions of one call must share a block range");
    if (hypo[i] < 0 || hypo[i] >= k) return fail(SPAN_E_INVALID, "hypo_ids[%d] = %d outside [0, %d)", i, hypo[i], k);
  }
  for (int i = 0; i < k; ++i) {
    const Session &src = sp->sessions[slots[hypo[i]]], &dst = sp->sessions[slots[i]];
    if (src.len > dst.max_len)
      return fail(SPAN_E_TOO_LONG, "session %d (max_len %d) cannot take the %d cached tokens of session %d",
                  ids[i], dst.max_len, src.len, ids[hypo[i]]);
  }
  // Plan.  New page list of entry i = the source's list; a source whose last page is partly
  // filled keeps that page for one of its continuations (itself if it names itself, else the
  // first that names it) and every other continuation gets a copy in a fresh page, because
  // each session appends into its last page.
  std::vector<std::vector<int>> plan(k);
  std::vector<int> keeper(k, -1);              // per source: the entry that keeps its partial page
  std::vector<std::pair<int, int>> copies;     // (entry, source page) needing a fresh page
  for (int i = 0; i < k; ++i)
    if (hypo[i] == i) keeper[i] = i;
  for (int i = 0; i < k; ++i) {
    const int src = hypo[i];
    const Session &s = sp->sessions[slots[src]];
    plan[i] = s.pages;
    if (s.len % SPAN_PAGE == 0) continue;      // all pages full (or none): shared as they are
    if (keeper[src] < 0) keeper[src] = i;
    if (keeper[src] != i) copies.push_back({i, s.pages.back()});
  }
  // pages that lose their last reference come back before the fresh ones are taken
  std::vector<int> ref = sp->page_ref;
  for (int i = 0; i < k; ++i)
    for (int pg : sp->sessions[slots[i]].pages) --ref[pg];
  for (int i = 0; i < k; ++i)
    for (int pg : plan[i]) ++ref[pg];
  for (auto &c : copies) --ref[c.second];      // these entries will list a fresh page instead
  size_t released = 0;                         // distinct pages nobody lists any more
  {
    std::vector<char> seen(ref.size(), 0);
    for (int i = 0; i < k; ++i)
      for (int pg : sp->sessions[slots[i]].pages)
        if (ref[pg] == 0 && !seen[pg]) { seen[pg] = 1; ++released; }
  }
  if (copies.size() > sp->free_pages.size() + released)
    return fail(SPAN_E_CACHE_FULL, "need %zu KV pages for partial-page copies, %zu free", copies.size(),
                sp->free_pages.size() + released);

  // Commit (host), then enqueue the copies and the page-table rows.  What the commit overwrites is kept
  // until the enqueue has succeeded: a call that returns an error leaves every session as it was.
  const std::vector<int> free_before = sp->free_pages, ref_before = sp->page_ref;
  std::vector<std::vector<int>> pages_before(k);
  std::vector<int> len_before(k);
  for (int i = 0; i < k; ++i) { pages_before[i] = sp->sessions[slots[i]].pages; len_before[i] = sp->sessions[slots[i]].len; }
  {
    std::vector<char> seen(ref.size(), 0);
    for (int i = 0; i < k; ++i)
      for (int pg : sp->sessions[slots[i]].pages)
        if (ref[pg] == 0 && !seen[pg]) { seen[pg] = 1; sp->free_pages.push_back(pg); }
  }
  PageCopies pc{};
  for (auto &c : copies) {
    const int fresh = sp->free_pages.back();
    sp->free_pages.pop_back();
    ref[fresh] = 1;
    plan[c.first].back() = fresh;
    pc.src[pc.n] = c.second; pc.dst[pc.n] = fresh; ++pc.n;
  }
  sp->page_ref.swap(ref);
  std::vector<int> lens(k);
  for (int i = 0; i < k; ++i) lens[i] = sp->sessions[slots[hypo[i]]].len;
  std::vector<int> upd_idx, upd_val;
  for (int i = 0; i < k; ++i) {
    Session &d = sp->sessions[slots[i]];
    for (size_t j = 0; j < plan[i].size(); ++j)
      if (j >= d.pages.size() || d.pages[j] != plan[i][j]) {
        upd_idx.push_back(slots[i] * sp->L.pps + (int)j);
        upd_val.push_back(plan[i][j]);
      }
    d.pages.swap(plan[i]);
    d.len = lens[i];
  }
  if (sp->cfg.dry_run) return SPAN_OK;
  hipStream_t st = (hipStream_t)stream;
  const Session &any = sp->sessions[slots[0]];
  if (sp->L.bits == 32) launch_f32_page_copy(sp->f32.pool, any.first_block, any.n_blocks, pc, st);
  else launch_kv_page_copy(sp->pool, any.first_block, any.n_blocks, pc, st);
  push_page_table(sp, upd_idx, upd_val, st);
  const int rc = hip_check("span_reorder kernels");
  if (rc != SPAN_OK) {
    sp->free_pages = free_before;
    sp->page_ref = ref_before;
    for (int i = 0; i < k; ++i) { sp->sessions[slots[i]].pages = pages_before[i]; sp->sessions[slots[i]].len = len_before[i]; }
  }
  return rc;
}

int span_replay(span_t *sp, int n, const span_session_t *ids, const int *ntok, const void *x, void *y, void *stream) {
  if (!sp) return fail(SPAN_E_INVALID, "null span");
  if (n < 0 || n > SPAN_MAX_CALL_SESSIONS) return fail(SPAN_E_INVALID, "n_sessions %d outside [0, %d]", n, SPAN_MAX_CALL_SESSIONS);
  if (n > 0 && (!ids || !ntok)) return fail(SPAN_E_INVALID, "null session or token-count array");
  long long total = 0;
  for (int i = 0; i < n; ++i) {
    Session *s = find_session(sp, ids[i]);
    if (!s) return fail(SPAN_E_BAD_SESSION, "session %d is not open", ids[i]);
    if (s->len != 0) return fail(SPAN_E_NOT_EMPTY, "replay needs an empty session; %d holds %d tokens", ids[i], s->len);
    if (ntok[i] < 0) return fail(SPAN_E_INVALID, "negative token count for session %d", ids[i]);
    for (int j = 0; j < i; ++j)
      if (ids[j] == ids[i]) return fail(SPAN_E_DUPLICATE, "session %d listed twice", ids[i]);
    total += ntok[i];
  }
  const int C = sp->cfg.max_batch_tokens;
  const size_t row_bytes = (size_t)sp->cfg.d_model * (sp->cfg.io_dtype == SPAN_IO_F32 ? 4 : 2);
  // walk the row space in chunks of at most C rows; a chunk may end inside a session
  int si = 0, done_in_si = 0;
  long long row = 0;
  while (row < total) {
    span_session_t cid[SPAN_MAX_CALL_SESSIONS];
    int cnt[SPAN_MAX_CALL_SESSIONS];
    int k = 0, room = C;
    while (room > 0 && si < n) {
      const int left = ntok[si] - done_in_si;
      if (left == 0) { ++si; done_in_si = 0; continue; }
      const int take = left < room ? left : room;
      cid[k] = ids[si]; cnt[k] = take; ++k;
      room -= take; done_in_si += take;
    }
    const char *xc = x ? (const char *)x + (size_t)row * row_bytes : nullptr;
    char *yc = y ? (char *)y + (size_t)row * row_bytes : nullptr;
    int rc = forward_impl(sp, k, cid, cnt, xc, yc, (hipStream_t)stream);
    if (rc != SPAN_OK) {
      std::string keep = g_err;
      for (int i = 0; i < n; ++i) release_session_pages(sp, *find_session(sp, ids[i]));
      g_err = keep;
      return rc;
    }
    row += C - room;
  }
  return SPAN_OK;
}

// ---- training-time passes ---------------------------------------------------------------------
namespace {
struct TrainLayout {
  int Kup, KT_nq, KT_up, nt_q, nt_f;
  size_t wt_block_bytes, o_qkv, o_o, o_up, o_down;
  int max_pages;
  size_t o_q, o_pool, o_pool2, o_pt, o_twt, o_qt, o_dot;
  int ld_t;
  size_t o_xs, o_x1, o_os, o_lse, o_pre, o_dres, o_dh, o_da, o_dob, o_dqkv, o_delta, o_tqkv, o_tup, scratch_bytes;
};
TrainLayout train_layout(const span_config &c, const Layout &L, int max_tokens) {
  TrainLayout t{};
  t.Kup = (L.llama ? 2 : 1) * L.F;
  t.KT_nq = round_up(L.nqkv, 128) / 32;
  t.KT_up = round_up(t.Kup, 128) / 32;
  t.nt_q = round_up(L.qdim / 16, 16);
  t.nt_f = round_up(ceil_div(L.F, 16), 16);
  size_t o = 0;
  auto mat = [&](int nt, int KT) { return align256((size_t)nt * 16 * KT * 32 * 2); };
  t.o_qkv = o;  o += mat(L.nt_o, t.KT_nq);      // rows d_model, K = q | k | v features
  t.o_o = o;    o += mat(t.nt_q, L.KT_d);       // rows q features, K = d_model
  t.o_up = o;   o += mat(L.nt_o, t.KT_up);      // rows d_model, K = gate | up (or up) features
  t.o_down = o; o += mat(t.nt_f, L.KT_d);       // rows d_ff, K = d_model
  t.wt_block_bytes = L.bits == 16 ? o : 0;      // compressed spans keep no transposed copies (see o_twt)
  const size_t M = (size_t)round_up(max_tokens, 16), nb = c.n_blocks, Mpad = round_up(max_tokens, 256);
  o = 0;
  t.o_xs = o;    o += align256(nb * M * L.d * 4);
  t.o_x1 = o;    o += align256(nb * M * L.d * 4);
  t.max_pages = (int)(M / SPAN_PAGE) + SPAN_MAX_CALL;            // every sequence may end in a partly filled page
  const size_t pool_bytes = nb * t.max_pages * 2 * c.n_kv_heads * SPAN_PAGE * c.head_dim * 2;
  t.o_q = o;     o += align256(nb * M * L.qdim * 2);
  t.o_pool = o;  o += align256(pool_bytes);
  t.o_pool2 = o; o += align256(pool_bytes);
  t.o_pt = o;    o += align256((size_t)SPAN_MAX_CALL * L.pps * 4);
  t.o_os = o;    o += align256(nb * M * L.qdim * 4);
  t.o_lse = o;   o += align256(nb * M * c.n_q_heads * 4);
  t.o_pre = o;   o += align256(nb * M * t.Kup * 4);
  t.o_dres = o;  o += align256(M * L.d * 4);
  t.o_dh = o;    o += align256(M * L.d * 4);
  t.o_da = o;    o += align256(M * L.F * 4);
  t.o_dob = o;   o += align256(M * L.qdim * 4);
  t.o_dqkv = o;  o += align256(M * L.nqkv * 4);
  t.o_delta = o; o += align256(M * c.n_q_heads * 4);
  t.o_tqkv = o;  o += align256(Mpad * t.KT_nq * 32 * 2);
  t.o_tup = o;   o += align256(Mpad * t.KT_up * 32 * 2);
  t.ld_t = (t.max_pages + 2) * SPAN_PAGE;                      // a 32-query step may read past a sequence's last page
  t.o_qt = o;    o += align256((size_t)L.qdim * t.ld_t * 2);
  t.o_dot = o;   o += align256((size_t)L.qdim * t.ld_t * 2);
  // compressed weights: one matrix at a time is expanded to bf16 (the span's workspace) and turned here
  t.o_twt = o;
  if (L.bits != 16) {
    size_t mx = (size_t)L.nt_o * t.KT_nq;
    if ((size_t)t.nt_q * L.KT_d > mx) mx = (size_t)t.nt_q * L.KT_d;
    if ((size_t)L.nt_o * t.KT_up > mx) mx = (size_t)L.nt_o * t.KT_up;
    if ((size_t)t.nt_f * L.KT_d > mx) mx = (size_t)t.nt_f * L.KT_d;
    o += align256(mx * 1024);
  }
  t.scratch_bytes = o;
  return t;
}

struct TrainCall {
  BatchMeta meta{};
  int M = 0;
};
int train_check(span_t *sp, int fb, int nb, int n_seq, const int *lens, TrainCall *tc) {
  if (!sp) return fail(SPAN_E_INVALID, "null span");
  if (!sp->train.on) return fail(SPAN_E_INVALID, "span_train_attach has not been called on this span");
  if (fb < 0 || nb < 1 || fb + nb > sp->cfg.n_blocks)
    return fail(SPAN_E_INVALID, "block range [%d, %d) outside the span's %d blocks", fb, fb + nb, sp->cfg.n_blocks);
  if (n_seq < 0 || n_seq > SPAN_MAX_CALL_SESSIONS || (n_seq > 0 && !lens))
    return fail(SPAN_E_INVALID, "n_seq %d outside [0, %d], or null lens", n_seq, SPAN_MAX_CALL_SESSIONS);
  long long total = 0;
  for (int i = 0; i < n_seq; ++i) {
    if (lens[i] < 0) return fail(SPAN_E_INVALID, "negative length of sequence %d", i);
    if (lens[i] > sp->cfg.max_session_tokens)
      return fail(SPAN_E_TOO_LONG, "sequence %d: %d tokens exceed max_session_tokens %d", i, lens[i], sp->cfg.max_session_tokens);
    total += lens[i];
    if (total > sp->train.max_tokens)
      return fail(SPAN_E_TOO_MANY_TOKENS, "call carries more than the attached max_tokens = %d tokens", sp->train.max_tokens);
    if (lens[i] == 0) continue;
    const int k = tc->meta.n_sess++;
    tc->meta.cu[k + 1] = tc->meta.cu[k] + lens[i];
    tc->meta.slot[k] = k;
  }
  tc->M = (int)total;
  return SPAN_OK;
}

constexpr int TRAIN_K_CHUNK = 256;   // k tiles (of 32) per launch of a split contraction
constexpr int TRAIN_SPLIT_MIN_TOKENS = 1024;

// One projection of a training-time pass on forward-format weights: the skinny kernel for up to 64
// rows, else the tiled one; compressed weights as in the inference path (stream the codes, or expand
// the matrix to bf16 scratch first).  scales = null: wp is a bf16 pack whatever the span's format.
void train_linear(span_t *sp, const bf16_t *wp, const float *scales, int nt_pad, const bf16_t *xp, int x_RT, int KT,
                  int n_pairs, int M, const EpiArgs &e, const BatchMeta &meta, hipStream_t st) {
  const bool packed_bf16 = sp->L.bits == 16 || !scales;
  QWeights qw{(const uint8_t *)wp, scales, nt_pad, sp->L.bits, {}, {}};
  for (int i = 0; i < 4; ++i) { qw.lut_lo[i] = sp->levels.lut_lo[i]; qw.lut_hi[i] = sp->levels.lut_hi[i]; }
  if (!packed_bf16 && M > 64) launch_expand_q(qw, KT / 2, sp->expand, st);
  auto go = [&] {
    if (packed_bf16) {
      if (M <= 64) launch_gemv(wp, nt_pad, xp, x_RT, KT, n_pairs, ceil_div(M, 16), sp->share, e, meta, st);
      else if (e.kind == EPI_PLAIN && KT > 2 * TRAIN_K_CHUNK && M > TRAIN_SPLIT_MIN_TOKENS) {
        // A very long contraction (the transposed gate/up projection: k = 2 d_ff) streams operands far
        // larger than the memory-side cache and the chip clocks down under the DRAM traffic (measured:
        // 1.0 GHz against 1.4-1.5 for the other projections).  Cut along k into launches whose operands
        // stay cached; the plain epilogue adds the pieces up in fp32, in a fixed order.  (Up to 1024 tokens
        // there is one band of token tiles, the weights are read once anyway, and splitting only costs.)
        for (int k0 = 0; k0 < KT; k0 += TRAIN_K_CHUNK) {
          EpiArgs ec = e;
          ec.accumulate = k0 > 0;
          const int kc = KT - k0 < TRAIN_K_CHUNK ? KT - k0 : TRAIN_K_CHUNK;
          launch_gemm(wp + (size_t)k0 * nt_pad * 512, nt_pad, xp + (size_t)k0 * x_RT * 512, x_RT, kc, M, ec, meta, st);
        }
      } else launch_gemm(wp, nt_pad, xp, x_RT, KT, M, e, meta, st);
    } else if (M <= 64) launch_gemvq(qw, xp, x_RT, KT / 2, n_pairs, ceil_div(M, 16), sp->share, e, meta, st);
    else launch_gemm(sp->expand, nt_pad, xp, x_RT, KT, M, e, meta, st);
  };
  if (!sp->profiling) { go(); return; }
  ProfRecord r{M <= 64 ? SPAN_K_SKINNY : SPAN_K_TILED, nullptr, nullptr};
  if (hipEventCreateWithFlags(&r.a, hipEventDisableSystemFence) != hipSuccess ||
      hipEventCreateWithFlags(&r.b, hipEventDisableSystemFence) != hipSuccess) { go(); return; }
  (void)hipEventRecord(r.a, st);
  go();
  (void)hipEventRecord(r.b, st);
  sp->prof.push_back(r);
}

// A backward projection dX = dY W: the transposed bf16 pack of a bf16 span, or, for a compressed
// span, the forward matrix expanded to bf16 and turned for this call.
struct FwdMatrix { const bf16_t *wp; const float *scales; int nt_pad, KT, order, rows0, N, K; };
void train_linear_t(span_t *sp, const bf16_t *wt_packed, const FwdMatrix &f, int d_RT, int d_KT, const bf16_t *xp,
                    int x_RT, int n_pairs, int M, const EpiArgs &e, const BatchMeta &meta, hipStream_t st) {
  const bf16_t *w = wt_packed;
  if (sp->L.bits != 16) {
    QWeights qw{(const uint8_t *)f.wp, f.scales, f.nt_pad, sp->L.bits, {}, {}};
    for (int i = 0; i < 4; ++i) { qw.lut_lo[i] = sp->levels.lut_lo[i]; qw.lut_hi[i] = sp->levels.lut_hi[i]; }
    launch_expand_q(qw, f.KT / 2, sp->expand, st);
    TransposeArgs ta{sp->expand, f.nt_pad, f.order, f.rows0, sp->cfg.head_dim, f.N, f.K, sp->train.t_wt, d_RT};
    launch_transpose_t16(ta, d_KT, st);
    w = sp->train.t_wt;
  }
  train_linear(sp, w, nullptr, d_RT, xp, x_RT, d_KT, n_pairs, M, e, meta, st);
}

// Forward sweep over whole sequences; keeps, per block, the rows the backward sweep needs.
// y (optional): output of the last block.  Without y the last block stops after its
// gate/up projection (its output is not needed to back-propagate).
void train_forward_sweep(span_t *sp, const TrainCall &tc, int fb, int nb, const void *x, void *y, hipStream_t st) {
  const span_config &c = sp->cfg;
  const Layout &L = sp->L;
  span_t::Train &T = sp->train;
  const int M = tc.M;
  const int x_RT = M <= 64 ? ceil_div(M, 16) : round_up(M, gemm_token_tile(M)) / 16;
  const size_t cap = (size_t)round_up(T.max_tokens, 16);
  const size_t row_d = (size_t)M * L.d * 4;
  int q_tiles = 0;
  for (int i = 0; i < tc.meta.n_sess; ++i) q_tiles += ceil_div(tc.meta.cu[i + 1] - tc.meta.cu[i], attn_prefill_q_tile());
  launch_train_page_table(T.pt, L.pps, tc.meta, st);
  for (int bi = 0; bi < nb; ++bi) {
    const BlockWeights &w = sp->blocks[fb + bi];
    float *xs = T.xs + bi * cap * L.d, *x1 = T.x1 + bi * cap * L.d;
    NormArgs n1{};
    n1.x_in = bi == 0 ? x : nullptr; n1.x_f32 = c.io_dtype == SPAN_IO_F32;
    n1.resid = xs; n1.gain = w.norm1_g; n1.bias = L.llama ? nullptr : w.norm1_b;
    n1.layernorm = !L.llama; n1.eps = c.norm_eps; n1.d = L.d; n1.RT = x_RT; n1.M = M; n1.h_out = sp->h;
    launch_norm(n1, st);

    EpiArgs e{};
    e.kind = EPI_QKV; e.M = M; e.N = L.nqkv; e.bias = L.llama ? nullptr : w.b_qkv;
    e.n_q_heads = c.n_q_heads; e.n_kv_heads = c.n_kv_heads; e.head_dim = c.head_dim; e.rotary = L.llama;
    e.rope = sp->rope; e.q_out = T.q + bi * cap * L.qdim; e.pool = T.pool; e.pool2 = T.pool2; e.block = bi;
    e.page_table = T.pt; e.pages_per_session = L.pps;
    train_linear(sp, w.w_qkv, w.s_qkv, L.nt_qkv, sp->h, x_RT, L.KT_d, L.nqkv / 32, M, e, tc.meta, st);

    // the prefill attention kernel of the inference path, on the call's own pages
    AttnArgs a{};
    a.q = e.q_out; a.pool = T.pool; a.block = bi; a.page_table = T.pt; a.pages_per_session = L.pps;
    a.n_q_heads = c.n_q_heads; a.n_kv_heads = c.n_kv_heads; a.head_dim = c.head_dim;
    a.alibi = L.llama ? nullptr : sp->alibi; a.o_out = sp->o; a.o_RT = x_RT; a.n_splits = 1; a.split_pp = 1;
    a.o_f32 = T.o + bi * cap * L.qdim; a.lse_out = T.lse + bi * cap * c.n_q_heads;
    launch_attn_prefill(a, tc.meta, q_tiles, st);

    (void)hipMemcpyAsync(x1, xs, row_d, hipMemcpyDeviceToDevice, st);
    EpiArgs eo{};
    eo.kind = EPI_RESID; eo.M = M; eo.N = L.d; eo.bias = L.llama ? nullptr : w.b_o; eo.resid = x1;
    train_linear(sp, w.w_o, w.s_o, L.nt_o, sp->o, x_RT, L.KT_q, L.d / 32, M, eo, tc.meta, st);

    NormArgs n2 = n1;
    n2.x_in = nullptr; n2.resid = x1; n2.gain = w.norm2_g; n2.bias = L.llama ? nullptr : w.norm2_b;
    launch_norm(n2, st);

    const bool last = bi == nb - 1;
    EpiArgs eu{};
    eu.M = M; eu.N = L.F; eu.act_out = sp->act; eu.act_RT = x_RT; eu.gu_plain = T.pre + bi * cap * T.Kup;
    if (L.llama) { eu.kind = EPI_SWIGLU; train_linear(sp, w.w_up, w.s_up, L.nt_up, sp->h, x_RT, L.KT_d, L.F / 16, M, eu, tc.meta, st); }
    else { eu.kind = EPI_GELU; eu.bias = w.b_up; train_linear(sp, w.w_up, w.s_up, L.nt_up, sp->h, x_RT, L.KT_d, L.F / 32, M, eu, tc.meta, st); }
    if (last && !y) break;

    float *out = last ? T.dh : T.xs + (bi + 1) * cap * L.d;
    (void)hipMemcpyAsync(out, x1, row_d, hipMemcpyDeviceToDevice, st);
    EpiArgs ed{};
    ed.kind = EPI_RESID; ed.M = M; ed.N = L.d; ed.bias = L.llama ? nullptr : w.b_down; ed.resid = out;
    if (last) { ed.y = y; ed.y_f32 = c.io_dtype == SPAN_IO_F32; }
    train_linear(sp, w.w_down, w.s_down, L.nt_down, sp->act, x_RT, L.KT_f, L.d / 32, M, ed, tc.meta, st);
  }
}

void train_backward_sweep(span_t *sp, const TrainCall &tc, int fb, int nb, const void *grad_y, void *grad_x,
                          hipStream_t st) {
  const span_config &c = sp->cfg;
  const Layout &L = sp->L;
  span_t::Train &T = sp->train;
  const int M = tc.M;
  const int x_RT = M <= 64 ? ceil_div(M, 16) : round_up(M, gemm_token_tile(M)) / 16;
  const size_t cap = (size_t)round_up(T.max_tokens, 16);
  const int io32 = c.io_dtype == SPAN_IO_F32;
  launch_rows_to_f32(grad_y, io32, T.dres, (size_t)M * L.d, st);
  auto plain = [&](float *out, int N) {
    EpiArgs e{};
    e.kind = EPI_PLAIN; e.M = M; e.N = N; e.out = out;
    return e;
  };
  for (int bi = nb - 1; bi >= 0; --bi) {
    const BlockWeights &w = sp->blocks[fb + bi];
    const char *wt = T.wt + (size_t)(fb + bi) * T.wt_block_bytes;
    const float *xs = T.xs + bi * cap * L.d, *x1 = T.x1 + bi * cap * L.d;
    // MLP: y = x1 + act(norm2(x1) W_up^T) W_down^T
    launch_pack_act_f32(T.dres, sp->h, M, L.d, L.KT_d, x_RT, st);
    const FwdMatrix f_down{w.w_down, w.s_down, L.nt_down, L.KT_f, PACK_NATURAL, 0, L.d, L.F};
    if (M > 64) {
      // the tiled kernels apply the activation's derivative in their epilogue and write the next input
      EpiArgs ea{};
      ea.kind = EPI_ACTBWD; ea.M = M; ea.N = L.F; ea.gated = L.llama; ea.gu_plain = T.pre + bi * cap * T.Kup;
      ea.act_out = T.t_up; ea.act_RT = x_RT;
      train_linear_t(sp, (const bf16_t *)(wt + T.o_down), f_down, T.nt_f, L.KT_d, sp->h, x_RT, ceil_div(L.F, 32), M, ea, tc.meta, st);
    } else {
      train_linear_t(sp, (const bf16_t *)(wt + T.o_down), f_down, T.nt_f, L.KT_d, sp->h, x_RT, ceil_div(L.F, 32), M,
                     plain(T.da, L.F), tc.meta, st);
      launch_act_bwd_pack(T.pre + bi * cap * T.Kup, T.da, T.t_up, M, L.F, L.llama, T.KT_up, x_RT, st);
    }
    train_linear_t(sp, (const bf16_t *)(wt + T.o_up),
                   FwdMatrix{w.w_up, w.s_up, L.nt_up, L.KT_d, L.llama ? PACK_GATEUP : PACK_NATURAL, L.F, T.Kup, L.d},
                   L.nt_o, T.KT_up, T.t_up, x_RT, L.d / 32, M, plain(T.dh, L.d), tc.meta, st);
    launch_norm_bwd(x1, w.norm2_g, T.dh, T.dres, M, L.d, c.norm_eps, !L.llama, st);
    // attention: x1 = x + attn(norm1(x)) W_o^T
    launch_pack_act_f32(T.dres, sp->h, M, L.d, L.KT_d, x_RT, st);
    train_linear_t(sp, (const bf16_t *)(wt + T.o_o), FwdMatrix{w.w_o, w.s_o, L.nt_o, L.KT_q, PACK_NATURAL, 0, L.d, L.qdim},
                   T.nt_q, L.KT_d, sp->h, x_RT, L.qdim / 32, M, plain(T.dob, L.qdim), tc.meta, st);
    TrainAttnArgs a{};
    a.q = T.q + bi * cap * L.qdim; a.pool = T.pool; a.pool2 = T.pool2; a.block = bi; a.page_table = T.pt;
    a.pages_per_seq = L.pps; a.n_q_heads = c.n_q_heads; a.n_kv_heads = c.n_kv_heads; a.head_dim = c.head_dim;
    a.alibi = L.llama ? nullptr : sp->alibi;
    a.o = T.o + bi * cap * L.qdim; a.lse = T.lse + bi * cap * c.n_q_heads;
    a.d_o = T.dob; a.delta = T.delta; a.dqkv = T.dqkv; a.q_t = T.q_t; a.do_t = T.do_t; a.ld_t = T.ld_t;
    launch_attn_train_bwd(a, tc.meta, M, st);
    launch_qkv_bwd_pack(T.dqkv, sp->rope, T.t_qkv, M, c.n_q_heads, c.n_kv_heads, c.head_dim, L.llama, T.KT_nq, x_RT,
                        tc.meta, st);
    train_linear_t(sp, (const bf16_t *)(wt + T.o_qkv), FwdMatrix{w.w_qkv, w.s_qkv, L.nt_qkv, L.KT_d, PACK_HEADS, 0, L.nqkv, L.d},
                   L.nt_o, T.KT_nq, T.t_qkv, x_RT, L.d / 32, M, plain(T.dh, L.d), tc.meta, st);
    launch_norm_bwd(xs, w.norm1_g, T.dh, T.dres, M, L.d, c.norm_eps, !L.llama, st);
  }
  launch_rows_from_f32(T.dres, grad_x, io32, (size_t)M * L.d, st);
}
}  // namespace

int span_train_sizes(const span_config *cfg, int max_tokens, size_t *weight_t_bytes, size_t *scratch_bytes) {
  if (!cfg) return fail(SPAN_E_INVALID, "null config");
  Layout L;
  int rc = make_layout(*cfg, L);
  if (rc) return rc;
  if (L.bits == 32) return fail(SPAN_E_INVALID, "the training-time passes exist for the bf16 kernels only (weight_bits 32 is inference only)");
  if (max_tokens < 1 || max_tokens > cfg->max_batch_tokens)
    return fail(SPAN_E_INVALID, "max_tokens %d outside [1, max_batch_tokens = %d]", max_tokens, cfg->max_batch_tokens);
  const TrainLayout t = train_layout(*cfg, L, max_tokens);
  if (weight_t_bytes) *weight_t_bytes = t.wt_block_bytes * cfg->n_blocks;
  if (scratch_bytes) *scratch_bytes = t.scratch_bytes;
  return SPAN_OK;
}

int span_train_attach(span_t *sp, const span_block_weights *weights, void *weight_t_arena, void *scratch, int max_tokens,
                      void *stream) {
  if (!sp || !scratch) return fail(SPAN_E_INVALID, "null argument");
  if (sp->cfg.dry_run) return fail(SPAN_E_INVALID, "dry-run span holds no data");
  const span_config &c = sp->cfg;
  const Layout &L = sp->L;
  if (L.bits == 32) return fail(SPAN_E_INVALID, "the training-time passes exist for the bf16 kernels only (weight_bits 32 is inference only)");
  if (L.bits == 16 && (!weights || !weight_t_arena)) return fail(SPAN_E_INVALID, "null weights or arena");
  if (max_tokens < 1 || max_tokens > c.max_batch_tokens)
    return fail(SPAN_E_INVALID, "max_tokens %d outside [1, max_batch_tokens = %d]", max_tokens, c.max_batch_tokens);
  for (int b = 0; L.bits == 16 && b < c.n_blocks; ++b) {
    const span_block_weights &w = weights[b];
    if (!w.wq || !w.wk || !w.wv || !w.wo || !w.w_up || !w.w_down || (L.llama && !w.w_gate))
      return fail(SPAN_E_INVALID, "block %d: a required weight pointer is null", b);
  }
  const TrainLayout t = train_layout(c, L, max_tokens);
  hipStream_t st = (hipStream_t)stream;
  span_t::Train &T = sp->train;
  T.on = false;                        // stays off if the set-up below fails
  T.max_tokens = max_tokens;
  T.Kup = t.Kup; T.KT_nq = t.KT_nq; T.KT_up = t.KT_up; T.nt_q = t.nt_q; T.nt_f = t.nt_f;
  T.wt_block_bytes = t.wt_block_bytes; T.o_qkv = t.o_qkv; T.o_o = t.o_o; T.o_up = t.o_up; T.o_down = t.o_down;
  T.wt = (char *)weight_t_arena;
  char *sc = (char *)scratch;
  T.xs = (float *)(sc + t.o_xs); T.x1 = (float *)(sc + t.o_x1); T.q = (bf16_t *)(sc + t.o_q);
  T.pool = KvPool{(bf16_t *)(sc + t.o_pool), t.max_pages, c.n_kv_heads, c.head_dim};
  T.pool2 = KvPool{(bf16_t *)(sc + t.o_pool2), t.max_pages, c.n_kv_heads, c.head_dim};
  T.pt = (int *)(sc + t.o_pt);
  T.o = (float *)(sc + t.o_os); T.lse = (float *)(sc + t.o_lse); T.pre = (float *)(sc + t.o_pre);
  T.dres = (float *)(sc + t.o_dres); T.dh = (float *)(sc + t.o_dh); T.da = (float *)(sc + t.o_da);
  T.dob = (float *)(sc + t.o_dob); T.dqkv = (float *)(sc + t.o_dqkv); T.delta = (float *)(sc + t.o_delta);
  T.t_qkv = (bf16_t *)(sc + t.o_tqkv); T.t_up = (bf16_t *)(sc + t.o_tup); T.t_wt = (bf16_t *)(sc + t.o_twt);
  T.q_t = (bf16_t *)(sc + t.o_qt); T.do_t = (bf16_t *)(sc + t.o_dot); T.ld_t = t.ld_t;
  // the k padding of the packed inputs must stay finite: it meets zero weights
  launch_fill_u32((uint32_t *)scratch, t.scratch_bytes / 4, 0u, st);
  for (int b = 0; L.bits == 16 && b < c.n_blocks; ++b) {
    const span_block_weights &w = weights[b];
    char *base = T.wt + (size_t)b * t.wt_block_bytes;
    PackTArgs p{};
    p.src[0] = (const bf16_t *)w.wq; p.src[1] = (const bf16_t *)w.wk; p.src[2] = (const bf16_t *)w.wv;
    p.rows[0] = L.qdim; p.rows[1] = L.kvdim; p.rows[2] = L.kvdim;
    p.ld = L.d; p.KT = t.KT_nq; p.RT = L.nt_o; p.dst = (bf16_t *)(base + t.o_qkv);
    launch_pack_weight_t(p, L.nt_o, st);
    p = PackTArgs{};
    p.src[0] = (const bf16_t *)w.wo; p.rows[0] = L.d; p.ld = L.qdim; p.KT = L.KT_d; p.RT = t.nt_q; p.dst = (bf16_t *)(base + t.o_o);
    launch_pack_weight_t(p, t.nt_q, st);
    p = PackTArgs{};
    if (L.llama) { p.src[0] = (const bf16_t *)w.w_gate; p.rows[0] = L.F; p.src[1] = (const bf16_t *)w.w_up; p.rows[1] = L.F; }
    else { p.src[0] = (const bf16_t *)w.w_up; p.rows[0] = L.F; }
    p.ld = L.d; p.KT = t.KT_up; p.RT = L.nt_o; p.dst = (bf16_t *)(base + t.o_up);
    launch_pack_weight_t(p, L.nt_o, st);
    p = PackTArgs{};
    p.src[0] = (const bf16_t *)w.w_down; p.rows[0] = L.d; p.ld = L.F; p.KT = L.KT_d; p.RT = t.nt_f; p.dst = (bf16_t *)(base + t.o_down);
    launch_pack_weight_t(p, t.nt_f, st);
  }
  int rc = hip_check("span_train_attach kernels");
  if (rc) return rc;
  T.on = true;
  return SPAN_OK;
}

int span_train_forward(span_t *sp, int fb, int nb, int n_seq, const int *lens, const void *x, void *y, void *stream) {
  TrainCall tc;
  int rc = train_check(sp, fb, nb, n_seq, lens, &tc);
  if (rc) return rc;
  if (tc.M == 0) return SPAN_OK;
  if (!x || !y) return fail(SPAN_E_INVALID, "null x or y");
  train_forward_sweep(sp, tc, fb, nb, x, y, (hipStream_t)stream);
  return hip_check("span_train_forward kernels");
}

int span_backward(span_t *sp, int fb, int nb, int n_seq, const int *lens, const void *x, const void *grad_y,
                  void *grad_x, void *y_out, void *stream) {
  TrainCall tc;
  int rc = train_check(sp, fb, nb, n_seq, lens, &tc);
  if (rc) return rc;
  if (tc.M == 0) return SPAN_OK;
  if (!x || !grad_y || !grad_x) return fail(SPAN_E_INVALID, "null x, grad_y or grad_x");
  train_forward_sweep(sp, tc, fb, nb, x, y_out, (hipStream_t)stream);
  train_backward_sweep(sp, tc, fb, nb, grad_y, grad_x, (hipStream_t)stream);
  return hip_check("span_backward kernels");
}

int span_debug_free_pages(span_t *sp, int *n_free) {
  if (!sp || !n_free) return fail(SPAN_E_INVALID, "null argument");
  *n_free = (int)sp->free_pages.size();
  return SPAN_OK;
}

int span_debug_page_table(span_t *sp, span_session_t id, int32_t *pages_out, int *n_pages) {
  if (!sp || !n_pages) return fail(SPAN_E_INVALID, "null argument");
  Session *s = find_session(sp, id);
  if (!s) return fail(SPAN_E_BAD_SESSION, "session %d is not open", id);
  *n_pages = (int)s->pages.size();
  if (pages_out) for (size_t i = 0; i < s->pages.size(); ++i) pages_out[i] = s->pages[i];
  return SPAN_OK;
}

int span_debug_read_kv(span_t *sp, span_session_t id, int block, int pos0, int n, void *k_out, void *v_out, void *stream) {
  if (!sp || !k_out || !v_out) return fail(SPAN_E_INVALID, "null argument");
  if (sp->cfg.dry_run) return fail(SPAN_E_INVALID, "dry-run span holds no data");
  int slot;
  Session *s = find_session(sp, id, &slot);
  if (!s) return fail(SPAN_E_BAD_SESSION, "session %d is not open", id);
  if (block < 0 || block >= s->n_blocks) return fail(SPAN_E_INVALID, "block %d outside the session's range", block);
  if (pos0 < 0 || n < 0 || pos0 + n > s->len) return fail(SPAN_E_INVALID, "positions [%d, %d) outside the cached %d", pos0, pos0 + n, s->len);
  if (n == 0) return SPAN_OK;
  if (sp->L.bits == 32)
    launch_f32_kv_gather(sp->f32.pool, s->first_block + block, sp->page_table + (size_t)slot * sp->L.pps, pos0, n,
                         (float *)k_out, (float *)v_out, (hipStream_t)stream);
  else
  launch_kv_gather(sp->pool, s->first_block + block, sp->page_table + (size_t)slot * sp->L.pps, pos0, n,
                   (bf16_t *)k_out, (bf16_t *)v_out, (hipStream_t)stream);
  return hip_check("kv gather");
}

int span_debug_tap(span_t *sp, int what, int block, span_session_t id, int head, int q0, int nq, void *out, size_t out_bytes) {
  if (!sp) return fail(SPAN_E_INVALID, "null span");
  if (what == 0) {                                      // disarm everything
    for (auto &t : sp->taps) t = span_t::Tap{};
    return SPAN_OK;
  }
  if (what < SPAN_TAP_Q_ROT || what > SPAN_TAP_LOGITS) return fail(SPAN_E_INVALID, "unknown tap %d", what);
  if (sp->cfg.dry_run) return fail(SPAN_E_INVALID, "dry-run span holds no data");
  if (sp->L.bits == 32) return fail(SPAN_E_INVALID, "taps exist for the bf16 kernels only (this span runs in single precision)");
  if (!out) return fail(SPAN_E_INVALID, "null argument");
  Session *s = find_session(sp, id);
  if (!s) return fail(SPAN_E_BAD_SESSION, "session %d is not open", id);
  if (block < 0 || block >= s->n_blocks) return fail(SPAN_E_INVALID, "block %d outside the session's range", block);
  if (q0 < 0 || nq < 1) return fail(SPAN_E_INVALID, "need q0 >= 0, nq >= 1");
  if (what == SPAN_TAP_LOGITS && (head < 0 || head >= sp->cfg.n_q_heads)) return fail(SPAN_E_INVALID, "head %d outside [0, %d)", head, sp->cfg.n_q_heads);
  span_t::Tap &t = sp->taps[what - 1];
  t = span_t::Tap{};
  t.armed = true; t.block = block; t.session = id; t.head = head; t.q0 = q0; t.nq = nq; t.out = out; t.out_bytes = out_bytes;
  return SPAN_OK;
}

int span_debug_profile(span_t *sp, int enable) {
  if (!sp) return fail(SPAN_E_INVALID, "null span");
  if (enable) clear_profile(sp);
  sp->profiling = enable != 0 && !sp->cfg.dry_run;
  return SPAN_OK;
}

int span_debug_profile_read(span_t *sp, int cls, int *n_launches, float *total_ms) {
  if (!sp || !n_launches || !total_ms) return fail(SPAN_E_INVALID, "null argument");
  if (cls < 0 || cls >= SPAN_K_CLASSES) return fail(SPAN_E_INVALID, "kernel class %d out of range", cls);
  int n = 0;
  float tot = 0.0f;
  for (auto &r : sp->prof) {
    if (r.cls != cls) continue;
    if (hipEventSynchronize(r.b) != hipSuccess) return hip_check("profile event synchronize");
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return hip_check("profile event elapsed");
    tot += ms; ++n;
  }
  *n_launches = n; *total_ms = tot;
  return SPAN_OK;
}

size_t span_op_linear_scratch(int M, int N, int K) {
  if (M < 1 || N < 1 || K < 1) return 0;
  const size_t kp = round_up(K, 128);
  return align256((size_t)round_up(ceil_div(N, 16), 16) * 16 * kp * 2) + align256((size_t)round_up(M, 256) * kp * 2) +
         align256(gemv_share_part_bytes()) + align256((size_t)ceil_div(N, 32) * 4);
}

int span_op_linear(const void *x, const void *w, float *y, int M, int N, int K, int path, void *scratch, void *stream) {
  if (!x || !w || !y || !scratch) return fail(SPAN_E_INVALID, "null argument");
  if (M < 1 || N < 16 || N % 16 || K < 8 || K % 8) return fail(SPAN_E_INVALID, "need M >= 1, N %% 16 == 0, K %% 8 == 0");
  if (path == 0 && M > 64) return fail(SPAN_E_INVALID, "the skinny path takes at most 64 rows");
  if (path != 0 && path != 1) return fail(SPAN_E_INVALID, "path must be 0 or 1");
  hipStream_t st = (hipStream_t)stream;
  const int KT = round_up(K, 128) / 32, nt = round_up(ceil_div(N, 16), 16);
  bf16_t *wp = (bf16_t *)scratch;
  bf16_t *xp = (bf16_t *)((char *)scratch + align256((size_t)nt * 16 * KT * 32 * 2));
  char *shp = (char *)xp + align256((size_t)round_up(M, 256) * KT * 32 * 2);
  GemvShare share{0, (f32x4 *)shp, (unsigned *)(shp + align256(gemv_share_part_bytes()))};
  PackArgs p{};
  p.order = PACK_NATURAL; p.src[0] = (const bf16_t *)w; p.rows[0] = N; p.K = K; p.KT = KT; p.RT = nt; p.dst = wp;
  launch_pack_weight(p, nt, st);
  const int x_RT = path == 0 ? ceil_div(M, 16) : round_up(M, gemm_token_tile(M)) / 16;
  launch_pack_act((const bf16_t *)x, xp, M, K, KT, x_RT, st);
  EpiArgs e{};
  e.kind = EPI_PLAIN; e.M = M; e.N = N; e.out = y;
  BatchMeta meta{};
  meta.n_sess = 1; meta.cu[1] = M;
  if (path == 0) {
    launch_fill_u32((uint32_t *)share.count, (size_t)ceil_div(N, 32), 0u, st);
    launch_gemv(wp, nt, xp, x_RT, KT, ceil_div(N, 32), ceil_div(M, 16), share, e, meta, st);
  }
  else launch_gemm(wp, nt, xp, x_RT, KT, M, e, meta, st);
  return hip_check("span_op_linear");
}

namespace {
struct LowbitScratch { size_t o_codes, o_scales, o_absmax, o_x, o_share, o_count, total; int nt, KT; };
LowbitScratch lowbit_layout(int M, int N, int K) {
  LowbitScratch l{};
  l.KT = round_up(K, 128) / 32; l.nt = round_up(ceil_div(N, 16), 16);
  size_t o = 0;
  l.o_codes = o;  o += align256((size_t)l.nt * 16 * l.KT * 32);
  l.o_scales = o; o += align256((size_t)l.nt * 16 * (l.KT / 2) * 4);
  l.o_absmax = o; o += align256((size_t)l.nt * 16 * (l.KT / 2) * 4);
  l.o_x = o;      o += align256((size_t)round_up(M, 64) * l.KT * 32 * 2);
  l.o_share = o;  o += align256(gemv_share_part_bytes());
  l.o_count = o;  o += align256((size_t)ceil_div(N, 32) * 4);
  l.total = o;
  return l;
}
int lowbit_encode(const void *w, int N, int K, int bits, const float *levels, char *sc, const LowbitScratch &l,
                  QuantArgs *qout, LevelTable *ltout, hipStream_t st) {
  if (bits != 8 && bits != 4) return fail(SPAN_E_INVALID, "bits must be 8 or 4");
  QuantArgs q{};
  q.bits = bits;
  if (bits == 4) {
    if (!levels) return fail(SPAN_E_INVALID, "null levels");
    for (int i = 0; i < 16; ++i)
      if (!(levels[i] >= -1.0f && levels[i] <= 1.0f) || (i > 0 && !(levels[i] > levels[i - 1])))
        return fail(SPAN_E_INVALID, "levels must be 16 strictly ascending numbers in [-1, 1]");
    *ltout = make_level_table(levels);
    for (int i = 0; i < 15; ++i) q.mids[i] = ltout->mids[i];
  }
  q.codes = (uint8_t *)(sc + l.o_codes); q.scales = (float *)(sc + l.o_scales); q.absmax_out = (float *)(sc + l.o_absmax);
  PackArgs p{};
  p.order = PACK_NATURAL; p.src[0] = (const bf16_t *)w; p.rows[0] = N; p.K = K; p.KT = l.KT; p.RT = l.nt; p.dst = nullptr;
  launch_pack_weight_q(p, q, l.nt, st);
  *qout = q;
  return SPAN_OK;
}
}  // namespace

int span_debug_ceilings(const void *buf, size_t bytes, void *out, float *read_gbs, float *mfma_tflops, void *stream) {
  if (!buf || !out || !read_gbs || !mfma_tflops) return fail(SPAN_E_INVALID, "null argument");
  if (bytes < (1u << 20) || bytes % 16) return fail(SPAN_E_INVALID, "need at least 1 MiB, a multiple of 16 bytes");
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return hip_check("event create");
  const int iters = 4000;
  float best_r = 0.0f, best_m = 0.0f;
  for (int rep = 0; rep < 4; ++rep) {
    float ms = 0.0f;
    (void)hipEventRecord(a, st);
    launch_stream_read(buf, bytes, (uint32_t *)out, st);
    (void)hipEventRecord(b, st);
    (void)hipEventSynchronize(b);
    (void)hipEventElapsedTime(&ms, a, b);
    if (rep > 0 && ms > 0.0f) best_r = fmaxf(best_r, (float)(bytes / (ms * 1e-3) / 1e9));
    (void)hipEventRecord(a, st);
    launch_mfma_loop(buf, (float *)out, iters, st);
    (void)hipEventRecord(b, st);
    (void)hipEventSynchronize(b);
    (void)hipEventElapsedTime(&ms, a, b);
    const double flops = 256.0 * 4 * iters * 16 * 32768.0;
    if (rep > 0 && ms > 0.0f) best_m = fmaxf(best_m, (float)(flops / (ms * 1e-3) / 1e12));
  }
  (void)hipEventDestroy(a); (void)hipEventDestroy(b);
  *read_gbs = best_r; *mfma_tflops = best_m;
  return hip_check("span_debug_ceilings");
}

namespace {
int check_hidden_args(int M, int d, int block, const float *levels, Levels256 *t) {
  if (M < 1 || d < 1) return fail(SPAN_E_INVALID, "need M >= 1, d >= 1");
  if (block < 64 || block > 4096 || block % 64) return fail(SPAN_E_INVALID, "block must be a multiple of 64 in [64, 4096]");
  if (!levels) return fail(SPAN_E_INVALID, "null levels");
  for (int i = 0; i < 256; ++i) {
    if (!(levels[i] >= -1.0f && levels[i] <= 1.0f) || (i > 0 && !(levels[i] > levels[i - 1])))
      return fail(SPAN_E_INVALID, "levels must be 256 strictly ascending numbers in [-1, 1]");
    t->lv[i] = levels[i];
  }
  return SPAN_OK;
}
}  // namespace

int span_hidden_encode(const void *x, int x_f32, int M, int d, int block, const float *levels, void *codes_out,
                       float *absmax_out, void *stream) {
  if (!x || !codes_out || !absmax_out) return fail(SPAN_E_INVALID, "null argument");
  Levels256 t;
  int rc = check_hidden_args(M, d, block, levels, &t);
  if (rc) return rc;
  launch_hidden_encode(x, x_f32, M, d, block, t, (uint8_t *)codes_out, absmax_out, (hipStream_t)stream);
  return hip_check("span_hidden_encode");
}

int span_hidden_decode(const void *codes, const float *absmax, int M, int d, int block, const float *levels, int y_f32,
                       void *y, void *stream) {
  if (!codes || !absmax || !y) return fail(SPAN_E_INVALID, "null argument");
  Levels256 t;
  int rc = check_hidden_args(M, d, block, levels, &t);
  if (rc) return rc;
  launch_hidden_decode((const uint8_t *)codes, absmax, M, d, block, t, y_f32, y, (hipStream_t)stream);
  return hip_check("span_hidden_decode");
}

size_t span_op_lowbit_scratch(int M, int N, int K) {
  if (M < 1 || N < 1 || K < 1) return 0;
  return lowbit_layout(M, N, K).total;
}

int span_op_quantize(const void *w, int N, int K, int bits, const float *levels, void *codes_out, float *absmax_out,
                     void *scratch, void *stream) {
  if (!w || !codes_out || !absmax_out || !scratch) return fail(SPAN_E_INVALID, "null argument");
  if (N < 1 || K < 8 || K % 8) return fail(SPAN_E_INVALID, "need N >= 1, K %% 8 == 0");
  hipStream_t st = (hipStream_t)stream;
  const LowbitScratch l = lowbit_layout(1, N, K);
  QuantArgs q;
  LevelTable lt{};
  int rc = lowbit_encode(w, N, K, bits, levels, (char *)scratch, l, &q, &lt, st);
  if (rc) return rc;
  launch_unpack_codes(q, l.nt, N, K, (uint8_t *)codes_out, absmax_out, q.absmax_out, st);
  return hip_check("span_op_quantize");
}

int span_op_linear_lowbit(const void *x, const void *w, float *y, int M, int N, int K, int bits, const float *levels,
                          void *scratch, void *stream) {
  if (!x || !w || !y || !scratch) return fail(SPAN_E_INVALID, "null argument");
  if (M < 1 || M > 64 || N < 16 || N % 16 || K < 8 || K % 8)
    return fail(SPAN_E_INVALID, "need 1 <= M <= 64, N %% 16 == 0, K %% 8 == 0");
  hipStream_t st = (hipStream_t)stream;
  const LowbitScratch l = lowbit_layout(M, N, K);
  char *sc = (char *)scratch;
  QuantArgs q;
  LevelTable lt{};
  int rc = lowbit_encode(w, N, K, bits, levels, sc, l, &q, &lt, st);
  if (rc) return rc;
  bf16_t *xp = (bf16_t *)(sc + l.o_x);
  const int x_RT = ceil_div(M, 16);
  launch_pack_act((const bf16_t *)x, xp, M, K, l.KT, x_RT, st);
  GemvShare share{0, (f32x4 *)(sc + l.o_share), (unsigned *)(sc + l.o_count)};
  launch_fill_u32((uint32_t *)share.count, (size_t)ceil_div(N, 32), 0u, st);
  EpiArgs e{};
  e.kind = EPI_PLAIN; e.M = M; e.N = N; e.out = y;
  BatchMeta meta{};
  meta.n_sess = 1; meta.cu[1] = M;
  QWeights qw{q.codes, q.scales, l.nt, bits, {}, {}};
  for (int i = 0; i < 4; ++i) { qw.lut_lo[i] = lt.lut_lo[i]; qw.lut_hi[i] = lt.lut_hi[i]; }
  launch_gemvq(qw, xp, x_RT, l.KT / 2, ceil_div(N, 32), x_RT, share, e, meta, st);
  return hip_check("span_op_linear_lowbit");
}

namespace {
// Scratch of the stand-alone decode attention: a page pool holding the token-major caches, an identity
// page table, the ALiBi slopes and the partial results of the key splits.
struct AttnOpScratch { size_t o_pool, o_pt, o_slopes, o_part, total, part_entries; int pps; };
AttnOpScratch attn_op_layout(int B, int L_max, int Hq, int Hkv, int hd) {
  AttnOpScratch l{};
  l.pps = ceil_div(L_max, SPAN_PAGE);
  // a session has at most 64 splits (choose_splits), so B * Hkv * 64 partial results always suffice
  l.part_entries = std::min<size_t>(std::max<size_t>((size_t)B * Hkv, 4096), (size_t)B * Hkv * 64);
  size_t o = 0;
  l.o_pool = o;   o += align256((size_t)B * l.pps * 2 * Hkv * SPAN_PAGE * hd * 2);
  l.o_pt = o;     o += align256((size_t)B * l.pps * 4);
  l.o_slopes = o; o += align256((size_t)Hq * 4);
  l.o_part = o;   o += align256(l.part_entries * 16 * (hd + 2) * 4);
  l.total = o;
  return l;
}

int attn_op_check(const void *q, const void *k, const void *v, const int *lens, int B, int L_max, int Hq, int Hkv,
                  int hd, const float *out) {
  if (!q || !k || !v || !lens || !out) return fail(SPAN_E_INVALID, "null argument");
  if (B < 1 || B > SPAN_MAX_CALL_SESSIONS || L_max < 1 || (hd != 64 && hd != 128) || Hkv < 1 || Hq < 1 || Hq % Hkv || Hq / Hkv > 16)
    return fail(SPAN_E_INVALID, "bad attention shape");
  for (int b = 0; b < B; ++b)
    if (lens[b] < 1 || lens[b] > L_max) return fail(SPAN_E_INVALID, "lens[%d] = %d outside [1, %d]", b, lens[b], L_max);
  return SPAN_OK;
}

// Arguments already checked; `sc` holds attn_op_layout(...).total bytes.  Everything the kernels
// expect to start at zero (the pool's unused slots) is cleared here by a fill kernel, so the
// scratch may hold anything on entry.
int attn_op_enqueue(const void *q, const void *k, const void *v, const int *lens, int B, int L_max, int Hq, int Hkv,
                    int hd, int alibi, float *out, float *logits, char *sc, hipStream_t st) {
  const AttnOpScratch l = attn_op_layout(B, L_max, Hq, Hkv, hd);
  KvPool pool{(bf16_t *)(sc + l.o_pool), B * l.pps, Hkv, hd};
  int *pt = (int *)(sc + l.o_pt);
  float *slopes = (float *)(sc + l.o_slopes);
  BatchMeta meta{};
  meta.n_sess = B;
  for (int b = 0; b < B; ++b) { meta.cu[b + 1] = b + 1; meta.past[b] = lens[b] - 1; meta.slot[b] = b; }
  launch_fill_u32((uint32_t *)(sc + l.o_pool), (l.o_pt - l.o_pool) / 4, 0u, st);
  launch_iota(pt, B * l.pps, st);
  launch_kv_scatter(pool, 0, pt, l.pps, (const bf16_t *)k, (const bf16_t *)v, B, L_max, meta, st);
  if (alibi) launch_alibi_slopes(slopes, Hq, st);
  AttnArgs a{};
  a.q = (const bf16_t *)q; a.pool = pool; a.block = 0; a.page_table = pt; a.pages_per_session = l.pps;
  a.n_q_heads = Hq; a.n_kv_heads = Hkv; a.head_dim = hd; a.alibi = alibi ? slopes : nullptr;
  a.o_out = nullptr; a.o_RT = 0; a.n_splits = choose_splits(meta, Hkv, l.part_entries, &a.split_pp);
  a.part = (float *)(sc + l.o_part); a.logits = logits; a.logits_ld = L_max;
  launch_attn_decode(a, meta, st);
  launch_attn_merge(a, meta, out, st);
  return hip_check("span_op_attn_decode");
}

// ---- scratch of span_op_attn_decode_static: one array per GPU, owned by the library's code object.
// Host code never uses the array's name as an address (on the host it is only a handle for
// hipGetSymbolAddress); the device address is looked up once per device and kept.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)SPAN_STATIC_SCRATCH_MIB << 20;
constexpr int STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char static_scratch[STATIC_SCRATCH_BYTES];
std::mutex g_static_mu;
void *g_static_ptr[STATIC_MAX_DEVICES] = {};

int static_scratch_ptr(char **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) {
    (void)hipGetLastError();
    return fail(SPAN_E_HIP, "no current HIP device (or device index beyond %d)", STATIC_MAX_DEVICES - 1);
  }
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch));
    if (e != hipSuccess || !p) {
      (void)hipGetLastError();
      return fail(SPAN_E_HIP, "hipGetSymbolAddress(static scratch) on device %d: %s", dev, hipGetErrorString(e));
    }
    g_static_ptr[dev] = p;
  }
  *out = (char *)g_static_ptr[dev];
  return SPAN_OK;
}
}  // namespace

size_t span_op_attn_decode_scratch(int B, int L_max, int Hq, int Hkv, int hd) {
  if (B < 1 || L_max < 1 || Hq < 1 || Hkv < 1 || hd < 1) return 0;
  return attn_op_layout(B, L_max, Hq, Hkv, hd).total;
}

int span_op_attn_decode(const void *q, const void *k, const void *v, const int *lens, int B, int L_max, int Hq,
                        int Hkv, int hd, int alibi, float *out, float *logits, void *scratch, void *stream) {
  if (!scratch) return fail(SPAN_E_INVALID, "null argument");
  const int rc = attn_op_check(q, k, v, lens, B, L_max, Hq, Hkv, hd, out);
  if (rc) return rc;
  return attn_op_enqueue(q, k, v, lens, B, L_max, Hq, Hkv, hd, alibi, out, logits, (char *)scratch, (hipStream_t)stream);
}

int span_op_attn_decode_static(const void *q, const void *k, const void *v, const int *lens, int B, int L_max, int Hq,
                               int Hkv, int hd, int alibi, float *out, float *logits, void *stream) {
  int rc = attn_op_check(q, k, v, lens, B, L_max, Hq, Hkv, hd, out);
  if (rc) return rc;
  const size_t need = attn_op_layout(B, L_max, Hq, Hkv, hd).total;
  if (need > STATIC_SCRATCH_BYTES)
    return fail(SPAN_E_INVALID, "this shape needs %zu bytes of scratch; the built-in scratch holds %zu (use span_op_attn_decode)",
                need, STATIC_SCRATCH_BYTES);
  char *sc = nullptr;
  rc = static_scratch_ptr(&sc);
  if (rc) return rc;
  return attn_op_enqueue(q, k, v, lens, B, L_max, Hq, Hkv, hd, alibi, out, logits, sc, (hipStream_t)stream);
}

}  // extern "C"

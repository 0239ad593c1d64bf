// Host-side launch interface between the C ABI (span_api.hip) and the kernel files.
#pragma once
#include "common.h"

enum PackOrder { PACK_NATURAL = 0, PACK_HEADS = 1, PACK_GATEUP = 2 };

struct PackArgs {
  int order;
  const bf16_t *src[3];   // NATURAL: src[0]; GATEUP: gate, up; HEADS: wq, wk, wv
  int rows[3];
  int K, KT;              // source columns, padded k tiles of the destination
  int RT;                 // row tiles per k step of the destination (k-major T16)
  int head_dim;           // HEADS only
  bf16_t *dst;
};

// k_linear.hip
void launch_pack_weight(const PackArgs &a, int n_phys_tiles, hipStream_t s);
void launch_pack_act(const bf16_t *x, bf16_t *dst, int M, int K, int KT, int m_tiles, hipStream_t s);
// Memory through which workgroups of the skinny kernel that share a tile pair combine their
// pieces: `part` holds gemv_share_part_bytes() bytes, `count` one zero-initialised counter per
// tile pair (the kernel leaves them zero).  L is filled in by the launcher.
#define GEMV_MAX_GRID 256   // = compute units
struct GemvShare {
  int L;
  f32x4 *part;
  unsigned *count;
};
size_t gemv_share_part_bytes();
// weights: k-major T16 with w_RT row tiles per k step; activations likewise with x_RT
void launch_gemv(const bf16_t *wp, int w_RT, const bf16_t *xp, int x_RT, int KT, int n_pairs, int m_tiles,
                 const GemvShare &sh, const EpiArgs &epi, const BatchMeta &meta, hipStream_t s);
// ---- k_lowbit.hip: block-wise low-bit weights ------------------------------------------------
struct QuantArgs {
  int bits;              // 8 or 4
  float mids[15];        // codebook format: midpoints of the 16 levels (fp32)
  uint8_t *codes;        // packed destination
  float *scales;         // [k block][row]: absmax / 127 (int8) or absmax (codebook)
  float *absmax_out;     // optional, same layout: the plain absmax (encoder tests)
};
struct QWeights {
  const uint8_t *codes;
  const float *scales;
  int RT;                       // row tiles per k block
  int bits;
  uint32_t lut_lo[4], lut_hi[4];  // codebook format: low / high bytes of the 16 bf16 levels, four per dword
};
// the 16 levels of the codebook format as used: rounded to bf16 (their precision on the matrix
// core), with the midpoints between neighbours that decide the codes
struct LevelTable {
  float rounded[16];
  float mids[15];
  uint16_t bits[16];
  uint32_t lut_lo[4], lut_hi[4];   // bytes of bits[], level 4j+i in byte i of dword j
};
LevelTable make_level_table(const float *levels);
// a.KT counts 32-k tiles (a multiple of 4); the packed form has a.KT / 2 blocks of 64 k
void launch_pack_weight_q(const PackArgs &a, const QuantArgs &q, int n_phys_tiles, hipStream_t s);
void launch_unpack_codes(const QuantArgs &q, int RT, int N, int K, uint8_t *codes_out, float *absmax_out,
                         const float *absmax_packed, hipStream_t s);
// 8-bit block-wise codec of hidden states (256 ascending levels, absmax per `block` features of a row)
struct Levels256 { float lv[256]; };
void launch_hidden_encode(const void *x, int x_f32, int M, int d, int block, const Levels256 &t, uint8_t *codes,
                          float *absmax, hipStream_t s);
void launch_hidden_decode(const uint8_t *codes, const float *absmax, int M, int d, int block, const Levels256 &t,
                          int y_f32, void *y, hipStream_t s);
// packed codes -> bf16 T16 tiles (dst: w.RT row tiles x 2*KU k tiles, k-major)
void launch_expand_q(const QWeights &w, int KU, bf16_t *dst, hipStream_t s);
void launch_gemvq(const QWeights &w, const bf16_t *xp, int x_RT, int KU, int n_pairs, int m_tiles,
                  const GemvShare &sh, const EpiArgs &epi, const BatchMeta &meta, hipStream_t s);

void launch_gemm(const bf16_t *wp, int w_RT, const bf16_t *xp, int x_RT, int KT, int M, const EpiArgs &epi,
                 const BatchMeta &meta, hipStream_t s);
int gemm_token_tile(int M);     // tokens per workgroup tile the tiled kernel will use for M rows

// k_attn.hip
struct AttnArgs {
  const bf16_t *q;          // [M][Hq*hd] row-major
  KvPool pool;
  int block;
  const int *page_table;
  int pages_per_session;
  int n_q_heads, n_kv_heads, head_dim;
  const float *alibi;       // per q head slopes or null
  bf16_t *o_out;            // T16 [M][Hq*hd] with o_RT row tiles per k step
  int o_RT;
  // decode (split-KV) only
  int n_splits;             // splits along the keys (grid size; at most 64)
  int split_pp;             // page pairs (32 keys) per split
  float *part;              // partial (m, l, O) per (session, kv head, split)
  float *logits;            // optional tap [B][Hq][logits_ld]
  int logits_ld;
  // prefill only, optional (training-time forward): what the backward pass needs later
  float *lse_out;           // [M][Hq] log2 of the sum of 2^(logit * log2 e) over each query's keys
  float *o_f32;             // [M][Hq*hd] the output rows in fp32
  // prefill only, optional test tap: the scaled (and ALiBi-biased) logits of query head tap_head for the new
  // tokens [tap_q0, tap_q0 + tap_nq) of the call's tap_sess-th session go to
  // tap_logits[(token - tap_q0) * tap_ld + key position]; entries of future keys are not written
  float *tap_logits;
  int tap_sess, tap_head, tap_q0, tap_nq, tap_ld;
};
size_t attn_decode_part_floats(int n_sess, int n_kv_heads, int n_splits, int head_dim);
void launch_attn_decode(const AttnArgs &a, const BatchMeta &meta, hipStream_t s);
void launch_attn_merge(const AttnArgs &a, const BatchMeta &meta, float *o_f32 /* optional [M][Hq*hd] */,
                       hipStream_t s);
void launch_attn_prefill(const AttnArgs &a, const BatchMeta &meta, int total_q_tiles, hipStream_t s);
int attn_prefill_q_tile();   // queries per workgroup tile of the prefill kernel
// copy whole pages (keys and values of all kv heads) for blocks [first_block, first_block + n_blocks)
struct PageCopies {
  int n;
  int src[64], dst[64];
};
void launch_kv_page_copy(const KvPool &pool, int first_block, int n_blocks, const PageCopies &pc, hipStream_t s);
void launch_kv_gather(const KvPool &pool, int block, const int *page_table_row, int pos0, int n,
                      bf16_t *k_out, bf16_t *v_out, hipStream_t s);
void launch_kv_scatter(const KvPool &pool, int block, const int *page_table, int pages_per_session,
                       const bf16_t *k, const bf16_t *v, int B, int L_max, const BatchMeta &lens, hipStream_t s);

// k_f32.hip: single-precision mode (fp32 weights, cache and arithmetic)
struct F32Pool {            // [block][page][K | V][kv head][slot][hd] fp32
  float *base;
  int max_pages, n_kv_heads, head_dim;
};
struct F32Block {           // canonical row-major fp32 matrices [out, in] and vectors of one block (null where the
  const float *norm1_g, *norm1_b, *wq, *bq, *wk, *bk, *wv, *bv, *wo, *bo;      // block style has none)
  const float *norm2_g, *norm2_b, *w_gate, *w_up, *b_up, *w_down, *b_down;
};
struct F32Call {
  const float *x_in;        // the call's input rows [M][d]
  float *resid, *h, *q, *o, *act;   // [M][d], [M][d], [M][Hq*hd], [M][Hq*hd], [M][F]
  int d, Hq, Hkv, hd, F, layernorm, rotary;
  float eps;
  const float *rope, *alibi;
  F32Pool pool;
  const int *page_table;
  int pps;
};
// one block of a forward call: norm, q/k/v (+ rotary, cache append), attention, output projection, norm, MLP;
// first = read the call's input instead of the residual stream; y = the call's output rows (last block) or null
void launch_f32_block(const F32Call &c, const F32Block &w, const BatchMeta &meta, int block, bool first, float *y,
                      hipStream_t s);
void launch_f32_kv_gather(const F32Pool &pool, int block, const int *page_table_row, int pos0, int n, float *k_out,
                          float *v_out, hipStream_t s);
void launch_f32_page_copy(const F32Pool &pool, int first_block, int n_blocks, const struct PageCopies &pc, hipStream_t s);

// k_misc.hip
struct NormArgs {
  const void *x_in;     // first block: the call's input rows (io dtype); else null
  int x_f32;
  float *resid;         // [M][d] fp32 residual stream (written when x_in != null, read otherwise)
  const float *gain, *bias;   // bias null for RMSNorm
  int layernorm;
  float eps;
  int d, RT, M;
  bf16_t *h_out;        // T16 with RT row tiles per k step
  float *shift_out;     // LayerNorm, optional: [M] receives the row means (start of the chain described at EpiArgs::shift)
};
void launch_norm(const NormArgs &a, hipStream_t s);
// tiled kernels' fused norm: partial sums [n_parts][ld rows][2] -> row_stat[row] = (1/sqrt(var + eps), mean)
void launch_row_stat(const float *tstat, int n_parts, int ld, float *row_stat, int M, int d, float eps, int center,
                     float *shift /* LayerNorm: shift[m] += the row's (shifted) mean; else null */, hipStream_t s);
void launch_fill_u32(uint32_t *p, size_t n, uint32_t v, hipStream_t s);
void launch_bf16_to_f32(const bf16_t *src, float *dst, int n, hipStream_t s);
void launch_rope_table(float *dst, int n_pos, int head_dim, double base, hipStream_t s);
void launch_alibi_slopes(float *dst, int n_heads, hipStream_t s);
struct PtUpdate {
  int n;
  int idx[120];
  int val[120];
};
void launch_pt_update(int *page_table, const PtUpdate &u, hipStream_t s);
void launch_iota(int *p, int n, hipStream_t s);
// ceiling probes (roofline report): out >= 4096 words / 65536 floats
void launch_stream_read(const void *src, size_t bytes, uint32_t *out, hipStream_t s);
void launch_mfma_loop(const void *seed, float *out, int iters, hipStream_t s);
// out[n] = (add ? add[n] : 0) + sum_k W[n][k] v[k] for row-major bf16 W [N, K] (set-up only)
void launch_rowdot(const bf16_t *w, const bf16_t *v, const float *add, float *out, int N, int K, hipStream_t s);

// ---- k_backward.hip: training-time passes (whole sequences, no cache) ---------------------------
// destination = T16 of the matrix whose row n, column k is S[k][n], S = src[0..2] stacked
// (row-major bf16 with `ld` columns; unused sources have rows = 0)
struct PackTArgs {
  const bf16_t *src[3];
  int rows[3];
  int ld;
  int KT, RT;
  bf16_t *dst;
};
void launch_pack_weight_t(const PackTArgs &a, int n_row_tiles, hipStream_t s);
// transposed copy of a packed bf16 matrix W [N logical rows][K]: dst = T16 of W^T (K rows, N columns)
struct TransposeArgs {
  const bf16_t *src;       // T16, physical row order `order`, s_RT row tiles per k step
  int s_RT, order, rows0, head_dim;   // rows0: GATEUP = rows of the gate matrix; head_dim: HEADS
  int N, K;
  bf16_t *dst;             // T16 with d_RT row tiles per k step (all of them are written)
  int d_RT;
};
void launch_transpose_t16(const TransposeArgs &a, int d_KT, hipStream_t s);
void launch_pack_act_f32(const float *x, bf16_t *dst, int M, int K, int KT, int RT, hipStream_t s);
void launch_rows_to_f32(const void *src, int src_f32, float *dst, size_t n, hipStream_t s);
void launch_rows_from_f32(const float *src, void *dst, int dst_f32, size_t n, hipStream_t s);
// acc[M][d] += gradient w.r.t. the norm's input x, given dy = gradient of its output
void launch_norm_bwd(const float *x, const float *gain, const float *dy, float *acc, int M, int d, float eps,
                     int layernorm, hipStream_t s);
// pre = [gate | up] ([M][2F], gated) or the GELU input ([M][F]); da [M][F]; dst = T16 of d(pre)
void launch_act_bwd_pack(const float *pre, const float *da, bf16_t *dst, int M, int F, int gated, int KT, int RT,
                         hipStream_t s);
void launch_qkv_bwd_pack(const float *dqkv, const float *rope, bf16_t *dst, int M, int n_q_heads, int n_kv_heads,
                         int hd, int rotary, int KT, int RT, const BatchMeta &meta, hipStream_t s);
struct TrainAttnArgs {
  const bf16_t *q;         // [M][Hq*hd] queries after the rotary embedding
  KvPool pool, pool2;      // keys / values of the call's sequences in pages: pool = (K row-wise, V transposed) as
                           // the forward kernel reads them, pool2 = (V row-wise, K transposed)
  int block;               // block index inside the pools
  const int *page_table;   // [sequence][pages_per_seq]
  int pages_per_seq;
  int n_q_heads, n_kv_heads, head_dim;
  const float *alibi;      // per q head slopes or null
  const float *o;          // [M][Hq*hd] forward output rows
  const float *lse;        // [M][Hq] as written by the forward kernel (base 2)
  const float *d_o;        // [M][Hq*hd] gradient of o
  float *delta;            // [M][Hq] scratch: do . o
  float *dqkv;             // [M][nqkv] gradient of [q | k | v] (q, k: after the rotary embedding)
  bf16_t *q_t, *do_t;      // scratch [Hq*hd][ld_t]: transposed bf16 copies of q and d_o (column = 16 * first page of the
  int ld_t;                // token's sequence + its position), written by the launcher before the dk/dv kernel
};
// meta: sequence i owns rows [cu[i], cu[i+1]) and row slot[i] of the page table; past = 0
void launch_attn_train_bwd(const TrainAttnArgs &a, const BatchMeta &meta, int M, hipStream_t s);
// page_table[i][j] = (pages of sequences before i) + j: the sequences' pages laid out one after the other
void launch_train_page_table(int *page_table, int pages_per_seq, const BatchMeta &meta, hipStream_t s);

// Attention over the paged, server-held KV cache.
//
// One wave handles NCT tiles of 16 "columns" against a range of keys, 32 keys (two pages)
// per iteration:
//   S^T = K . Q^T      v_mfma_f32_16x16x32_bf16, row operand = K page tile as stored,
//                      column operand = queries; a lane ends up with 8 logits of ONE column
//   softmax            running max / sum per column: in-lane over the 8 logits, then two
//                      wavefront shuffles across the four 16-lane groups
//   O^T += V^T . P^T   same instruction, row operand = V page tile as stored (values are
//                      kept transposed in the page), column operand = the lane's own 8
//                      probabilities; the rescale factor of a column lives in the same
//                      lanes as its accumulator, so no cross-lane traffic is needed.
// Columns are query tokens of one head (prefill / replay, any past length) or the query
// heads that share one kv head for a single new token (decode step, split along keys and
// merged by a second small kernel).
#include "common.h"
#include "launch.h"

namespace {

constexpr int PREFILL_NCT = 2;     // 32 queries per wave

// Prefill launches one workgroup per (query tile, kv head): its waves are the query heads
// that share the kv head, so they stream the same K/V pages at the same time and the
// pages are fetched from HBM once per group (L1/L2 hits for the other waves).
constexpr int PREFILL_MAX_WAVES = 8;

// TAP: a second instantiation that also writes logits to memory for the tests (prefill: those of one (session,
// head, query range); decode: all, for the stand-alone operator); the kernels the serving path runs carry none
// of that code.
template <int HD, int NCT, bool DECODE, bool BIAS, bool TAP = false>
__global__ __launch_bounds__(DECODE ? 64 : 64 * PREFILL_MAX_WAVES) void attn_kernel(AttnArgs a, BatchMeta meta) {
  constexpr int KS = HD / 32;      // k-steps of the QK product == 16-byte chunks per lane per page
  constexpr int HB = HD / 16;      // 16-row blocks of O^T
  constexpr int QT = 16 * NCT;
  const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
  const int G = a.n_q_heads / a.n_kv_heads;
  const float scale = rsqrtf((float)HD);

  int s, kvh, T, t0 = 0, split = 0;
  int head_of_col;                 // query head of this lane's column
  if (DECODE) {
    kvh = blockIdx.x; split = blockIdx.y; s = blockIdx.z;      // the kv heads of a page are adjacent in memory: launch them together
    T = 1;
    head_of_col = kvh * G + min(c, G - 1);
  } else {
    int tile = gridDim.x - 1 - blockIdx.x;       // long (late) tiles of a session are scheduled first
    s = 0;
    while (true) {
      int nt = ceil_div(meta.cu[s + 1] - meta.cu[s], QT);
      if (tile < nt) break;
      tile -= nt; ++s;
    }
    T = meta.cu[s + 1] - meta.cu[s];
    t0 = tile * QT;
    const int wpb = min(G, PREFILL_MAX_WAVES), parts = ceil_div(G, wpb);
    kvh = blockIdx.y / parts;
    const int hg = (blockIdx.y % parts) * wpb + (threadIdx.x >> 6);
    if (hg >= G) return;
    head_of_col = kvh * G + hg;
  }
  const int past = meta.past[s];
  const int *ptrow = a.page_table + (size_t)meta.slot[s] * a.pages_per_session;
  const int n_pg = ceil_div(past + T, SPAN_PAGE);
  const float slope = BIAS ? a.alibi[head_of_col] : 0.0f;

  // queries -> column operands
  bf16x8 Q[NCT][KS];
  int qpos[NCT], mrow[NCT];
  bool col_valid[NCT];
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) {
    int t = DECODE ? 0 : t0 + ct * 16 + c;
    col_valid[ct] = DECODE ? (c < G) : (t < T);
    t = min(t, T - 1);
    mrow[ct] = meta.cu[s] + t;
    qpos[ct] = past + t;
    const bf16_t *qp = a.q + ((size_t)mrow[ct] * a.n_q_heads + head_of_col) * HD + g * 8;
#pragma unroll
    for (int j = 0; j < KS; ++j) Q[ct][j] = *(const bf16x8 *)(qp + j * 32);
  }

  // key range in units of page pairs
  int pp0, pp1;
  if (DECODE) {
    // every split covers the same number of page pairs (a.split_pp), so a session gets splits
    // in proportion to its length and all waves of a ragged batch do about the same work
    const int npp = ceil_div(past + 1, 32);
    pp0 = split * a.split_pp;
    if (pp0 >= npp) return;
    pp1 = min(pp0 + a.split_pp, npp);
  } else {
    const int qmax = past + min(t0 + QT, T) - 1;
    pp0 = 0;
    pp1 = ceil_div(qmax + 1, 32);
  }

  f32x4 O[NCT][HB];
  float m_run[NCT], l_run[NCT];
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) {
    m_run[ct] = -INFINITY; l_run[ct] = 0.0f;
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) O[ct][hb] = f32x4{0, 0, 0, 0};
  }

  // K/V tiles of one iteration (two pages); the decode kernel keeps the next iteration's
  // tiles in flight while it works on the current ones
  struct Tiles { bf16x8 KA[KS], KB[KS]; u32x4 VA[KS], VB[KS]; };
  // The page ids of the next 64 pages of the session sit in a register, one per lane, and a step takes its two
  // with v_readlane: a scalar load of the page-table entry in every step costs its whole latency, because the
  // wave cannot issue the step's K/V loads (nor anything after them) before the entry is back.
  int pg_base = 2 * pp0;
  int my_pg = ptrow[min(pg_base + lane, n_pg - 1)];
  auto load_tiles = [&](int pp, Tiles &t) {
    if (2 * pp + 1 >= pg_base + 64) {        // uniform over the wave; steps come in increasing order
      pg_base = 2 * pp;
      my_pg = ptrow[min(pg_base + lane, n_pg - 1)];
    }
    const int pgA = __builtin_amdgcn_readlane(my_pg, 2 * pp - pg_base);
    const int pgB = __builtin_amdgcn_readlane(my_pg, 2 * pp + 1 - pg_base);      // (past the session's last page: its last page again)
    const bf16_t *kA = a.pool.base + a.pool.k_off(a.block, pgA, kvh) + lane * 8;
    const bf16_t *kB = a.pool.base + a.pool.k_off(a.block, pgB, kvh) + lane * 8;
    const bf16_t *vA = a.pool.base + a.pool.v_off(a.block, pgA, kvh) + lane * 8;
    const bf16_t *vB = a.pool.base + a.pool.v_off(a.block, pgB, kvh) + lane * 8;
#pragma unroll
    for (int j = 0; j < KS; ++j) {
      if (DECODE) {      // every K/V tile is read once per step: stream it past the caches
        t.KA[j] = __builtin_nontemporal_load((const bf16x8 *)(kA + j * 512));
        t.KB[j] = __builtin_nontemporal_load((const bf16x8 *)(kB + j * 512));
        t.VA[j] = __builtin_nontemporal_load((const u32x4 *)(vA + j * 512));
        t.VB[j] = __builtin_nontemporal_load((const u32x4 *)(vB + j * 512));
      } else {
        t.KA[j] = *(const bf16x8 *)(kA + j * 512);
        t.KB[j] = *(const bf16x8 *)(kB + j * 512);
        t.VA[j] = *(const u32x4 *)(vA + j * 512);
        t.VB[j] = *(const u32x4 *)(vB + j * 512);
      }
    }
  };
  Tiles cur, nxt;
  if (DECODE && pp0 < pp1) load_tiles(pp0, cur);

  // Softmax in base 2: logits are scaled by log2(e)/sqrt(hd) so that a probability costs one
  // v_exp_f32; the running maximum and sum (and the decode partials) live in that domain.
  const float scale2 = scale * 1.4426950408889634f, slope2 = slope * 1.4426950408889634f;
  // one 32-key step; MASK = some key of the step may lie in a query's future (only the steps on
  // the causal diagonal); BIAS (ALiBi) is fixed per kernel
  auto step = [&](int pp, auto mask_) {
    constexpr bool MASK = decltype(mask_)::value;
    const bf16x8 (&KA)[KS] = cur.KA;
    const bf16x8 (&KB)[KS] = cur.KB;
    const u32x4 (&VA)[KS] = cur.VA;
    const u32x4 (&VB)[KS] = cur.VB;
    const int kposA = pp * 32 + g * 4, kposB = kposA + 16;

    bf16x8 P[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
      f32x4 sA = {0, 0, 0, 0}, sB = {0, 0, 0, 0};
#pragma unroll
      for (int j = 0; j < KS; ++j) {
        sA = __builtin_amdgcn_mfma_f32_16x16x32_bf16(KA[j], Q[ct][j], sA, 0, 0, 0);
        sB = __builtin_amdgcn_mfma_f32_16x16x32_bf16(KB[j], Q[ct][j], sB, 0, 0, 0);
      }
      float sv[8];
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int kp = (i < 4 ? kposA + i : kposB + (i - 4));
        const float raw = i < 4 ? sA[i] : sB[i - 4];
        float v = raw * scale2;
        if (BIAS) v -= slope2 * (float)(qpos[ct] - kp);
        if (DECODE && TAP && kp <= qpos[ct] && c < G)     // (decode: the operator test's logits output)
          a.logits[((size_t)s * a.n_q_heads + head_of_col) * a.logits_ld + kp] = raw * scale - slope * (float)(qpos[ct] - kp);
        if constexpr (TAP && !DECODE) {
          const int tq = qpos[ct] - past - a.tap_q0;
          if (s == a.tap_sess && head_of_col == a.tap_head && col_valid[ct] && tq >= 0 && tq < a.tap_nq && kp <= qpos[ct])
            a.tap_logits[(size_t)tq * a.tap_ld + kp] = raw * scale - slope * (float)(qpos[ct] - kp);
        }
        if (MASK) v = kp <= qpos[ct] ? v : -INFINITY;
        sv[i] = v;
        mx = fmaxf(mx, v);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      // the accumulator is rescaled only when some column's maximum moved (rare after the first
      // steps of a long row); the test is uniform over the wave
      if (__any(mx > m_run[ct])) {
        const float m_new = fmaxf(m_run[ct], mx);
        const float alpha = __builtin_amdgcn_exp2f(m_run[ct] - m_new);
        l_run[ct] *= alpha;
        m_run[ct] = m_new;
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) O[ct][hb] *= alpha;
      }
      float ps = 0.0f, pv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) { pv[i] = __builtin_amdgcn_exp2f(sv[i] - m_run[ct]); ps += pv[i]; }
      l_run[ct] += ps;
      u32x4 pk;
      pk.x = pack_bf16x2(pv[0], pv[1]); pk.y = pack_bf16x2(pv[2], pv[3]);
      pk.z = pack_bf16x2(pv[4], pv[5]); pk.w = pack_bf16x2(pv[6], pv[7]);
      P[ct] = __builtin_bit_cast(bf16x8, pk);
    }
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
      const int c2 = hb >> 1;
      u32x4 vv;
      if (hb & 1) { vv.x = VA[c2].z; vv.y = VA[c2].w; vv.z = VB[c2].z; vv.w = VB[c2].w; }
      else        { vv.x = VA[c2].x; vv.y = VA[c2].y; vv.z = VB[c2].x; vv.w = VB[c2].y; }
      const bf16x8 Vop = __builtin_bit_cast(bf16x8, vv);
#pragma unroll
      for (int ct = 0; ct < NCT; ++ct)
        O[ct][hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Vop, P[ct], O[ct][hb], 0, 0, 0);
    }
  };
  // the first position any column of this wave holds: steps that end at or before it need no mask
  const int q_first = DECODE ? past : past + t0;
  // steps [pp0, pp_clear) lie wholly in every column's past, the rest touch the causal diagonal
  const int pp_clear = min(pp1, max(pp0, (q_first + 1) / 32));
  for (int pp = pp0; pp < pp_clear; ++pp) {
    if (DECODE) { if (pp + 1 < pp1) load_tiles(pp + 1, nxt); }
    else load_tiles(pp, cur);
    step(pp, std::false_type{});
    if (DECODE) cur = nxt;
  }
  for (int pp = pp_clear; pp < pp1; ++pp) {
    if (DECODE) { if (pp + 1 < pp1) load_tiles(pp + 1, nxt); }
    else load_tiles(pp, cur);
    step(pp, std::true_type{});
    if (DECODE) cur = nxt;
  }

#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) {
    float l = l_run[ct];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (DECODE) {
      // partial result of this split: [HD values | m | l] per column
      if (c < G) {
        float *pp = a.part + ((((size_t)s * a.n_kv_heads + kvh) * a.n_splits + split) * 16 + c) * (HD + 2);
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) *(f32x4 *)(pp + hb * 16 + g * 4) = O[ct][hb];
        if (g == 0) { pp[HD] = m_run[ct]; pp[HD + 1] = l; }
      }
    } else if (col_valid[ct]) {
      const float inv = 1.0f / l;
#pragma unroll
      for (int hb = 0; hb < HB; ++hb) {
        f32x4 o = O[ct][hb] * inv;
        u32x2 w;
        w.x = pack_bf16x2(o.x, o.y); w.y = pack_bf16x2(o.z, o.w);
        *(u32x2 *)(a.o_out + t16_off(mrow[ct], head_of_col * HD + hb * 16 + g * 4, a.o_RT)) = w;
        if (a.o_f32) *(f32x4 *)(a.o_f32 + ((size_t)mrow[ct] * a.n_q_heads + head_of_col) * HD + hb * 16 + g * 4) = o;
      }
      if (a.lse_out && g == 0) a.lse_out[(size_t)mrow[ct] * a.n_q_heads + head_of_col] = m_run[ct] + __log2f(l);
    }
  }
}

// Merge the split partials of one (session, query head).  One wave: lane sp first takes
// split sp's (max, sum) so that the softmax weights of all splits are formed in parallel;
// then every lane owns HD/64 head dimensions and walks the splits with the weights
// broadcast by shuffles (independent loads, no serial dependency through memory).
template <int HD>
__global__ __launch_bounds__(64) void attn_merge_kernel(AttnArgs a, BatchMeta meta, float *o_f32) {
  const int head = blockIdx.x, s = blockIdx.y, lane = threadIdx.x;
  const int G = a.n_q_heads / a.n_kv_heads;
  const int kvh = head / G, c = head % G;
  const float *base = a.part + (((size_t)s * a.n_kv_heads + kvh) * a.n_splits * 16 + c) * (HD + 2);
  const size_t stride = (size_t)16 * (HD + 2);
  // splits that hold part of this session: the first ceil(pairs / split_pp)
  const int n_valid = ceil_div(ceil_div(meta.past[s] + 1, 32), a.split_pp);
  float m = -INFINITY, l = 0.0f;
  if (lane < n_valid) { m = base[lane * stride + HD]; l = base[lane * stride + HD + 1]; }
  float M = m;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
  const float w = __builtin_amdgcn_exp2f(m - M);   // (the partials' maxima are in base 2) empty or absent split: m = -inf -> weight 0
  float den = w * l;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) den += __shfl_xor(den, o);
  constexpr int PER = HD / 64;
  float num[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) num[e] = 0.0f;
  // sixteen splits per round, all loads of a round issued before the first use (they do not
  // depend on the weights, so the first round overlaps the (max, sum) loads above as well)
  for (int sp0 = 0; sp0 < n_valid; sp0 += 16) {
    float v[16][PER];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
      for (int e = 0; e < PER; ++e) v[i][e] = sp0 + i < n_valid ? base[(sp0 + i) * stride + e * 64 + lane] : 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float ws = __shfl(w, sp0 + i);
#pragma unroll
      for (int e = 0; e < PER; ++e) num[e] += ws * v[i][e];
    }
  }
  const int mrow = meta.cu[s];
  const float inv = 1.0f / den;
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int h = e * 64 + lane;
    const float o = num[e] * inv;
    if (a.o_out) a.o_out[t16_off(mrow, head * HD + h, a.o_RT)] = f32_to_bf16(o);
    if (o_f32) o_f32[((size_t)mrow * a.n_q_heads + head) * HD + h] = o;
  }
}

__global__ void kv_gather_kernel(KvPool pool, int block, const int *ptrow, int pos0, int n, bf16_t *k_out,
                                 bf16_t *v_out) {
  const int hd = pool.head_dim, Hkv = pool.n_kv_heads;
  const size_t total = (size_t)n * Hkv * hd;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int h = i % hd, kh = (i / hd) % Hkv, t = i / ((size_t)hd * Hkv);
    const int pos = pos0 + t, pg = ptrow[pos >> 4], sl = pos & 15;
    if (k_out) k_out[i] = pool.base[pool.k_off(block, pg, kh) + kpage_off(sl, h)];
    if (v_out) v_out[i] = pool.base[pool.v_off(block, pg, kh) + vpage_off(sl, h)];
  }
}

// One workgroup per (copy, block): a page's keys and values of all kv heads are one contiguous run.
__global__ __launch_bounds__(256) void kv_page_copy_kernel(KvPool pool, int first_block, PageCopies pc) {
  const int blk = first_block + blockIdx.y;
  const size_t n16 = (size_t)2 * pool.n_kv_heads * pool.head_elems() / 8;      // 16-byte chunks per page
  const u32x4 *src = (const u32x4 *)(pool.base + pool.k_off(blk, pc.src[blockIdx.x], 0));
  u32x4 *dst = (u32x4 *)(pool.base + pool.k_off(blk, pc.dst[blockIdx.x], 0));
  for (size_t i = threadIdx.x; i < n16; i += blockDim.x) dst[i] = src[i];
}

// token-major [B][L_max][Hkv][hd] caches -> pages (operator tests)
__global__ void kv_scatter_kernel(KvPool pool, int block, const int *page_table, int pps, const bf16_t *k,
                                  const bf16_t *v, int B, int L_max, BatchMeta lens) {
  const int hd = pool.head_dim, Hkv = pool.n_kv_heads;
  const size_t total = (size_t)B * L_max * Hkv * hd;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int h = i % hd, kh = (i / hd) % Hkv;
    const int pos = (i / ((size_t)hd * Hkv)) % L_max, b = i / ((size_t)hd * Hkv * L_max);
    if (pos > lens.past[b]) continue;           // session b holds past[b] + 1 tokens
    const int pg = page_table[(size_t)lens.slot[b] * pps + (pos >> 4)], sl = pos & 15;
    pool.base[pool.k_off(block, pg, kh) + kpage_off(sl, h)] = k[i];
    pool.base[pool.v_off(block, pg, kh) + vpage_off(sl, h)] = v[i];
  }
}

}  // namespace

size_t attn_decode_part_floats(int n_sess, int n_kv_heads, int n_splits, int head_dim) {
  return (size_t)n_sess * n_kv_heads * n_splits * 16 * (head_dim + 2);
}

int attn_prefill_q_tile() { return 16 * PREFILL_NCT; }

template <int HD, bool BIAS>
static void launch_attn_decode_hb(const AttnArgs &a, const BatchMeta &meta, hipStream_t s) {
  dim3 grid(a.n_kv_heads, a.n_splits, meta.n_sess);
  if (a.logits) hipLaunchKernelGGL((attn_kernel<HD, 1, true, BIAS, true>), grid, dim3(64), 0, s, a, meta);
  else hipLaunchKernelGGL((attn_kernel<HD, 1, true, BIAS, false>), grid, dim3(64), 0, s, a, meta);
}

void launch_attn_decode(const AttnArgs &a, const BatchMeta &meta, hipStream_t s) {
  if (a.head_dim == 128) {
    if (a.alibi) launch_attn_decode_hb<128, true>(a, meta, s);
    else launch_attn_decode_hb<128, false>(a, meta, s);
  } else {
    if (a.alibi) launch_attn_decode_hb<64, true>(a, meta, s);
    else launch_attn_decode_hb<64, false>(a, meta, s);
  }
}

void launch_attn_merge(const AttnArgs &a, const BatchMeta &meta, float *o_f32, hipStream_t s) {
  dim3 grid(a.n_q_heads, meta.n_sess);
  if (a.head_dim == 128) {
    hipLaunchKernelGGL((attn_merge_kernel<128>), grid, dim3(64), 0, s, a, meta, o_f32);
  } else {
    hipLaunchKernelGGL((attn_merge_kernel<64>), grid, dim3(64), 0, s, a, meta, o_f32);
  }
}

void launch_attn_prefill(const AttnArgs &a, const BatchMeta &meta, int total_q_tiles, hipStream_t s) {
  const int G = a.n_q_heads / a.n_kv_heads;
  const int wpb = G < PREFILL_MAX_WAVES ? G : PREFILL_MAX_WAVES, parts = (G + wpb - 1) / wpb;
  dim3 grid(total_q_tiles, a.n_kv_heads * parts), block(64 * wpb);
  if (a.tap_logits) {
    if (a.head_dim == 128) {
      if (a.alibi) hipLaunchKernelGGL((attn_kernel<128, PREFILL_NCT, false, true, true>), grid, block, 0, s, a, meta);
      else hipLaunchKernelGGL((attn_kernel<128, PREFILL_NCT, false, false, true>), grid, block, 0, s, a, meta);
    } else {
      if (a.alibi) hipLaunchKernelGGL((attn_kernel<64, PREFILL_NCT, false, true, true>), grid, block, 0, s, a, meta);
      else hipLaunchKernelGGL((attn_kernel<64, PREFILL_NCT, false, false, true>), grid, block, 0, s, a, meta);
    }
    return;
  }
  if (a.head_dim == 128) {
    if (a.alibi) hipLaunchKernelGGL((attn_kernel<128, PREFILL_NCT, false, true>), grid, block, 0, s, a, meta);
    else hipLaunchKernelGGL((attn_kernel<128, PREFILL_NCT, false, false>), grid, block, 0, s, a, meta);
  } else {
    if (a.alibi) hipLaunchKernelGGL((attn_kernel<64, PREFILL_NCT, false, true>), grid, block, 0, s, a, meta);
    else hipLaunchKernelGGL((attn_kernel<64, PREFILL_NCT, false, false>), grid, block, 0, s, a, meta);
  }
}

void launch_kv_page_copy(const KvPool &pool, int first_block, int n_blocks, const PageCopies &pc, hipStream_t s) {
  if (pc.n < 1) return;
  hipLaunchKernelGGL(kv_page_copy_kernel, dim3(pc.n, n_blocks), dim3(256), 0, s, pool, first_block, pc);
}

void launch_kv_gather(const KvPool &pool, int block, const int *page_table_row, int pos0, int n, bf16_t *k_out,
                      bf16_t *v_out, hipStream_t s) {
  size_t total = (size_t)n * pool.n_kv_heads * pool.head_dim;
  int grid = (int)min((size_t)4096, (total + 255) / 256);
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(kv_gather_kernel, dim3(grid), dim3(256), 0, s, pool, block, page_table_row, pos0, n, k_out,
                     v_out);
}

void launch_kv_scatter(const KvPool &pool, int block, const int *page_table, int pages_per_session,
                       const bf16_t *k, const bf16_t *v, int B, int L_max, const BatchMeta &lens, hipStream_t s) {
  size_t total = (size_t)B * L_max * pool.n_kv_heads * pool.head_dim;
  int grid = (int)min((size_t)4096, (total + 255) / 256);
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(kv_scatter_kernel, dim3(grid), dim3(256), 0, s, pool, block, page_table, pages_per_session,
                     k, v, B, L_max, lens);
}

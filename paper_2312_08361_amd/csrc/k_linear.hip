// Projection kernels: weight packing, the weight-streaming skinny kernel used by decode
// steps, and the LDS-tiled MFMA kernel used by prefill / cache replay.
#include <atomic>

#include "common.h"
#include "epilogue.h"
#include "launch.h"

// ------------------------------------------------------------------------------------
// Packing: canonical row-major [rows, K] bf16 -> T16 tiles in the physical tile order the
// epilogues expect.  One wave per (k tile, physical row tile).
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void pack_weight_kernel(PackArgs a) {
  const int kt = blockIdx.x, pt = blockIdx.y, lane = threadIdx.x;
  const int g = lane >> 4, r = lane & 15;
  const bf16_t *src = nullptr;
  int row = -1, rows = 0;
  if (a.order == PACK_NATURAL) {
    src = a.src[0]; rows = a.rows[0]; row = pt * 16 + r;
  } else if (a.order == PACK_GATEUP) {
    int which = pt & 1;
    src = a.src[which]; rows = a.rows[which]; row = (pt >> 1) * 16 + r;
  } else {  // PACK_HEADS: [q heads | k heads | v heads], tiles (a, a+HT/2) adjacent
    const int HT = a.head_dim >> 4;
    int head = pt / HT, j = pt % HT;
    int lt = (j >> 1) + (j & 1) * (HT >> 1);
    int lrow = (head * HT + lt) * 16 + r;          // row in the concatenated matrix
    if (lrow < a.rows[0]) { src = a.src[0]; rows = a.rows[0]; row = lrow; }
    else if (lrow < a.rows[0] + a.rows[1]) { src = a.src[1]; rows = a.rows[1]; row = lrow - a.rows[0]; }
    else { src = a.src[2]; rows = a.rows[2]; row = lrow - a.rows[0] - a.rows[1]; }
  }
  const int k = kt * 32 + g * 8;
  u32x4 v = {0, 0, 0, 0};
  if (src && row >= 0 && row < rows && k < a.K) v = *(const u32x4 *)(src + (size_t)row * a.K + k);
  *(u32x4 *)(a.dst + ((size_t)kt * a.RT + pt) * 512 + lane * 8) = v;
}

void launch_pack_weight(const PackArgs &a, int n_phys_tiles, hipStream_t s) {
  hipLaunchKernelGGL(pack_weight_kernel, dim3(a.KT, n_phys_tiles), dim3(64), 0, s, a);
}

// row-major bf16 activations [M, K] -> T16 (rows beyond M and k beyond K are zero)
__global__ __launch_bounds__(64) void pack_act_kernel(const bf16_t *x, bf16_t *dst, int M, int K, int KT) {
  const int kt = blockIdx.x, mt = blockIdx.y, lane = threadIdx.x;
  const int g = lane >> 4, r = lane & 15;
  const int row = mt * 16 + r, k = kt * 32 + g * 8;
  u32x4 v = {0, 0, 0, 0};
  if (row < M && k < K) v = *(const u32x4 *)(x + (size_t)row * K + k);
  *(u32x4 *)(dst + ((size_t)kt * gridDim.y + mt) * 512 + lane * 8) = v;
}

void launch_pack_act(const bf16_t *x, bf16_t *dst, int M, int K, int KT, int m_tiles, hipStream_t s) {
  hipLaunchKernelGGL(pack_act_kernel, dim3(KT, m_tiles), dim3(64), 0, s, x, dst, M, K, KT);
}

// ------------------------------------------------------------------------------------
// Weight-streaming skinny kernel (decode).  HBM-bound: every weight byte is read exactly
// once, as 1 KiB fully coalesced wave loads straight into MFMA operand registers.
//
// Work is the flat sequence of (tile pair, k tile) items, pair-major; a pair is 32 output
// rows.  Workgroup g owns items [g*L, (g+1)*L): whole pairs when L is a multiple of KT, and
// otherwise a share that makes every compute unit stream the same number of bytes whatever
// the pair count is (320 pairs on 256 CUs would otherwise take two rounds).  For each pair
// it touches, the workgroup's waves take the k tiles of its range in turn, U at a time (so the
// whole chip sweeps one contiguous region of the matrix at any moment: 1.5 us per launch faster
// at the 70B shape than giving every wave one contiguous eighth of the range), partial sums meet
// in LDS and waves 0..MT-1 hold the result.  A pair covered completely goes straight to the fused epilogue.
// A pair shared with neighbouring workgroups goes through memory: each sharer stores its
// piece, then bumps the pair's counter; whoever brings the counter to the number of pieces
// adds all pieces in workgroup order (so the sum does not depend on who came last), runs the
// epilogue and clears the counter for the next launch.  Nobody waits for anybody.
// Tokens (<= 16*MT) are the MFMA column operand, read from a T16 activation buffer that
// stays L2-resident.
// ------------------------------------------------------------------------------------
template <int MT, int WAVES, int U, int EPI>
__global__ __launch_bounds__(WAVES * 64) void gemv_kernel(const bf16_t *__restrict__ wp, int w_RT,
                                                          const bf16_t *__restrict__ xp, int x_RT, int KT,
                                                          int n_pairs, GemvShare sh, EpiArgs epi, BatchMeta meta) {
  __shared__ f32x4 red[WAVES][2][MT][64];
  __shared__ float stat[WAVES][2][64];
  __shared__ int finisher;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // fused norm, consumer side: sum the producer's per-workgroup partials of each token's
  // row statistics (fixed order, so the result does not depend on scheduling).  A wave
  // covers PPW partials x TOK tokens per load; the loads are independent of the weight
  // stream that follows and stay in flight behind it.
  constexpr int TOK = 16 * MT, PPW = 64 / TOK, SJ = 8;
  float sreg[SJ], treg[SJ];
  const int st_sub = lane / TOK, st_tok = lane % TOK;
  const bool st_on = epi.stat_in && st_sub < PPW && st_tok < epi.M;
#pragma unroll
  for (int j = 0; j < SJ; ++j) {
    const int q = (j * WAVES + wave) * PPW + st_sub;
    const bool ok = st_on && q < epi.stat_parts;
    sreg[j] = ok ? epi.stat_in[(size_t)q * 128 + st_tok] : 0.0f;
    treg[j] = ok ? epi.stat_in[(size_t)q * 128 + 64 + st_tok] : 0.0f;
  }
  // the epilogue lanes (waves 0..MT-1) own token em, output rows er4..er4+3 of both tiles
  const int el = wave * 16 + (lane & 15), em = epi.m0 + el, er4 = (lane >> 4) * 4;
  const bool e_on = wave < MT && em < epi.M;
  TokInfo ti = token_info(meta, e_on ? em : 0);

  const bf16x8 *xb = (const bf16x8 *)xp + lane;
  // Token rows past the end of the call are padding: their lanes take zeros instead of loading.  The
  // activation tiles share the vector memory path with the weight stream, and with 8 tokens in a
  // 16-row tile half of their requests carried nothing (measured: 69.7 -> 67.5 us per launch at the
  // 70B shape, 413 -> 426 decode steps/s).
  bool x_on[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) x_on[mt] = epi.m0 + mt * 16 + (lane & 15) < epi.M;
  const size_t wst = (size_t)w_RT * 64, xst = (size_t)x_RT * 64;
  const long total = (long)n_pairs * KT;
  const long f0 = (long)blockIdx.x * sh.L;
  const long f1 = f0 + sh.L < total ? f0 + sh.L : total;
  bool first = true;

  for (long f = f0; f < f1;) {            // uniform over the workgroup
    const int p = (int)(f / KT), ka = (int)(f - (long)p * KT);
    const int kb = (f1 - f) < (long)(KT - ka) ? ka + (int)(f1 - f) : KT;
    // what the epilogue needs besides the sums is fetched ahead of the weight stream
    EpiPre pre{};
    if (e_on) pre = epilogue_prefetch<EPI>(epi, ti, em, p, er4);

    // the waves of a workgroup take the k tiles of its range in turn, U at a time, so that at any moment the
    // whole chip reads one contiguous region of the matrix
    const int n_grp = (kb - ka) / U;
    // tiles (kt, 2p) and (kt, 2p+1) are adjacent: one 2 KiB run per k step
    const bf16x8 *w0 = (const bf16x8 *)wp + (size_t)(2 * p) * 64 + lane;
    const bf16x8 *w1 = w0 + 64;

    f32x4 acc0[MT], acc1[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) { acc0[mt] = f32x4{0, 0, 0, 0}; acc1[mt] = f32x4{0, 0, 0, 0}; }

    for (int j = wave; j < n_grp; j += WAVES) {
      const int kt = ka + j * U;
      bf16x8 a0[U], a1[U], b[U][MT];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        a0[u] = __builtin_nontemporal_load(w0 + (kt + u) * wst);
        a1[u] = __builtin_nontemporal_load(w1 + (kt + u) * wst);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) b[u][mt] = x_on[mt] ? xb[(kt + u) * xst + mt * 64] : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          acc0[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[u], b[u][mt], acc0[mt], 0, 0, 0);
          acc1[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1[u], b[u][mt], acc1[mt], 0, 0, 0);
        }
    }
    for (int kt = ka + n_grp * U + wave; kt < kb; kt += WAVES) {
      bf16x8 a0 = __builtin_nontemporal_load(w0 + kt * wst);
      bf16x8 a1 = __builtin_nontemporal_load(w1 + kt * wst);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        bf16x8 b = x_on[mt] ? xb[kt * xst + mt * 64] : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        acc0[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b, acc0[mt], 0, 0, 0);
        acc1[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b, acc1[mt], 0, 0, 0);
      }
    }

    if (first && epi.stat_in) {
      float ss = 0.0f, s1 = 0.0f;
#pragma unroll
      for (int j = 0; j < SJ; ++j) { ss += sreg[j]; s1 += treg[j]; }
      if (st_on)
        for (int q = (SJ * WAVES + wave) * PPW + st_sub; q < epi.stat_parts; q += WAVES * PPW) {
          ss += epi.stat_in[(size_t)q * 128 + st_tok];
          s1 += epi.stat_in[(size_t)q * 128 + 64 + st_tok];
        }
      stat[wave][0][lane] = ss; stat[wave][1][lane] = s1;
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) { red[wave][0][mt][lane] = acc0[mt]; red[wave][1][mt][lane] = acc1[mt]; }
    __syncthreads();

    f32x4 v0 = f32x4{0, 0, 0, 0}, v1 = v0;
    if (wave < MT) {
      v0 = red[0][0][wave][lane]; v1 = red[0][1][wave][lane];
#pragma unroll
      for (int w = 1; w < WAVES; ++w) { v0 += red[w][0][wave][lane]; v1 += red[w][1][wave][lane]; }
      if (first && e_on && epi.stat_in) {
        float ss = 0.0f, s1 = 0.0f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w)
#pragma unroll
          for (int q = 0; q < PPW; ++q) { ss += stat[w][0][q * TOK + el]; s1 += stat[w][1][q * TOK + el]; }
        const float inv_d = 1.0f / (float)epi.norm_d;
        ti.mu = epi.norm_center ? s1 * inv_d : 0.0f;
        ti.r = rsqrtf(fmaxf(ss * inv_d - ti.mu * ti.mu, 0.0f) + epi.norm_eps);   // one-pass variance: rounding may leave it a hair below zero
        // the sums are of values shifted by the previous norm's mean: leave this norm's mean for the next producer
        if (epi.shift && blockIdx.x == 0 && er4 == 0) epi.shift[em] += ti.mu;
      }
    }
    first = false;

    bool finish = ka == 0 && kb == KT;
    if (!finish) {
      // shared pair: pieces come from workgroups g_first..g_last.  A workgroup's piece lives in
      // its slot 0 when the piece starts the workgroup's range, else in slot 1 (then it is
      // the last thing the workgroup does, so the two never collide).
      const int g_first = (int)(((long)p * KT) / sh.L), g_last = (int)(((long)(p + 1) * KT - 1) / sh.L);
      const int g = blockIdx.x;
      float *mine = (float *)(sh.part + ((size_t)g * 2 + (f == f0 ? 0 : 1)) * (2 * MT * 64));
      // The pieces travel as device-scope atomic accesses, which are coherent between the
      // L2 caches of the chip's dies without flushing or invalidating anything; a piece is
      // complete in memory (stores acknowledged, then the workgroup barrier) before thread 0
      // bumps the counter, and the finisher reads only after it has seen the final count.
      if (wave < MT) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          __hip_atomic_store(mine + (wave * 64 + lane) * 4 + i, v0[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(mine + ((MT + wave) * 64 + lane) * 4 + i, v1[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's piece has been acknowledged
      __syncthreads();
      if (threadIdx.x == 0) {
        const unsigned old = __hip_atomic_fetch_add(sh.count + p, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = old == (unsigned)(g_last - g_first);
        if (last) __hip_atomic_store(sh.count + p, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        finisher = last;
      }
      __syncthreads();
      finish = finisher != 0;
      if (finish && wave < MT) {
        v0 = f32x4{0, 0, 0, 0}; v1 = v0;
        for (int gi = g_first; gi <= g_last; ++gi) {
          const bool starts_here = (long)gi * sh.L >= (long)p * KT;
          const float *pc = (const float *)(sh.part + ((size_t)gi * 2 + (starts_here ? 0 : 1)) * (2 * MT * 64));
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            v0[i] += __hip_atomic_load(pc + (wave * 64 + lane) * 4 + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            v1[i] += __hip_atomic_load(pc + ((MT + wave) * 64 + lane) * 4 + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
        }
      }
    }
    if (finish && e_on) epilogue_pair_k<EPI>(epi, ti, em, p, er4, v0, v1, &pre);
    f += kb - ka;
    if (f < f1) __syncthreads();          // red[] and `finisher` are reused by the next pair
  }
}

// Work split of the skinny kernel: `grid` workgroups of `L` k tiles each (see above).
static void gemv_split(int n_pairs, int KT, int *grid, int *L) {
  // Whole pairs load the CUs evenly when their number is a multiple of the CU count, and well enough
  // when there are many short ones (two workgroups run per CU and the stream stays saturated while the
  // last ones finish: 7B gate/up, 688 pairs of 128 k tiles, 2360 -> 2456 steps/s).  Otherwise one
  // workgroup per CU, each with an equal share of the k tiles (measured on the 70B q/k/v projection:
  // 256 workgroups beat 512 and more; with long pairs the shares also win at 1344 pairs of 448 k
  // tiles, the BLOOM q/k/v).  At least half a pair each, so a pair never spans more than three workgroups.
  if (n_pairs % GEMV_MAX_GRID == 0 || n_pairs < 1 || (n_pairs >= 2 * GEMV_MAX_GRID && KT <= 256)) { *grid = n_pairs; *L = KT; return; }
  const long total = (long)n_pairs * KT;
  const int g = 2 * n_pairs < GEMV_MAX_GRID ? 2 * n_pairs : GEMV_MAX_GRID;
  int l = (int)((total + g - 1) / g);
  *L = l;
  *grid = (int)((total + l - 1) / l);
}

template <int MT, int EPI>
static void launch_gemv_me(const bf16_t *wp, int w_RT, const bf16_t *xp, int x_RT, int KT, int n_pairs,
                           const GemvShare &share, const EpiArgs &epi, const BatchMeta &meta, hipStream_t s) {
  GemvShare sh = share;
  int grid;
  gemv_split(n_pairs, KT, &grid, &sh.L);
  if (sh.L >= 64) {
    hipLaunchKernelGGL((gemv_kernel<MT, 8, 4, EPI>), dim3(grid), dim3(512), 0, s, wp, w_RT, xp, x_RT, KT, n_pairs, sh, epi, meta);
  } else {
    hipLaunchKernelGGL((gemv_kernel<MT, 4, 2, EPI>), dim3(grid), dim3(256), 0, s, wp, w_RT, xp, x_RT, KT, n_pairs, sh, epi, meta);
  }
}

template <int MT>
static void launch_gemv_mt(const bf16_t *wp, int w_RT, const bf16_t *xp, int x_RT, int KT, int n_pairs,
                           const GemvShare &sh, const EpiArgs &epi, const BatchMeta &meta, hipStream_t s) {
  switch (epi.kind) {
    case EPI_PLAIN: launch_gemv_me<MT, EPI_PLAIN>(wp, w_RT, xp, x_RT, KT, n_pairs, sh, epi, meta, s); break;
    case EPI_QKV: launch_gemv_me<MT, EPI_QKV>(wp, w_RT, xp, x_RT, KT, n_pairs, sh, epi, meta, s); break;
    case EPI_RESID: launch_gemv_me<MT, EPI_RESID>(wp, w_RT, xp, x_RT, KT, n_pairs, sh, epi, meta, s); break;
    case EPI_SWIGLU: launch_gemv_me<MT, EPI_SWIGLU>(wp, w_RT, xp, x_RT, KT, n_pairs, sh, epi, meta, s); break;
    default: launch_gemv_me<MT, EPI_GELU>(wp, w_RT, xp, x_RT, KT, n_pairs, sh, epi, meta, s); break;
  }
}

size_t gemv_share_part_bytes() { return (size_t)GEMV_MAX_GRID * 2 * (2 * 4 * 64) * sizeof(f32x4); }

void launch_gemv(const bf16_t *wp, int w_RT, const bf16_t *xp, int x_RT, int KT, int n_pairs, int m_tiles,
                 const GemvShare &sh, const EpiArgs &epi, const BatchMeta &meta, hipStream_t s) {
  switch (m_tiles) {
    case 1: launch_gemv_mt<1>(wp, w_RT, xp, x_RT, KT, n_pairs, sh, epi, meta, s); break;
    case 2: launch_gemv_mt<2>(wp, w_RT, xp, x_RT, KT, n_pairs, sh, epi, meta, s); break;
    case 3: launch_gemv_mt<3>(wp, w_RT, xp, x_RT, KT, n_pairs, sh, epi, meta, s); break;
    default: launch_gemv_mt<4>(wp, w_RT, xp, x_RT, KT, n_pairs, sh, epi, meta, s); break;
  }
}

// ------------------------------------------------------------------------------------
// LDS-tiled MFMA kernels (prefill / replay).  Both operands are T16, so a stage (32 k) is a
// set of 1 KiB tiles copied verbatim: coalesced global reads, conflict-free ds_read_b128 of
// v_mfma_f32_32x32x16_bf16 operands.  Two kernels share tile mapping and epilogues:
//   gemmd_kernel  256 rows x 256 tokens, for long calls (the replay path): tiles go
//                 memory -> LDS directly, eight waves
//   gemm_kernel   256 rows x 64 or 128 tokens, for short calls and for projections whose
//                 256-token tiles would leave compute units idle: tiles staged through
//                 registers, four waves
// Both require KT % 4 == 0.
//
// gemm_kernel: workgroup tile 256 weight rows x (64*WTOK) tokens, 4 waves as 2 x 2, each wave
// 128 rows x (32*WTOK) tokens.  Data path global -> registers -> LDS, with the loads of stage
// s+4 issued during stage s (four rotating register sets), so about three stages of MFMA work
// cover the memory latency.  Inside a stage the 32 MFMAs run as 8 rows of 4; between rows the
// wave issues two operand reads for the next k step, two LDS writes of the next stage and one
// global load.  Two LDS stage buffers, one barrier per stage.
// ------------------------------------------------------------------------------------
#include "tile_map.h"

// Epilogue of the tiled kernels for one token row of a lane: eight fragments (two 32-row blocks x
// four) of four values from each tile of a pair, 64 of the 128 features the wave holds of that row
// (the lane 32 further on holds the other 64).  With the norm fused across kernels (see EpiArgs) a
// consumer takes the row's (1/sigma, mean) from row_stat, and a producer adds up the new residual
// values and leaves the row's partial sums over each quad (64 features) of the wave in tstat_out.
// NV = quads (64 weight rows) this wave holds: 2, or 1 in the narrower tiles of gemmd_kernel; quad_end = quads of
// the matrix (the last narrower tile of a part may reach past it: those quads are dropped).
template <int EPI, int CT, int CI, int NV = 2>
__device__ __forceinline__ void tile_epilogue(const EpiArgs &epi, const BatchMeta &meta, f32x16 (&acc)[4][CT], int m,
                                              int quad0, int quad_end, int gq) {
  const bool on = m < epi.M;
  TokInfo ti = token_info(meta, on ? m : 0);
  if (on && epi.row_stat) { ti.r = epi.row_stat[2 * (size_t)m]; ti.mu = epi.row_stat[2 * (size_t)m + 1]; }
  float ss[2] = {0.0f, 0.0f}, s1[2] = {0.0f, 0.0f};
  static_for<4 * NV>([&](auto c_) {
    constexpr int c = decltype(c_)::value, v = c >> 2, j = c & 3;
    f32x4 v0, v1;
    v0.x = acc[2 * v][CI][4 * j + 0]; v0.y = acc[2 * v][CI][4 * j + 1];
    v0.z = acc[2 * v][CI][4 * j + 2]; v0.w = acc[2 * v][CI][4 * j + 3];
    v1.x = acc[2 * v + 1][CI][4 * j + 0]; v1.y = acc[2 * v + 1][CI][4 * j + 1];
    v1.z = acc[2 * v + 1][CI][4 * j + 2]; v1.w = acc[2 * v + 1][CI][4 * j + 3];
    if (on && quad0 + v < quad_end) {
      const int p = (quad0 + v) * 2 + (j >> 1), r4 = (j & 1) * 8 + gq * 4;
      if constexpr (EPI == EPI_RESID) {
        if (epi.tstat_out) {                 // producer: the new residual values are needed here as well
          const EpiPre pre = epilogue_prefetch<EPI_RESID>(epi, ti, m, p, r4);
          // (features past the model width are padding: they count for nothing)
          const int nA = (2 * p) * 16 + r4;
          const f32x4 zero = {0, 0, 0, 0};
          const f32x4 n0 = nA < epi.N ? v0 + pre.a - pre.shift : zero, n1 = nA + 16 < epi.N ? v1 + pre.b - pre.shift : zero;
          ss[v] += (n0.x * n0.x + n0.y * n0.y + n0.z * n0.z + n0.w * n0.w) + (n1.x * n1.x + n1.y * n1.y + n1.z * n1.z + n1.w * n1.w);
          s1[v] += (n0.x + n0.y + n0.z + n0.w) + (n1.x + n1.y + n1.z + n1.w);
          epilogue_pair_k<EPI>(epi, ti, m, p, r4, v0, v1, &pre);
        } else {
          epilogue_pair_k<EPI>(epi, ti, m, p, r4, v0, v1);
        }
      } else {
        epilogue_pair_k<EPI>(epi, ti, m, p, r4, v0, v1);
      }
    }
  });
  if constexpr (EPI == EPI_RESID) {
    if (epi.tstat_out) {                     // uniform over the workgroup: one pair of partial sums per (row, quad)
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const float a = ss[v] + __shfl_xor(ss[v], 32), b = s1[v] + __shfl_xor(s1[v], 32);
        if (on && gq == 0 && quad0 + v < quad_end) {
          float *t = epi.tstat_out + ((size_t)(quad0 + v) * epi.tstat_ld + m) * 2;
          t[0] = a; t[1] = b;
        }
      }
    }
  }
}

template <int WTOK, int EPI>
__global__ __launch_bounds__(256) void gemm_kernel(const bf16_t *__restrict__ wp, int w_RT,
                                                    const bf16_t *__restrict__ xp, int x_RT, int KT, int NW, int NM, TileBands tb,
                                                    EpiArgs epi, BatchMeta meta) {
  constexpr int W_TILES = 16, X_TILES = 4 * WTOK;
  constexpr int STAGE_TILES = W_TILES + X_TILES;              // one k tile (32 k) per stage
  constexpr int LOADS = STAGE_TILES / 4;                      // 1 KiB tiles per wave per stage (8, 6, 5)
  constexpr int STAGE_BYTES = STAGE_TILES * 1024;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wn = wave & 1, wm = wave >> 1;

  int wg_n, wg_m;
  if (!tile_of_block(tb, NW, NM, blockIdx.x, wg_n, wg_m)) return;

  // tile t of a stage: t < 16 weight row tile t, else token tile t-16; wave w copies tiles
  // w*LOADS...  Loads go through buffer resources (scalar base + scalar offset + 16*lane), so a
  // load costs one instruction and no vector address arithmetic; reads past a matrix return 0.
  const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
      (void *)(wp + (size_t)wg_n * W_TILES * 512), 0, (unsigned)(((size_t)w_RT * KT - (size_t)wg_n * W_TILES) * 1024), 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
      (void *)(xp + (size_t)wg_m * X_TILES * 512), 0, (unsigned)(((size_t)x_RT * KT - (size_t)wg_m * X_TILES) * 1024), 0x00020000);
  unsigned soff[LOADS], sstep[LOADS];
  const unsigned loff = lane * 16;
#pragma unroll
  for (int i = 0; i < LOADS; ++i) {
    const int t = wave * LOADS + i;
    soff[i] = (t < W_TILES ? t : t - W_TILES) * 1024;
    sstep[i] = (t < W_TILES ? w_RT : x_RT) * 1024;
  }
  const int NS = KT;
  u32x4 G[4][LOADS];                                          // staging registers of four stages
  // soff[i] walks forward one stage per load of tile i; past the last stage it stays put
  // (re-loads the last stage, unused)
  auto gload = [&](auto set_, int stage, int i) {
    constexpr int set = decltype(set_)::value;
    const bool is_w = wave * LOADS + i < W_TILES;
    G[set][i] = is_w ? __builtin_amdgcn_raw_buffer_load_b128(rs_w, loff, soff[i], 0)
                     : __builtin_amdgcn_raw_buffer_load_b128(rs_x, loff, soff[i], 0);
    soff[i] += stage + 1 < NS ? sstep[i] : 0;
  };
  char *const wdst = smem + wave * LOADS * 1024 + lane * 16;
  auto lwrite = [&](auto set_, int buf, int i) {
    constexpr int set = decltype(set_)::value;
    *(u32x4 *)(wdst + buf * STAGE_BYTES + i * 1024) = G[set][i];
  };

  f32x16 acc[4][WTOK];
#pragma unroll
  for (int bi = 0; bi < 4; ++bi)
#pragma unroll
    for (int ci = 0; ci < WTOK; ++ci)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[bi][ci][e] = 0.0f;

  const int gq = lane >> 5, r32 = lane & 31;
  int a_off[4], b_off[WTOK];
#pragma unroll
  for (int bi = 0; bi < 4; ++bi) {
    const int quad = wn * 2 + (bi >> 1), e = bi & 1;
    const int tile = quad * 4 + e + ((r32 >> 4) << 1);
    a_off[bi] = tile * 1024 + (gq * 16 + (r32 & 15)) * 16;
  }
#pragma unroll
  for (int ci = 0; ci < WTOK; ++ci) {
    const int tile = (wm * WTOK + ci) * 2 + (r32 >> 4);
    b_off[ci] = (W_TILES + tile) * 1024 + (gq * 16 + (r32 & 15)) * 16;
  }
  bf16x8 A0[4], B0[WTOK], A1[4], B1[WTOK];
#define PIN __builtin_amdgcn_sched_barrier(0)

  // prologue: stages 0..3 in flight, stage 0 into LDS buffer 0
  static_for<4>([&](auto j_) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) gload(j_, decltype(j_)::value, i);
  });
#pragma unroll
  for (int i = 0; i < LOADS; ++i) lwrite(std::integral_constant<int, 0>{}, 0, i);
  __syncthreads();
#pragma unroll
  for (int bi = 0; bi < 4; ++bi) A0[bi] = *(const bf16x8 *)(smem + a_off[bi]);
#pragma unroll
  for (int ci = 0; ci < WTOK; ++ci) B0[ci] = *(const bf16x8 *)(smem + b_off[ci]);

  // One stage = 32 MFMAs (8 rows of 4).  With a single wave per SIMD every other instruction
  // must slip into the shadow of an MFMA (32 cycles), so the stage's 16 operand reads, LOADS
  // LDS writes and LOADS global loads are dealt out one per MFMA:
  //   after MFMA 0..7   : read operand set 1 of this stage (needed from MFMA 16)
  //   after MFMA 6..13  : write stage s+1 (registers) to the other LDS buffer
  //   after MFMA 15     : barrier (stage s+1 visible to all)
  //   after MFMA 16..23 : read operand set 0 of stage s+1 (needed from the next MFMA 0)
  //   after MFMA 24..31 : global loads of stage s+4 into the registers just freed
  for (int s0 = 0; s0 < NS; s0 += 4) {
    static_for<4>([&](auto j_) {
      constexpr int j = decltype(j_)::value;
      constexpr int cur = j & 1, nxt = cur ^ 1;               // LDS buffers of stage s and s+1
      using SetNext = std::integral_constant<int, (j + 1) & 3>;   // registers holding stage s+1
      const int s = s0 + j;
      static_for<32>([&](auto m_) {
        constexpr int m = decltype(m_)::value;
        constexpr int half = m / 16, bi = (m % 16) / 4, ci = m % 4;
        if constexpr (ci < WTOK) {
          PIN;
          if constexpr (half == 0)
            acc[bi][ci] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A0[bi], B0[ci], acc[bi][ci], 0, 0, 0);
          else
            acc[bi][ci] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1[bi], B1[ci], acc[bi][ci], 0, 0, 0);
          PIN;
        }
        // ---- the shadow of MFMA m
        if constexpr (m < 8) {                                   // operand set 1 of stage s
          const char *b = smem + cur * STAGE_BYTES + 512;
          if constexpr (m < 4) A1[m] = *(const bf16x8 *)(b + a_off[m]);
          else if constexpr (m - 4 < WTOK) B1[m - 4] = *(const bf16x8 *)(b + b_off[m - 4]);
        }
        if constexpr (m >= 6 && m < 14) {
          if constexpr (m - 6 < LOADS) lwrite(SetNext{}, nxt, m - 6);
        }
        if constexpr (m == 15) { PIN; __syncthreads(); }
        if constexpr (m >= 16 && m < 24) {                       // operand set 0 of stage s+1
          const char *b = smem + nxt * STAGE_BYTES;
          if constexpr (m < 20) A0[m - 16] = *(const bf16x8 *)(b + a_off[m - 16]);
          else if constexpr (m - 20 < WTOK) B0[m - 20] = *(const bf16x8 *)(b + b_off[m - 20]);
        }
        if constexpr (m >= 24) {
          if constexpr (m - 24 < LOADS) gload(j_, s + 4, m - 24);
        }
      });
      PIN;
    });
  }
#undef PIN

  static_for<WTOK>([&](auto ci_) {
    constexpr int ci = decltype(ci_)::value;
    tile_epilogue<EPI, WTOK, ci>(epi, meta, acc, (wg_m * X_TILES + (wm * WTOK + ci) * 2) * 16 + r32, wg_n * 4 + wn * 2, w_RT / 4, gq);
  });
}

// gemmd_kernel: the stage tiles go from memory straight into LDS (buffer loads with the LDS
// modifier): no staging registers and no LDS store instructions, whose data path was the
// busiest unit of the register-staged kernel at this tile size (its LDS data FIFO was full
// for a fifth of the run).  2 x WM waves; WM = 4 puts two waves on every SIMD, each wave
// 128 rows x 64 tokens.  A ring of NB LDS stage buffers; the copies of stage s+NB-1 are
// issued during the first MFMAs of stage s, one per MFMA; one barrier per stage.
// Measured on the 70B shapes (16384 tokens): 1.26-1.30 PFLOP/s against 1.19 for the
// register-staged kernel; ring depth 3, 4 or 5 and the position of the copies inside the stage
// made no measurable difference, flat instead of buffer addressing cost about 2 %.
#define WAITCNT_VM_LGKM0(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4))
// HQ = quads (64 weight rows) per tile: 4 = the 256-row tile; 3, 2, 1 = narrower tiles for the last weight rows of
// a matrix whose 256-row tiles do not come out in whole rounds of 256 workgroups (the launcher cuts the rows into
// a part of 256-row tiles in whole rounds and a part of narrower tiles, see launch_gemm).  A wave of the "wn = 0"
// half holds NQ0 quads, one of the "wn = 1" half NQ1: (2,2), (2,1), (1,1), (1,0).  With unequal halves the waves
// are paired so that every SIMD runs one of each (waves w and w + 4 share a SIMD), i.e. the matrix work per
// SIMD, and with it the tile's time, shrinks with the tile's height.  quad_base = first quad of the part.
template <int WM, int EPI, int NB = 4, int HQ = 4>
__global__ __launch_bounds__(128 * WM) void gemmd_kernel(const bf16_t *__restrict__ wp, int w_RT,
                                                          const bf16_t *__restrict__ xp, int x_RT, int KT, int NW, int NM, TileBands tb,
                                                          int quad_base, EpiArgs epi, BatchMeta meta) {
  constexpr int NQ0 = HQ >= 3 ? 2 : 1, NQ1 = HQ - NQ0;
  // 2 x WM waves; a wave owns 128 rows x (256 / WM) tokens = 4 x CT blocks of 32 x 32
  constexpr int W_TILES = 16, X_TILES = 16, CT = 8 / WM, NWAVES = 2 * WM;
  constexpr int STAGE_TILES = W_TILES + X_TILES;
  constexpr int LOADS = STAGE_TILES / NWAVES;
  constexpr int STAGE_BYTES = STAGE_TILES * 1024;
  constexpr int H = 4 * CT;                                  // MFMAs per k step (half a stage)
  typedef __attribute__((address_space(3))) void *lds_ptr;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wn = (NQ0 == NQ1 ? wave : wave ^ (wave >> 2)) & 1, wm = wave >> 1;
  const int q_first = wn * NQ0;                               // first quad of this wave inside the tile

  int wg_n, wg_m;
  if (!tile_of_block(tb, NW, NM, blockIdx.x, wg_n, wg_m)) return;
  const int rt0 = (quad_base + wg_n * HQ) * 4;                // first weight row tile of the workgroup's tile

  // tile t of a stage: t < 16 weight row tile t, else token tile t-16; wave w copies tiles
  // w*LOADS...  Copies are buffer loads with the LDS modifier: scalar base (resource) + scalar
  // offset + 16*lane, so a copy costs one instruction and no vector address arithmetic, and
  // its address travels as a 32-bit offset (flat addressing sends 64 bits per lane and was
  // measurably slower).  Waves 0..NWAVES/2-1 copy weight tiles, the others token tiles.
  const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
      (void *)(wp + (size_t)rt0 * 512), 0, (unsigned)(((size_t)w_RT * KT - (size_t)rt0) * 1024), 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
      (void *)(xp + (size_t)wg_m * X_TILES * 512), 0, (unsigned)(((size_t)x_RT * KT - (size_t)wg_m * X_TILES) * 1024), 0x00020000);
  const bool is_w = wave < NWAVES / 2;
  const bool copies = !is_w || wave < HQ;                     // weight wave q copies quad q of the tile: only the tile's own
  const __amdgpu_buffer_rsrc_t rs = is_w ? rs_w : rs_x;
  const unsigned sstep = (is_w ? w_RT : x_RT) * 1024;
  // a wave's LOADS tiles are adjacent both in memory and in LDS, so they share one scalar
  // offset and one LDS base (M0); the instruction's immediate offset, which applies to both
  // sides, selects the tile within a group of four
  constexpr int NG = LOADS / 4;
  unsigned soff[NG];
  const unsigned loff = lane * 16;
#pragma unroll
  for (int g = 0; g < NG; ++g) soff[g] = ((wave % (NWAVES / 2)) * LOADS + 4 * g) * 1024;
  const int NS = KT;
  char *const wdst = smem + wave * LOADS * 1024;
  // copy tile i of `stage` into LDS buffer `buf`; past the last stage the source stays put
  auto dma = [&](int buf, int stage, auto i_) {
    constexpr int i = decltype(i_)::value, g = i / 4;
#if defined(__HIP_DEVICE_COMPILE__)   // the builtin exists in the device pass only
    if (HQ == 4 || copies)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr)(wdst + buf * STAGE_BYTES + g * 4096), 16, loff, soff[g], (i % 4) * 1024, 0);
#endif
    if constexpr (i % 4 == 3) soff[g] += stage + 1 < NS ? sstep : 0;
  };

  f32x16 acc[4][CT];
#pragma unroll
  for (int bi = 0; bi < 4; ++bi)
#pragma unroll
    for (int ci = 0; ci < CT; ++ci)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[bi][ci][e] = 0.0f;

  const int gq = lane >> 5, r32 = lane & 31;
  int a_off[4], b_off[CT];
#pragma unroll
  for (int bi = 0; bi < 4; ++bi) {
    const int quad = q_first + (bi >> 1), e = bi & 1;
    const int tile = quad * 4 + e + ((r32 >> 4) << 1);
    a_off[bi] = tile * 1024 + (gq * 16 + (r32 & 15)) * 16;
  }
#pragma unroll
  for (int ci = 0; ci < CT; ++ci) {
    const int tile = (wm * CT + ci) * 2 + (r32 >> 4);
    b_off[ci] = (W_TILES + tile) * 1024 + (gq * 16 + (r32 & 15)) * 16;
  }
  bf16x8 A0[4], B0[CT], A1[4], B1[CT];
#define PIN __builtin_amdgcn_sched_barrier(0)

  // the loop and the epilogue for a wave that holds NQ quads (2 * NQ blocks of 32 rows)
  auto body = [&](auto nq_) {
  constexpr int NQ = decltype(nq_)::value, NBI = 2 * NQ;

  // prologue: stages 0..NB-2 on their way, stage 0 landed
#pragma unroll
  for (int st = 0; st < NB - 1; ++st)
    static_for<LOADS>([&](auto i_) { dma(st, st, i_); });
  WAITCNT_VM_LGKM0((NB - 2) * LOADS);
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int bi = 0; bi < NBI; ++bi) A0[bi] = *(const bf16x8 *)(smem + a_off[bi]);
#pragma unroll
  for (int ci = 0; ci < CT; ++ci) B0[ci] = *(const bf16x8 *)(smem + b_off[ci]);

  // Stage s lives in buffer s % NB (a ring).  Per stage, after MFMA
  //   0 ..        : one operand read of set 1 of this stage and one copy of stage s+NB-1 (into
  //                 the buffer of stage s-1, which nobody reads any more since the last barrier)
  //   H-1         : wait until this wave's copies of stage s+1 have landed (the younger ones
  //                 may still fly) and all its LDS reads are back; barrier
  //   H ..        : read operand set 0 of stage s+1
  int bcur = 0;
  for (int s0 = 0; s0 < NS; s0 += 4) {
    static_for<4>([&](auto j_) {
      constexpr int j = decltype(j_)::value;
      const int s = s0 + j;
      const int bnxt = bcur == NB - 1 ? 0 : bcur + 1, bfill = bcur == 0 ? NB - 1 : bcur - 1;
      const char *const pc = smem + bcur * STAGE_BYTES + 512, *const pn = smem + bnxt * STAGE_BYTES;
      static_for<2 * H>([&](auto m_) {
        constexpr int m = decltype(m_)::value;
        constexpr int half = m / H, bi = (m % H) / CT, ci = m % CT;
        PIN;
        if constexpr (bi < NBI) {
          if constexpr (half == 0)
            acc[bi][ci] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A0[bi], B0[ci], acc[bi][ci], 0, 0, 0);
          else
            acc[bi][ci] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1[bi], B1[ci], acc[bi][ci], 0, 0, 0);
        }
        PIN;
        if constexpr (m < 4 + CT) {
          if constexpr (m < 4) { if constexpr (m < NBI) A1[m] = *(const bf16x8 *)(pc + a_off[m]); }
          else if constexpr (NBI > 0) B1[m - 4] = *(const bf16x8 *)(pc + b_off[m - 4]);
        }
        if constexpr (m < LOADS) dma(bfill, s + NB - 1, m_);
        if constexpr (m == H - 1) { PIN; WAITCNT_VM_LGKM0((NB - 2) * LOADS); __builtin_amdgcn_s_barrier(); }
        if constexpr (m >= H && m < H + 4 + CT) {
          if constexpr (m < H + 4) { if constexpr (m - H < NBI) A0[m - H] = *(const bf16x8 *)(pn + a_off[m - H]); }
          else if constexpr (NBI > 0) B0[m - H - 4] = *(const bf16x8 *)(pn + b_off[m - H - 4]);
        }
      });
      PIN;
      bcur = bnxt;
    });
  }
#undef PIN
  WAITCNT_VM_LGKM0(0);     // no copy may still be in flight when the workgroup's LDS is released

  if constexpr (NQ > 0)
    static_for<CT>([&](auto ci_) {
      constexpr int ci = decltype(ci_)::value;
      tile_epilogue<EPI, CT, ci, NQ>(epi, meta, acc, (wg_m * X_TILES + (wm * CT + ci) * 2) * 16 + r32,
                                     quad_base + wg_n * HQ + q_first, w_RT / 4, gq);
    });
  };
  if constexpr (NQ0 == NQ1) body(std::integral_constant<int, NQ0>{});
  else if (wn == 0) body(std::integral_constant<int, NQ0>{});
  else body(std::integral_constant<int, NQ1>{});
}

// The tiled kernels need more dynamic LDS than the default limit: raised once per kernel instantiation
// and device (thread-safe; a bit per device).  On failure nothing is launched and the HIP error stays
// pending for the caller's check after the enqueue.
template <auto KERNEL>
static bool ensure_dynamic_lds(int bytes) {
  static std::atomic<unsigned long long> done{0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
  if ((done.load(std::memory_order_acquire) >> dev) & 1ull) return true;
  if (hipFuncSetAttribute(reinterpret_cast<const void *>(KERNEL), hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
    return false;
  done.fetch_or(1ull << dev, std::memory_order_release);
  return true;
}

// one part of the weight rows: n_quads quads from quad_base on, as tiles of HQ quads
template <int WM, int EPI, int HQ>
static void launch_gemmd_part(const bf16_t *wp, int w_RT, const bf16_t *xp, int x_RT, int KT, int M, int quad_base, int n_quads,
                              const EpiArgs &epi, const BatchMeta &meta, hipStream_t s) {
  constexpr int NB = 4, smem = 32 * 1024 * NB;
  const int NW = ceil_div(n_quads, HQ), NM = ceil_div(M, 256);
  const TileBands tb = make_bands(NW, NM, KT, 256);
  const int grid = tb.b0[tb.n_rem];
  if (!ensure_dynamic_lds<&gemmd_kernel<WM, EPI, NB, HQ>>(smem)) return;
  hipLaunchKernelGGL((gemmd_kernel<WM, EPI, NB, HQ>), dim3(grid), dim3(128 * WM), smem, s, wp, w_RT, xp, x_RT, KT, NW, NM, tb,
                     quad_base, epi, meta);
}

template <int WM, int EPI>
static void launch_gemmd_e(const bf16_t *wp, int w_RT, const bf16_t *xp, int x_RT, int KT, int M,
                           const EpiArgs &epi, const BatchMeta &meta, hipStream_t s) {
  const RowParts rp = plan_row_parts(w_RT / 4, ceil_div(M, 256));
  for (int i = 0; i < rp.n; ++i) {
    switch (rp.hq[i]) {
      case 4: launch_gemmd_part<WM, EPI, 4>(wp, w_RT, xp, x_RT, KT, M, rp.quad_base[i], rp.n_quads[i], epi, meta, s); break;
      case 3: launch_gemmd_part<WM, EPI, 3>(wp, w_RT, xp, x_RT, KT, M, rp.quad_base[i], rp.n_quads[i], epi, meta, s); break;
      case 2: launch_gemmd_part<WM, EPI, 2>(wp, w_RT, xp, x_RT, KT, M, rp.quad_base[i], rp.n_quads[i], epi, meta, s); break;
      default: launch_gemmd_part<WM, EPI, 1>(wp, w_RT, xp, x_RT, KT, M, rp.quad_base[i], rp.n_quads[i], epi, meta, s); break;
    }
  }
}

template <int WM>
static void launch_gemmd(const bf16_t *wp, int w_RT, const bf16_t *xp, int x_RT, int KT, int M,
                         const EpiArgs &epi, const BatchMeta &meta, hipStream_t s) {
  switch (epi.kind) {
    case EPI_PLAIN: launch_gemmd_e<WM, EPI_PLAIN>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s); break;
    case EPI_QKV: launch_gemmd_e<WM, EPI_QKV>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s); break;
    case EPI_RESID: launch_gemmd_e<WM, EPI_RESID>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s); break;
    case EPI_SWIGLU: launch_gemmd_e<WM, EPI_SWIGLU>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s); break;
    case EPI_ACTBWD: launch_gemmd_e<WM, EPI_ACTBWD>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s); break;
    default: launch_gemmd_e<WM, EPI_GELU>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s); break;
  }
}

template <int WTOK, int EPI>
static void launch_gemm_we(const bf16_t *wp, int w_RT, const bf16_t *xp, int x_RT, int KT, int M,
                           const EpiArgs &epi, const BatchMeta &meta, hipStream_t s) {
  constexpr int TOKT = 64 * WTOK;
  constexpr int smem = (16 + 4 * WTOK) * 1024 * 2;            // two stage buffers
  const int NW = w_RT / 16, NM = ceil_div(M, TOKT);
  const TileBands tb = make_bands(NW, NM, KT, TOKT);
  const int grid = tb.b0[tb.n_rem];
  if (!ensure_dynamic_lds<&gemm_kernel<WTOK, EPI>>(smem)) return;
  hipLaunchKernelGGL((gemm_kernel<WTOK, EPI>), dim3(grid), dim3(256), smem, s, wp, w_RT, xp, x_RT, KT, NW, NM, tb, epi, meta);
}

template <int WTOK>
static void launch_gemm_w(const bf16_t *wp, int w_RT, const bf16_t *xp, int x_RT, int KT, int M,
                          const EpiArgs &epi, const BatchMeta &meta, hipStream_t s) {
  switch (epi.kind) {
    case EPI_PLAIN: launch_gemm_we<WTOK, EPI_PLAIN>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s); break;
    case EPI_QKV: launch_gemm_we<WTOK, EPI_QKV>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s); break;
    case EPI_RESID: launch_gemm_we<WTOK, EPI_RESID>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s); break;
    case EPI_SWIGLU: launch_gemm_we<WTOK, EPI_SWIGLU>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s); break;
    case EPI_ACTBWD: launch_gemm_we<WTOK, EPI_ACTBWD>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s); break;
    default: launch_gemm_we<WTOK, EPI_GELU>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s); break;
  }
}

int gemm_token_tile(int M) { return M > 512 ? 256 : (M > 256 ? 128 : 64); }

void launch_gemm(const bf16_t *wp, int w_RT, const bf16_t *xp, int x_RT, int KT, int M, const EpiArgs &epi,
                 const BatchMeta &meta, hipStream_t s) {
  // The activation buffers are padded for gemm_token_tile(M); a smaller tile may still be the better
  // choice when the larger one leaves compute units without a tile (7B shape, 2048 tokens: the 16 x 8
  // tiles of the attention output projection fill half the chip).  Cost = rounds of 256 workgroups x
  // tokens per tile / relative speed of the kernel (measured on full rounds: 1, 0.72, 0.5).
  int tt = gemm_token_tile(M);
  {
    const int NW = w_RT / 16;
    double best = 1e30;
    int pick = tt;
    const int cand[3] = {256, 128, 64};
    const double speed[3] = {1.0, 0.72, 0.5};
    for (int i = 0; i < 3; ++i) {
      if (cand[i] > tt) continue;
      const long tiles = (long)NW * ((M + cand[i] - 1) / cand[i]);
      double cost = (double)((tiles + GEMV_MAX_GRID - 1) / GEMV_MAX_GRID) * cand[i] / speed[i];
      if (cand[i] == 256) cost = plan_row_parts(w_RT / 4, ceil_div(M, 256)).cost / 4.0 * 256;   // 256-token tiles may be cut into two parts
      if (cost < best - 1e-9) { best = cost; pick = cand[i]; }
    }
    tt = pick;
  }
  if (tt == 256) launch_gemmd<4>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s);
  else if (tt == 128) launch_gemm_w<2>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s);
  else launch_gemm_w<1>(wp, w_RT, xp, x_RT, KT, M, epi, meta, s);
}

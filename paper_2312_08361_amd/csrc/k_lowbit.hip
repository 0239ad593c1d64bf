// Block-wise low-bit weights (Section 3.1, "Compression": 8-bit weights, 4-bit NormalFloat):
// the encoder that packs canonical bf16 weights into codes + one fp32 scale per 64 input
// features of a row, and the weight-streaming decode kernel that consumes them.
//
// Format (an absmax block format; rows = output features, blocks run along the input features):
//   int8      code = round_to_nearest_even(w / absmax * 127), w' = code * (absmax / 127)
//   codebook  code = number of midpoints of 16 ascending levels that lie strictly below
//             w / absmax (= index of the nearest level, ties to the lower one), w' = level * absmax
// all in fp32, in exactly this order of operations (the integer codes are compared bit for bit
// with an independent CPU implementation).
//
// Packed layout.  A unit is 16 rows x 64 k (one scale block per row), units are k-major like
// T16 tiles (the row tiles of one k block are adjacent):
//   int8      1 KiB per unit; lane (r = lane % 16, g = lane / 16) owns 16 bytes:
//             bytes 0..7  = k 8g..8g+7 of the block's first 32 k,  bytes 8..15 = the same of its
//             second 32 k; each half converts to one v_mfma_f32_16x16x32_bf16 operand
//   codebook  512 B per unit, stored as pairs of row tiles (the decode kernel always works on
//             pairs): lane owns 16 bytes = [8 bytes of tile 2p | 8 bytes of tile 2p+1]; a dword
//             holds the 8 codes of one 32-k step, k index i in nibble i, so that a byte is the two
//             codes of one bf16 pair of the MFMA operand (the decode kernel looks bytes up)
//   scales    fp32 [k block][row]: int8 stores absmax / 127, codebook stores absmax
// The decode kernel multiplies *unscaled* codes on the matrix core (exact in bf16) into a
// fresh accumulator per 64-k block and applies the four row scales a lane needs with one
// fp32 multiply-add per accumulator register.
#include "common.h"
#include "epilogue.h"
#include "launch.h"
#include <string.h>

namespace {

__device__ __forceinline__ int phys_tile_row(const PackArgs &a, int pt, int r, const bf16_t **src, int *rows) {
  int row = -1;
  *src = nullptr; *rows = 0;
  if (a.order == PACK_NATURAL) {
    *src = a.src[0]; *rows = a.rows[0]; row = pt * 16 + r;
  } else if (a.order == PACK_GATEUP) {
    const int which = pt & 1;
    *src = a.src[which]; *rows = a.rows[which]; row = (pt >> 1) * 16 + r;
  } else {
    const int HT = a.head_dim >> 4;
    const int head = pt / HT, j = pt % HT;
    const int lt = (j >> 1) + (j & 1) * (HT >> 1);
    const int lrow = (head * HT + lt) * 16 + r;
    if (lrow < a.rows[0]) { *src = a.src[0]; *rows = a.rows[0]; row = lrow; }
    else if (lrow < a.rows[0] + a.rows[1]) { *src = a.src[1]; *rows = a.rows[1]; row = lrow - a.rows[0]; }
    else { *src = a.src[2]; *rows = a.rows[2]; row = lrow - a.rows[0] - a.rows[1]; }
  }
  return row;
}

// One wave per (k block, physical row tile).  Lane (r, g) holds the 16 values it will own in
// the packed unit; the row's absmax is the maximum over its four lanes.
__global__ __launch_bounds__(64) void pack_weight_q_kernel(PackArgs a, QuantArgs q) {
  const int ku = blockIdx.x, pt = blockIdx.y, lane = threadIdx.x;
  const int g = lane >> 4, r = lane & 15;
  const bf16_t *src;
  int rows;
  const int row = phys_tile_row(a, pt, r, &src, &rows);
  float v[16];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int k = ku * 64 + h * 32 + g * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool ok = src && row >= 0 && row < rows && k + i < a.K;
      v[h * 8 + i] = ok ? bf16_to_f32(src[(size_t)row * a.K + k + i]) : 0.0f;
    }
  }
  float am = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; ++i) am = fmaxf(am, fabsf(v[i]));
  am = fmaxf(am, __shfl_xor(am, 16));
  am = fmaxf(am, __shfl_xor(am, 32));
  const float safe = am > 0.0f ? am : 1.0f;
  uint32_t code[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const float t = v[i] / safe;                       // fp32 division, correctly rounded
    if (q.bits == 8) {
      code[i] = (uint32_t)(__float2int_rn(t * 127.0f) & 0xFF);
    } else {
      uint32_t c = 0;
#pragma unroll
      for (int j = 0; j < 15; ++j) c += t > q.mids[j] ? 1u : 0u;
      code[i] = c;
    }
  }
  if (q.bits == 8) {
    u32x4 w;
    w.x = code[0] | code[1] << 8 | code[2] << 16 | code[3] << 24;
    w.y = code[4] | code[5] << 8 | code[6] << 16 | code[7] << 24;
    w.z = code[8] | code[9] << 8 | code[10] << 16 | code[11] << 24;
    w.w = code[12] | code[13] << 8 | code[14] << 16 | code[15] << 24;
    *(u32x4 *)(q.codes + ((size_t)ku * a.RT + pt) * 1024 + lane * 16) = w;
  } else {
    u32x2 w;
    w.x = w.y = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) { w.x |= code[i] << (4 * i); w.y |= code[8 + i] << (4 * i); }
    *(u32x2 *)(q.codes + ((size_t)ku * (a.RT / 2) + (pt >> 1)) * 1024 + lane * 16 + (pt & 1) * 8) = w;
  }
  if (g == 0) {
    q.scales[((size_t)ku * a.RT + pt) * 16 + r] = q.bits == 8 ? am / 127.0f : am;
    if (q.absmax_out) q.absmax_out[((size_t)ku * a.RT + pt) * 16 + r] = am;
  }
}

// packed -> row-major codes (one byte per code) and absmax, for the bit-exact encoder test
__global__ void unpack_codes_kernel(QuantArgs q, int RT, int N, int K, uint8_t *codes_out, float *absmax_out,
                                    const float *absmax_packed) {
  const int KU = ceil_div(K, 64);
  const size_t total = (size_t)N * K;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int n = idx / K, k = idx % K;
    const int ku = k >> 6, h = (k >> 5) & 1, g = (k >> 3) & 3, i = k & 7, pt = n >> 4, r = n & 15;
    const int lane = g * 16 + r, j = h * 8 + i;
    uint8_t c;
    if (q.bits == 8) c = q.codes[((size_t)ku * RT + pt) * 1024 + lane * 16 + j];
    else {
      const int nib = i + 8 * h;                                     // nibble inside the lane's 8 bytes of this tile
      const uint8_t b = q.codes[((size_t)ku * (RT / 2) + (pt >> 1)) * 1024 + lane * 16 + (pt & 1) * 8 + (nib >> 1)];
      c = (nib & 1) ? (b >> 4) : (b & 15);
    }
    codes_out[idx] = c;
    if (k % 64 == 0) absmax_out[(size_t)n * KU + ku] = absmax_packed[((size_t)ku * RT + pt) * 16 + r];
  }
}

// eight int8 codes (two dwords) -> one MFMA operand; small integers are exact in bf16
__device__ __forceinline__ bf16x8 cvt_i8x8(uint32_t lo, uint32_t hi) {
  u32x4 o;
  auto two = [](uint32_t x, int sh) -> uint32_t {
    const float f0 = (float)(int)(int8_t)(x >> sh), f1 = (float)(int)(int8_t)(x >> (sh + 8));
    return (__float_as_uint(f0) >> 16) | (__float_as_uint(f1) & 0xFFFF0000u);
  };
  o.x = two(lo, 0); o.y = two(lo, 16); o.z = two(hi, 0); o.w = two(hi, 16);
  return __builtin_bit_cast(bf16x8, o);
}

// eight 4-bit codes (one dword, k index i in nibble i) -> one MFMA operand, without memory access (the expansion
// kernel's way; the decode kernel looks bytes up in an LDS table, which is twice as fast).  The 16 bf16 levels are
// split into a table of low bytes and a table of high bytes (four dwords each, in scalar registers); v_perm_b32
// looks four codes up at a time: two 8-entry lookups by the low three code bits, a third permute picks between
// them by the fourth bit, then low and high bytes are interleaved into bf16 values and even and odd k into pairs.
__device__ __forceinline__ bf16x8 cvt_c4x8(uint32_t x, const uint32_t (&lo)[4], const uint32_t (&hi)[4]) {
  const uint32_t x4 = x >> 4;
  const uint32_t se = x & 0x07070707u, so = x4 & 0x07070707u;                  // low three bits of the even / odd nibbles
  const uint32_t me = ((x >> 1) & 0x04040404u) | 0x03020100u;                 // byte i of the first (0) or second (4) lookup
  const uint32_t mo = ((x4 >> 1) & 0x04040404u) | 0x03020100u;
  auto look = [&](const uint32_t (&t)[4], uint32_t s, uint32_t m) {
    const uint32_t a = __builtin_amdgcn_perm(t[1], t[0], s), b = __builtin_amdgcn_perm(t[3], t[2], s);
    return __builtin_amdgcn_perm(b, a, m);
  };
  const uint32_t le = look(lo, se, me), he = look(hi, se, me), lod = look(lo, so, mo), hod = look(hi, so, mo);
  const uint32_t e01 = __builtin_amdgcn_perm(he, le, 0x05010400u), e23 = __builtin_amdgcn_perm(he, le, 0x07030602u);     // k 0, 2 | k 4, 6
  const uint32_t o01 = __builtin_amdgcn_perm(hod, lod, 0x05010400u), o23 = __builtin_amdgcn_perm(hod, lod, 0x07030602u); // k 1, 3 | k 5, 7
  u32x4 o;
  o.x = __builtin_amdgcn_perm(o01, e01, 0x05040100u);    // k 0, 1
  o.y = __builtin_amdgcn_perm(o01, e01, 0x07060302u);    // k 2, 3
  o.z = __builtin_amdgcn_perm(o23, e23, 0x05040100u);    // k 4, 5
  o.w = __builtin_amdgcn_perm(o23, e23, 0x07060302u);    // k 6, 7
  return __builtin_bit_cast(bf16x8, o);
}

// Packed codes -> bf16 T16 tiles (code value times block scale, rounded to bf16) for the tiled
// MFMA kernels of long calls: a compressed matrix is expanded into a scratch buffer right before
// the projection that uses it.  A packed unit (16 rows x 64 k) becomes the T16 tiles of the same
// row tile at k tiles 2*ku and 2*ku+1, and a lane's 16 codes are exactly its two 16-byte chunks
// there.  One wave per (k block, row tile).
template <int BITS>
__global__ __launch_bounds__(64) void expand_q_kernel(QWeights w, bf16_t *dst) {
  const int ku = blockIdx.x, pt = blockIdx.y, lane = threadIdx.x;
  const float sc = w.scales[((size_t)ku * w.RT + pt) * 16 + (lane & 15)];
  bf16x8 lo, hi;
  if (BITS == 8) {
    const u32x4 q = *((const u32x4 *)w.codes + ((size_t)ku * w.RT + pt) * 64 + lane);
    lo = cvt_i8x8(q.x, q.y); hi = cvt_i8x8(q.z, q.w);
  } else {
    const u32x2 q = *(const u32x2 *)(w.codes + ((size_t)ku * (w.RT / 2) + (pt >> 1)) * 1024 + lane * 16 + (pt & 1) * 8);
    lo = cvt_c4x8(q.x, w.lut_lo, w.lut_hi); hi = cvt_c4x8(q.y, w.lut_lo, w.lut_hi);
  }
  u32x4 o0, o1;
  o0.x = pack_bf16x2((float)lo[0] * sc, (float)lo[1] * sc); o0.y = pack_bf16x2((float)lo[2] * sc, (float)lo[3] * sc);
  o0.z = pack_bf16x2((float)lo[4] * sc, (float)lo[5] * sc); o0.w = pack_bf16x2((float)lo[6] * sc, (float)lo[7] * sc);
  o1.x = pack_bf16x2((float)hi[0] * sc, (float)hi[1] * sc); o1.y = pack_bf16x2((float)hi[2] * sc, (float)hi[3] * sc);
  o1.z = pack_bf16x2((float)hi[4] * sc, (float)hi[5] * sc); o1.w = pack_bf16x2((float)hi[6] * sc, (float)hi[7] * sc);
  *(u32x4 *)(dst + ((size_t)(2 * ku) * w.RT + pt) * 512 + lane * 8) = o0;
  *(u32x4 *)(dst + ((size_t)(2 * ku + 1) * w.RT + pt) * 512 + lane * 8) = o1;
}

// ------------------------------------------------------------------------------------
// Weight-streaming decode kernel for packed low-bit weights.  Same work split, cross-wave
// reduction, sharing through memory and fused epilogues as the bf16 kernel; a k unit here is one
// 64-k block, and a workgroup owns PP adjacent tile pairs at a time (its "group"): with codes
// of 1 or 1/2 byte the activation tiles are as many bytes as the weights they meet, so every
// activation load is used for 32 * PP weight rows.
//
// The tokens are the MFMA row operand and the weight rows the column operand, so a lane's
// accumulator registers belong to ONE weight row (lane % 16) and four tokens: the block scale
// is a single float per lane.  The result is transposed inside the wave through LDS before the
// epilogue, which wants one token and four rows per lane.
// ------------------------------------------------------------------------------------
template <int MT, int EPI, int BITS, int PP>
__global__ __launch_bounds__(512) void gemvq_kernel(QWeights w, const bf16_t *__restrict__ xp, int x_RT, int KU,
                                                    int n_groups, GemvShare sh, EpiArgs epi, BatchMeta meta) {
  constexpr int WAVES = 8, U = 2, NE = MT * PP;      // NE waves run epilogues: wave = j * MT + mt
  static_assert(NE <= 4, "at most four (pair, token tile) results per workgroup");
  __shared__ f32x4 red[WAVES][PP][2][MT][64];
  __shared__ float stat[WAVES][2][64];
  __shared__ int finisher;
  __shared__ __attribute__((aligned(16))) float tr[NE][2][16][20];   // per-wave transpose buffers (rows padded to 20 floats)
  // codebook format: the bf16 pair of every byte (two codes): one LDS read per pair of codes instead of 23 vector
  // operations per eight (a stand-alone loop converts 9.3 TB/s of codes this way against 4.9 by byte permutes)
  __shared__ uint32_t c4tab[BITS == 4 ? 256 : 1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if constexpr (BITS == 4) {
    if (threadIdx.x < 256) {
      auto level = [&](int c) -> uint32_t {
        const int j = c >> 2, sh = 8 * (c & 3);
        const uint32_t l = j == 0 ? w.lut_lo[0] : (j == 1 ? w.lut_lo[1] : (j == 2 ? w.lut_lo[2] : w.lut_lo[3]));
        const uint32_t h = j == 0 ? w.lut_hi[0] : (j == 1 ? w.lut_hi[1] : (j == 2 ? w.lut_hi[2] : w.lut_hi[3]));
        return ((l >> sh) & 0xFFu) | (((h >> sh) & 0xFFu) << 8);
      };
      c4tab[threadIdx.x] = level(threadIdx.x & 15) | (level(threadIdx.x >> 4) << 16);
    }
    __syncthreads();
  }
  auto cvt_tab = [&](uint32_t x) -> bf16x8 {
    u32x4 o;
    o.x = c4tab[x & 255u]; o.y = c4tab[(x >> 8) & 255u]; o.z = c4tab[(x >> 16) & 255u]; o.w = c4tab[x >> 24];
    return __builtin_bit_cast(bf16x8, o);
  };

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
  const int e_mt = wave % MT, e_j = wave / MT;        // epilogue role of this wave (if wave < NE)
  const int el = e_mt * 16 + (lane & 15), em = epi.m0 + el, er4 = (lane >> 4) * 4;
  const bool e_on = wave < NE && em < epi.M;
  TokInfo ti = token_info(meta, e_on ? em : 0);

  const bf16x8 *xb = (const bf16x8 *)xp + lane;
  // token rows past the end of the call are padding: their lanes take zeros instead of loading
  bool x_on[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) x_on[mt] = epi.m0 + mt * 16 + (lane & 15) < epi.M;
  const size_t xst = (size_t)x_RT * 64;
  const long total = (long)n_groups * KU;
  const long f0 = (long)blockIdx.x * sh.L;
  const long f1 = f0 + sh.L < total ? f0 + sh.L : total;
  bool first = true;

  for (long f = f0; f < f1;) {
    const int gp = (int)(f / KU), ka = (int)(f - (long)gp * KU);
    const int kb = (f1 - f) < (long)(KU - ka) ? ka + (int)(f1 - f) : KU;
    const int p_mine = gp * PP + e_j;                  // the pair this wave's epilogue handles
    EpiPre pre{};
    if (e_on) pre = epilogue_prefetch<EPI>(epi, ti, em, p_mine, er4);

    // the waves take the k units of the range in turn, U at a time (see gemv_kernel)
    const int n_grp = (kb - ka) / U;
    // codes of the group in k unit ku: int8 two 1 KiB units per pair, codebook one 1 KiB unit per
    // pair; the pairs of a group are adjacent
    constexpr int QPP = BITS == 8 ? 2 : 1;             // 16-byte loads per pair and unit
    const u32x4 *wq = (const u32x4 *)w.codes + (size_t)(gp * PP) * QPP * 64 + lane;
    const size_t wst = BITS == 8 ? (size_t)w.RT * 64 : (size_t)(w.RT / 2) * 64;
    const float *sc = w.scales + (size_t)(2 * gp * PP) * 16 + (lane & 15);
    const size_t sst = (size_t)w.RT * 16;              // floats per k unit

    f32x4 acc0[PP][MT], acc1[PP][MT];
#pragma unroll
    for (int j = 0; j < PP; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) { acc0[j][mt] = f32x4{0, 0, 0, 0}; acc1[j][mt] = f32x4{0, 0, 0, 0}; }

    auto unit = [&](const u32x4 (&q)[PP * QPP], const float (&s)[PP * 2], const bf16x8 (&b0)[MT], const bf16x8 (&b1)[MT]) {
#pragma unroll
      for (int j = 0; j < PP; ++j) {
        bf16x8 A0l, A0h, A1l, A1h;
        if constexpr (BITS == 8) {
          A0l = cvt_i8x8(q[2 * j].x, q[2 * j].y); A0h = cvt_i8x8(q[2 * j].z, q[2 * j].w);
          A1l = cvt_i8x8(q[2 * j + 1].x, q[2 * j + 1].y); A1h = cvt_i8x8(q[2 * j + 1].z, q[2 * j + 1].w);
        } else {
          A0l = cvt_tab(q[j].x); A0h = cvt_tab(q[j].y);
          A1l = cvt_tab(q[j].z); A1h = cvt_tab(q[j].w);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          f32x4 t0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b0[mt], A0l, f32x4{0, 0, 0, 0}, 0, 0, 0);
          t0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b1[mt], A0h, t0, 0, 0, 0);
          f32x4 t1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b0[mt], A1l, f32x4{0, 0, 0, 0}, 0, 0, 0);
          t1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b1[mt], A1h, t1, 0, 0, 0);
          acc0[j][mt] += s[2 * j] * t0;
          acc1[j][mt] += s[2 * j + 1] * t1;
        }
      }
    };
    auto load_unit = [&](int ku, u32x4 (&q)[PP * QPP], float (&s)[PP * 2], bf16x8 (&b0)[MT], bf16x8 (&b1)[MT]) {
#pragma unroll
      for (int i = 0; i < PP * QPP; ++i) q[i] = __builtin_nontemporal_load(wq + ku * wst + i * 64);
#pragma unroll
      for (int i = 0; i < PP * 2; ++i) s[i] = sc[ku * sst + i * 16];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        b0[mt] = x_on[mt] ? xb[(size_t)(2 * ku) * xst + mt * 64] : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        b1[mt] = x_on[mt] ? xb[(size_t)(2 * ku + 1) * xst + mt * 64] : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      }
    };

    for (int jg = wave; jg < n_grp; jg += WAVES) {
      const int ku = ka + jg * U;
      u32x4 q[U][PP * QPP];
      float s[U][PP * 2];
      bf16x8 b0[U][MT], b1[U][MT];
#pragma unroll
      for (int u = 0; u < U; ++u) load_unit(ku + u, q[u], s[u], b0[u], b1[u]);
#pragma unroll
      for (int u = 0; u < U; ++u) unit(q[u], s[u], b0[u], b1[u]);
    }
    for (int ku = ka + n_grp * U + wave; ku < kb; ku += WAVES) {
      u32x4 q[PP * QPP];
      float s[PP * 2];
      bf16x8 b0[MT], b1[MT];
      load_unit(ku, q, s, b0, b1);
      unit(q, s, b0, b1);
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
    for (int j = 0; j < PP; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) { red[wave][j][0][mt][lane] = acc0[j][mt]; red[wave][j][1][mt][lane] = acc1[j][mt]; }
    __syncthreads();

    f32x4 v0 = f32x4{0, 0, 0, 0}, v1 = v0;
    if (wave < NE) {
      v0 = red[0][e_j][0][e_mt][lane]; v1 = red[0][e_j][1][e_mt][lane];
#pragma unroll
      for (int ww = 1; ww < WAVES; ++ww) { v0 += red[ww][e_j][0][e_mt][lane]; v1 += red[ww][e_j][1][e_mt][lane]; }
      if (first && e_on && epi.stat_in) {
        float ss = 0.0f, s1 = 0.0f;
#pragma unroll
        for (int ww = 0; ww < WAVES; ++ww)
#pragma unroll
          for (int q = 0; q < PPW; ++q) { ss += stat[ww][0][q * TOK + el]; s1 += stat[ww][1][q * TOK + el]; }
        const float inv_d = 1.0f / (float)epi.norm_d;
        ti.mu = epi.norm_center ? s1 * inv_d : 0.0f;
        ti.r = rsqrtf(fmaxf(ss * inv_d - ti.mu * ti.mu, 0.0f) + epi.norm_eps);   // one-pass variance: rounding may leave it a hair below zero
      }
    }
    first = false;

    bool finish = ka == 0 && kb == KU;
    if (!finish) {
      // group shared with neighbouring workgroups: pieces meet in memory (see the bf16 kernel)
      const int g_first = (int)(((long)gp * KU) / sh.L), g_last = (int)(((long)(gp + 1) * KU - 1) / sh.L);
      const int g = blockIdx.x;
      float *mine = (float *)(sh.part + ((size_t)g * 2 + (f == f0 ? 0 : 1)) * (2 * 4 * 64));
      if (wave < NE) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          __hip_atomic_store(mine + ((wave * 2) * 64 + lane) * 4 + i, v0[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(mine + ((wave * 2 + 1) * 64 + lane) * 4 + i, v1[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (threadIdx.x == 0) {
        const unsigned old = __hip_atomic_fetch_add(sh.count + gp, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = old == (unsigned)(g_last - g_first);
        if (last) __hip_atomic_store(sh.count + gp, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        finisher = last;
      }
      __syncthreads();
      finish = finisher != 0;
      if (finish && wave < NE) {
        v0 = f32x4{0, 0, 0, 0}; v1 = v0;
        for (int gi = g_first; gi <= g_last; ++gi) {
          const bool starts_here = (long)gi * sh.L >= (long)gp * KU;
          const float *pc = (const float *)(sh.part + ((size_t)gi * 2 + (starts_here ? 0 : 1)) * (2 * 4 * 64));
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            v0[i] += __hip_atomic_load(pc + ((wave * 2) * 64 + lane) * 4 + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            v1[i] += __hip_atomic_load(pc + ((wave * 2 + 1) * 64 + lane) * 4 + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
        }
      }
    }
    if (finish && wave < NE) {
      // [token 4*(lane/16)+i][row lane%16] -> [token lane%16][rows 4*(lane/16)+j] inside the wave
      float *t0 = &tr[wave][0][0][0], *t1 = &tr[wave][1][0][0];
      *(f32x4 *)(t0 + (lane & 15) * 20 + er4) = v0;
      *(f32x4 *)(t1 + (lane & 15) * 20 + er4) = v1;
#pragma unroll
      for (int j = 0; j < 4; ++j) { v0[j] = t0[(er4 + j) * 20 + (lane & 15)]; v1[j] = t1[(er4 + j) * 20 + (lane & 15)]; }
    }
    if (finish && e_on) epilogue_pair_k<EPI>(epi, ti, em, p_mine, er4, v0, v1, &pre);
    f += kb - ka;
    if (f < f1) __syncthreads();
  }
}

template <int MT, int EPI, int BITS, int PP>
void launch_gemvq_pp(const QWeights &w, const bf16_t *xp, int x_RT, int KU, int n_pairs, const GemvShare &share,
                     const EpiArgs &epi, const BatchMeta &meta, hipStream_t s) {
  GemvShare sh = share;
  const int n_groups = n_pairs / PP;
  int grid;
  // whole groups when they divide evenly over the CUs or are many (two workgroups run per CU; measured
  // against equal shares: 4-bit 70B 713 -> 747 steps/s, BLOOM 554 -> 569, int8 unchanged or slightly up)
  if (n_groups % GEMV_MAX_GRID == 0 || n_groups >= 2 * GEMV_MAX_GRID) { grid = n_groups; sh.L = KU; }
  else {
    const long total = (long)n_groups * KU;
    const int g = 2 * n_groups < GEMV_MAX_GRID ? 2 * n_groups : GEMV_MAX_GRID;
    sh.L = (int)((total + g - 1) / g);
    grid = (int)((total + sh.L - 1) / sh.L);
  }
  hipLaunchKernelGGL((gemvq_kernel<MT, EPI, BITS, PP>), dim3(grid), dim3(512), 0, s, w, xp, x_RT, KU, n_groups, sh, epi, meta);
}

template <int MT, int EPI>
void launch_gemvq_me(const QWeights &w, const bf16_t *xp, int x_RT, int KU, int n_pairs, const GemvShare &share,
                     const EpiArgs &epi, const BatchMeta &meta, hipStream_t s) {
  // Two pairs per workgroup pay off for the 4-bit format only (its activation tiles are twice the
  // bytes of its codes): measured on the 70B shapes, +2.5 % there, but -17 % for int8, whose
  // pair counts then stop being multiples of the CU count.  Needs MT * PP <= 4 and an even count.
  constexpr int PPMAX = MT <= 2 ? 2 : 1;
  if (w.bits == 8) launch_gemvq_pp<MT, EPI, 8, 1>(w, xp, x_RT, KU, n_pairs, share, epi, meta, s);
  else if (PPMAX == 2 && n_pairs % 2 == 0) launch_gemvq_pp<MT, EPI, 4, PPMAX>(w, xp, x_RT, KU, n_pairs, share, epi, meta, s);
  else launch_gemvq_pp<MT, EPI, 4, 1>(w, xp, x_RT, KU, n_pairs, share, epi, meta, s);
}

template <int MT>
void launch_gemvq_mt(const QWeights &w, const bf16_t *xp, int x_RT, int KU, int n_pairs, const GemvShare &sh,
                     const EpiArgs &epi, const BatchMeta &meta, hipStream_t s) {
  switch (epi.kind) {
    case EPI_PLAIN: launch_gemvq_me<MT, EPI_PLAIN>(w, xp, x_RT, KU, n_pairs, sh, epi, meta, s); break;
    case EPI_QKV: launch_gemvq_me<MT, EPI_QKV>(w, xp, x_RT, KU, n_pairs, sh, epi, meta, s); break;
    case EPI_RESID: launch_gemvq_me<MT, EPI_RESID>(w, xp, x_RT, KU, n_pairs, sh, epi, meta, s); break;
    case EPI_SWIGLU: launch_gemvq_me<MT, EPI_SWIGLU>(w, xp, x_RT, KU, n_pairs, sh, epi, meta, s); break;
    default: launch_gemvq_me<MT, EPI_GELU>(w, xp, x_RT, KU, n_pairs, sh, epi, meta, s); break;
  }
}

// ------------------------------------------------------------------------------------
// Hidden states between pipeline stages (Section 3.1, "Compression", last paragraph): 8-bit
// block-wise quantisation.  One wave per (block of a row): absmax by wavefront shuffles, then
// for every element the number of midpoints of the 256 levels that lie strictly below
// x / absmax (binary search over the midpoints in LDS) = index of the nearest level.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void hidden_encode_kernel(const void *x, int x_f32, int d, int block, Levels256 t,
                                                           uint8_t *codes, float *absmax) {
  __shared__ float mids[256];
  const int lane = threadIdx.x, b = blockIdx.x, m = blockIdx.y, nb = gridDim.x;
  for (int i = lane; i < 255; i += 64) mids[i] = (t.lv[i] + t.lv[i + 1]) * 0.5f;
  __syncthreads();
  const int k0 = b * block, per = block / 64;
  auto load = [&](int k) -> float {
    if (k >= d) return 0.0f;
    return x_f32 ? ((const float *)x)[(size_t)m * d + k] : bf16_to_f32(((const bf16_t *)x)[(size_t)m * d + k]);
  };
  float am = 0.0f;
  for (int i = 0; i < per; ++i) am = fmaxf(am, fabsf(load(k0 + i * 64 + lane)));
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) am = fmaxf(am, __shfl_xor(am, o));
  const float safe = am > 0.0f ? am : 1.0f;
  for (int i = 0; i < per; ++i) {
    const int k = k0 + i * 64 + lane;
    if (k >= d) continue;
    const float r = load(k) / safe;
    int c = 0;
#pragma unroll
    for (int step = 128; step > 0; step >>= 1)
      if (c + step <= 255 && mids[c + step - 1] < r) c += step;
    codes[(size_t)m * d + k] = (uint8_t)c;
  }
  if (lane == 0) absmax[(size_t)m * nb + b] = am;
}

__global__ void hidden_decode_kernel(const uint8_t *codes, const float *absmax, int M, int d, int block, Levels256 t,
                                     int y_f32, void *y) {
  __shared__ float lv[256];
  for (int i = threadIdx.x; i < 256; i += blockDim.x) lv[i] = t.lv[i];
  __syncthreads();
  const int nb = ceil_div(d, block);
  const size_t total = (size_t)M * d;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int m = idx / d, k = idx % d;
    const float v = lv[codes[idx]] * absmax[(size_t)m * nb + k / block];
    if (y_f32) ((float *)y)[idx] = v;
    else ((bf16_t *)y)[idx] = f32_to_bf16(v);
  }
}

}  // namespace

LevelTable make_level_table(const float *levels) {
  LevelTable lt{};
  for (int i = 0; i < 16; ++i) {
    uint32_t u;
    memcpy(&u, &levels[i], 4);
    u += 0x7FFFu + ((u >> 16) & 1u);                   // round to nearest even, as everywhere
    lt.bits[i] = (uint16_t)(u >> 16);
    u = (uint32_t)lt.bits[i] << 16;
    memcpy(&lt.rounded[i], &u, 4);
  }
  for (int i = 0; i < 15; ++i) lt.mids[i] = (lt.rounded[i] + lt.rounded[i + 1]) * 0.5f;
  for (int i = 0; i < 16; ++i) {
    lt.lut_lo[i / 4] |= (uint32_t)(lt.bits[i] & 0xFF) << (8 * (i % 4));
    lt.lut_hi[i / 4] |= (uint32_t)(lt.bits[i] >> 8) << (8 * (i % 4));
  }
  return lt;
}

void launch_pack_weight_q(const PackArgs &a, const QuantArgs &q, int n_phys_tiles, hipStream_t s) {
  hipLaunchKernelGGL(pack_weight_q_kernel, dim3(a.KT / 2, n_phys_tiles), dim3(64), 0, s, a, q);
}

void launch_unpack_codes(const QuantArgs &q, int RT, int N, int K, uint8_t *codes_out, float *absmax_out,
                         const float *absmax_packed, hipStream_t s) {
  const size_t total = (size_t)N * K;
  int grid = (int)((total + 255) / 256);
  if (grid > 4096) grid = 4096;
  hipLaunchKernelGGL(unpack_codes_kernel, dim3(grid), dim3(256), 0, s, q, RT, N, K, codes_out, absmax_out, absmax_packed);
}

void launch_hidden_encode(const void *x, int x_f32, int M, int d, int block, const Levels256 &t, uint8_t *codes,
                          float *absmax, hipStream_t s) {
  hipLaunchKernelGGL(hidden_encode_kernel, dim3(ceil_div(d, block), M), dim3(64), 0, s, x, x_f32, d, block, t, codes, absmax);
}

void launch_hidden_decode(const uint8_t *codes, const float *absmax, int M, int d, int block, const Levels256 &t,
                          int y_f32, void *y, hipStream_t s) {
  const size_t total = (size_t)M * d;
  int grid = (int)((total + 255) / 256);
  if (grid > 4096) grid = 4096;
  hipLaunchKernelGGL(hidden_decode_kernel, dim3(grid), dim3(256), 0, s, codes, absmax, M, d, block, t, y_f32, y);
}

void launch_expand_q(const QWeights &w, int KU, bf16_t *dst, hipStream_t s) {
  if (w.bits == 8) hipLaunchKernelGGL((expand_q_kernel<8>), dim3(KU, w.RT), dim3(64), 0, s, w, dst);
  else hipLaunchKernelGGL((expand_q_kernel<4>), dim3(KU, w.RT), dim3(64), 0, s, w, dst);
}

void launch_gemvq(const QWeights &w, const bf16_t *xp, int x_RT, int KU, int n_pairs, int m_tiles,
                  const GemvShare &sh, const EpiArgs &epi, const BatchMeta &meta, hipStream_t s) {
  switch (m_tiles) {
    case 1: launch_gemvq_mt<1>(w, xp, x_RT, KU, n_pairs, sh, epi, meta, s); break;
    case 2: launch_gemvq_mt<2>(w, xp, x_RT, KU, n_pairs, sh, epi, meta, s); break;
    case 3: launch_gemvq_mt<3>(w, xp, x_RT, KU, n_pairs, sh, epi, meta, s); break;
    default: launch_gemvq_mt<4>(w, xp, x_RT, KU, n_pairs, sh, epi, meta, s); break;
  }
}

// Fused epilogues shared by the weight-streaming (decode) and the LDS-tiled (prefill)
// projection kernels.  Both kernels use the packed weights as the MFMA row operand and
// the tokens as the column operand, so each lane ends up with, for one token m, four
// consecutive output rows of physical weight tile 2p (v0) and the same four rows of
// tile 2p+1 (v1).  The packing order of the weight tiles makes that pair exactly what
// each epilogue needs:
//   q/k/v projection : tiles (a, a + hd/32) of one head  -> the two halves of rotary pairs
//   gate/up          : gate rows and the same up rows    -> SwiGLU
//   others           : two consecutive row tiles
#pragma once
#include "common.h"

struct TokInfo {
  int pos;    // absolute position of the token in its session
  int slot;   // row of the session in the device page table
  float r;    // fused norm: 1/sqrt(var + eps) of the token's input row (1 when not fused)
  float mu;   // fused LayerNorm: mean of the row (0 otherwise)
};

__device__ __forceinline__ TokInfo token_info(const BatchMeta &meta, int m) {
  TokInfo t{0, 0, 1.0f, 0.0f};
  int s = 0;
  // sessions per call are few (<= 64): a linear scan is cheaper than it looks
  while (s + 1 < meta.n_sess && m >= meta.cu[s + 1]) ++s;
  t.pos = meta.past[s] + (m - meta.cu[s]);
  t.slot = meta.slot[s];
  return t;
}

// (the hardware reciprocal is good to one unit in the last place; the result is rounded to bf16)
__device__ __forceinline__ float silu_f(float z) { return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }
__device__ __forceinline__ float gelu_tanh_f(float z) {
  const float c = 0.7978845608028654f;   // sqrt(2/pi)
  float u = c * (z + 0.044715f * z * z * z);
  // tanh(u) = 1 - 2 / (exp(2u) + 1), safe for large |u|
  float t = 1.0f - 2.0f * __builtin_amdgcn_rcpf(__expf(2.0f * u) + 1.0f);
  return 0.5f * z * (1.0f + t);
}

// d gelu_tanh(z) / dz
__device__ __forceinline__ float gelu_tanh_grad(float z) {
  const float c = 0.7978845608028654f, k = 0.044715f;
  const float u = c * (z + k * z * z * z);
  const float t = 1.0f - 2.0f / (__expf(2.0f * u) + 1.0f);
  return 0.5f * (1.0f + t) + 0.5f * z * (1.0f - t * t) * c * (1.0f + 3.0f * k * z * z);
}

__device__ __forceinline__ void store_bf16x4(bf16_t *dst, f32x4 v) {
  u32x2 w;
  w.x = pack_bf16x2(v.x, v.y);
  w.y = pack_bf16x2(v.z, v.w);
  *(u32x2 *)dst = w;
}

// Epilogue operands that do not depend on the accumulators.  The skinny kernel fetches them
// before it starts streaming weights, so its tail is only arithmetic and stores; the tiled
// kernel passes no prefetch and the epilogue loads them in place.
struct EpiPre {
  f32x4 a, b;   // QKV: (cos, sin) x 4 of the rotary pairs;  RESID: residual (+ bias) of the two tiles
  f32x4 c, d;   // RESID: gains of the next norm for the two tiles
  int pg;       // QKV: page of the token's position
  float shift;  // RESID, fused LayerNorm: the row's shift (see EpiArgs)
};

template <int KIND>
__device__ __forceinline__ EpiPre epilogue_prefetch(const EpiArgs &a, const TokInfo &ti, int m, int p, int r4) {
  EpiPre pre{};
  if constexpr (KIND == EPI_QKV) {
    const int hd = a.head_dim, half = hd >> 1, pairs_per_head = hd >> 5;
    const int head = p / pairs_per_head;
    if (head < a.n_q_heads + 2 * a.n_kv_heads) {
      const int lo = (p % pairs_per_head) * 16 + r4;
      if (a.rotary && head < a.n_q_heads + a.n_kv_heads) {
        const float *cs = a.rope + ((size_t)ti.pos * half + lo) * 2;
        pre.a = *(const f32x4 *)cs; pre.b = *(const f32x4 *)(cs + 4);
      }
      if (head >= a.n_q_heads) pre.pg = a.page_table[(size_t)ti.slot * a.pages_per_session + (ti.pos >> 4)];
    }
  } else if constexpr (KIND == EPI_RESID) {
    const int n0 = (2 * p) * 16 + r4;
    if (a.h_out && a.shift) pre.shift = a.shift[m];
    if (n0 < a.N) {
      pre.a = *(const f32x4 *)(a.resid + (size_t)m * a.N + n0);
      if (a.bias) pre.a += *(const f32x4 *)(a.bias + n0);
      if (a.h_out) pre.c = *(const f32x4 *)(a.next_gain + n0);
    }
    if (n0 + 16 < a.N) {
      pre.b = *(const f32x4 *)(a.resid + (size_t)m * a.N + n0 + 16);
      if (a.bias) pre.b += *(const f32x4 *)(a.bias + n0 + 16);
      if (a.h_out) pre.d = *(const f32x4 *)(a.next_gain + n0 + 16);
    }
  }
  return pre;
}

// Finish a norm that the producer kernel left half done (see EpiArgs): features n..n+3.
__device__ __forceinline__ f32x4 finish_norm(const EpiArgs &a, const TokInfo &ti, f32x4 v, int n) {
  if (!a.stat_in) return v;
  if (a.norm_center) v -= ti.mu * *(const f32x4 *)(a.wg + n);
  return v * ti.r;
}

// One (token, tile pair, row quad) fragment.  `m` < a.M is checked by the caller.
// KIND is a compile-time EpiKind: the tiled kernel instantiates one kernel per kind so
// that its accumulator indexing stays static.
template <int KIND>
__device__ __forceinline__ void epilogue_pair_k(const EpiArgs &a, const TokInfo &ti, int m, int p,
                                                int r4, f32x4 v0, f32x4 v1, const EpiPre *pre = nullptr) {
  switch (KIND) {
    case EPI_PLAIN: {
      int n0 = (2 * p) * 16 + r4, n1 = n0 + 16;
      float *o0 = a.out + (size_t)m * a.N + n0, *o1 = o0 + 16;
      if (a.accumulate) {
        if (n0 < a.N) v0 += *(const f32x4 *)o0;
        if (n1 < a.N) v1 += *(const f32x4 *)o1;
      }
      if (n0 < a.N) *(f32x4 *)o0 = v0;
      if (n1 < a.N) *(f32x4 *)o1 = v1;
    } break;

    case EPI_RESID: {
      int n0 = (2 * p) * 16 + r4;
      float ss = 0.0f, s1 = 0.0f;
      const float sh = (a.h_out && a.shift) ? (pre ? pre->shift : a.shift[m]) : 0.0f;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        int n = n0 + 16 * t;
        if (n >= a.N) continue;
        f32x4 v = t ? v1 : v0;
        float *rp = a.resid + (size_t)m * a.N + n;
        if (pre) v += t ? pre->b : pre->a;
        else {
          if (a.bias) v += *(const f32x4 *)(a.bias + n);
          v += *(const f32x4 *)rp;
        }
        *(f32x4 *)rp = v;
        if (a.y) {
          if (a.y_f32) *(f32x4 *)((float *)a.y + (size_t)m * a.N + n) = v;
          else store_bf16x4((bf16_t *)a.y + (size_t)m * a.N + n, v);
        }
        if (a.h_out) {
          const f32x4 gn = pre ? (t ? pre->d : pre->c) : *(const f32x4 *)(a.next_gain + n);
          const f32x4 vc = v - sh;
          store_bf16x4(a.h_out + t16_off(m, n, a.h_RT), vc * gn);
          ss += vc.x * vc.x + vc.y * vc.y + vc.z * vc.z + vc.w * vc.w;
          s1 += vc.x + vc.y + vc.z + vc.w;
        }
      }
      if (a.h_out && a.stat_out) {
        // the four lanes that share this token (lane ^ 16, lane ^ 32) hold the other rows of the pair
        ss += __shfl_xor(ss, 16); ss += __shfl_xor(ss, 32);
        s1 += __shfl_xor(s1, 16); s1 += __shfl_xor(s1, 32);
        if (r4 == 0) { a.stat_out[(size_t)p * 128 + m] = ss; a.stat_out[(size_t)p * 128 + 64 + m] = s1; }
      }
    } break;

    case EPI_SWIGLU: {
      int f = p * 16 + r4;
      if (f >= a.N) break;
      v0 *= ti.r; v1 *= ti.r;          // fused RMSNorm (r == 1 when the input was normalised already)
      if (a.gu_plain) {
        *(f32x4 *)(a.gu_plain + (size_t)m * 2 * a.N + f) = v0;
        *(f32x4 *)(a.gu_plain + (size_t)m * 2 * a.N + a.N + f) = v1;
      }
      f32x4 o;
      o.x = silu_f(v0.x) * v1.x; o.y = silu_f(v0.y) * v1.y;
      o.z = silu_f(v0.z) * v1.z; o.w = silu_f(v0.w) * v1.w;
      store_bf16x4(a.act_out + t16_off(m, f, a.act_RT), o);
    } break;

    case EPI_GELU: {
      int f0 = (2 * p) * 16 + r4;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        int f = f0 + 16 * t;
        if (f >= a.N) continue;
        f32x4 v = finish_norm(a, ti, t ? v1 : v0, f);
        if (a.bias) v += *(const f32x4 *)(a.bias + f);
        if (a.gu_plain) *(f32x4 *)(a.gu_plain + (size_t)m * a.N + f) = v;
        f32x4 o;
        o.x = gelu_tanh_f(v.x); o.y = gelu_tanh_f(v.y); o.z = gelu_tanh_f(v.z); o.w = gelu_tanh_f(v.w);
        store_bf16x4(a.act_out + t16_off(m, f, a.act_RT), o);
      }
    } break;

    case EPI_ACTBWD: {
      // a = silu(g) * u:  dg = da * u * sig(g) * (1 + g * (1 - sig(g))),  du = da * silu(g);  a = gelu(z): dz = da * gelu'(z)
      const int F = a.N, f0 = (2 * p) * 16 + r4;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int f = f0 + 16 * t;
        if (f >= F) continue;
        const f32x4 d = t ? v1 : v0;
        if (a.gated) {
          const float *gp = a.gu_plain + (size_t)m * 2 * F + f;
          const f32x4 g = *(const f32x4 *)gp, u = *(const f32x4 *)(gp + F);
          f32x4 dg, du;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float sg = 1.0f / (1.0f + __expf(-g[i]));
            dg[i] = d[i] * u[i] * sg * (1.0f + g[i] * (1.0f - sg));
            du[i] = d[i] * g[i] * sg;
          }
          store_bf16x4(a.act_out + t16_off(m, f, a.act_RT), dg);
          store_bf16x4(a.act_out + t16_off(m, F + f, a.act_RT), du);
        } else {
          const f32x4 z = *(const f32x4 *)(a.gu_plain + (size_t)m * F + f);
          f32x4 dz;
#pragma unroll
          for (int i = 0; i < 4; ++i) dz[i] = d[i] * gelu_tanh_grad(z[i]);
          store_bf16x4(a.act_out + t16_off(m, f, a.act_RT), dz);
        }
      }
    } break;

    case EPI_QKV: {
      const int hd = a.head_dim, half = hd >> 1;
      const int pairs_per_head = hd >> 5;            // (hd/16 tiles) / 2
      const int head = p / pairs_per_head;            // index over [q heads | k heads | v heads]
      if (head >= a.n_q_heads + 2 * a.n_kv_heads) break;
      const int lo = (p % pairs_per_head) * 16 + r4;  // dims lo..lo+3 and lo+half..lo+half+3
      v0 = finish_norm(a, ti, v0, head * hd + lo);
      v1 = finish_norm(a, ti, v1, head * hd + lo + half);
      if (a.bias) {
        v0 += *(const f32x4 *)(a.bias + (size_t)head * hd + lo);
        v1 += *(const f32x4 *)(a.bias + (size_t)head * hd + lo + half);
      }
      const bool is_v = head >= a.n_q_heads + a.n_kv_heads;
      if (a.rotary && !is_v) {
        const float *cs = a.rope + ((size_t)ti.pos * half + lo) * 2;
        const f32x4 c01 = pre ? pre->a : *(const f32x4 *)cs;           // (cos,sin) x 4
        const f32x4 c23 = pre ? pre->b : *(const f32x4 *)(cs + 4);
        f32x4 x = v0, y = v1;
        v0.x = x.x * c01.x - y.x * c01.y;  v1.x = x.x * c01.y + y.x * c01.x;
        v0.y = x.y * c01.z - y.y * c01.w;  v1.y = x.y * c01.w + y.y * c01.z;
        v0.z = x.z * c23.x - y.z * c23.y;  v1.z = x.z * c23.y + y.z * c23.x;
        v0.w = x.w * c23.z - y.w * c23.w;  v1.w = x.w * c23.w + y.w * c23.z;
      }
      if (head < a.n_q_heads) {
        bf16_t *q = a.q_out + ((size_t)m * a.n_q_heads + head) * hd;
        store_bf16x4(q + lo, v0);
        store_bf16x4(q + lo + half, v1);
      } else {
        const int pg = pre ? pre->pg : a.page_table[(size_t)ti.slot * a.pages_per_session + (ti.pos >> 4)];
        const int sl = ti.pos & 15;
        if (!is_v) {
          bf16_t *kp = a.pool.base + a.pool.k_off(a.block, pg, head - a.n_q_heads);
          store_bf16x4(kp + kpage_off(sl, lo), v0);
          store_bf16x4(kp + kpage_off(sl, lo + half), v1);
          if (a.pool2.base) {
            bf16_t *kt = a.pool2.base + a.pool2.v_off(a.block, pg, head - a.n_q_heads);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              kt[vpage_off(sl, lo + i)] = f32_to_bf16(v0[i]);
              kt[vpage_off(sl, lo + half + i)] = f32_to_bf16(v1[i]);
            }
          }
        } else {
          bf16_t *vp = a.pool.base + a.pool.v_off(a.block, pg, head - a.n_q_heads - a.n_kv_heads);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            vp[vpage_off(sl, lo + i)] = f32_to_bf16(v0[i]);
            vp[vpage_off(sl, lo + half + i)] = f32_to_bf16(v1[i]);
          }
          if (a.pool2.base) {
            bf16_t *vr = a.pool2.base + a.pool2.k_off(a.block, pg, head - a.n_q_heads - a.n_kv_heads);
            store_bf16x4(vr + kpage_off(sl, lo), v0);
            store_bf16x4(vr + kpage_off(sl, lo + half), v1);
          }
        }
      }
    } break;
  }
}

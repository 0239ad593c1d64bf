// Training-time passes through a span (Section 3.3 of the paper: the servers keep their weights
// frozen, back-propagate through their blocks and return the gradient with respect to their
// input activations; whole sequences, no attention cache).
//
// The projections of the backward pass are the same kernels as in the forward pass, run on
// transposed packed copies of the weights (dX = dY W is a projection with W^T as the weight);
// the forward sweep is the inference path's own kernels (projections with fused epilogues,
// prefill attention) writing into pages that belong to the call.  This file holds what
// surrounds them: packing of transposed weights and of fp32 rows into the projections' T16
// input format, the derivatives of the norms, of the gated activation and of the rotary
// embedding, and the attention backward kernels.
#include "common.h"
#include "epilogue.h"
#include "launch.h"

// ------------------------------------------------------------------------------------
// W^T packing: the destination is the T16 form of the matrix whose row n, column k is
// S[k][n], S = the sources stacked on top of each other (row-major bf16, `ld` columns).
// One wave per (k tile, row tile); set-up only.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void pack_weight_t_kernel(PackTArgs a) {
  const int kt = blockIdx.x, pt = blockIdx.y, lane = threadIdx.x;
  const int g = lane >> 4, r = lane & 15;
  const int n = pt * 16 + r;
  bf16_t v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    int k = kt * 32 + g * 8 + i;
    bf16_t e = 0;
    if (n < a.ld) {
      if (k < a.rows[0]) e = a.src[0][(size_t)k * a.ld + n];
      else if (k < a.rows[0] + a.rows[1]) e = a.src[1][(size_t)(k - a.rows[0]) * a.ld + n];
      else if (k < a.rows[0] + a.rows[1] + a.rows[2]) e = a.src[2][(size_t)(k - a.rows[0] - a.rows[1]) * a.ld + n];
    }
    v[i] = e;
  }
  u32x4 w;
  w.x = v[0] | ((uint32_t)v[1] << 16); w.y = v[2] | ((uint32_t)v[3] << 16);
  w.z = v[4] | ((uint32_t)v[5] << 16); w.w = v[6] | ((uint32_t)v[7] << 16);
  *(u32x4 *)(a.dst + ((size_t)kt * a.RT + pt) * 512 + lane * 8) = w;
}

void launch_pack_weight_t(const PackTArgs &a, int n_row_tiles, hipStream_t s) {
  hipLaunchKernelGGL(pack_weight_t_kernel, dim3(a.KT, n_row_tiles), dim3(64), 0, s, a);
}

// ------------------------------------------------------------------------------------
// Transposed copy of a packed bf16 matrix (compressed spans: a matrix is expanded to bf16 tiles for
// one call, then turned for the backward projection).  Source: T16 in the physical row order of
// the forward packs (see PackOrder) with s_RT row tiles per k step; destination: T16 of the
// matrix whose row k, column n is W[n][k] with n in *logical* order ([q | k | v], [gate | up]).
// One wave per destination tile; each lane gathers its eight values.
// ------------------------------------------------------------------------------------
__device__ __forceinline__ int physical_row(const TransposeArgs &a, int n) {
  if (a.order == PACK_NATURAL) return n;
  if (a.order == PACK_GATEUP) {
    const bool up = n >= a.rows0;
    const int f = up ? n - a.rows0 : n;
    return ((f >> 4) * 2 + (up ? 1 : 0)) * 16 + (f & 15);
  }
  // PACK_HEADS: within a head, logical tile lt sits at physical tile j, with (lt, lt + HT/2) adjacent
  const int HT = a.head_dim >> 4, head = n / a.head_dim, within = n % a.head_dim;
  const int lt = within >> 4;
  const int j = lt < (HT >> 1) ? 2 * lt : 2 * (lt - (HT >> 1)) + 1;
  return (head * HT + j) * 16 + (within & 15);
}

__global__ __launch_bounds__(64) void transpose_t16_kernel(TransposeArgs a) {
  const int kt = blockIdx.x, pt = blockIdx.y, lane = threadIdx.x;
  const int g = lane >> 4, r = lane & 15;
  const int row = pt * 16 + r;                 // = k of the source
  uint32_t v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int n = kt * 32 + g * 8 + i;         // logical source row
    v[i] = (row < a.K && n < a.N) ? a.src[t16_off(physical_row(a, n), row, a.s_RT)] : 0;
  }
  u32x4 w;
  w.x = v[0] | (v[1] << 16); w.y = v[2] | (v[3] << 16); w.z = v[4] | (v[5] << 16); w.w = v[6] | (v[7] << 16);
  *(u32x4 *)(a.dst + ((size_t)kt * a.d_RT + pt) * 512 + lane * 8) = w;
}

void launch_transpose_t16(const TransposeArgs &a, int d_KT, hipStream_t s) {
  hipLaunchKernelGGL(transpose_t16_kernel, dim3(d_KT, a.d_RT), dim3(64), 0, s, a);
}

// ------------------------------------------------------------------------------------
// The three kernels below write T16 tiles of projection inputs.  A workgroup of four waves
// covers one row tile and PACK_KPB consecutive k tiles: a wave takes four of the 16 rows, and
// 16 lanes read 512 consecutive bytes of one row (four k tiles) per step; every lane ends up
// with exactly one 16-byte chunk of a tile.
// ------------------------------------------------------------------------------------
#define PACK_KPB 16
#define PACK_TILE_VARS                                                                      \
  const int mt = blockIdx.y, lane = threadIdx.x & 63;                                       \
  const int r = (threadIdx.x >> 6) * 4 + (lane >> 4), g = lane & 3;
#define PACK_TILE_FOR(KT_)                                                                  \
  for (int kt = blockIdx.x * PACK_KPB + ((lane >> 2) & 3); kt < (blockIdx.x + 1) * PACK_KPB && kt < (KT_); kt += 4)
#define PACK_TILE_LOOP(KT_) PACK_TILE_VARS PACK_TILE_FOR(KT_)
static inline dim3 pack_grid(int KT, int M) { return dim3(ceil_div(KT, PACK_KPB), ceil_div(M, 16)); }

// fp32 rows [M][K] -> T16 bf16 with RT row tiles per k step (rows >= M and k >= K are zero)
__global__ __launch_bounds__(256) void pack_act_f32_kernel(const float *x, bf16_t *dst, int M, int K, int KT, int RT) {
  PACK_TILE_LOOP(KT) {
  const int row = mt * 16 + r, k = kt * 32 + g * 8;
  u32x4 w = {0, 0, 0, 0};
  if (row < M && k < K) {
    const f32x4 a = *(const f32x4 *)(x + (size_t)row * K + k);
    const f32x4 b = *(const f32x4 *)(x + (size_t)row * K + k + 4);
    w.x = pack_bf16x2(a.x, a.y); w.y = pack_bf16x2(a.z, a.w);
    w.z = pack_bf16x2(b.x, b.y); w.w = pack_bf16x2(b.z, b.w);
  }
  *(u32x4 *)(dst + ((size_t)kt * RT + mt) * 512 + (g * 16 + r) * 8) = w;
  }
}

void launch_pack_act_f32(const float *x, bf16_t *dst, int M, int K, int KT, int RT, hipStream_t s) {
  if (M < 1) return;
  hipLaunchKernelGGL(pack_act_f32_kernel, pack_grid(KT, M), dim3(256), 0, s, x, dst, M, K, KT, RT);
}

// ------------------------------------------------------------------------------------
// rows between the caller's dtype and the fp32 working buffers
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rows_to_f32_kernel(const void *src, int src_f32, float *dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = src_f32 ? ((const float *)src)[i] : bf16_to_f32(((const bf16_t *)src)[i]);
}
__global__ __launch_bounds__(256) void rows_from_f32_kernel(const float *src, void *dst, int dst_f32, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) {
    if (dst_f32) ((float *)dst)[i] = src[i];
    else ((bf16_t *)dst)[i] = f32_to_bf16(src[i]);
  }
}
void launch_rows_to_f32(const void *src, int src_f32, float *dst, size_t n, hipStream_t s) {
  if (n) hipLaunchKernelGGL(rows_to_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, src, src_f32, dst, n);
}
void launch_rows_from_f32(const float *src, void *dst, int dst_f32, size_t n, hipStream_t s) {
  if (n) hipLaunchKernelGGL(rows_from_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, src, dst, dst_f32, n);
}

// ------------------------------------------------------------------------------------
// Norm backward, one workgroup per row.  With y = xhat * gain (+ beta), xhat = (x - mu) * r,
// r = rsqrt(var + eps) (mu = 0 and var = mean x^2 for RMSNorm), and dy the gradient of y:
//   dxh = dy * gain
//   RMSNorm:   dx = r * (dxh - x * r^2 * mean(dxh * x))
//   LayerNorm: dx = r * (dxh - mean(dxh) - xhat * mean(dxh * xhat))
// The result is ADDED to `acc` (the gradient that reaches x through the residual branch).
// ------------------------------------------------------------------------------------
__device__ __forceinline__ float block_sum_256(float v, float *red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  const int wave = threadIdx.x >> 6;
  __syncthreads();                       // red may still be read from the previous call
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

template <bool LN>
__global__ __launch_bounds__(256) void norm_bwd_kernel(const float *__restrict__ x, const float *__restrict__ gain,
                                                       const float *__restrict__ dy, float *__restrict__ acc,
                                                       int d, float eps) {
  __shared__ float red[4];
  const size_t row = blockIdx.x;
  const float *xr = x + row * d, *dr = dy + row * d;
  float *ar = acc + row * d;
  float s1 = 0.f, s2 = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) { const float v = xr[i]; s1 += v; s2 += v * v; }
  s2 = block_sum_256(s2, red);
  float mu = 0.f, var;
  if (LN) {
    s1 = block_sum_256(s1, red);
    mu = s1 / d;
    var = s2 / d - mu * mu;
    // the subtraction above loses digits when |mu| is large against the spread: redo it centred
    float c2 = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) { const float v = xr[i] - mu; c2 += v * v; }
    var = block_sum_256(c2, red) / d;
  } else {
    var = s2 / d;
  }
  const float r = rsqrtf(var + eps);
  float a = 0.f, b = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float dxh = dr[i] * gain[i];
    const float xh = (xr[i] - mu) * r;
    a += dxh * xh;
    b += dxh;
  }
  a = block_sum_256(a, red) / d;
  b = LN ? block_sum_256(b, red) / d : 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float dxh = dr[i] * gain[i];
    const float xh = (xr[i] - mu) * r;
    ar[i] += r * (dxh - b - xh * a);
  }
}

void launch_norm_bwd(const float *x, const float *gain, const float *dy, float *acc, int M, int d, float eps,
                     int layernorm, hipStream_t s) {
  if (M < 1) return;
  if (layernorm) hipLaunchKernelGGL((norm_bwd_kernel<true>), dim3(M), dim3(256), 0, s, x, gain, dy, acc, d, eps);
  else hipLaunchKernelGGL((norm_bwd_kernel<false>), dim3(M), dim3(256), 0, s, x, gain, dy, acc, d, eps);
}

// ------------------------------------------------------------------------------------
// Activation backward, written straight into the T16 input of the next projection.
//   gated (Llama): a = silu(g) * u, pre = [g | u] ([M][2F]), da [M][F]:
//                  dg = da * u * sig(g) * (1 + g * (1 - sig(g))),  du = da * silu(g);  out columns [dg | du]
//   plain (BLOOM): a = gelu_tanh(z), pre = z ([M][F]):  dz = da * gelu'(z)
// ------------------------------------------------------------------------------------
template <bool GATED>
__global__ __launch_bounds__(256) void act_bwd_pack_kernel(const float *__restrict__ pre, const float *__restrict__ da,
                                                           bf16_t *dst, int M, int F, int KT, int RT) {
  PACK_TILE_LOOP(KT) {
    const int row = mt * 16 + r, k = kt * 32 + g * 8;
    const int Kc = GATED ? 2 * F : F;
    if (GATED && k >= F && k < Kc) continue;          // written by the lane that holds the gate column k - F
    float o[8] = {0, 0, 0, 0, 0, 0, 0, 0}, o2[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (row < M && k < F) {
      float zv[8], uv[8], dv[8];
      const float *zp = pre + (size_t)row * Kc + k, *dp = da + (size_t)row * F + k;
      *(f32x4 *)zv = *(const f32x4 *)zp; *(f32x4 *)(zv + 4) = *(const f32x4 *)(zp + 4);
      *(f32x4 *)dv = *(const f32x4 *)dp; *(f32x4 *)(dv + 4) = *(const f32x4 *)(dp + 4);
      if (GATED) {
        *(f32x4 *)uv = *(const f32x4 *)(zp + F); *(f32x4 *)(uv + 4) = *(const f32x4 *)(zp + F + 4);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float sg = 1.0f / (1.0f + __expf(-zv[i]));
          o[i] = dv[i] * uv[i] * sg * (1.0f + zv[i] * (1.0f - sg));
          o2[i] = dv[i] * zv[i] * sg;
        }
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = dv[i] * gelu_tanh_grad(zv[i]);
      }
    }
    u32x4 w;
    w.x = pack_bf16x2(o[0], o[1]); w.y = pack_bf16x2(o[2], o[3]);
    w.z = pack_bf16x2(o[4], o[5]); w.w = pack_bf16x2(o[6], o[7]);
    *(u32x4 *)(dst + ((size_t)kt * RT + mt) * 512 + (g * 16 + r) * 8) = w;
    if (GATED && k < F) {
      const int k2 = k + F;                            // the up column of the same feature
      w.x = pack_bf16x2(o2[0], o2[1]); w.y = pack_bf16x2(o2[2], o2[3]);
      w.z = pack_bf16x2(o2[4], o2[5]); w.w = pack_bf16x2(o2[6], o2[7]);
      *(u32x4 *)(dst + ((size_t)(k2 >> 5) * RT + mt) * 512 + ((((k2 >> 3) & 3) * 16 + r)) * 8) = w;
    }
  }
}

void launch_act_bwd_pack(const float *pre, const float *da, bf16_t *dst, int M, int F, int gated, int KT, int RT,
                         hipStream_t s) {
  if (M < 1) return;
  if (gated) hipLaunchKernelGGL((act_bwd_pack_kernel<true>), pack_grid(KT, M), dim3(256), 0, s, pre, da, dst, M, F, KT, RT);
  else hipLaunchKernelGGL((act_bwd_pack_kernel<false>), pack_grid(KT, M), dim3(256), 0, s, pre, da, dst, M, F, KT, RT);
}

// ------------------------------------------------------------------------------------
// Gradient of [q | k | v] ([M][nqkv] fp32, q and k taken after the rotary embedding) -> T16
// input of the transposed q/k/v projection.  The rotation (a, b) -> (a c - b s, a s + b c) of
// a pair (dim, dim + hd/2) is undone on the gradient by its transpose.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void qkv_bwd_pack_kernel(const float *__restrict__ dqkv, const float *__restrict__ rope,
                                                           bf16_t *dst, int M, int n_q_heads, int n_kv_heads, int hd,
                                                           int rotary, int KT, int RT, BatchMeta meta) {
  PACK_TILE_VARS
  const int row = mt * 16 + r;
  const int pos = rotary && row < M ? token_info(meta, row).pos : 0;     // once per thread, not per tile
  PACK_TILE_FOR(KT) {
  const int k = kt * 32 + g * 8;
  const int nqkv = (n_q_heads + 2 * n_kv_heads) * hd;
  float o[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (row < M && k < nqkv) {
    const float *src = dqkv + (size_t)row * nqkv;
    const int head = k / hd, dim = k % hd, half = hd >> 1;
    if (rotary && head < n_q_heads + n_kv_heads) {
      const bool hi = dim >= half;
      const int lo = hi ? dim - half : dim;
      const float *cs = rope + ((size_t)pos * half + lo) * 2;
      const float *pa = src + head * hd + lo;
      float a8[8], b8[8], cs16[16];
      *(f32x4 *)a8 = *(const f32x4 *)pa;          *(f32x4 *)(a8 + 4) = *(const f32x4 *)(pa + 4);
      *(f32x4 *)b8 = *(const f32x4 *)(pa + half); *(f32x4 *)(b8 + 4) = *(const f32x4 *)(pa + half + 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) *(f32x4 *)(cs16 + 4 * i) = *(const f32x4 *)(cs + 4 * i);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float c = cs16[2 * i], sn = cs16[2 * i + 1];
        o[i] = hi ? -sn * a8[i] + c * b8[i] : c * a8[i] + sn * b8[i];
      }
    } else {
      *(f32x4 *)o = *(const f32x4 *)(src + k); *(f32x4 *)(o + 4) = *(const f32x4 *)(src + k + 4);
    }
  }
  u32x4 w;
  w.x = pack_bf16x2(o[0], o[1]); w.y = pack_bf16x2(o[2], o[3]);
  w.z = pack_bf16x2(o[4], o[5]); w.w = pack_bf16x2(o[6], o[7]);
  *(u32x4 *)(dst + ((size_t)kt * RT + mt) * 512 + (g * 16 + r) * 8) = w;
  }
}

void launch_qkv_bwd_pack(const float *dqkv, const float *rope, bf16_t *dst, int M, int n_q_heads, int n_kv_heads,
                         int hd, int rotary, int KT, int RT, const BatchMeta &meta, hipStream_t s) {
  if (M < 1) return;
  hipLaunchKernelGGL(qkv_bwd_pack_kernel, pack_grid(KT, M), dim3(256), 0, s, dqkv, rope, dst, M, n_q_heads,
                     n_kv_heads, hd, rotary, KT, RT, meta);
}

// ------------------------------------------------------------------------------------
// Attention backward over whole sequences (causal, one sequence attends to itself only).
// The forward pass is the prefill kernel of the inference path run on pages that belong to
// the call; it leaves, per query, the output row o and the log-sum-exp of its logits (base 2).
// With p = softmax probabilities, dp = do . v, delta = do . o:
//     ds = p * (dp - delta),   dq = ds K / sqrt(hd),   dk = ds^T Q / sqrt(hd),   dv = p^T do.
// All five contractions run on v_mfma_f32_16x16x32_bf16 with operands read straight from
// memory in the layouts the forward pass stored (no LDS, no barriers):
//   dq kernel   one wave per (32 queries, query head), walking the keys 32 at a time like the
//               forward kernel:  S^T = K Q^T,  dP^T = V dO^T  (row operands = row-wise K / V page
//               tiles, column operands = the wave's queries),  dQ^T += K^T dS^T  (row operand =
//               transposed K page tiles, column operand = the lane's own 8 values of dS^T).
//   dk/dv kernel one wave per (page of 16 keys, kv head), eight consecutive pages per workgroup, walking
//               the later queries 32 at a time and the query heads of the group together (the operands
//               that depend on the step only pass through LDS once per workgroup):  S = Q K^T,  dP = dO V^T  (column operands =
//               the page's K / V tile, kept in registers),  dV^T += dO^T P,  dK^T += Q^T dS  (row
//               operands = 16-byte reads of transposed bf16 copies of the q / do rows, column
//               operands = the lane's own 8 values).
// The contraction index of the second product of each pair is permuted (lane group g holds
// keys / queries g*4..g*4+3 of two 16-wide sub-tiles); both operands use the same permutation.
// ------------------------------------------------------------------------------------
namespace {
constexpr int BWD_NCT = 2;          // 32 queries per wave in the dq kernel
constexpr int BWD_MAX_WAVES = 8;
constexpr float LOG2E = 1.4426950408889634f;

__device__ __forceinline__ bf16x8 pack8(const float *v) {
  u32x4 w;
  w.x = pack_bf16x2(v[0], v[1]); w.y = pack_bf16x2(v[2], v[3]);
  w.z = pack_bf16x2(v[4], v[5]); w.w = pack_bf16x2(v[6], v[7]);
  return __builtin_bit_cast(bf16x8, w);
}
__device__ __forceinline__ bf16x8 pack8(f32x4 a, f32x4 b) {
  u32x4 w;
  w.x = pack_bf16x2(a.x, a.y); w.y = pack_bf16x2(a.z, a.w);
  w.z = pack_bf16x2(b.x, b.y); w.w = pack_bf16x2(b.z, b.w);
  return __builtin_bit_cast(bf16x8, w);
}

template <int HD, bool BIAS>
__global__ __launch_bounds__(64 * BWD_MAX_WAVES) void attn_bwd_dq_kernel(TrainAttnArgs a, BatchMeta meta) {
  constexpr int KS = HD / 32, HB = HD / 16, NCT = BWD_NCT, QT = 16 * NCT;
  const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
  const int G = a.n_q_heads / a.n_kv_heads;
  int tile = gridDim.x - 1 - blockIdx.x, s = 0;
  while (true) {
    const int nt = ceil_div(meta.cu[s + 1] - meta.cu[s], QT);
    if (tile < nt) break;
    tile -= nt; ++s;
  }
  const int T = meta.cu[s + 1] - meta.cu[s], t0 = tile * QT;
  const int wpb = min(G, BWD_MAX_WAVES), parts = ceil_div(G, wpb);
  const int kvh = blockIdx.y / parts;
  const int hg = (blockIdx.y % parts) * wpb + (threadIdx.x >> 6);
  if (hg >= G) return;
  const int head = kvh * G + hg;
  const int *ptrow = a.page_table + (size_t)meta.slot[s] * a.pages_per_seq;
  const int n_pg = ceil_div(T, SPAN_PAGE);
  const float scale = rsqrtf((float)HD), scale2 = scale * LOG2E;
  const float slope2 = BIAS ? a.alibi[head] * LOG2E : 0.0f;
  const int qdim = a.n_q_heads * HD, nqkv = qdim + 2 * a.n_kv_heads * HD;

  bf16x8 Q[NCT][KS], DO[NCT][KS];
  float delta[NCT], lse2[NCT];
  int qpos[NCT], mrow[NCT];
  bool valid[NCT];
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) {
    int t = t0 + ct * 16 + c;
    valid[ct] = t < T;
    t = min(t, T - 1);
    qpos[ct] = t;
    mrow[ct] = meta.cu[s] + t;
    const size_t off = (size_t)mrow[ct] * qdim + head * HD + g * 8;
    float dl = 0.0f;
#pragma unroll
    for (int j = 0; j < KS; ++j) {
      Q[ct][j] = *(const bf16x8 *)(a.q + off + j * 32);
      const f32x4 x0 = *(const f32x4 *)(a.d_o + off + j * 32), x1 = *(const f32x4 *)(a.d_o + off + j * 32 + 4);
      const f32x4 o0 = *(const f32x4 *)(a.o + off + j * 32), o1 = *(const f32x4 *)(a.o + off + j * 32 + 4);
      dl += x0.x * o0.x + x0.y * o0.y + x0.z * o0.z + x0.w * o0.w + x1.x * o1.x + x1.y * o1.y + x1.z * o1.z + x1.w * o1.w;
      DO[ct][j] = pack8(x0, x1);
    }
    dl += __shfl_xor(dl, 16);
    dl += __shfl_xor(dl, 32);
    delta[ct] = dl;
    lse2[ct] = a.lse[(size_t)mrow[ct] * a.n_q_heads + head];
    if (valid[ct] && g == 0) a.delta[(size_t)mrow[ct] * a.n_q_heads + head] = dl;
  }

  f32x4 dQ[NCT][HB];
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) dQ[ct][hb] = f32x4{0, 0, 0, 0};

  const int pp1 = ceil_div(min(t0 + QT, T), 32);
  for (int pp = 0; pp < pp1; ++pp) {
    const int pgA = ptrow[2 * pp], pgB = ptrow[min(2 * pp + 1, n_pg - 1)];
    const bf16_t *kA = a.pool.base + a.pool.k_off(a.block, pgA, kvh) + lane * 8;
    const bf16_t *kB = a.pool.base + a.pool.k_off(a.block, pgB, kvh) + lane * 8;
    const bf16_t *vA = a.pool2.base + a.pool2.k_off(a.block, pgA, kvh) + lane * 8;
    const bf16_t *vB = a.pool2.base + a.pool2.k_off(a.block, pgB, kvh) + lane * 8;
    const bf16_t *tA = a.pool2.base + a.pool2.v_off(a.block, pgA, kvh) + lane * 8;
    const bf16_t *tB = a.pool2.base + a.pool2.v_off(a.block, pgB, kvh) + lane * 8;
    bf16x8 KA[KS], KB[KS], VA[KS], VB[KS];
    u32x4 TA[KS], TB[KS];
#pragma unroll
    for (int j = 0; j < KS; ++j) {
      KA[j] = *(const bf16x8 *)(kA + j * 512); KB[j] = *(const bf16x8 *)(kB + j * 512);
      VA[j] = *(const bf16x8 *)(vA + j * 512); VB[j] = *(const bf16x8 *)(vB + j * 512);
      TA[j] = *(const u32x4 *)(tA + j * 512);  TB[j] = *(const u32x4 *)(tB + j * 512);
    }
    const int kposA = pp * 32 + g * 4, kposB = kposA + 16;
    bf16x8 DS[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
      f32x4 sA = {0, 0, 0, 0}, sB = {0, 0, 0, 0}, dA = {0, 0, 0, 0}, dB = {0, 0, 0, 0};
#pragma unroll
      for (int j = 0; j < KS; ++j) {
        sA = __builtin_amdgcn_mfma_f32_16x16x32_bf16(KA[j], Q[ct][j], sA, 0, 0, 0);
        sB = __builtin_amdgcn_mfma_f32_16x16x32_bf16(KB[j], Q[ct][j], sB, 0, 0, 0);
        dA = __builtin_amdgcn_mfma_f32_16x16x32_bf16(VA[j], DO[ct][j], dA, 0, 0, 0);
        dB = __builtin_amdgcn_mfma_f32_16x16x32_bf16(VB[j], DO[ct][j], dB, 0, 0, 0);
      }
      float ds[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int kp = i < 4 ? kposA + i : kposB + (i - 4);
        float v = (i < 4 ? sA[i] : sB[i - 4]) * scale2;
        if (BIAS) v -= slope2 * (float)(qpos[ct] - kp);
        const float p = kp <= qpos[ct] ? __builtin_amdgcn_exp2f(v - lse2[ct]) : 0.0f;
        ds[i] = p * ((i < 4 ? dA[i] : dB[i - 4]) - delta[ct]);
      }
      DS[ct] = pack8(ds);
    }
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
      const int c2 = hb >> 1;
      u32x4 kk;
      if (hb & 1) { kk.x = TA[c2].z; kk.y = TA[c2].w; kk.z = TB[c2].z; kk.w = TB[c2].w; }
      else        { kk.x = TA[c2].x; kk.y = TA[c2].y; kk.z = TB[c2].x; kk.w = TB[c2].y; }
      const bf16x8 Kop = __builtin_bit_cast(bf16x8, kk);
#pragma unroll
      for (int ct = 0; ct < NCT; ++ct)
        dQ[ct][hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Kop, DS[ct], dQ[ct][hb], 0, 0, 0);
    }
  }
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) {
    if (!valid[ct]) continue;
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
      *(f32x4 *)(a.dqkv + (size_t)mrow[ct] * nqkv + head * HD + hb * 16 + g * 4) = dQ[ct][hb] * scale;
  }
}

constexpr int DKV_WAVES = 8;        // consecutive key pages per workgroup, one wave each

// Transposed bf16 copy of token rows: dst[n][col(m)] = src[m][n], col(m) = 16 * (first page of m's
// sequence) + position of m in its sequence, so that a sequence's columns start 16-aligned whatever
// the lengths before it.  The dk/dv kernel reads its row operands (contraction over queries) from
// these copies with 16-byte loads.
__global__ __launch_bounds__(256) void transpose_rows_kernel(const void *src, int src_f32, bf16_t *dst, int M, int N,
                                                             int ld, const int *page_table, int pps, BatchMeta meta) {
  __shared__ bf16_t tile[32][34];
  const int n0 = blockIdx.x * 32, m0 = blockIdx.y * 32, tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int r = ty; r < 32; r += 8) {
    const int m = m0 + r, n = n0 + tx;
    bf16_t v = 0;
    if (m < M && n < N)
      v = src_f32 ? f32_to_bf16(((const float *)src)[(size_t)m * N + n]) : ((const bf16_t *)src)[(size_t)m * N + n];
    tile[r][tx] = v;
  }
  __syncthreads();
  const int m = m0 + tx;
  if (m >= M) return;
  int s0, s1, sq = 0;
  while (sq + 1 < meta.n_sess && m >= meta.cu[sq + 1]) ++sq;
  s0 = meta.cu[sq]; s1 = meta.cu[sq + 1]; (void)s1;
  const size_t col = (size_t)page_table[(size_t)meta.slot[sq] * pps] * SPAN_PAGE + (m - s0);
  for (int r = ty; r < 32; r += 8) {
    const int n = n0 + r;
    if (n < N) dst[(size_t)n * ld + col] = tile[tx][r];
  }
}

// One workgroup per (group of DKV_WAVES consecutive key pages of a sequence, kv head), one wave per page.
// All waves walk the same steps -- (32 queries, query head) from the group's first page to the end of the
// sequence -- so the operands that depend on the step only (the q / do rows and their transposed copies,
// 32 KiB per step at hd = 128) are fetched once per workgroup into LDS, the next step's while the current
// one computes, and every wave reads them from there.  (Fetched per wave, these operands are re-read for
// every 16 keys: 43 GB per block at 4096 tokens, which is what bounded the first version.)
template <int HD, bool BIAS>
__global__ __launch_bounds__(64 * DKV_WAVES) void attn_bwd_dkv_kernel(TrainAttnArgs a, BatchMeta meta) {
  constexpr int KS = HD / 32, HB = HD / 16;
  constexpr int SLOTS = 4 * KS + 2 * HB;        // 1 KiB operand fragments of a step: q[u][j], do[u][j], q^T[hb], do^T[hb]
  constexpr int PER = SLOTS / DKV_WAVES;        // fragments a wave fetches per step
  static_assert(SLOTS % DKV_WAVES == 0, "fragments must divide among the waves");
  __shared__ u32x4 stage[2][SLOTS * 64];
  __shared__ float row_stat[2][64];           // per step: log-sum-exp of its 32 queries, then their delta
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, c = lane & 15, g = lane >> 4;
  const int G = a.n_q_heads / a.n_kv_heads, kvh = blockIdx.y;
  int grp = blockIdx.x, s = 0;
  while (true) {
    const int ng = ceil_div(ceil_div(meta.cu[s + 1] - meta.cu[s], SPAN_PAGE), DKV_WAVES);
    if (grp < ng) break;
    grp -= ng; ++s;
  }
  const int T = meta.cu[s + 1] - meta.cu[s], row0 = meta.cu[s], n_pg = ceil_div(T, SPAN_PAGE);
  const int pj = grp * DKV_WAVES + wave;
  const bool have = pj < n_pg;                  // a wave without a page still fetches and meets the barriers
  const int *ptrow = a.page_table + (size_t)meta.slot[s] * a.pages_per_seq;
  const int pg = ptrow[min(pj, n_pg - 1)];
  const size_t col0 = (size_t)ptrow[0] * SPAN_PAGE;       // the sequence's first column in the transposed copies
  const float scale = rsqrtf((float)HD), scale2 = scale * LOG2E;
  const int qdim = a.n_q_heads * HD, kvdim = a.n_kv_heads * HD, nqkv = qdim + 2 * kvdim;
  bf16x8 K[KS], V[KS];
  {
    const bf16_t *kp = a.pool.base + a.pool.k_off(a.block, pg, kvh) + lane * 8;
    const bf16_t *vp = a.pool2.base + a.pool2.k_off(a.block, pg, kvh) + lane * 8;
#pragma unroll
    for (int j = 0; j < KS; ++j) { K[j] = *(const bf16x8 *)(kp + j * 512); V[j] = *(const bf16x8 *)(vp + j * 512); }
  }
  const int kpos = pj * SPAN_PAGE + c;          // the key of this lane's column
  f32x4 dK[HB], dV[HB];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) { dK[hb] = f32x4{0, 0, 0, 0}; dV[hb] = f32x4{0, 0, 0, 0}; }

  // Steps: it -> query tile qt_first + it / G, head kvh * G + it % G.  A step takes 32 queries as two MFMA
  // row tiles; row r of tile u is query qt0 + (r/4)*8 + u*4 + r%4, so that the eight accumulator rows a lane
  // group g ends up with (rows g*4.. of both tiles) are the eight consecutive queries qt0 + g*8 ..: the
  // contraction index of the second products in memory order.
  const int qt_first = (grp * DKV_WAVES * SPAN_PAGE) & ~31;
  const int n_steps = ceil_div(T - qt_first, 32) * G;
  u32x4 fr[PER];
  float fs = 0.0f;
  auto fetch = [&](int it) {
    const int qt0 = qt_first + (it / G) * 32, head = kvh * G + it % G;
    if (wave == DKV_WAVES - 1) {
      const size_t r = (size_t)(row0 + min(qt0 + (lane & 31), T - 1)) * a.n_q_heads + head;
      fs = lane < 32 ? a.lse[r] : a.delta[r];
    }
    static_for<PER>([&](auto i_) {
      constexpr int i = decltype(i_)::value;
      const int sl = wave + i * DKV_WAVES;                 // uniform over the wave
      if (sl < 4 * KS) {
        const int u = (sl % (2 * KS)) / KS, j = sl % KS;
        const size_t row = (size_t)(row0 + min(qt0 + (c >> 2) * 8 + u * 4 + (c & 3), T - 1));
        const size_t off = row * qdim + head * HD + g * 8 + j * 32;
        if (sl < 2 * KS) fr[i] = *(const u32x4 *)(a.q + off);
        else fr[i] = __builtin_bit_cast(u32x4, pack8(*(const f32x4 *)(a.d_o + off), *(const f32x4 *)(a.d_o + off + 4)));
      } else {
        const int hb = (sl - 4 * KS) % HB;
        const size_t off = (size_t)(head * HD + hb * 16 + c) * a.ld_t + col0 + qt0 + g * 8;
        fr[i] = *(const u32x4 *)((sl < 4 * KS + HB ? a.q_t : a.do_t) + off);
      }
    });
  };
  auto stash = [&](int b) {
    static_for<PER>([&](auto i_) {
      constexpr int i = decltype(i_)::value;
      stage[b][(wave + i * DKV_WAVES) * 64 + lane] = fr[i];
    });
    if (wave == DKV_WAVES - 1) row_stat[b][lane] = fs;
  };

  // Fragments are fetched two steps ahead and written to LDS one step ahead: a fetch has a whole step
  // to arrive before the wave needs its registers back.  Two buffers are enough: the buffer of step
  // it + 1 is that of step it - 1, which every wave has left at the barrier ending that step.
  fetch(0);
  stash(0);
  if (n_steps > 1) fetch(1);
  __syncthreads();
  for (int it = 0; it < n_steps; ++it) {
    if (it + 1 < n_steps) stash((it + 1) & 1);    // (conditions are uniform over the workgroup)
    if (it + 2 < n_steps) fetch(it + 2);
    const int qt0 = qt_first + (it / G) * 32, head = kvh * G + it % G;
    // steps whose queries all precede the page contribute nothing
    if (have && qt0 + 31 >= pj * SPAN_PAGE) {
      const u32x4 *st = stage[it & 1];
      const float slope2 = BIAS ? a.alibi[head] * LOG2E : 0.0f;
      f32x4 S[2], DP[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        f32x4 sacc = {0, 0, 0, 0}, dacc = {0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < KS; ++j) {
          const bf16x8 qa = __builtin_bit_cast(bf16x8, st[(u * KS + j) * 64 + lane]);
          const bf16x8 da = __builtin_bit_cast(bf16x8, st[(2 * KS + u * KS + j) * 64 + lane]);
          sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa, K[j], sacc, 0, 0, 0);
          dacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(da, V[j], dacc, 0, 0, 0);
        }
        S[u] = sacc; DP[u] = dacc;
      }
      float pv[8], dsv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int tq = qt0 + g * 8 + e;
        const float lse = row_stat[it & 1][g * 8 + e], dl = row_stat[it & 1][32 + g * 8 + e];
        float v = S[e >> 2][e & 3] * scale2;
        if (BIAS) v -= slope2 * (float)(tq - kpos);
        const float p = (tq < T && kpos <= tq) ? __builtin_amdgcn_exp2f(v - lse) : 0.0f;
        pv[e] = p;
        dsv[e] = p * (DP[e >> 2][e & 3] - dl);
      }
      const bf16x8 Pb = pack8(pv), DSb = pack8(dsv);
#pragma unroll
      for (int hb = 0; hb < HB; ++hb) {
        const bf16x8 qt = __builtin_bit_cast(bf16x8, st[(4 * KS + hb) * 64 + lane]);
        const bf16x8 gt = __builtin_bit_cast(bf16x8, st[(4 * KS + HB + hb) * 64 + lane]);
        dV[hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gt, Pb, dV[hb], 0, 0, 0);
        dK[hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qt, DSb, dK[hb], 0, 0, 0);
      }
    }
    __syncthreads();
  }
  if (have && kpos < T) {
    float *dst = a.dqkv + (size_t)(row0 + kpos) * nqkv + qdim + kvh * HD + g * 4;
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
      *(f32x4 *)(dst + hb * 16) = dK[hb] * scale;
      *(f32x4 *)(dst + kvdim + hb * 16) = dV[hb];
    }
  }
}

__global__ __launch_bounds__(64) void train_page_table_kernel(int *pt, int pps, BatchMeta meta) {
  const int s = blockIdx.x;
  int base = 0;
  for (int i = 0; i < s; ++i) base += ceil_div(meta.cu[i + 1] - meta.cu[i], SPAN_PAGE);
  const int np = ceil_div(meta.cu[s + 1] - meta.cu[s], SPAN_PAGE);
  for (int j = threadIdx.x; j < np; j += 64) pt[(size_t)meta.slot[s] * pps + j] = base + j;
}
}  // namespace

void launch_train_page_table(int *page_table, int pages_per_seq, const BatchMeta &meta, hipStream_t s) {
  if (meta.n_sess < 1) return;
  hipLaunchKernelGGL(train_page_table_kernel, dim3(meta.n_sess), dim3(64), 0, s, page_table, pages_per_seq, meta);
}

void launch_attn_train_bwd(const TrainAttnArgs &a, const BatchMeta &meta, int M, hipStream_t s) {
  if (M < 1) return;
  {
    const int N = a.n_q_heads * a.head_dim;
    const dim3 gt(ceil_div(N, 32), ceil_div(M, 32));
    hipLaunchKernelGGL(transpose_rows_kernel, gt, dim3(256), 0, s, (const void *)a.q, 0, a.q_t, M, N, a.ld_t, a.page_table,
                       a.pages_per_seq, meta);
    hipLaunchKernelGGL(transpose_rows_kernel, gt, dim3(256), 0, s, (const void *)a.d_o, 1, a.do_t, M, N, a.ld_t, a.page_table,
                       a.pages_per_seq, meta);
  }
  const int G = a.n_q_heads / a.n_kv_heads;
  const int wpb = G < BWD_MAX_WAVES ? G : BWD_MAX_WAVES, parts = (G + wpb - 1) / wpb;
  int q_tiles = 0, pages = 0;                 // pages: groups of DKV_WAVES key pages, per sequence
  for (int i = 0; i < meta.n_sess; ++i) {
    q_tiles += ceil_div(meta.cu[i + 1] - meta.cu[i], 16 * BWD_NCT);
    pages += ceil_div(ceil_div(meta.cu[i + 1] - meta.cu[i], SPAN_PAGE), DKV_WAVES);
  }
  const dim3 gq(q_tiles, a.n_kv_heads * parts), bq(64 * wpb), gk(pages, a.n_kv_heads);
  if (a.head_dim == 128) {
    if (a.alibi) {
      hipLaunchKernelGGL((attn_bwd_dq_kernel<128, true>), gq, bq, 0, s, a, meta);
      hipLaunchKernelGGL((attn_bwd_dkv_kernel<128, true>), gk, dim3(64 * DKV_WAVES), 0, s, a, meta);
    } else {
      hipLaunchKernelGGL((attn_bwd_dq_kernel<128, false>), gq, bq, 0, s, a, meta);
      hipLaunchKernelGGL((attn_bwd_dkv_kernel<128, false>), gk, dim3(64 * DKV_WAVES), 0, s, a, meta);
    }
  } else {
    if (a.alibi) {
      hipLaunchKernelGGL((attn_bwd_dq_kernel<64, true>), gq, bq, 0, s, a, meta);
      hipLaunchKernelGGL((attn_bwd_dkv_kernel<64, true>), gk, dim3(64 * DKV_WAVES), 0, s, a, meta);
    } else {
      hipLaunchKernelGGL((attn_bwd_dq_kernel<64, false>), gq, bq, 0, s, a, meta);
      hipLaunchKernelGGL((attn_bwd_dkv_kernel<64, false>), gk, dim3(64 * DKV_WAVES), 0, s, a, meta);
    }
  }
}

// Training-time passes through a span (Section 3.3 of the paper: the servers keep their weights
// frozen, back-propagate through their blocks and return the gradient with respect to their
// input activations; whole sequences, no attention cache).
//
// The contractions of the backward pass are the same projection kernels as the forward pass,
// run on transposed packed copies of the weights (dX = dY W is a projection with W^T as the
// weight).  This file holds what surrounds them: packing of transposed weights and of fp32
// rows into the projections' T16 input format, the derivatives of the norms, of the gated
// activation and of the rotary embedding, and causal attention over whole sequences, forward
// and backward, on plain fp32 rows.
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
// fp32 rows [M][K] -> T16 bf16 with RT row tiles per k step (rows >= M and k >= K are zero)
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void pack_act_f32_kernel(const float *x, bf16_t *dst, int M, int K, int RT) {
  const int kt = blockIdx.x, mt = blockIdx.y, lane = threadIdx.x;
  const int g = lane & 3, r = lane >> 2;          // four lanes read 128 consecutive bytes of one row
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

void launch_pack_act_f32(const float *x, bf16_t *dst, int M, int K, int KT, int RT, hipStream_t s) {
  hipLaunchKernelGGL(pack_act_f32_kernel, dim3(KT, ceil_div(M, 16)), dim3(64), 0, s, x, dst, M, K, RT);
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
__device__ __forceinline__ float gelu_tanh_grad(float z) {
  const float c = 0.7978845608028654f, k = 0.044715f;
  const float u = c * (z + k * z * z * z);
  const float t = 1.0f - 2.0f / (__expf(2.0f * u) + 1.0f);
  return 0.5f * (1.0f + t) + 0.5f * z * (1.0f - t * t) * c * (1.0f + 3.0f * k * z * z);
}

template <bool GATED>
__global__ __launch_bounds__(64) void act_bwd_pack_kernel(const float *__restrict__ pre, const float *__restrict__ da,
                                                          bf16_t *dst, int M, int F, int RT) {
  const int kt = blockIdx.x, mt = blockIdx.y, lane = threadIdx.x;
  const int g = lane & 3, r = lane >> 2;          // four lanes read 128 consecutive bytes of one row
  const int row = mt * 16 + r, k = kt * 32 + g * 8;
  const int Kc = GATED ? 2 * F : F;
  float o[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (row < M && k < Kc) {
    if (GATED) {
      const bool up = k >= F;
      const int f = up ? k - F : k;
      const float *gp = pre + (size_t)row * 2 * F + f, *upp = gp + F, *dp = da + (size_t)row * F + f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float gv = gp[i], uv = upp[i], dv = dp[i];
        const float sg = 1.0f / (1.0f + __expf(-gv));
        o[i] = up ? dv * gv * sg : dv * uv * sg * (1.0f + gv * (1.0f - sg));
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = da[(size_t)row * F + k + i] * gelu_tanh_grad(pre[(size_t)row * F + k + i]);
    }
  }
  u32x4 w;
  w.x = pack_bf16x2(o[0], o[1]); w.y = pack_bf16x2(o[2], o[3]);
  w.z = pack_bf16x2(o[4], o[5]); w.w = pack_bf16x2(o[6], o[7]);
  *(u32x4 *)(dst + ((size_t)kt * RT + mt) * 512 + (g * 16 + r) * 8) = w;
}

void launch_act_bwd_pack(const float *pre, const float *da, bf16_t *dst, int M, int F, int gated, int KT, int RT,
                         hipStream_t s) {
  if (M < 1) return;
  if (gated) hipLaunchKernelGGL((act_bwd_pack_kernel<true>), dim3(KT, ceil_div(M, 16)), dim3(64), 0, s, pre, da, dst, M, F, RT);
  else hipLaunchKernelGGL((act_bwd_pack_kernel<false>), dim3(KT, ceil_div(M, 16)), dim3(64), 0, s, pre, da, dst, M, F, RT);
}

// ------------------------------------------------------------------------------------
// Gradient of [q | k | v] ([M][nqkv] fp32, q and k taken after the rotary embedding) -> T16
// input of the transposed q/k/v projection.  The rotation (a, b) -> (a c - b s, a s + b c) of
// a pair (dim, dim + hd/2) is undone on the gradient by its transpose.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void qkv_bwd_pack_kernel(const float *__restrict__ dqkv, const float *__restrict__ rope,
                                                          bf16_t *dst, int M, int n_q_heads, int n_kv_heads, int hd,
                                                          int rotary, int RT, BatchMeta meta) {
  const int kt = blockIdx.x, mt = blockIdx.y, lane = threadIdx.x;
  const int g = lane & 3, r = lane >> 2;          // four lanes read 128 consecutive bytes of one row
  const int row = mt * 16 + r, k = kt * 32 + g * 8;
  const int nqkv = (n_q_heads + 2 * n_kv_heads) * hd;
  float o[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (row < M && k < nqkv) {
    const float *src = dqkv + (size_t)row * nqkv;
    const int head = k / hd, dim = k % hd, half = hd >> 1;
    if (rotary && head < n_q_heads + n_kv_heads) {
      const int pos = token_info(meta, row).pos;
      const bool hi = dim >= half;
      const int lo = hi ? dim - half : dim;
      const float *cs = rope + ((size_t)pos * half + lo) * 2;
      const float *pa = src + head * hd + lo, *pb = pa + half;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float c = cs[2 * i], sn = cs[2 * i + 1];
        o[i] = hi ? -sn * pa[i] + c * pb[i] : c * pa[i] + sn * pb[i];
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = src[k + i];
    }
  }
  u32x4 w;
  w.x = pack_bf16x2(o[0], o[1]); w.y = pack_bf16x2(o[2], o[3]);
  w.z = pack_bf16x2(o[4], o[5]); w.w = pack_bf16x2(o[6], o[7]);
  *(u32x4 *)(dst + ((size_t)kt * RT + mt) * 512 + (g * 16 + r) * 8) = w;
}

void launch_qkv_bwd_pack(const float *dqkv, const float *rope, bf16_t *dst, int M, int n_q_heads, int n_kv_heads,
                         int hd, int rotary, int KT, int RT, const BatchMeta &meta, hipStream_t s) {
  if (M < 1) return;
  hipLaunchKernelGGL(qkv_bwd_pack_kernel, dim3(KT, ceil_div(M, 16)), dim3(64), 0, s, dqkv, rope, dst, M, n_q_heads,
                     n_kv_heads, hd, rotary, RT, meta);
}

// ------------------------------------------------------------------------------------
// Causal attention over whole sequences on fp32 rows [M][nqkv] = [q heads | k heads | v heads].
// One wave per (token, query head); a lane owns HD/64 consecutive dims of the head, so a key
// or value row is one coalesced read and a logit one wave reduction.  Logit of query m and key
// j (same sequence, j <= m): q.k / sqrt(hd) - slope * (m - j).
// ------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ __forceinline__ void seq_range(const BatchMeta &meta, int m, int &s0, int &s1) {
  int s = 0;
  while (s + 1 < meta.n_sess && m >= meta.cu[s + 1]) ++s;
  s0 = meta.cu[s]; s1 = meta.cu[s + 1];
}

template <int HD>
__global__ __launch_bounds__(256) void attn_train_fwd_kernel(TrainAttnArgs a, BatchMeta meta) {
  constexpr int E = HD / 64;
  const int lane = threadIdx.x & 63, m = blockIdx.x;
  const int h = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (h >= a.n_q_heads) return;
  const int kh = h / (a.n_q_heads / a.n_kv_heads);
  const int qdim = a.n_q_heads * HD, kvdim = a.n_kv_heads * HD, nqkv = qdim + 2 * kvdim;
  int s0, s1;
  seq_range(meta, m, s0, s1);
  const float scale = rsqrtf((float)HD);
  const float slope = a.alibi ? a.alibi[h] : 0.0f;
  float q[E], acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) { q[e] = a.qkv[(size_t)m * nqkv + h * HD + lane * E + e] * scale; acc[e] = 0.f; }
  float mx = -INFINITY, l = 0.f;
  const float *kp = a.qkv + qdim + kh * HD + lane * E;
  for (int j = s0; j <= m; ++j) {
    const float *kr = kp + (size_t)j * nqkv, *vr = kr + kvdim;
    float part = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) part += q[e] * kr[e];
    const float s = wave_sum(part) - slope * (float)(m - j);
    const float mn = fmaxf(mx, s);
    const float corr = __expf(mx - mn), p = __expf(s - mn);
    l = l * corr + p;
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = acc[e] * corr + p * vr[e];
    mx = mn;
  }
  const float inv = 1.0f / l;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const float o = acc[e] * inv;
    const int col = h * HD + lane * E + e;
    a.o[(size_t)m * qdim + col] = o;
    a.o_t16[t16_off(m, col, a.o_RT)] = f32_to_bf16(o);
  }
  if (lane == 0) a.lse[(size_t)m * a.n_q_heads + h] = mx + __logf(l);
}

// gradient of the queries; also delta[m][h] = do . o, which the key/value kernel needs
template <int HD>
__global__ __launch_bounds__(256) void attn_train_bwd_dq_kernel(TrainAttnArgs a, BatchMeta meta) {
  constexpr int E = HD / 64;
  const int lane = threadIdx.x & 63, m = blockIdx.x;
  const int h = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (h >= a.n_q_heads) return;
  const int kh = h / (a.n_q_heads / a.n_kv_heads);
  const int qdim = a.n_q_heads * HD, kvdim = a.n_kv_heads * HD, nqkv = qdim + 2 * kvdim;
  int s0, s1;
  seq_range(meta, m, s0, s1);
  const float scale = rsqrtf((float)HD);
  const float slope = a.alibi ? a.alibi[h] : 0.0f;
  float q[E], go[E], dq[E];
  float dl = 0.f;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int col = h * HD + lane * E + e;
    q[e] = a.qkv[(size_t)m * nqkv + col] * scale;
    go[e] = a.d_o[(size_t)m * qdim + col];
    dl += go[e] * a.o[(size_t)m * qdim + col];
    dq[e] = 0.f;
  }
  dl = wave_sum(dl);
  const float lse = a.lse[(size_t)m * a.n_q_heads + h];
  if (lane == 0) a.delta[(size_t)m * a.n_q_heads + h] = dl;
  const float *kp = a.qkv + qdim + kh * HD + lane * E;
  for (int j = s0; j <= m; ++j) {
    const float *kr = kp + (size_t)j * nqkv, *vr = kr + kvdim;
    float ps = 0.f, pd = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) { ps += q[e] * kr[e]; pd += go[e] * vr[e]; }
    const float s = wave_sum(ps) - slope * (float)(m - j);
    const float dp = wave_sum(pd);
    const float ds = __expf(s - lse) * (dp - dl);
#pragma unroll
    for (int e = 0; e < E; ++e) dq[e] += ds * kr[e];
  }
#pragma unroll
  for (int e = 0; e < E; ++e) a.dqkv[(size_t)m * nqkv + h * HD + lane * E + e] = dq[e] * scale;
}

// gradient of the keys and values: one wave per (token j, kv head), over the queries m >= j of
// the sequence and the query heads of the group
template <int HD>
__global__ __launch_bounds__(256) void attn_train_bwd_dkv_kernel(TrainAttnArgs a, BatchMeta meta) {
  constexpr int E = HD / 64;
  const int lane = threadIdx.x & 63, j = blockIdx.x;
  const int kh = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (kh >= a.n_kv_heads) return;
  const int group = a.n_q_heads / a.n_kv_heads;
  const int qdim = a.n_q_heads * HD, kvdim = a.n_kv_heads * HD, nqkv = qdim + 2 * kvdim;
  int s0, s1;
  seq_range(meta, j, s0, s1);
  const float scale = rsqrtf((float)HD);
  float k[E], v[E], dk[E], dv[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    k[e] = a.qkv[(size_t)j * nqkv + qdim + kh * HD + lane * E + e] * scale;
    v[e] = a.qkv[(size_t)j * nqkv + qdim + kvdim + kh * HD + lane * E + e];
    dk[e] = 0.f; dv[e] = 0.f;
  }
  for (int m = j; m < s1; ++m) {
    for (int hg = 0; hg < group; ++hg) {
      const int h = kh * group + hg;
      const float *qr = a.qkv + (size_t)m * nqkv + h * HD + lane * E;
      const float *gr = a.d_o + (size_t)m * qdim + h * HD + lane * E;
      float qv[E], gv[E];
      float ps = 0.f, pd = 0.f;
#pragma unroll
      for (int e = 0; e < E; ++e) { qv[e] = qr[e]; gv[e] = gr[e]; ps += qv[e] * k[e]; pd += gv[e] * v[e]; }
      const float slope = a.alibi ? a.alibi[h] : 0.0f;
      const float s = wave_sum(ps) - slope * (float)(m - j);
      const float dp = wave_sum(pd);
      const float p = __expf(s - a.lse[(size_t)m * a.n_q_heads + h]);
      const float ds = p * (dp - a.delta[(size_t)m * a.n_q_heads + h]);
#pragma unroll
      for (int e = 0; e < E; ++e) { dv[e] += p * gv[e]; dk[e] += ds * qv[e]; }
    }
  }
#pragma unroll
  for (int e = 0; e < E; ++e) {
    a.dqkv[(size_t)j * nqkv + qdim + kh * HD + lane * E + e] = dk[e] * scale;
    a.dqkv[(size_t)j * nqkv + qdim + kvdim + kh * HD + lane * E + e] = dv[e];
  }
}

void launch_attn_train_fwd(const TrainAttnArgs &a, const BatchMeta &meta, int M, hipStream_t s) {
  if (M < 1) return;
  const dim3 grid(M, ceil_div(a.n_q_heads, 4));
  if (a.head_dim == 128) hipLaunchKernelGGL((attn_train_fwd_kernel<128>), grid, dim3(256), 0, s, a, meta);
  else hipLaunchKernelGGL((attn_train_fwd_kernel<64>), grid, dim3(256), 0, s, a, meta);
}

void launch_attn_train_bwd(const TrainAttnArgs &a, const BatchMeta &meta, int M, hipStream_t s) {
  if (M < 1) return;
  const dim3 gq(M, ceil_div(a.n_q_heads, 4)), gk(M, ceil_div(a.n_kv_heads, 4));
  if (a.head_dim == 128) {
    hipLaunchKernelGGL((attn_train_bwd_dq_kernel<128>), gq, dim3(256), 0, s, a, meta);
    hipLaunchKernelGGL((attn_train_bwd_dkv_kernel<128>), gk, dim3(256), 0, s, a, meta);
  } else {
    hipLaunchKernelGGL((attn_train_bwd_dq_kernel<64>), gq, dim3(256), 0, s, a, meta);
    hipLaunchKernelGGL((attn_train_bwd_dkv_kernel<64>), gk, dim3(256), 0, s, a, meta);
  }
}

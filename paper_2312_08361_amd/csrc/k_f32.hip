// Single-precision mode of the span (span_config.weight_bits == 32): fp32 weights, fp32 attention cache,
// fp32 arithmetic throughout, for the configuration that asks for fp32 weights (a tiny span) and for
// checking the path's control logic -- sessions, pages, positions, head mapping -- against the oracle
// without bf16 rounding in the way.  Plain kernels, one wave per output element or per (token, head);
// no matrix cores (their fp32 form would change nothing at these sizes).  Every reduction has a fixed
// order, so results are reproducible run to run.
#include "common.h"
#include "epilogue.h"
#include "launch.h"

namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// x . w over K elements, lanes striding over k; every lane returns the sum
__device__ __forceinline__ float wave_dot(const float *__restrict__ x, const float *__restrict__ w, int K, int lane) {
  float acc = 0.0f;
  for (int k = lane; k < K; k += 64) acc = fmaf(x[k], w[k], acc);
  return wave_sum(acc);
}

__device__ __forceinline__ float silu_exact(float z) { return z / (1.0f + expf(-z)); }
__device__ __forceinline__ float gelu_tanh_exact(float z) {
  const float c = 0.7978845608028654f;
  return 0.5f * z * (1.0f + tanhf(c * (z + 0.044715f * z * z * z)));
}

// element offsets in the fp32 pool: [block][page][K | V][kv head][slot][hd]
__device__ __forceinline__ size_t f32_kv_off(const F32Pool &p, int blk, int pg, int which, int kh, int slot) {
  return (((((size_t)blk * p.max_pages + pg) * 2 + which) * p.n_kv_heads + kh) * SPAN_PAGE + slot) * p.head_dim;
}

// One workgroup (one wave) per token row: h = norm(x) * g (+ b); the first block of a call also
// copies the call's input rows into the residual stream.
__global__ __launch_bounds__(64) void f32_norm_kernel(const float *x_in, float *resid, const float *gain, const float *bias,
                                                      int layernorm, float eps, int d, float *h) {
  const int m = blockIdx.x, lane = threadIdx.x;
  const float *src = x_in ? x_in + (size_t)m * d : resid + (size_t)m * d;
  float s = 0.0f;
  for (int k = lane; k < d; k += 64) s += layernorm ? src[k] : src[k] * src[k];
  s = wave_sum(s);
  float mean = 0.0f, rstd;
  if (layernorm) {
    mean = s / (float)d;
    float q = 0.0f;
    for (int k = lane; k < d; k += 64) { const float c = src[k] - mean; q += c * c; }
    rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
  } else {
    rstd = 1.0f / sqrtf(s / (float)d + eps);
  }
  for (int k = lane; k < d; k += 64) {
    const float v = src[k];
    if (x_in) resid[(size_t)m * d + k] = v;
    float o = (v - mean) * rstd * gain[k];
    if (layernorm) o += bias[k];
    h[(size_t)m * d + k] = o;
  }
}

// q/k/v projection + bias + rotary + cache append.  One wave per (token, head, i < hd/2): the two
// outputs i and i + hd/2 of the head, which the rotary embedding mixes.
__global__ __launch_bounds__(64) void f32_qkv_kernel(F32Block w, const float *h, int d, int Hq, int Hkv, int hd, int rotary,
                                                     const float *rope, float *q_out, F32Pool pool, int block,
                                                     const int *page_table, int pps, BatchMeta meta) {
  const int half = hd >> 1, lane = threadIdx.x;
  const int unit = blockIdx.x, m = blockIdx.y;
  const int head = unit / half, i = unit % half;
  const float *W, *bvec;
  int hl;                                              // head index inside its matrix
  if (head < Hq) { W = w.wq; bvec = w.bq; hl = head; }
  else if (head < Hq + Hkv) { W = w.wk; bvec = w.bk; hl = head - Hq; }
  else { W = w.wv; bvec = w.bv; hl = head - Hq - Hkv; }
  const int n0 = hl * hd + i, n1 = n0 + half;
  const float *x = h + (size_t)m * d;
  float a = wave_dot(x, W + (size_t)n0 * d, d, lane), b = wave_dot(x, W + (size_t)n1 * d, d, lane);
  if (bvec) { a += bvec[n0]; b += bvec[n1]; }
  const TokInfo ti = token_info(meta, m);
  const bool is_v = head >= Hq + Hkv;
  if (rotary && !is_v) {
    const float c = rope[((size_t)ti.pos * half + i) * 2], s = rope[((size_t)ti.pos * half + i) * 2 + 1];
    const float ra = a * c - b * s, rb = a * s + b * c;
    a = ra; b = rb;
  }
  if (lane != 0) return;
  if (head < Hq) {
    float *q = q_out + ((size_t)m * Hq + head) * hd;
    q[i] = a; q[i + half] = b;
  } else {
    const int pg = page_table[(size_t)ti.slot * pps + (ti.pos >> 4)];
    float *dst = pool.base + f32_kv_off(pool, block, pg, is_v ? 1 : 0, hl, ti.pos & 15);
    dst[i] = a; dst[i + half] = b;
  }
}

// Attention of one (token, query head) over the session's cache, keys in order, running softmax.
// A lane owns hd/64 dimensions of the head.
template <int PER>
__global__ __launch_bounds__(64) void f32_attn_kernel(const float *q, F32Pool pool, int block, const int *page_table, int pps,
                                                      int Hq, int Hkv, const float *alibi, float *o_out, BatchMeta meta) {
  constexpr int HD = 64 * PER;
  const int head = blockIdx.x, m = blockIdx.y, lane = threadIdx.x;
  const TokInfo ti = token_info(meta, m);
  const int kh = head / (Hq / Hkv);
  const float scale = 1.0f / sqrtf((float)HD), slope = alibi ? alibi[head] : 0.0f;
  float qv[PER], o[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) { qv[e] = q[((size_t)m * Hq + head) * HD + e * 64 + lane]; o[e] = 0.0f; }
  float mx = -INFINITY, l = 0.0f;
  const int *ptrow = page_table + (size_t)ti.slot * pps;
  for (int j = 0; j <= ti.pos; ++j) {
    const int pg = ptrow[j >> 4];
    const float *k = pool.base + f32_kv_off(pool, block, pg, 0, kh, j & 15);
    const float *v = pool.base + f32_kv_off(pool, block, pg, 1, kh, j & 15);
    float part = 0.0f;
#pragma unroll
    for (int e = 0; e < PER; ++e) part = fmaf(qv[e], k[e * 64 + lane], part);
    const float s = wave_sum(part) * scale - slope * (float)(ti.pos - j);
    const float m_new = fmaxf(mx, s);
    const float alpha = expf(mx - m_new), p = expf(s - m_new);      // first key: exp(-inf) = 0
    l = l * alpha + p;
#pragma unroll
    for (int e = 0; e < PER; ++e) o[e] = o[e] * alpha + p * v[e * 64 + lane];
    mx = m_new;
  }
#pragma unroll
  for (int e = 0; e < PER; ++e) o_out[((size_t)m * Hq + head) * HD + e * 64 + lane] = o[e] / l;
}

// resid[m][n] += x[m] . W[n] (+ b[n]); optionally the call's output row as well
__global__ __launch_bounds__(64) void f32_resid_kernel(const float *x, int K, const float *W, const float *bvec, float *resid,
                                                       int N, float *y) {
  const int n = blockIdx.x, m = blockIdx.y, lane = threadIdx.x;
  float v = wave_dot(x + (size_t)m * K, W + (size_t)n * K, K, lane);
  if (lane != 0) return;
  if (bvec) v += bvec[n];
  v += resid[(size_t)m * N + n];
  resid[(size_t)m * N + n] = v;
  if (y) y[(size_t)m * N + n] = v;
}

// act[m][f] = silu(h . Wg[f]) * (h . Wu[f])   or   gelu(h . W1[f] + b1[f])
__global__ __launch_bounds__(64) void f32_up_kernel(const float *h, int d, const float *w_gate, const float *w_up,
                                                    const float *b_up, int F, float *act) {
  const int f = blockIdx.x, m = blockIdx.y, lane = threadIdx.x;
  const float *x = h + (size_t)m * d;
  float u = wave_dot(x, w_up + (size_t)f * d, d, lane);
  float a;
  if (w_gate) a = silu_exact(wave_dot(x, w_gate + (size_t)f * d, d, lane)) * u;
  else a = gelu_tanh_exact(u + b_up[f]);
  if (lane == 0) act[(size_t)m * F + f] = a;
}

__global__ void f32_kv_gather_kernel(F32Pool pool, int block, const int *ptrow, int pos0, int n, float *k_out, float *v_out) {
  const int hd = pool.head_dim, Hkv = pool.n_kv_heads;
  const size_t total = (size_t)n * Hkv * hd;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int h = i % hd, kh = (i / hd) % Hkv, t = i / ((size_t)hd * Hkv);
    const int pos = pos0 + t, pg = ptrow[pos >> 4];
    if (k_out) k_out[i] = pool.base[f32_kv_off(pool, block, pg, 0, kh, pos & 15) + h];
    if (v_out) v_out[i] = pool.base[f32_kv_off(pool, block, pg, 1, kh, pos & 15) + h];
  }
}

// one workgroup per (copy, block): a page's keys and values of all kv heads are one contiguous run
__global__ __launch_bounds__(256) void f32_page_copy_kernel(F32Pool pool, int first_block, PageCopies pc) {
  const int blk = first_block + blockIdx.y;
  const size_t n4 = (size_t)2 * pool.n_kv_heads * SPAN_PAGE * pool.head_dim / 4;
  const f32x4 *src = (const f32x4 *)(pool.base + f32_kv_off(pool, blk, pc.src[blockIdx.x], 0, 0, 0));
  f32x4 *dst = (f32x4 *)(pool.base + f32_kv_off(pool, blk, pc.dst[blockIdx.x], 0, 0, 0));
  for (size_t i = threadIdx.x; i < n4; i += blockDim.x) dst[i] = src[i];
}

}  // namespace

void launch_f32_block(const F32Call &c, const F32Block &w, const BatchMeta &meta, int block, bool first, float *y,
                      hipStream_t s) {
  const int M = meta.cu[meta.n_sess];
  const int nqkv_heads = c.Hq + 2 * c.Hkv;
  hipLaunchKernelGGL(f32_norm_kernel, dim3(M), dim3(64), 0, s, first ? c.x_in : nullptr, c.resid, w.norm1_g, w.norm1_b,
                     c.layernorm, c.eps, c.d, c.h);
  hipLaunchKernelGGL(f32_qkv_kernel, dim3(nqkv_heads * (c.hd / 2), M), dim3(64), 0, s, w, c.h, c.d, c.Hq, c.Hkv, c.hd,
                     c.rotary, c.rope, c.q, c.pool, block, c.page_table, c.pps, meta);
  if (c.hd == 128)
    hipLaunchKernelGGL(f32_attn_kernel<2>, dim3(c.Hq, M), dim3(64), 0, s, c.q, c.pool, block, c.page_table, c.pps, c.Hq,
                       c.Hkv, c.alibi, c.o, meta);
  else
    hipLaunchKernelGGL(f32_attn_kernel<1>, dim3(c.Hq, M), dim3(64), 0, s, c.q, c.pool, block, c.page_table, c.pps, c.Hq,
                       c.Hkv, c.alibi, c.o, meta);
  hipLaunchKernelGGL(f32_resid_kernel, dim3(c.d, M), dim3(64), 0, s, c.o, c.Hq * c.hd, w.wo, w.bo, c.resid, c.d, (float *)nullptr);
  hipLaunchKernelGGL(f32_norm_kernel, dim3(M), dim3(64), 0, s, (const float *)nullptr, c.resid, w.norm2_g, w.norm2_b,
                     c.layernorm, c.eps, c.d, c.h);
  hipLaunchKernelGGL(f32_up_kernel, dim3(c.F, M), dim3(64), 0, s, c.h, c.d, w.w_gate, w.w_up, w.b_up, c.F, c.act);
  hipLaunchKernelGGL(f32_resid_kernel, dim3(c.d, M), dim3(64), 0, s, c.act, c.F, w.w_down, w.b_down, c.resid, c.d, y);
}

void launch_f32_kv_gather(const F32Pool &pool, int block, const int *page_table_row, int pos0, int n, float *k_out,
                          float *v_out, hipStream_t s) {
  const size_t total = (size_t)n * pool.n_kv_heads * pool.head_dim;
  int grid = (int)((total + 255) / 256);
  if (grid > 4096) grid = 4096;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(f32_kv_gather_kernel, dim3(grid), dim3(256), 0, s, pool, block, page_table_row, pos0, n, k_out, v_out);
}

void launch_f32_page_copy(const F32Pool &pool, int first_block, int n_blocks, const PageCopies &pc, hipStream_t s) {
  if (pc.n < 1) return;
  hipLaunchKernelGGL(f32_page_copy_kernel, dim3(pc.n, n_blocks), dim3(256), 0, s, pool, first_block, pc);
}

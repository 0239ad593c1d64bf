// Shared device-side types and memory layouts of the block-span kernels (gfx950 only).
//
// Layouts (all bf16 unless noted)
// -------------------------------
// T16: a matrix X[rows, K] stored as tiles of 16 rows x 32 k.  Tile (rt, kt) is one
//      contiguous 1 KiB block at tile index rt*s_rt + kt*s_kt.  All buffers are k-major
//      (s_rt = 1, s_kt = number of row tiles): the row tiles of one k step are adjacent, so
//      a workgroup that needs many row tiles of the same k reads one long contiguous run
//      and concurrent workgroups spread over all memory channels (a row-tile-major order
//      puts them a power-of-two stride apart, i.e. all on one channel).
//      Inside a tile, 16-byte chunk number (g*16 + r) holds
//      X[rt*16 + r][kt*32 + g*8 .. +8].  A 64-lane wave that loads chunk `lane` gets
//      exactly the operand registers of v_mfma_f32_16x16x32_bf16 (row = lane%16,
//      k-group = lane/16) with one fully coalesced 1 KiB read; two such tiles form an
//      operand of v_mfma_f32_32x32x16_bf16.  Packed weights, and every activation
//      buffer that feeds a projection, use T16.
// K page: keys of 16 consecutive tokens of one kv head: [hd/32][64 chunks][8], chunk
//      (g*16 + slot) of k-step j holds K[slot][j*32 + g*8 .. +8]   (= T16 with rows = slots).
// V page: values of the same 16 tokens, transposed for the P.V product:
//      [hd/32][64 chunks][2][4]; chunk (g*16 + r) of c2, half `par`, holds
//      V[slot g*4 .. +4][(2*c2 + par)*16 + r].
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;   // raw bf16 bits
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#include <utility>

// compile-time loop: f(std::integral_constant<int, 0>{}) ... f(<N-1>); indices stay
// constant expressions whatever the optimiser's unrolling heuristics decide
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

#define SPAN_PAGE 16
#define SPAN_MAX_CALL 64

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ inline int round_up(int a, int b) { return ceil_div(a, b) * b; }

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// round to nearest, ties to even (inputs are finite on this path)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// two at a time with the hardware conversion (v_cvt_pk_bf16_f32, round to nearest even)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// element offset of X[row][k] in a k-major T16 buffer with RT row tiles per k step
__host__ __device__ __forceinline__ size_t t16_off(int row, int k, int RT) {
  return ((size_t)(k >> 5) * RT + (row >> 4)) * 512 + ((((k & 31) >> 3) * 16 + (row & 15)) << 3) + (k & 7);
}
// element offset inside a K page (16 slots x hd) of K[slot][h]
__device__ __forceinline__ int kpage_off(int slot, int h) {
  return (h >> 5) * 512 + ((((h & 31) >> 3) * 16 + slot) << 3) + (h & 7);
}
// element offset inside a V page of V[slot][h]
__device__ __forceinline__ int vpage_off(int slot, int h) {
  int c = h >> 4, r = h & 15;
  return (((c >> 1) * 64 + (slot >> 2) * 16 + r) * 2 + (c & 1)) * 4 + (slot & 3);
}

// Per-call batch description, passed by value to the kernels that need to know which
// session a token row belongs to.  Rows are grouped by session: session i owns rows
// [cu[i], cu[i+1]); it held past[i] tokens before this call; slot[i] is its row in the
// device page table.
struct BatchMeta {
  int n_sess;
  int cu[SPAN_MAX_CALL + 1];
  int past[SPAN_MAX_CALL];
  int slot[SPAN_MAX_CALL];
};

// Addressing of the paged KV pool: page `pg` of block `blk`, kv head `kh`.
struct KvPool {
  bf16_t *base;
  int max_pages, n_kv_heads, head_dim;
  __host__ __device__ size_t head_elems() const { return (size_t)SPAN_PAGE * head_dim; }
  __host__ __device__ size_t k_off(int blk, int pg, int kh) const {
    return ((((size_t)blk * max_pages + pg) * 2 + 0) * n_kv_heads + kh) * head_elems();
  }
  __host__ __device__ size_t v_off(int blk, int pg, int kh) const {
    return ((((size_t)blk * max_pages + pg) * 2 + 1) * n_kv_heads + kh) * head_elems();
  }
};

// What a projection kernel does with its accumulators.
enum EpiKind {
  EPI_PLAIN = 0,   // out[m][n] = acc (fp32)                      -- operator tests
  EPI_QKV = 1,     // + bias, rotary, q -> q buffer, k/v -> pages
  EPI_RESID = 2,   // resid[m][n] += acc + bias, optional cast to y
  EPI_SWIGLU = 3,  // a[m][f] = silu(gate) * up  -> T16
  EPI_GELU = 4,    // a[m][f] = gelu(acc + bias) -> T16
  EPI_ACTBWD = 5   // backward pass, tiled kernels only: acc = gradient of a[m][f]; writes the gradient of the
                   // pre-activations (gate | up, or the GELU input) as the T16 input of the next projection
};

struct EpiArgs {
  int kind;
  int M;                 // valid token rows
  int m0;                // skinny kernels: row of the call that the launch's first token row is (a launch may
                         // cover the tail rows of a longer call; M stays the call's row count)
  int N;                 // valid logical output features
  // EPI_PLAIN
  float *out;
  int accumulate;        // out += acc instead of out = acc (a contraction split along k over several launches)
  // bias (fp32, indexed by logical feature) or null
  const float *bias;
  // EPI_QKV
  int n_q_heads, n_kv_heads, head_dim, rotary;
  const float *rope;     // [pos][hd/2][2] = (cos, sin)
  bf16_t *q_out;         // [M][Hq*hd] row-major
  KvPool pool;
  int block;             // absolute block index in the pool
  const int *page_table; // device [max_sessions][pages_per_session]
  int pages_per_session;
  // EPI_RESID
  float *resid;          // [M][N] fp32
  void *y;               // optional final output [M][N]
  int y_f32;
  // EPI_SWIGLU / EPI_GELU
  bf16_t *act_out;       // T16 with act_RT row tiles per k step
  int act_RT;
  // training-time passes (no cache): what the backward pass needs later, in fp32 row-major
  KvPool pool2;          // EPI_QKV, base != null: second copy of the new keys and values with the layouts swapped
                         // (keys in the transposed V-page layout, values in the row-wise K-page layout): the
                         // operands of the attention backward pass
  float *gu_plain;       // EPI_SWIGLU: [M][2 N] gate | up before the activation; EPI_GELU: [M][N] likewise
                         // (EPI_ACTBWD reads them back)
  int gated;             // EPI_ACTBWD: 1 = SwiGLU, 0 = GELU

  // ---- norm fused across the skinny (decode) kernels; all null / 0 otherwise -------------
  // Producer side (EPI_RESID): besides the new residual x', emit bf16(x' * next_gain) as the
  // next projection's T16 input and, per workgroup, the partial sums of x'^2 (and of x' for
  // LayerNorm) of its 32 features: stat_out[part][0/1][64 tokens].
  const float *next_gain;
  bf16_t *h_out;
  int h_RT;
  float *stat_out;
  // Consumer side (EPI_QKV / EPI_SWIGLU / EPI_GELU): the input was only scaled by the gain;
  // finish the norm on the accumulators: y = r * (acc - mu * wg) + bias', with
  // r = rsqrt(var + eps) from the producer's partial sums, wg = W.gain (LayerNorm only) and
  // bias' = W.beta + bias folded into `bias` by the host.
  const float *stat_in;
  int stat_parts;
  // The same fusion in the tiled kernels (long calls).  Producer (EPI_RESID with next_gain / h_out set and
  // stat_out null): per (token row, 128 features) the partial sums go to tstat_out[part][tstat_ld rows][2];
  // a small kernel turns them into row_stat[row] = (1/sqrt(var + eps), mean), which the consumer's
  // epilogue reads instead of summing partials itself (stat_in is then just non-null).
  float *tstat_out;
  int tstat_ld;
  const float *row_stat;
  int norm_d;
  float norm_eps;
  int norm_center;       // 1 = LayerNorm (subtract the mean), 0 = RMSNorm
  const float *wg;
  // LayerNorm only: shift[m] = the mean the previous norm found for token row m.  A producer writes
  // bf16((x' - shift) * gain) and sums (x' - shift), (x' - shift)^2, so that neither the bf16 rounding of
  // the projection's input nor the one-pass variance loses digits when a row's mean is large against its
  // spread (the residual stream's mean moves little from one norm to the next); the consumer's formula is
  // unchanged (its mean is the shifted one) and it adds that mean to shift[m] for the next producer.
  float *shift;
};

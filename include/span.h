/*
 * span.h -- C ABI of the block-span inference server path for MI355X (gfx950).
 *
 * One `span_t` is what the paper calls a server: a set of consecutive transformer
 * blocks resident on one GPU (Section 3.2), serving many client sessions at once
 * (Section 4.2, concurrent clients).  The calls mirror the life cycle of an inference
 * stream in Algorithm 2 (rpc_inference): open -> send(inputs) repeatedly -> close, and
 * the cache replay of Algorithm 3 (a fresh stream receives all stored past inputs in
 * one request and returns the outputs of every position).
 *
 * General rules
 *  - Every function returns SPAN_OK (0) or a negative span_status.  Nothing throws,
 *    nothing aborts.  span_last_error() gives a thread-local message for the last
 *    failure on the calling thread.
 *  - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *    ordinary host memory.  The library never allocates or frees device memory: the
 *    caller provides three arenas (packed weights, KV page pool, workspace) whose sizes
 *    come from span_query_sizes() and which must stay alive until span_destroy().
 *  - Kernels are enqueued on the hipStream_t the caller passes (as void*); the call
 *    returns after enqueueing.  Host-side session state (lengths, page tables) is
 *    updated at enqueue time.  The caller synchronises the stream before reading y.
 *    Calls on one span must be issued from one thread at a time and on one stream (or on
 *    streams the caller orders itself): the workspace is shared by consecutive calls.
 *  - A call that returns an error leaves every session's length and page table as they
 *    were (Algorithm 1 records an input as sent only after the send succeeded, and then
 *    retries, so a failed request must not advance the server-side cache).
 *  - The product path has no CPU fallback: without a GPU every compute call fails with
 *    SPAN_E_HIP, except on a span created with `dry_run` (host bookkeeping only).
 */
#ifndef SPAN_H_
#define SPAN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPAN_MAX_CALL_SESSIONS 64   /* sessions batched in one forward / replay call   */

typedef enum span_status {
  SPAN_OK = 0,
  SPAN_E_INVALID = -1,        /* bad argument or configuration                          */
  SPAN_E_BAD_SESSION = -2,    /* handle is not an open session of this span             */
  SPAN_E_CACHE_FULL = -3,     /* not enough free KV pages for the request               */
  SPAN_E_TOO_LONG = -4,       /* session length would exceed the max_len it was opened with */
  SPAN_E_MIXED_SPANS = -5,    /* sessions of one call are open on different block ranges */
  SPAN_E_DUPLICATE = -6,      /* the same session appears twice in one call             */
  SPAN_E_HIP = -7,            /* a HIP runtime call failed (message has the HIP error)  */
  SPAN_E_TOO_MANY_TOKENS = -8,/* a forward call carries more tokens than max_batch_tokens */
  SPAN_E_NOT_EMPTY = -9,      /* replay on a session that already holds tokens          */
  SPAN_E_NO_SLOT = -10        /* max_sessions sessions are already open                 */
} span_status;

enum { SPAN_ARCH_LLAMA = 0, SPAN_ARCH_BLOOM = 1 };
enum { SPAN_IO_BF16 = 0, SPAN_IO_F32 = 1 };

/*
 * Shape of the span.  The paper takes the block from Llama 2 / BLOOM by citation
 * (Section 4.2); the two styles are
 *   LLAMA: RMSNorm, q/k/v projections without bias, rotary position embedding
 *          (half-split pairing, position = index of the token in its session),
 *          grouped-query attention, SwiGLU MLP;
 *   BLOOM: LayerNorm, projections with bias, ALiBi logit bias -slope_h*(i-j),
 *          multi-head attention, tanh-GELU MLP.
 * Constraints: head_dim in {64,128}; n_q_heads % n_kv_heads == 0 with a ratio <= 16;
 * d_model, n_q_heads*head_dim multiples of 32; d_ff a multiple of 16; page_tokens == 16.
 */
typedef struct span_config {
  int32_t arch;              /* SPAN_ARCH_*                                             */
  int32_t n_blocks;          /* blocks held by this server                              */
  int32_t d_model;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  int32_t d_ff;
  float   norm_eps;
  float   rope_base;         /* LLAMA only                                              */
  int32_t page_tokens;       /* tokens per KV page (16)                                 */
  int32_t max_pages;         /* pages in the KV pool (each page spans all blocks)       */
  int32_t max_sessions;      /* simultaneously open sessions                            */
  int32_t max_session_tokens;/* upper bound on any session's max_len                    */
  int32_t max_batch_tokens;  /* most tokens one span_forward call may carry; span_replay
                                splits longer requests into chunks of this size         */
  int32_t io_dtype;          /* SPAN_IO_*: element type of x and y                      */
  int32_t dry_run;           /* 1: host bookkeeping only, no device work (tests, sizing) */
  int32_t weight_bits;       /* 0 or 16: weights kept in bf16; 8 or 4: compressed, see below;
                                32: single-precision mode, see below                        */
  float   levels[16];        /* weight_bits == 4: the 16 ascending levels of the codebook     */
} span_config;

/*
 * Compressed weights (Section 3.1, "Compression": the paper's servers hold 8-bit weights for
 * BLOOM and 4-bit NormalFloat weights for Llama 2).  With weight_bits 8 or 4, span_create()
 * encodes every projection matrix into an absmax block format and keeps only that:
 * a row [in_features] is cut into blocks of 64 consecutive input features, a block is stored
 * as its largest magnitude (fp32) and one code per element,
 *   8: code = round_to_nearest_even(w / absmax * 127),         w' = code * (absmax / 127)
 *   4: code = index of the level nearest to w / absmax (ties to the lower level; levels[] is
 *      any strictly ascending table in [-1, 1], e.g. the NormalFloat one; the library rounds
 *      the levels to bf16, the precision in which they meet the hidden states),
 *                                                             w' = levels[code] * absmax
 * decided in fp32 in the order written.  The span then computes with the dequantised matrices
 * w'; hidden states, norms, biases and the attention cache are unchanged.  Calls of up to 64
 * tokens stream the codes through the weight-streaming kernels (the products with the codes are
 * exact, the block scale is applied in fp32).  Longer calls expand one matrix at a time into a
 * bf16 scratch copy (w' rounded to bf16) for the tiled kernels; the workspace grows by the size of
 * the largest matrix in bf16.
 */

/*
 * Single-precision mode (weight_bits == 32): the canonical weights are fp32 (same shapes, row-major),
 * io_dtype must be SPAN_IO_F32, and the span keeps fp32 copies of the weights, an fp32 attention cache
 * (kv_bytes doubles) and computes every step in fp32 with plain (non-matrix-core) kernels.  It is
 * the mode of the configuration that specifies fp32 weights (a tiny two-block span) and the way to
 * check sessions, pages, positions and head mapping against the oracle without bf16 rounding;
 * it is not tuned (one wave per output element) and takes at most 65535 tokens per call.
 * Sessions, span_forward / span_replay / span_reorder and the span_debug_* readers work as in bf16
 * mode (span_debug_read_kv then returns fp32); span_debug_tap and the training-time passes return
 * SPAN_E_INVALID.
 */

/*
 * Canonical weights of one block: device pointers to bf16 (fp32 in single-precision mode), row-major
 * [out_features, in_features] for matrices (y = x W^T + b), plain vectors otherwise.
 * LLAMA uses norm1_g, wq, wk, wv, wo, norm2_g, w_gate, w_up, w_down (others NULL);
 * BLOOM uses everything except w_gate.  Shapes: wq [Hq*hd, d], wk/wv [Hkv*hd, d],
 * wo [d, Hq*hd], w_gate/w_up [d_ff, d], w_down [d, d_ff].
 * span_create() copies them into its own packed layout; the caller may free them after
 * the stream passed to span_create() has been synchronised.
 */
typedef struct span_block_weights {
  const void *norm1_g, *norm1_b;
  const void *wq, *bq, *wk, *bk, *wv, *bv;
  const void *wo, *bo;
  const void *norm2_g, *norm2_b;
  const void *w_gate, *w_up, *b_up;
  const void *w_down, *b_down;
} span_block_weights;

typedef struct span_t span_t;           /* opaque server state                          */
typedef int32_t span_session_t;         /* session handle; never reused while open      */

/* Bytes the caller must provide for the three device arenas (each 256-byte aligned). */
int span_query_sizes(const span_config *cfg, size_t *weight_bytes, size_t *kv_bytes,
                     size_t *workspace_bytes);

/*
 * Build a server.  `weights` is a host array of n_blocks structs holding device
 * pointers (ignored when cfg->dry_run).  Packing kernels and a clear of the workspace
 * are enqueued on `stream`.  On success *out owns only host metadata.
 */
int span_create(const span_config *cfg, const span_block_weights *weights,
                void *weight_arena, void *kv_arena, void *workspace, void *stream,
                span_t **out);
int span_destroy(span_t *span);

/*
 * Algorithm 2, set-up: open a stream with an empty attention cache for every local
 * layer.  A client may ask for the whole span or a sub-segment of it (Appendix D):
 * blocks [first_block, first_block + n_blocks).  max_len bounds the session's tokens.
 */
int span_session_open(span_t *span, int first_block, int n_blocks, int max_len,
                      span_session_t *out);
/* Close a stream (Algorithm 1, stream.close()); its pages return to the pool. */
int span_session_close(span_t *span, span_session_t session);
int span_session_length(span_t *span, span_session_t session, int *len);

/*
 * Algorithm 2, loop body, batched over sessions: for each listed session, n_tokens[i]
 * new hidden-state rows go through every block of the session's range in order; each
 * block attends over the session's cached keys/values plus the new ones, and the new
 * keys/values are appended to the cache.  n_tokens[i] == 1 is a decode step, > 1 a
 * prefix or a chunk of one, 0 leaves the session untouched.
 *   sessions  host [n_sessions], distinct, all open on the same block range
 *   n_tokens  host [n_sessions], each >= 0, sum <= max_batch_tokens
 *   x         device [sum n_tokens, d_model], io_dtype, rows grouped by session in order
 *   y         device [sum n_tokens, d_model], io_dtype: outputs of every position
 */
int span_forward(span_t *span, int n_sessions, const span_session_t *sessions,
                 const int *n_tokens, const void *x, void *y, void *stream);

/*
 * Cache replay (Algorithm 3, the send of past inputs to a fresh stream): sessions that must be empty receive all
 * stored past inputs at once; y_all holds the outputs of all positions (they feed the
 * next replacement server).  Same layout as span_forward; the total may exceed
 * max_batch_tokens (processed in chunks, cf. the 1024-token micro-batches of Section 4.2).
 * On error the sessions are left empty.
 */
int span_replay(span_t *span, int n_sessions, const span_session_t *sessions,
                const int *n_tokens, const void *x_past, void *y_all, void *stream);

/*
 * Cache reordering for search-based decoding (Section 3.1, last paragraph, and the appendix
 * on beam search): the listed sessions are a beam; after the call sessions[i] continues from
 * the attention cache that sessions[hypo_ids[i]] held before it (a gather over the beam).
 * An entry named several times is cloned, an entry named by nobody loses its cache.
 *   sessions  host [k], distinct, all open on the same block range, 1 <= k <= 64
 *   hypo_ids  host [k], each in [0, k) (0-based; the paper's example counts from 1)
 * The paged cache makes this mostly bookkeeping: full pages are shared by reference, only a
 * source's last, partly filled page is copied for every additional session that continues
 * from it (each session appends into a page of its own).  Needs at most k free pages; with
 * too few the call fails with SPAN_E_CACHE_FULL and nothing has changed.  A source longer
 * than a target's max_len gives SPAN_E_TOO_LONG.  The copies and the page-table update are
 * enqueued on `stream`.
 */
int span_reorder(span_t *span, int k, const span_session_t *sessions, const int *hypo_ids,
                 void *stream);

/*
 * Training-time passes (Section 3.3, "Fine-tuning": the servers keep their parameters frozen,
 * run back-propagation through their blocks and return the gradient with respect to their input
 * activations; forward and backward passes process whole sequences in one go, so there is no
 * session and no attention cache).  A batch is n_seq sequences laid one after the other in x:
 * sequence i owns rows [sum(lens[0..i)), ...) and its tokens sit at positions 0..lens[i]-1 with
 * causal attention among themselves.
 *
 *   span_train_sizes   bytes of the two extra arenas this needs for calls of at most max_tokens
 *                      tokens: transposed packed copies of the projection weights (dX = dY W is
 *                      a projection with W^T as the weight) and scratch that keeps every block's
 *                      intermediate rows between the forward and the backward sweep of one call.
 *   span_train_attach  packs the transposed copies from the same canonical weights that
 *                      span_create took (device, may be freed afterwards) and binds both arenas
 *                      (device, caller-owned, alive until span_destroy); max_tokens <=
 *                      max_batch_tokens.  A span with compressed weights keeps no transposed
 *                      copies (weight_t_bytes is 0; weights and weight_t_arena may be null): each
 *                      backward projection expands its matrix to bf16 in the workspace and turns
 *                      it in scratch for the call, so the gradient belongs to exactly the
 *                      function the forward pass computes with the dequantised weights.
 *   span_train_forward y = blocks [first_block, first_block + n_blocks) applied to x.
 *   span_backward      grad_x = (d y / d x)^T grad_y for the same function: the call runs the
 *                      forward sweep itself (a backward request carries the inputs again, the
 *                      server keeps nothing between requests), then the backward sweep.
 *                      y_out, if not null, receives the forward output as well.
 * x, grad_y, grad_x, y: device [sum(lens), d_model] in the span's io_dtype.  n_seq in
 * [0, SPAN_MAX_CALL_SESSIONS]; lens[i] in [0, max_session_tokens]; sum(lens) <= max_tokens.
 * Sessions and their caches are not touched; the calls share the span's workspace with
 * span_forward (same stream-ordering rule).  Errors: SPAN_E_INVALID (not attached, bad range,
 * null pointer), SPAN_E_TOO_LONG, SPAN_E_TOO_MANY_TOKENS, SPAN_E_HIP.
 */
int span_train_sizes(const span_config *cfg, int max_tokens, size_t *weight_t_bytes, size_t *scratch_bytes);
int span_train_attach(span_t *span, const span_block_weights *weights, void *weight_t_arena, void *scratch,
                      int max_tokens, void *stream);
int span_train_forward(span_t *span, int first_block, int n_blocks, int n_seq, const int *lens, const void *x,
                       void *y, void *stream);
int span_backward(span_t *span, int first_block, int n_blocks, int n_seq, const int *lens, const void *x,
                  const void *grad_y, void *grad_x, void *y_out, void *stream);

/*
 * Hidden states on their way between pipeline stages (Section 3.1, "Compression", last
 * paragraph: block-wise 8-bit quantisation halves the bytes a span's output takes on the wire).
 * Each row [d] is cut into blocks of `block` consecutive features (a multiple of 64, at most
 * 4096); a block becomes its absmax (fp32) and one byte per element, the index of the level
 * nearest to x / absmax (fp32; ties to the lower level) among `levels`, 256 strictly ascending
 * numbers in [-1, 1] on the host (the dynamic 8-bit data type is one such table).
 *   encode: x device [M, d] (fp32 if x_f32 else bf16) -> codes_out device uint8 [M, d],
 *           absmax_out device fp32 [M, ceil(d / block)]
 *   decode: y[m][k] = levels[codes[m][k]] * absmax[m][k / block], device [M, d] (fp32 if y_f32
 *           else bf16, rounded to nearest even)
 * Stateless: no span, no scratch; kernels are enqueued on `stream`.
 */
int span_hidden_encode(const void *x, int x_f32, int M, int d, int block, const float *levels,
                       void *codes_out, float *absmax_out, void *stream);
int span_hidden_decode(const void *codes, const float *absmax, int M, int d, int block,
                       const float *levels, int y_f32, void *y, void *stream);

/* ---- introspection for tests (not used by the serving path) ----------------------- */

/*
 * The encoder of the compressed-weight formats on its own: w device bf16 [N, K] row-major ->
 * codes_out device uint8 [N, K] (int8 codes as two's-complement bytes, codebook codes 0..15)
 * and absmax_out device fp32 [N, ceil(K/64)].  levels: host [16], used when bits == 4.
 * scratch: span_op_lowbit_scratch(1, N, K) bytes.
 */
size_t span_op_lowbit_scratch(int M, int N, int K);
int span_op_quantize(const void *w, int N, int K, int bits, const float *levels, void *codes_out,
                     float *absmax_out, void *scratch, void *stream);
/*
 * y = x W'^T with W' the dequantised form of w (encoded as above, then multiplied by the
 * weight-streaming kernel).  x device bf16 [M, K], M <= 64; y device fp32 [M, N];
 * N a multiple of 16, K a multiple of 8.  scratch: span_op_lowbit_scratch(M, N, K) bytes.
 */
int span_op_linear_lowbit(const void *x, const void *w, float *y, int M, int N, int K, int bits,
                          const float *levels, void *scratch, void *stream);

/* Free pages left in the pool. */
int span_debug_free_pages(span_t *span, int *n_free);
/* Page ids of a session, in order; pages_out host [>= ceil(len/page_tokens)].  After
 * span_reorder two sessions may list the same (full) page. */
int span_debug_page_table(span_t *span, span_session_t session, int32_t *pages_out,
                          int *n_pages);
/*
 * Gather cached keys/values of positions [pos0, pos0+n) of one block (index local to
 * the session's range) into token-major bf16 (single-precision mode: fp32) device arrays [n, n_kv_heads, head_dim].
 */
int span_debug_read_kv(span_t *span, span_session_t session, int block, int pos0, int n,
                       void *k_out, void *v_out, void *stream);

/*
 * Taps into the path's own intermediates, for kernel-level parity of the attention inside a
 * real call (Algorithm 3's replay runs the multi-token attention kernel; the bar on
 * fp32-accumulated logits is checked on what that kernel itself computed).  A tap is armed
 * for the NEXT span_forward call (for span_replay: its first chunk of max_batch_tokens rows)
 * and disarmed when that call returns, whether it succeeded or not; one tap of each kind can be
 * armed at a time; what = 0 disarms all.  `session` must bring tokens in that call; q0, nq
 * select its new tokens [q0, q0 + nq) (0 = the first token of the session in the call); `block`
 * is local to the session's range.  `out` is device memory of out_bytes bytes, written by
 * work enqueued on the call's stream:
 *   SPAN_TAP_Q_ROT   bf16 [nq, n_q_heads * head_dim]   queries after bias and rotary embedding, as
 *                    the attention kernel reads them (`head` ignored)
 *   SPAN_TAP_K_ROT   bf16 [nq, n_kv_heads * head_dim]  keys of the same tokens after the rotary
 *                    embedding, read back from the cache pages (`head` ignored)
 *   SPAN_TAP_LOGITS  fp32 [nq, ld], ld = the session's length after the call: row i holds
 *                    logit(query token q0 + i of head `head`, key position j) = q.k / sqrt(head_dim)
 *                    (- slope_head * distance for BLOOM) for j <= the query's position; later
 *                    entries are left untouched.  Multi-token calls only (they run the attention
 *                    kernel of prefill / replay; a tapped call runs a variant of it that differs
 *                    only in these stores).
 * A tap that does not fit the call (session without tokens in it, range beyond its new tokens,
 * out_bytes too small, logits tap on a call of single tokens) makes that call fail with
 * SPAN_E_INVALID before anything is enqueued; sessions are unchanged.
 */
enum { SPAN_TAP_Q_ROT = 1, SPAN_TAP_K_ROT = 2, SPAN_TAP_LOGITS = 3 };
int span_debug_tap(span_t *span, int what, int block, span_session_t session, int head, int q0, int nq,
                   void *out, size_t out_bytes);

/*
 * Per-kernel timing for the roofline report.  While enabled, every kernel launch of
 * span_forward / span_replay is bracketed by HIP events on the caller's stream (this
 * perturbs step time slightly; leave it off when timing whole steps).  span_debug_profile
 * (span, 1) also clears earlier records.  span_debug_profile_read synchronises on the
 * recorded events and returns the number of launches and their summed duration in
 * milliseconds for one kernel class.
 */
enum {
  SPAN_K_NORM = 0,          /* RMSNorm / LayerNorm                                      */
  SPAN_K_SKINNY = 1,        /* weight-streaming projection (decode)                     */
  SPAN_K_TILED = 2,         /* LDS-tiled MFMA projection (prefill / replay)             */
  SPAN_K_ATTN_DECODE = 3,   /* split-KV decode attention                                */
  SPAN_K_ATTN_MERGE = 4,    /* merge of the split partials                              */
  SPAN_K_ATTN_PREFILL = 5,  /* causal attention over new + cached tokens                */
  SPAN_K_CLASSES = 6
};
int span_debug_profile(span_t *span, int enable);
int span_debug_profile_read(span_t *span, int kernel_class, int *n_launches, float *total_ms);

/*
 * Practical ceilings of the device, printed beside the rooflines: the rate of a pure streaming
 * read of `bytes` of `buf` (device, 16-byte aligned, bytes a multiple of 16; GB/s) and of a
 * register-only loop of 32x32x16 bf16 MFMAs whose operands are the first 32 KiB of `buf`
 * (TFLOP/s; the rate depends on those bits through the chip's power management).  `out`: device
 * scratch of 256 KiB.  Synchronises the stream; each figure is the best of three runs.
 */
int span_debug_ceilings(const void *buf, size_t bytes, void *out, float *read_gbs, float *mfma_tflops,
                        void *stream);

/* ---- single operators, for kernel-level parity and micro-benchmarks --------------- */

/*
 * y[M,N] (fp32, device, row-major) = x[M,K] W[N,K]^T with bf16 x and W (device,
 * row-major), fp32 accumulation.  path 0 = weight-streaming skinny kernel (M <= 64),
 * path 1 = MFMA LDS-tiled kernel.  scratch: device, >= span_op_linear_scratch(M,N,K).
 */
size_t span_op_linear_scratch(int M, int N, int K);
int span_op_linear(const void *x, const void *w, float *y, int M, int N, int K, int path,
                   void *scratch, void *stream);

/*
 * Attention of one new query per session over token-major caches, through the paged
 * kernels.  q [B, Hq, hd] bf16; k, v [B, L_max, Hkv, hd] bf16 (session b uses the first
 * lens[b] rows; the query sits at position lens[b]-1, i.e. its own key is row lens[b]-1);
 * out [B, Hq, hd] fp32; logits (may be NULL) [B, Hq, L_max] fp32 receives the scaled
 * (and ALiBi-biased when alibi != 0) pre-softmax logits.  lens: host [B], 1..L_max.
 */
size_t span_op_attn_decode_scratch(int B, int L_max, int Hq, int Hkv, int hd);
int span_op_attn_decode(const void *q, const void *k, const void *v, const int *lens,
                        int B, int L_max, int Hq, int Hkv, int hd, int alibi, float *out,
                        float *logits, void *scratch, void *stream);

/*
 * span_op_attn_decode for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments (without `scratch`), same kernels, same results; the scratch is an array of
 * SPAN_STATIC_SCRATCH_MIB MiB that the library's code object itself holds on every GPU it is
 * loaded on, for the life of the process.  The call allocates and frees nothing (its first call
 * on a device looks the array's device address up, once).  A shape whose scratch
 * (span_op_attn_decode_scratch) exceeds the array returns SPAN_E_INVALID and enqueues nothing.
 * All calls on one GPU share the array, which keeps the previous call's contents; the call clears
 * what it needs cleared, with a kernel on `stream`.  Calls on one GPU must therefore not overlap:
 * issue them on one stream, or order the streams yourself; concurrent calls race.
 */
#define SPAN_STATIC_SCRATCH_MIB 64
int span_op_attn_decode_static(const void *q, const void *k, const void *v, const int *lens,
                               int B, int L_max, int Hq, int Hkv, int hd, int alibi, float *out,
                               float *logits, void *stream);

const char *span_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SPAN_H_ */

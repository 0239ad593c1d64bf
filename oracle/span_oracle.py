"""CPU oracle for a server's forward pass through a span of transformer blocks.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
path is checked against.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it; the product path never does and
shares no code, tables or constants with it.

What it follows
---------------
* Session semantics: Algorithm 2 (rpc_inference) of the paper.  A session holds
  one attention cache per local layer; each request runs
  ``inputs, new_kv = forward(layer, inputs, past_kv)`` layer by layer and appends
  ``new_kv``.  A multi-token request (the prefix of Algorithm 1, or the replay of
  past inputs in Algorithm 3) is the same call with T > 1 and returns the outputs
  of all T positions.
* What ``forward(layer, ...)`` computes: the paper names Llama 2 and BLOOM blocks
  by citation only (Section 4.2), so the block arithmetic below is the public
  textbook definition of those operators (pre-norm residual blocks; RMSNorm +
  rotary + grouped-query attention + SwiGLU for the Llama style; LayerNorm +
  ALiBi + multi-head attention + tanh-GELU MLP with biases for the BLOOM style).
  Block math overall is therefore "parity unpinned by the paper"; it is pinned by
  closed forms, invariants and library special cases in tests/test_oracle_*.py.
* Truth for caching: Section 2.1 / 3.2 -- cached generation is an exact
  reformulation of recomputing the whole sequence with causal attention.
  ``span_full`` is that plain definition (no cache at all); ``Session`` is the
  cached form.  They are compared by brute force in the tests.

Conventions (every reading of an under-specified point lives here)
------------------------------------------------------------------
* weights are [out_features, in_features]; y = x @ W.T (+ b).
* rotary: half-split pairing (i, i + head_dim/2), angle = pos * base**(-2i/head_dim),
  pos = absolute 0-based index of the token in the session.
* grouped-query attention: query head h reads kv head h // (n_q_heads // n_kv_heads).
* logits = q.k / sqrt(head_dim)  (BLOOM style: minus slope_h * (t - j)).
* ALiBi slopes for H heads: n0 = largest power of two <= H; 2**(-8k/n0), k=1..n0;
  then the odd-indexed terms 2**(-8(2k-1)/(2 n0)), k = 1..H-n0.
* LayerNorm: biased variance, eps inside the square root.
* GELU: tanh form.  SiLU: z / (1 + exp(-z)).
* BLOOM residual: taken from the block input (before LayerNorm).

All arithmetic runs in ``dtype`` (float64 by default) with no blocking, fusion or
reordering beyond the definitions above.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import numpy as np


# --------------------------------------------------------------------------- operators

def rms_norm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """x * rsqrt(mean(x^2) + eps) * g, row-wise."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def layer_norm(x: np.ndarray, g: np.ndarray, b: np.ndarray, eps: float) -> np.ndarray:
    """(x - mean) * rsqrt(var + eps) * g + b with the biased variance, row-wise."""
    mu = np.mean(x, axis=-1, keepdims=True)
    var = np.mean((x - mu) ** 2, axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def gelu_tanh(z: np.ndarray) -> np.ndarray:
    return 0.5 * z * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z ** 3)))


def rotary(u: np.ndarray, positions: np.ndarray, base: float) -> np.ndarray:
    """Rotate each head of u [T, H, hd] by its token's absolute position.

    Pair i is (u[..., i], u[..., i + hd/2]); it turns by the angle pos * base**(-2i/hd).
    """
    T, H, hd = u.shape
    half = hd // 2
    inv_freq = base ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]   # [T, half]
    c = np.cos(ang).astype(u.dtype)[:, None, :]
    s = np.sin(ang).astype(u.dtype)[:, None, :]
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def alibi_slopes(n_heads: int) -> np.ndarray:
    n0 = 1 << (n_heads.bit_length() - 1)            # largest power of two <= n_heads
    first = [2.0 ** (-8.0 * k / n0) for k in range(1, n0 + 1)]
    extra = [2.0 ** (-8.0 * (2 * k - 1) / (2 * n0)) for k in range(1, n_heads - n0 + 1)]
    return np.array(first + extra, dtype=np.float64)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention_with_cache(q: np.ndarray, k_all: np.ndarray, v_all: np.ndarray, n_past: int,
                         slopes: Optional[np.ndarray] = None, taps: Optional[dict] = None) -> np.ndarray:
    """Attention of T new tokens over a cache that already includes them.

    q      [T, Hq, hd]   queries of the new tokens (absolute positions n_past .. n_past+T-1)
    k_all  [n_past+T, Hkv, hd], v_all likewise: cached keys/values, new tokens appended.
    Query t sees keys j <= n_past + t.  Returns [T, Hq, hd].
    Written query by query so the causal limit is a slice bound, not a mask.
    """
    T, Hq, hd = q.shape
    Hkv = k_all.shape[1]
    group = Hq // Hkv
    out = np.zeros_like(q)
    scale = 1.0 / math.sqrt(hd)
    for t in range(T):
        pos = n_past + t
        for h in range(Hq):
            kh = h // group
            keys = k_all[: pos + 1, kh, :]                    # [pos+1, hd]
            logit = keys @ q[t, h, :] * scale
            if slopes is not None:
                logit = logit - slopes[h] * (pos - np.arange(pos + 1, dtype=q.dtype))
            p = softmax_rows(logit[None, :])[0]
            out[t, h, :] = p @ v_all[: pos + 1, kh, :]
            if taps is not None:
                taps.setdefault("logits", {})[(t, h)] = logit
                taps.setdefault("probs", {})[(t, h)] = p
    return out


def attention_full_masked(q: np.ndarray, k: np.ndarray, v: np.ndarray,
                          slopes: Optional[np.ndarray] = None, n_past: int = 0) -> np.ndarray:
    """Plain causal attention in matrix form: T x N logits, disallowed entries = -inf.

    With n_past = 0 this is textbook causal self-attention of a whole sequence
    (N x N logits, upper triangle masked).  With n_past > 0 the T queries sit at
    positions n_past .. n_past+T-1 of the N = n_past+T keys.
    """
    T, Hq, hd = q.shape
    Hkv = k.shape[1]
    group = Hq // Hkv
    qpos = n_past + np.arange(T)
    kpos = np.arange(k.shape[0])
    allowed = kpos[None, :] <= qpos[:, None]                  # [query, key]
    dist = (qpos[:, None] - kpos[None, :]).astype(q.dtype)
    out = np.zeros_like(q)
    for h in range(Hq):
        kh = h // group
        s = (q[:, h, :] @ k[:, kh, :].T) / math.sqrt(hd)
        if slopes is not None:
            s = s - slopes[h] * dist
        s = np.where(allowed, s, -np.inf)
        out[:, h, :] = softmax_rows(s) @ v[:, kh, :]
    return out


# --------------------------------------------------------------------------- one block

def _lin(x: np.ndarray, w: Dict[str, np.ndarray], wname: str, bname: Optional[str], dtype) -> np.ndarray:
    y = x @ np.asarray(w[wname], dtype=dtype).T
    if bname is not None and bname in w:
        y = y + np.asarray(w[bname], dtype=dtype)
    return y


def _qkv(shape, w, x, positions, dtype):
    """Pre-attention norm, projections and the positional op of one block."""
    T = x.shape[0]
    if shape.arch == "llama":
        h = rms_norm(x, np.asarray(w["norm1_g"], dtype), shape.norm_eps)
    else:
        h = layer_norm(x, np.asarray(w["norm1_g"], dtype), np.asarray(w["norm1_b"], dtype), shape.norm_eps)
    q = _lin(h, w, "wq", "bq", dtype).reshape(T, shape.n_q_heads, shape.head_dim)
    k = _lin(h, w, "wk", "bk", dtype).reshape(T, shape.n_kv_heads, shape.head_dim)
    v = _lin(h, w, "wv", "bv", dtype).reshape(T, shape.n_kv_heads, shape.head_dim)
    if shape.arch == "llama":
        q = rotary(q, positions, shape.rope_base)
        k = rotary(k, positions, shape.rope_base)
    return q, k, v


def _after_attention(shape, w, x, o, dtype):
    """Output projection + residual, post-attention norm, MLP + residual."""
    T = x.shape[0]
    x1 = x + _lin(o.reshape(T, shape.q_dim), w, "wo", "bo", dtype)
    if shape.arch == "llama":
        m = rms_norm(x1, np.asarray(w["norm2_g"], dtype), shape.norm_eps)
        a = silu(_lin(m, w, "w_gate", None, dtype)) * _lin(m, w, "w_up", None, dtype)
    else:
        m = layer_norm(x1, np.asarray(w["norm2_g"], dtype), np.asarray(w["norm2_b"], dtype), shape.norm_eps)
        a = gelu_tanh(_lin(m, w, "w_up", "b_up", dtype))
    return x1 + _lin(a, w, "w_down", "b_down", dtype)


def block_forward(shape, w: Dict[str, np.ndarray], x: np.ndarray,
                  past_k: np.ndarray, past_v: np.ndarray, dtype=np.float64,
                  taps: Optional[dict] = None, matrix_attention: bool = False):
    """forward(layer, inputs, past_kv) of Algorithm 2: returns (outputs, new_k, new_v).

    x [T, d]; past_k / past_v [L, Hkv, hd] (L may be 0).  new_k / new_v are the T
    rows the caller appends to the layer's cache.  ``matrix_attention`` swaps the
    query-by-query attention for the masked-matrix form (same result, far fewer
    Python iterations; used for long sequences).
    """
    x = np.asarray(x, dtype=dtype)
    T, L = x.shape[0], past_k.shape[0]
    if T == 0:
        empty = np.zeros((0, shape.n_kv_heads, shape.head_dim), dtype)
        return x.copy(), empty, empty.copy()
    q, k, v = _qkv(shape, w, x, np.arange(L, L + T), dtype)
    k_all = np.concatenate([past_k, k], axis=0)
    v_all = np.concatenate([past_v, v], axis=0)
    slopes = alibi_slopes(shape.n_q_heads).astype(dtype) if shape.arch == "bloom" else None
    if taps is not None:
        taps["q"], taps["k"], taps["v"] = q, k, v
    if matrix_attention:
        o = attention_full_masked(q, k_all, v_all, slopes, L)
    else:
        o = attention_with_cache(q, k_all, v_all, L, slopes, taps)
    if taps is not None:
        taps["o"] = o
    return _after_attention(shape, w, x, o, dtype), k, v


# --------------------------------------------------------------------------- sessions (Algorithm 2)

class Session:
    """One inference stream on the blocks [first_block, first_block + n_blocks) of a span.

    ``forward(x)`` is one pass of Algorithm 2's loop body: x [T, d] goes through
    every local layer in order, each layer's new keys/values are appended to its
    cache, and the outputs of all T positions are returned.  ``length`` is the
    number of tokens cached so far.
    """

    def __init__(self, shape, weights: Sequence[Dict[str, np.ndarray]],
                 first_block: int = 0, n_blocks: Optional[int] = None, dtype=np.float64,
                 matrix_attention: bool = False):
        self.shape, self.weights, self.dtype = shape, weights, dtype
        self.matrix_attention = matrix_attention
        self.first_block = first_block
        self.n_blocks = shape.n_blocks - first_block if n_blocks is None else n_blocks
        empty = lambda: np.zeros((0, shape.n_kv_heads, shape.head_dim), dtype)
        self.k: List[np.ndarray] = [empty() for _ in range(self.n_blocks)]
        self.v: List[np.ndarray] = [empty() for _ in range(self.n_blocks)]
        self.length = 0

    def forward(self, x: np.ndarray, taps: Optional[List[dict]] = None) -> np.ndarray:
        inputs = np.asarray(x, dtype=self.dtype)
        for i in range(self.n_blocks):
            w = self.weights[self.first_block + i]
            tap = None
            if taps is not None:
                tap = {}
                taps.append(tap)
            inputs, new_k, new_v = block_forward(self.shape, w, inputs, self.k[i], self.v[i], self.dtype, tap,
                                                 self.matrix_attention)
            self.k[i] = np.concatenate([self.k[i], new_k], axis=0)
            self.v[i] = np.concatenate([self.v[i], new_v], axis=0)
        self.length += x.shape[0]
        return inputs


def replay(shape, weights, past_inputs: np.ndarray, first_block: int = 0,
           n_blocks: Optional[int] = None, dtype=np.float64):
    """Cache replay of Algorithm 3: a fresh session receives all stored past inputs at once.

    Returns (session with rebuilt caches, outputs for all positions).
    """
    s = Session(shape, weights, first_block, n_blocks, dtype)
    return s, s.forward(past_inputs)


def reorder(sessions: Sequence["Session"], hypo_ids: Sequence[int]) -> List["Session"]:
    """Cache reordering for search-based decoding (Section 3.1, last paragraph; appendix on beam
    search): the client sends one index per beam entry and entry i of the next beam continues
    from the attention cache that entry hypo_ids[i] held before the call (a gather).  An entry
    may be named several times (its cache is cloned: the clones grow independently afterwards)
    or not at all (its cache is dropped).  Indices are 0-based here; the paper's example counts
    from 1.

    Returns the sessions of the next beam; the inputs are left untouched.
    """
    out = []
    for src in hypo_ids:
        if not 0 <= src < len(sessions):
            raise IndexError(f"hypothesis index {src} outside the beam of {len(sessions)}")
        old = sessions[src]
        new = Session(old.shape, old.weights, old.first_block, old.n_blocks, old.dtype, old.matrix_attention)
        new.k = [a.copy() for a in old.k]
        new.v = [a.copy() for a in old.v]
        new.length = old.length
        out.append(new)
    return out


# --------------------------------------------------------------------------- no cache at all

def span_full(shape, weights, x: np.ndarray, first_block: int = 0,
              n_blocks: Optional[int] = None, dtype=np.float64) -> np.ndarray:
    """The span applied to a whole sequence x [N, d] with plain causal attention, no cache."""
    n_blocks = shape.n_blocks - first_block if n_blocks is None else n_blocks
    x = np.asarray(x, dtype=dtype)
    N = x.shape[0]
    slopes = alibi_slopes(shape.n_q_heads).astype(dtype) if shape.arch == "bloom" else None
    for i in range(n_blocks):
        w = weights[first_block + i]
        q, k, v = _qkv(shape, w, x, np.arange(N), dtype)
        o = attention_full_masked(q, k, v, slopes)
        x = _after_attention(shape, w, x, o, dtype)
    return x


# --------------------------------------------------------------------------- isolated pieces for kernel-level parity

def attention_logits(q: np.ndarray, keys: np.ndarray, head_dim: int,
                     slope: float = 0.0, q_pos: Optional[int] = None) -> np.ndarray:
    """Scaled logits of one query vector against keys [n, hd] (positions 0..n-1)."""
    s = keys.astype(np.float64) @ q.astype(np.float64) / math.sqrt(head_dim)
    if slope:
        s = s - slope * (q_pos - np.arange(keys.shape[0], dtype=np.float64))
    return s


def linear(x: np.ndarray, w: np.ndarray, b: Optional[np.ndarray] = None, dtype=np.float64) -> np.ndarray:
    """Textbook y = x W^T (+ b)."""
    y = np.asarray(x, dtype) @ np.asarray(w, dtype).T
    return y if b is None else y + np.asarray(b, dtype)

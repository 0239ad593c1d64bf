"""bf16 precision model of the block-span path -- TEST CODE, CPU only.

The HIP path computes every contraction on the matrix cores: bf16 operands, fp32 accumulation.
Its precision contract is therefore "the oracle's arithmetic, with every tensor that enters a
contraction (or is kept in the bf16 attention cache) rounded to bf16 first".  This module writes
that contract down in numpy, independently of the kernels: the oracle's own operators
(oracle/span_oracle.py) composed in the oracle's order, with ``workloads.bf16_round`` applied at the
named rounding points

    h   input of the q/k/v projection   (the normalised row, or the gain-scaled row: see below)
    q   queries after the positional op
    k   keys after the positional op    (also what the cache holds)
    v   values                          (also what the cache holds)
    p   un-normalised softmax weights exp(s - max), as the P.V product consumes them
        (the normaliser is the fp32 sum of the unrounded weights)
    o   attention output, input of the output projection
    m   input of the MLP up projection  (second norm)
    a   activation, input of the MLP down projection

and everything else (accumulation, norms, softmax, activation functions, the residual stream) in
``dtype``.  With no rounding point switched on the model IS the oracle (pinned in
tests/test_precision_model.py), so whatever separates the model from the oracle is the bf16 floor
of the contract itself, no kernel involved; and whatever separates the GPU from the model is what
the kernels add of their own (accumulation order, exp / reciprocal approximations).

Norm placement: a row can be rounded after normalisation, ``round(norm(x) * g)``, or before it,
``round(x * g)`` with the row's 1/sigma (and mean term) applied to the projection's fp32 result.
Both are the same function when nothing is rounded; the second is what a path does that folds the
norm into the neighbouring projections.  ``folded`` selects it per norm.  A folded LayerNorm rounds the row
shifted by the mean the previous norm of the chain found, ``round((x - c) * g)``: the residual stream's mean
moves little from one norm to the next, so the rounding stays relative to the row's spread, not to its mean.
"""
from __future__ import annotations

import math
from typing import Dict, FrozenSet, List, Optional, Sequence

import numpy as np

from oracle import span_oracle as so
from workloads import bf16_round

ALL_POINTS: FrozenSet[str] = frozenset("hqkvpoma")
NO_POINTS: FrozenSet[str] = frozenset()


def _rnd(x: np.ndarray, on: bool) -> np.ndarray:
    if not on:
        return x
    return bf16_round(np.asarray(x, dtype=np.float32)).astype(x.dtype)


def _normed_linear(shape, w: Dict[str, np.ndarray], x: np.ndarray, gname: str, bname: str,
                   mats: Sequence[tuple], rnd: bool, folded: bool, dtype, shift=None) -> List[np.ndarray]:
    """[norm(x) W_i^T + b_i for (W_i, b_i) in mats] with the input row rounded to bf16 (if rnd).
    shift [T, 1]: folded LayerNorm only, the per-row mean found by the previous norm (None = 0)."""
    g = np.asarray(w[gname], dtype)
    llama = shape.arch == "llama"
    if not folded:
        h = so.rms_norm(x, g, shape.norm_eps) if llama else \
            so.layer_norm(x, g, np.asarray(w[bname], dtype), shape.norm_eps)
        h = _rnd(h, rnd)
        return [so.linear(h, w[wn], w.get(bn) if bn else None, dtype) for wn, bn in mats]
    # folded: contraction on the gain-scaled row, 1/sigma and the mean / shift terms afterwards
    if llama:
        hs = _rnd(x * g, rnd)
        r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + dtype(shape.norm_eps))
        return [so.linear(hs, w[wn], None, dtype) * r for wn, bn in mats]
    c = np.zeros((x.shape[0], 1), dtype) if shift is None else np.asarray(shift, dtype)
    hs = _rnd((x - c) * g, rnd)
    mu = np.mean(x, axis=-1, keepdims=True)
    r = 1.0 / np.sqrt(np.mean((x - mu) ** 2, axis=-1, keepdims=True) + dtype(shape.norm_eps))
    beta = np.asarray(w[bname], dtype)
    out = []
    for wn, bn in mats:
        W = np.asarray(w[wn], dtype)
        y = r * (hs @ W.T - (mu - c) * (W @ g)[None, :]) + (W @ beta)[None, :]
        if bn and bn in w:
            y = y + np.asarray(w[bn], dtype)
        out.append(y)
    return out


def _attention(q: np.ndarray, k_all: np.ndarray, v_all: np.ndarray, n_past: int,
               slopes: Optional[np.ndarray], round_p: bool) -> np.ndarray:
    """Causal attention in matrix form, the softmax weights rounded before the P.V product."""
    T, Hq, hd = q.shape
    group = Hq // k_all.shape[1]
    qpos = n_past + np.arange(T)
    kpos = np.arange(k_all.shape[0])
    allowed = kpos[None, :] <= qpos[:, None]
    dist = (qpos[:, None] - kpos[None, :]).astype(q.dtype)
    out = np.zeros_like(q)
    for h in range(Hq):
        kh = h // group
        s = (q[:, h, :] @ k_all[:, kh, :].T) / math.sqrt(hd)
        if slopes is not None:
            s = s - slopes[h] * dist
        s = np.where(allowed, s, -np.inf)
        e = np.exp(s - np.max(s, axis=-1, keepdims=True))
        out[:, h, :] = (_rnd(e, round_p) @ v_all[:, kh, :]) / np.sum(e, axis=-1, keepdims=True)
    return out


def block_forward(shape, w: Dict[str, np.ndarray], x: np.ndarray, past_k: np.ndarray, past_v: np.ndarray,
                  points: FrozenSet[str] = ALL_POINTS, folded_norm1: bool = False, folded_norm2: bool = True,
                  dtype=np.float32, carry: Optional[dict] = None):
    """One block under the bf16 contract: returns (outputs, new_k, new_v) like the oracle's block_forward.
    past_k / past_v are what an earlier call of this function returned (already rounded if k / v are on).
    carry: optional dict through which consecutive blocks of a call hand on the per-row mean that the last norm
    found (key "shift"; used by folded LayerNorms only)."""
    x = np.asarray(x, dtype=dtype)
    T, L = x.shape[0], past_k.shape[0]
    llama = shape.arch == "llama"
    shift1 = carry.get("shift") if (carry is not None and folded_norm1) else None
    q, k, v = _normed_linear(shape, w, x, "norm1_g", "norm1_b", [("wq", "bq"), ("wk", "bk"), ("wv", "bv")],
                             "h" in points, folded_norm1, dtype, shift1)
    shift2 = None if llama else np.mean(x, axis=-1, keepdims=True)         # what norm 1 found: the shift of norm 2
    q = q.reshape(T, shape.n_q_heads, shape.head_dim)
    k = k.reshape(T, shape.n_kv_heads, shape.head_dim)
    v = v.reshape(T, shape.n_kv_heads, shape.head_dim)
    if llama:
        pos = np.arange(L, L + T)
        q, k = so.rotary(q, pos, shape.rope_base), so.rotary(k, pos, shape.rope_base)
    q, k, v = _rnd(q, "q" in points), _rnd(k, "k" in points), _rnd(v, "v" in points)
    k_all = np.concatenate([past_k, k], axis=0)
    v_all = np.concatenate([past_v, v], axis=0)
    slopes = None if llama else so.alibi_slopes(shape.n_q_heads).astype(dtype)
    o = _rnd(_attention(q, k_all, v_all, L, slopes, "p" in points), "o" in points)
    x1 = x + so.linear(o.reshape(T, shape.q_dim), w["wo"], w.get("bo"), dtype)
    if llama:
        gate, up = _normed_linear(shape, w, x1, "norm2_g", "norm2_b", [("w_gate", None), ("w_up", None)],
                                  "m" in points, folded_norm2, dtype)
        a = so.silu(gate) * up
    else:
        (z,) = _normed_linear(shape, w, x1, "norm2_g", "norm2_b", [("w_up", "b_up")], "m" in points, folded_norm2, dtype, shift2)
        if carry is not None:
            carry["shift"] = np.mean(x1, axis=-1, keepdims=True)           # what norm 2 found: the shift of the next block's norm 1
        a = so.gelu_tanh(z)
    y = x1 + so.linear(_rnd(a, "a" in points), w["w_down"], w.get("b_down"), dtype)
    return y, k, v


class Session:
    """The oracle's Session (Algorithm 2) under the bf16 contract.  ``fold_norms`` = the span folds every
    norm but its first into the neighbouring projections (False: every norm rounds the normalised row)."""

    def __init__(self, shape, weights, first_block: int = 0, n_blocks: Optional[int] = None,
                 points: FrozenSet[str] = ALL_POINTS, fold_norms: bool = True, dtype=np.float32):
        self.shape, self.weights, self.points, self.fold, self.dtype = shape, weights, points, fold_norms, dtype
        self.first_block = first_block
        self.n_blocks = shape.n_blocks - first_block if n_blocks is None else n_blocks
        empty = lambda: np.zeros((0, shape.n_kv_heads, shape.head_dim), dtype)
        self.k = [empty() for _ in range(self.n_blocks)]
        self.v = [empty() for _ in range(self.n_blocks)]
        self.length = 0

    def forward(self, x: np.ndarray, per_block: Optional[list] = None) -> np.ndarray:
        h = np.asarray(x, dtype=self.dtype)
        carry = {}
        for i in range(self.n_blocks):
            h, nk, nv = block_forward(self.shape, self.weights[self.first_block + i], h, self.k[i], self.v[i],
                                      self.points, self.fold and i > 0, self.fold, self.dtype, carry)
            self.k[i] = np.concatenate([self.k[i], nk], axis=0)
            self.v[i] = np.concatenate([self.v[i], nv], axis=0)
            if per_block is not None:
                per_block.append(h)
        self.length += x.shape[0]
        return h


# --------------------------------------------------------------------------- error measures (tests' bars)

def row_l2_rel(got: np.ndarray, ref: np.ndarray) -> np.ndarray:
    """per row: ||got - ref||_2 / ||ref||_2"""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return np.sqrt(np.sum((got - ref) ** 2, axis=-1)) / (np.sqrt(np.sum(ref * ref, axis=-1)) + 1e-300)


def elem_rel(got: np.ndarray, ref: np.ndarray) -> np.ndarray:
    """per element: |got - ref| / rms(ref row)"""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return np.abs(got - ref) / (np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True)) + 1e-300)

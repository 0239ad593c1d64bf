"""Training-time passes through a span: plain CPU reference (test infrastructure only).

Section 3.3 of the paper: for parameter-efficient fine-tuning the servers keep their weights
frozen, run back-propagation through their blocks and return the gradient with respect to
their *input activations*; forward and backward process whole sequences in one go, with no
attention cache.  So the backward pass of a span is

    grad_x = (d span(x) / d x)^T  grad_y ,      span = the blocks applied to whole sequences
                                                with causal attention,

which has a plain definition: the vector-Jacobian product of the forward definition.  This
module writes the forward definition a second time in torch (fp64, CPU) and lets torch's
reverse-mode differentiation form the product; the tests pin (a) this forward to the numpy
oracle's `span_full`, and (b) the product to central finite differences of the *numpy* forward,
so a slip in either copy shows.  Llama-style and BLOOM-style blocks, several sequences per call.

Nothing outside tests/, the smoke check and the benchmark's CPU leg may import this module.
"""
from typing import Dict, Sequence

import numpy as np
import torch

from oracle.span_oracle import alibi_slopes


def _t(a) -> torch.Tensor:
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def _block(shape, w: Dict[str, np.ndarray], x: torch.Tensor) -> torch.Tensor:
    """One block on one whole sequence x [N, d] (positions 0..N-1), causal attention."""
    n, d = x.shape
    hq, hkv, hd = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    llama = shape.arch == "llama"
    eps = shape.norm_eps

    def norm(v, g, b):
        if llama:
            return v * torch.rsqrt((v * v).mean(-1, keepdim=True) + eps) * _t(w[g])
        mu = v.mean(-1, keepdim=True)
        var = ((v - mu) ** 2).mean(-1, keepdim=True)
        return (v - mu) * torch.rsqrt(var + eps) * _t(w[g]) + _t(w[b])

    def lin(v, wn, bn):
        y = v @ _t(w[wn]).T
        if not llama:
            y = y + _t(w[bn])
        return y

    h = norm(x, "norm1_g", "norm1_b")
    q = lin(h, "wq", "bq").reshape(n, hq, hd)
    k = lin(h, "wk", "bk").reshape(n, hkv, hd)
    v = lin(h, "wv", "bv").reshape(n, hkv, hd)
    pos = torch.arange(n, dtype=torch.float64)
    if llama:
        half = hd // 2
        inv = shape.rope_base ** (-2.0 * torch.arange(half, dtype=torch.float64) / hd)
        ang = pos[:, None] * inv[None, :]
        cos, sin = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]

        def rot(u):
            a, b = u[..., :half], u[..., half:]
            return torch.cat([a * cos - b * sin, a * sin + b * cos], dim=-1)

        q, k = rot(q), rot(k)
    g = hq // hkv
    kk = k.repeat_interleave(g, dim=1)
    vv = v.repeat_interleave(g, dim=1)
    s = torch.einsum("thd,jhd->htj", q, kk) / np.sqrt(hd)
    if not llama:
        slopes = _t(alibi_slopes(hq))
        s = s - slopes[:, None, None] * (pos[None, :, None] - pos[None, None, :])
    mask = pos[None, None, :] > pos[None, :, None]
    s = s.masked_fill(mask, float("-inf"))
    p = torch.softmax(s, dim=-1)
    o = torch.einsum("htj,jhd->thd", p, vv).reshape(n, hq * hd)
    x1 = x + lin(o, "wo", "bo")
    m = norm(x1, "norm2_g", "norm2_b")
    if llama:
        gate = m @ _t(w["w_gate"]).T
        act = gate / (1.0 + torch.exp(-gate)) * (m @ _t(w["w_up"]).T)
        return x1 + act @ _t(w["w_down"]).T
    z = lin(m, "w_up", "b_up")
    act = 0.5 * z * (1.0 + torch.tanh(np.sqrt(2.0 / np.pi) * (z + 0.044715 * z ** 3)))
    return x1 + lin(act, "w_down", "b_down")


def span_forward_backward(shape, weights: Sequence[Dict[str, np.ndarray]], x: np.ndarray, grad_y: np.ndarray,
                          lens: Sequence[int], first_block: int = 0, n_blocks=None):
    """x, grad_y [sum(lens), d]: the sequences of the batch one after the other.
    Returns (y, grad_x) as fp64 numpy arrays."""
    n_blocks = shape.n_blocks - first_block if n_blocks is None else n_blocks
    with torch.enable_grad():
        xt = _t(x).clone().requires_grad_(True)
        outs, off = [], 0
        for n in lens:
            h = xt[off:off + n]
            for b in range(first_block, first_block + n_blocks):
                h = _block(shape, weights[b], h)
            outs.append(h)
            off += n
        y = torch.cat(outs) if outs else xt[:0]
        (y * _t(grad_y)).sum().backward()
    return y.detach().numpy(), xt.grad.numpy()

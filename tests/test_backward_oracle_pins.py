"""Pins for the training-time oracle (Section 3.3: servers back-propagate through frozen blocks
and return the gradient with respect to their input activations; whole sequences, no cache).

The backward pass is the vector-Jacobian product of the forward definition, so it is pinned
against that definition itself, evaluated by the *numpy* oracle (a second, separately written
copy of the forward): central finite differences along random and along single-coordinate
directions, linearity in grad_y, the causal structure of the Jacobian, the independence of the
sequences of a batch, composition over sub-spans, and a closed form for a degenerate block.
"""
import numpy as np
import pytest

from oracle import backward_oracle as bo
from oracle import span_oracle as so
from workloads import TINY, TINY_BLOOM, SpanShape, SpanWeights, draw_hidden

SHAPES = {"llama": TINY, "bloom": TINY_BLOOM}


def _inputs(shape, lens, seed=3):
    n = sum(lens)
    x = draw_hidden(shape, seed, 0, n).astype(np.float64)
    gy = np.random.default_rng(seed + 100).standard_normal((n, shape.d_model))
    return x, gy


@pytest.mark.parametrize("arch", ["llama", "bloom"])
def test_forward_copy_equals_numpy_forward(arch):
    shape = SHAPES[arch]
    w = SpanWeights(shape, seed=1)
    lens = [7, 12]
    x, gy = _inputs(shape, lens)
    y, _ = bo.span_forward_backward(shape, w, x, gy, lens)
    ref = np.concatenate([so.span_full(shape, w, x[:7]), so.span_full(shape, w, x[7:])])
    assert np.max(np.abs(y - ref)) <= 1e-10 * np.max(np.abs(ref))


@pytest.mark.parametrize("arch", ["llama", "bloom"])
def test_directional_derivatives_match_finite_differences_of_numpy_forward(arch):
    shape = SHAPES[arch]
    w = SpanWeights(shape, seed=2)
    n = 9
    x, gy = _inputs(shape, [n], seed=5)
    _, gx = bo.span_forward_backward(shape, w, x, gy, [n])
    rng = np.random.default_rng(0)
    f = lambda z: float(np.sum(so.span_full(shape, w, z) * gy))
    scale = np.sqrt(np.mean(x * x))
    dirs = [rng.standard_normal(x.shape) for _ in range(3)]
    for t, c in [(0, 0), (4, 17), (n - 1, shape.d_model - 1)]:           # single coordinates
        e = np.zeros_like(x)
        e[t, c] = 1.0
        dirs.append(e)
    for u in dirs:
        h = 1e-5 * scale
        fd = (f(x + h * u) - f(x - h * u)) / (2 * h)
        an = float(np.sum(gx * u))
        assert abs(fd - an) <= 1e-6 * max(abs(an), np.linalg.norm(gx) * np.linalg.norm(u) * 1e-3), (fd, an)


def test_linear_in_grad_y_and_zero():
    shape = TINY
    w = SpanWeights(shape, seed=1)
    lens = [5, 3]
    x, g1 = _inputs(shape, lens, seed=1)
    _, g2 = _inputs(shape, lens, seed=2)
    _, a = bo.span_forward_backward(shape, w, x, g1, lens)
    _, b = bo.span_forward_backward(shape, w, x, g2, lens)
    _, c = bo.span_forward_backward(shape, w, x, 2.0 * g1 - 3.0 * g2, lens)
    assert np.allclose(c, 2.0 * a - 3.0 * b, rtol=1e-9, atol=1e-12)
    _, z = bo.span_forward_backward(shape, w, x, np.zeros_like(g1), lens)
    assert np.all(z == 0)


@pytest.mark.parametrize("arch", ["llama", "bloom"])
def test_causal_structure(arch):
    """Output t depends on inputs 0..t only: a grad_y supported on token t gives a grad_x that
    vanishes after t, and is non-zero at t and (through attention) before it."""
    shape = SHAPES[arch]
    w = SpanWeights(shape, seed=4)
    n, t = 10, 6
    x, gy = _inputs(shape, [n], seed=7)
    g = np.zeros_like(gy)
    g[t] = gy[t]
    _, gx = bo.span_forward_backward(shape, w, x, g, [n])
    assert np.all(gx[t + 1:] == 0)
    assert np.linalg.norm(gx[t]) > 0 and np.linalg.norm(gx[0]) > 0 and np.linalg.norm(gx[t - 1]) > 0


def test_sequences_of_a_batch_are_independent():
    shape = TINY
    w = SpanWeights(shape, seed=1)
    lens = [6, 1, 9]
    x, gy = _inputs(shape, lens, seed=9)
    _, gx = bo.span_forward_backward(shape, w, x, gy, lens)
    off = 0
    for n in lens:
        _, one = bo.span_forward_backward(shape, w, x[off:off + n], gy[off:off + n], [n])
        assert np.allclose(gx[off:off + n], one, rtol=1e-12, atol=1e-14)
        off += n
    # an empty batch and an empty sequence are allowed
    _, e = bo.span_forward_backward(shape, w, x[:0], gy[:0], [])
    assert e.shape == (0, shape.d_model)
    _, e2 = bo.span_forward_backward(shape, w, x[:6], gy[:6], [6, 0])
    assert np.allclose(e2, gx[:6], rtol=1e-12, atol=1e-14)


def test_chain_rule_over_sub_spans():
    """Backward through blocks [0,2) = backward through block 1, then block 0 (what a chain of
    servers computes when each returns its input gradient to the previous one)."""
    shape = TINY
    w = SpanWeights(shape, seed=6)
    lens = [8, 5]
    x, gy = _inputs(shape, lens, seed=11)
    _, whole = bo.span_forward_backward(shape, w, x, gy, lens)
    mid, _ = bo.span_forward_backward(shape, w, x, gy, lens, first_block=0, n_blocks=1)
    _, g_mid = bo.span_forward_backward(shape, w, mid, gy, lens, first_block=1, n_blocks=1)
    _, g_in = bo.span_forward_backward(shape, w, x, g_mid, lens, first_block=0, n_blocks=1)
    assert np.allclose(whole, g_in, rtol=1e-9, atol=1e-12)


def test_single_token_closed_form():
    """A one-token sequence attends to itself only, so attention returns v and the attention half
    of a Llama-style block is x1 = x + Wo Rep(Wv rmsnorm(x)) (Rep: each kv head repeated for its
    group of query heads): with the MLP switched off (w_down = 0) the Jacobian is I + Wo Rep Wv J_norm,
    J_norm = r diag(g) (I - r^2 x x^T / d)."""
    shape = SpanShape("llama", 1, 64, 4, 2, 16, 96)
    base = SpanWeights(shape, seed=8)
    w = dict(base[0])
    w["w_down"] = np.zeros_like(w["w_down"])
    x = draw_hidden(shape, 1, 0, 1).astype(np.float64)
    gy = np.random.default_rng(1).standard_normal((1, 64))
    _, gx = bo.span_forward_backward(shape, [w], x, gy, [1])
    d = 64
    xv = x[0]
    r = 1.0 / np.sqrt(np.mean(xv * xv) + shape.norm_eps)
    j_norm = r * np.diag(np.asarray(w["norm1_g"], np.float64)) @ (np.eye(d) - (r * r / d) * np.outer(xv, xv))
    rep = np.zeros((shape.q_dim, shape.kv_dim))
    for h in range(shape.n_q_heads):
        kh = h // (shape.n_q_heads // shape.n_kv_heads)
        rep[h * 16:(h + 1) * 16, kh * 16:(kh + 1) * 16] = np.eye(16)
    jac = np.eye(d) + np.asarray(w["wo"], np.float64) @ rep @ np.asarray(w["wv"], np.float64) @ j_norm
    assert np.allclose(gx[0], jac.T @ gy[0], rtol=1e-9, atol=1e-12)

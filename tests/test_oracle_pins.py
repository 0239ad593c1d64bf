"""Pins for the CPU oracle: closed forms, invariants, special cases and brute force.

The paper fixes the *session semantics* (Algorithms 1-3: cached generation and
replay reach the same result as recomputing the sequence, Sections 2.1 and 3.2)
but prints no activations, so the block arithmetic is pinned by what the
mathematics fixes.  Each test is chosen so that a plausible slip in the oracle (a
dropped term, wrong index, transposed operand, off-by-one causal limit, wrong
head mapping) fails at least one of them.
"""
import math

import numpy as np
import pytest

from oracle import span_oracle as so
from workloads import SpanShape, SpanWeights, TINY, TINY_BLOOM, draw_hidden

TOL = 1e-9   # fp64 oracle; everything here is exact up to rounding order


def rel_err(a, b):
    """max |a-b| normalised by the per-row rms of b."""
    rms = np.sqrt(np.mean(b * b, axis=-1, keepdims=True)) + 1e-300
    return float(np.max(np.abs(a - b) / rms))


def weights_of(shape, seed=0):
    return SpanWeights(shape, seed=seed, bf16=False, cache=True)


def mutable(weights, shape):
    return [dict((k, v.astype(np.float64).copy()) for k, v in weights[b].items()) for b in range(shape.n_blocks)]


# ------------------------------------------------------------------ caching semantics (brute force)

@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
def test_cached_decode_equals_full_recompute(shape):
    """Sections 2.1/3.2: cached step n == last row of recomputing n+1 tokens from scratch."""
    W = weights_of(shape)
    x = draw_hidden(shape, 0, 0, 24, bf16=False)
    sess = so.Session(shape, W)
    y_prefix = sess.forward(x[:16])
    full16 = so.span_full(shape, W, x[:16])
    assert rel_err(y_prefix, full16) < TOL
    for n in range(16, 24):
        y = sess.forward(x[n:n + 1])
        full = so.span_full(shape, W, x[:n + 1])
        assert rel_err(y, full[-1:]) < TOL, n
    assert sess.length == 24


@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
def test_replay_rebuilds_incremental_cache(shape):
    """Algorithm 3: a fresh session fed all stored inputs ends in the same state and outputs."""
    W = weights_of(shape)
    x = draw_hidden(shape, 0, 0, 24, bf16=False)
    inc = so.Session(shape, W)
    outs = [inc.forward(x[:16])] + [inc.forward(x[n:n + 1]) for n in range(16, 24)]
    rep, y_all = so.replay(shape, W, x)
    assert rel_err(y_all, np.concatenate(outs)) < TOL
    for b in range(shape.n_blocks):
        assert rep.k[b].shape == inc.k[b].shape == (24, shape.n_kv_heads, shape.head_dim)
        assert np.max(np.abs(rep.k[b] - inc.k[b])) < 1e-10
        assert np.max(np.abs(rep.v[b] - inc.v[b])) < 1e-10
    # both continue identically
    nxt = draw_hidden(shape, 1, 7, 1, bf16=False)
    assert rel_err(rep.forward(nxt), inc.forward(nxt)) < TOL


@pytest.mark.parametrize("split", [0, 1, 7, 16, 23, 24])
def test_chunk_invariance(split):
    """Micro-batching (Section 4.2 footnote): feeding a sequence in two requests == one request."""
    W = weights_of(TINY)
    x = draw_hidden(TINY, 0, 0, 24, bf16=False)
    one = so.Session(TINY, W).forward(x)
    s = so.Session(TINY, W)
    two = np.concatenate([s.forward(x[:split]), s.forward(x[split:])])
    assert rel_err(two, one) < TOL and s.length == 24


def test_matrix_attention_path_equals_row_path():
    W = weights_of(TINY_BLOOM)
    x = draw_hidden(TINY_BLOOM, 0, 0, 20, bf16=False)
    a = so.Session(TINY_BLOOM, W)
    b = so.Session(TINY_BLOOM, W, matrix_attention=True)
    ya = np.concatenate([a.forward(x[:9]), a.forward(x[9:])])
    yb = np.concatenate([b.forward(x[:9]), b.forward(x[9:])])
    assert rel_err(ya, yb) < TOL


@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
def test_causality(shape):
    """Changing inputs after position t must leave outputs up to t bit-identical."""
    W = weights_of(shape)
    x = draw_hidden(shape, 0, 0, 12, bf16=False).astype(np.float64)
    x2 = x.copy()
    x2[8:] += 3.0
    for fn in (lambda z: so.span_full(shape, W, z), lambda z: so.Session(shape, W).forward(z)):
        y, y2 = fn(x), fn(x2)
        assert np.array_equal(y[:8], y2[:8])
        assert not np.allclose(y[8:], y2[8:])


def test_sub_span_sessions_compose():
    """A span served as two consecutive sub-segments (Appendix D) equals the whole span."""
    W = weights_of(TINY)
    x = draw_hidden(TINY, 0, 0, 10, bf16=False)
    whole = so.Session(TINY, W).forward(x)
    first = so.Session(TINY, W, first_block=0, n_blocks=1).forward(x)
    second = so.Session(TINY, W, first_block=1, n_blocks=1).forward(first)
    assert rel_err(second, whole) < TOL


# ------------------------------------------------------------------ rotary

def test_rotary_is_complex_multiplication():
    rng = np.random.default_rng(1)
    u = rng.standard_normal((5, 3, 8))
    pos = np.array([0, 1, 2, 77, 4100])
    out = so.rotary(u, pos, 10000.0)
    half = 4
    z = u[..., :half] + 1j * u[..., half:]
    theta = 10000.0 ** (-2.0 * np.arange(half) / 8)
    zr = z * np.exp(1j * pos[:, None, None] * theta[None, None, :])
    assert np.allclose(out[..., :half], zr.real, atol=1e-12)
    assert np.allclose(out[..., half:], zr.imag, atol=1e-12)
    assert np.array_equal(out[0], u[0])                                   # position 0 is the identity
    assert np.allclose(np.linalg.norm(out, axis=-1), np.linalg.norm(u, axis=-1))


def test_rotary_first_frequency_is_one_radian_per_position():
    u = np.zeros((1, 1, 4)); u[0, 0, 0] = 1.0      # pair 0 = (dim0, dim2), theta_0 = 1
    out = so.rotary(u, np.array([1]), 10000.0)
    assert np.allclose(out[0, 0], [math.cos(1.0), 0.0, math.sin(1.0), 0.0])
    # pair 1 = (dim1, dim3), theta_1 = base**(-2/4) = 0.01
    u = np.zeros((1, 1, 4)); u[0, 0, 1] = 1.0
    out = so.rotary(u, np.array([50]), 10000.0)
    assert np.allclose(out[0, 0], [0.0, math.cos(0.5), 0.0, math.sin(0.5)])


def test_rotary_logits_depend_only_on_relative_position():
    rng = np.random.default_rng(2)
    q, k = rng.standard_normal((1, 1, 16)), rng.standard_normal((1, 1, 16))
    def dot(m, n):
        return float(np.sum(so.rotary(q, np.array([m]), 10000.0) * so.rotary(k, np.array([n]), 10000.0)))
    assert abs(dot(9, 4) - dot(1009, 1004)) < 1e-9
    assert abs(dot(9, 4) - dot(9, 5)) > 1e-6


def test_shifting_all_positions_leaves_llama_attention_unchanged():
    """Relative-position property end to end: cache built at positions 3.. equals positions 0.."""
    shape = TINY
    W = weights_of(shape)
    w = W[0]
    x = draw_hidden(shape, 0, 0, 6, bf16=False).astype(np.float64)
    outs = []
    for shift in (0, 3):
        q, k, v = so._qkv(shape, w, x, np.arange(shift, shift + 6), np.float64)
        outs.append(so.attention_full_masked(q, k, v))
    assert np.allclose(outs[0], outs[1], atol=1e-10)


# ------------------------------------------------------------------ attention / softmax special cases

def test_zero_queries_give_running_mean_of_values():
    """Wq = 0 -> all logits 0 -> o_t = mean of v_j, j <= t (Llama style)."""
    shape = TINY
    W = mutable(weights_of(shape), shape)
    W[0]["wq"][:] = 0.0
    x = draw_hidden(shape, 0, 0, 7, bf16=False).astype(np.float64)
    taps = {}
    so.block_forward(shape, W[0], x, np.zeros((0, 2, 64)), np.zeros((0, 2, 64)), taps=taps)
    v, o = taps["v"], taps["o"]
    group = shape.n_q_heads // shape.n_kv_heads
    for t in range(7):
        for h in range(shape.n_q_heads):
            assert np.allclose(o[t, h], v[: t + 1, h // group].mean(axis=0), atol=1e-12)
            assert abs(taps["probs"][(t, h)].sum() - 1.0) < 1e-12


def test_zero_queries_bloom_give_geometric_weights():
    """BLOOM style with q = 0: p_j proportional to exp(-slope_h (t-j))."""
    shape = TINY_BLOOM
    W = mutable(weights_of(shape), shape)
    W[0]["wq"][:] = 0.0
    W[0]["bq"][:] = 0.0
    x = draw_hidden(shape, 0, 0, 6, bf16=False).astype(np.float64)
    taps = {}
    so.block_forward(shape, W[0], x, np.zeros((0, 4, 64)), np.zeros((0, 4, 64)), taps=taps)
    slopes = [2.0 ** -2, 2.0 ** -4, 2.0 ** -6, 2.0 ** -8]        # 4 heads: 2^(-8k/4)
    for h in range(4):
        r = math.exp(-slopes[h])
        wts = np.array([r ** (5 - j) for j in range(6)])
        assert np.allclose(taps["probs"][(5, h)], wts / wts.sum(), atol=1e-12)
        assert np.allclose(taps["o"][5, h], (wts / wts.sum()) @ taps["v"][:, h], atol=1e-12)


def test_attention_by_hand_on_two_tokens():
    """2 tokens, 1 head, hd=2: numbers small enough to do on paper."""
    q = np.array([[[1.0, 0.0]], [[0.0, 2.0]]])
    k = np.array([[[1.0, 1.0]], [[3.0, -1.0]]])
    v = np.array([[[10.0, 0.0]], [[0.0, 10.0]]])
    o = so.attention_with_cache(q, k, v, 0)
    assert np.allclose(o[0, 0], [10.0, 0.0])                      # first token sees only itself
    s = np.array([2.0, -2.0]) / math.sqrt(2.0)                     # q1.k0, q1.k1 scaled
    p = np.exp(s) / np.exp(s).sum()
    assert np.allclose(o[1, 0], [10 * p[0], 10 * p[1]])
    assert np.allclose(so.attention_full_masked(q, k, v), o)


def test_gqa_equals_mha_with_replicated_kv_heads():
    shape = TINY                                   # 4 q heads, 2 kv heads
    W = mutable(weights_of(shape), shape)
    mha = SpanShape("llama", 2, 256, 4, 4, 64, 688)
    W2 = []
    for w in W:
        w2 = dict(w)
        for name in ("wk", "wv"):
            blocks = w[name].reshape(2, 64, 256)
            w2[name] = np.repeat(blocks, 2, axis=0).reshape(4 * 64, 256)
        W2.append(w2)
    x = draw_hidden(shape, 0, 0, 9, bf16=False)
    assert rel_err(so.span_full(mha, W2, x), so.span_full(shape, W, x)) < TOL


def test_head_mapping_is_contiguous_groups():
    """Zero the values of kv head 1: exactly query heads 2,3 (not 1,3) go to zero output."""
    shape = TINY
    W = mutable(weights_of(shape), shape)
    W[0]["wv"][64:, :] = 0.0
    x = draw_hidden(shape, 0, 0, 5, bf16=False).astype(np.float64)
    taps = {}
    so.block_forward(shape, W[0], x, np.zeros((0, 2, 64)), np.zeros((0, 2, 64)), taps=taps)
    o = taps["o"]
    assert np.all(o[:, 2:] == 0.0) and np.all(np.abs(o[:, :2]).max(axis=(0, 2)) > 0)


# ------------------------------------------------------------------ residual path, norms, activations

@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
def test_zero_output_projections_make_span_identity(shape):
    W = mutable(weights_of(shape), shape)
    for w in W:
        w["wo"][:] = 0.0
        w["w_down"][:] = 0.0
        for b in ("bo", "b_down"):
            if b in w:
                w[b][:] = 0.0
    x = draw_hidden(shape, 0, 0, 5, bf16=False).astype(np.float64)
    assert np.array_equal(so.span_full(shape, W, x), x)
    assert np.array_equal(so.Session(shape, W).forward(x), x)


def test_residual_adds_each_branch_once():
    """With Wo = 0 the block is x + MLP(norm(x)); with W_down = 0 it is x + attn branch."""
    shape = TINY
    W = mutable(weights_of(shape), shape)
    w = W[0]
    x = draw_hidden(shape, 0, 0, 4, bf16=False).astype(np.float64)
    e = np.zeros((0, 2, 64))
    w_a = dict(w); w_a["wo"] = np.zeros_like(w["wo"])
    m = so.rms_norm(x, w["norm2_g"], shape.norm_eps)
    mlp = (so.silu(m @ w["w_gate"].T) * (m @ w["w_up"].T)) @ w["w_down"].T
    assert np.allclose(so.block_forward(shape, w_a, x, e, e)[0], x + mlp, atol=1e-12)
    w_b = dict(w); w_b["w_down"] = np.zeros_like(w["w_down"])
    taps = {}
    y = so.block_forward(shape, w_b, x, e, e, taps=taps)[0]
    assert np.allclose(y, x + taps["o"].reshape(4, -1) @ w["wo"].T, atol=1e-12)


def test_rms_norm_closed_forms():
    g = np.linspace(0.5, 1.5, 8)
    for c in (3.0, -0.25):
        out = so.rms_norm(np.full((1, 8), c), g, 1e-5)
        assert np.allclose(out[0], np.sign(c) * g / math.sqrt(1 + 1e-5 / c ** 2), atol=1e-14)
    x = np.random.default_rng(0).standard_normal((3, 8))
    assert np.allclose(so.rms_norm(1000 * x, g, 1e-5), so.rms_norm(x, g, 1e-11), atol=1e-9)
    assert np.allclose(np.mean(so.rms_norm(x, np.ones(8), 0.0) ** 2, axis=-1), 1.0)


def test_layer_norm_closed_forms():
    g, b = np.linspace(0.5, 1.5, 8), np.linspace(-1, 1, 8)
    assert np.allclose(so.layer_norm(np.full((1, 8), 7.0), g, b, 1e-5)[0], b)
    x = np.random.default_rng(0).standard_normal((3, 8))
    y = so.layer_norm(x, np.ones(8), np.zeros(8), 0.0)
    assert np.allclose(y.mean(axis=-1), 0.0, atol=1e-12) and np.allclose((y * y).mean(axis=-1), 1.0)
    # two-point input: variance is the biased one ((a-b)/2)^2
    y2 = so.layer_norm(np.array([[1.0, 3.0]]), np.ones(2), np.zeros(2), 0.0)
    assert np.allclose(y2, [[-1.0, 1.0]])


def test_activation_values():
    assert so.silu(np.array([0.0]))[0] == 0.0
    assert abs(so.silu(np.array([1.0]))[0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    assert abs(so.silu(np.array([-20.0]))[0]) < 1e-7
    z = np.array([-3.0, -1.0, 0.0, 0.5, 2.0])
    erf_gelu = 0.5 * z * (1.0 + np.array([math.erf(v / math.sqrt(2)) for v in z]))
    assert np.max(np.abs(so.gelu_tanh(z) - erf_gelu)) < 1e-3     # tanh form tracks the exact GELU
    assert so.gelu_tanh(np.array([0.0]))[0] == 0.0
    assert abs(so.gelu_tanh(np.array([10.0]))[0] - 10.0) < 1e-9


def test_alibi_slopes():
    for n in (4, 8, 64, 128):
        s = so.alibi_slopes(n)
        assert np.allclose(s, [2.0 ** (-8.0 * k / n) for k in range(1, n + 1)])
    s = so.alibi_slopes(112)
    assert len(s) == 112 and np.allclose(s[:64], so.alibi_slopes(64))
    assert np.allclose(s[64:], so.alibi_slopes(128)[0::2][:48])
    assert np.allclose(s[1:64] / s[:63], 2.0 ** (-8 / 64)) and np.allclose(s[65:] / s[64:-1], 2.0 ** (-8 / 64))


def test_linear_is_x_times_w_transposed():
    x = np.array([[1.0, 2.0, 3.0]])
    w = np.array([[1.0, 0.0, 0.0], [0.0, 1.0, 1.0]])          # 2 outputs, 3 inputs
    assert np.array_equal(so.linear(x, w, np.array([10.0, 20.0])), [[11.0, 25.0]])


# ------------------------------------------------------------------ sessions are independent

def test_sessions_do_not_interact():
    W = weights_of(TINY)
    xa, xb = draw_hidden(TINY, 0, 0, 6, bf16=False), draw_hidden(TINY, 0, 1, 9, bf16=False)
    sa, sb = so.Session(TINY, W), so.Session(TINY, W)
    ya1, yb1 = sa.forward(xa[:3]), sb.forward(xb[:5])
    yb2, ya2 = sb.forward(xb[5:]), sa.forward(xa[3:])
    assert rel_err(np.concatenate([ya1, ya2]), so.span_full(TINY, W, xa)) < TOL
    assert rel_err(np.concatenate([yb1, yb2]), so.span_full(TINY, W, xb)) < TOL


def test_fp32_mode_tracks_fp64():
    W = weights_of(TINY)
    x = draw_hidden(TINY, 0, 0, 24, bf16=False)
    y64 = so.span_full(TINY, W, x)
    y32 = so.span_full(TINY, W, x, dtype=np.float32)
    assert y32.dtype == np.float32 and rel_err(y32.astype(np.float64), y64) < 1e-5


# ----------------------------------------------------------------------------- cache reordering (beam search)

def _beam(n, tokens=5):
    """n sessions of the tiny span with distinct histories; returns (sessions, histories)."""
    W = SpanWeights(TINY, seed=0, bf16=False, cache=True)
    sessions, hist = [], []
    for i in range(n):
        x = draw_hidden(TINY, 11, i, tokens + i)          # different lengths too
        s = so.Session(TINY, W)
        s.forward(x)
        sessions.append(s)
        hist.append(x)
    return W, sessions, hist


def test_reorder_follows_the_papers_worked_example():
    """Appendix on beam search: indices [2, 2, 1, 3, 2] (from 1).  The fixture holds what the paper
    says about the outcome; each new entry must hold exactly the cache of the entry it names."""
    import os
    lines = [l.strip() for l in open(os.path.join(os.path.dirname(__file__), "golden", "beam_reorder_example.txt"))
             if l.strip() and not l.startswith("#")]
    fields = dict(l.split(":", 1) for l in lines)
    idx = [int(v) for v in fields["indices"].split()]
    pairs = [tuple(int(v) for v in p.split("<-")) for p in (fields["stated"] + " " + fields["from_list"]).split()]
    dropped = [int(v) for v in fields["discarded"].split()]
    W, old, _ = _beam(5)
    new = so.reorder(old, [i - 1 for i in idx])
    assert len(new) == 5 and sorted(p[0] for p in pairs) == [1, 2, 3, 4, 5]
    for place, src in pairs:
        assert new[place - 1].length == old[src - 1].length
        for b in range(TINY.n_blocks):
            assert np.array_equal(new[place - 1].k[b], old[src - 1].k[b])
            assert np.array_equal(new[place - 1].v[b], old[src - 1].v[b])
    lengths_after = {s.length for s in new}
    for d in dropped:                                         # histories have distinct lengths
        assert old[d - 1].length not in lengths_after


def test_reordered_beam_continues_like_fresh_sessions_with_the_source_histories():
    """Cloning a cache must equal having processed the source's whole history (the cached form
    is an exact reformulation, Section 2.1): after a reorder every entry's next outputs equal a
    full recomputation over (source history + new tokens); clones of one source then grow
    independently."""
    W, old, hist = _beam(3)
    hypo = [1, 1, 0]
    new = so.reorder(old, hypo)
    steps = [draw_hidden(TINY, 12, i, 3) for i in range(3)]    # different continuations per entry
    for i, s in enumerate(new):
        y = s.forward(steps[i])
        full = so.span_full(TINY, W, np.concatenate([hist[hypo[i]], steps[i]]))
        assert np.max(np.abs(y - full[-3:])) < 1e-9
    # the untouched inputs still hold their own caches
    assert [s.length for s in old] == [5, 6, 7]
    # identity and composition
    same = so.reorder(new, [0, 1, 2])
    assert all(np.array_equal(a.k[0], b.k[0]) for a, b in zip(same, new))
    p, q = [2, 0, 0], [1, 2, 1]
    two = so.reorder(so.reorder(new, p), q)
    one = so.reorder(new, [p[j] for j in q])
    assert all(np.array_equal(a.v[1], b.v[1]) and a.length == b.length for a, b in zip(two, one))
    with pytest.raises(IndexError):
        so.reorder(new, [3])

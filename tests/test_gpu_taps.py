"""Kernel-level parity of the attention inside real calls, through span_debug_tap.

The bar "<= 1e-3 on fp32-accumulated attention logits" is a statement about the kernel's
accumulation, not about bf16 rounding of its operands: the oracle's logit routine is therefore fed
the path's OWN post-rotary bf16 queries (tap) and the keys the cache holds (read through the page
table), and what the multi-token attention kernel -- the one a cache replay (Algorithm 3) and every
prompt chunk run -- computed is compared with that, normalised by the row's largest |logit|.
Covered: past > 0 and = 0, ALiBi on / off, head_dim 64 / 128, query ranges that cross tile
boundaries and the causal diagonal, a ragged batch with a single-token session beside the tapped
one, and a replay.  The tapped queries and keys themselves are checked against the oracle's q / k."""
import numpy as np
import pytest
import torch

from gpu_util import *  # noqa: F401,F403
from workloads import SpanShape

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]

SHAPES = {
    "llama-hd64-gqa": SpanShape("llama", 2, 256, 8, 2, 64, 352),
    "llama-hd128-gqa": SpanShape("llama", 2, 512, 8, 2, 128, 704),
    "bloom-hd64": SpanShape("bloom", 2, 256, 4, 4, 64, 512),
    "bloom-hd128": SpanShape("bloom", 2, 384, 3, 3, 128, 768),       # 3 heads: slopes beyond the power-of-two rule
}


def make(shape, seed=11):
    W = SpanWeights(shape, seed=seed, bf16=True, cache=True)
    cfg = config_for(shape, max_pages=96, max_sessions=6, max_session_tokens=320, max_batch_tokens=512, io_f32=True)
    return SpanServer(cfg, W, DEV), W


def tap_buffers(shape, nq, ld):
    q = torch.full((nq, shape.q_dim), float("nan"), dtype=torch.bfloat16, device=DEV)
    k = torch.full((nq, shape.kv_dim), float("nan"), dtype=torch.bfloat16, device=DEV)
    lg = torch.full((nq, ld), float("nan"), dtype=torch.float32, device=DEV)
    return q, k, lg


def arm(srv, block, sess, head, q0, nq, bufs):
    q, k, lg = bufs
    B.span_debug_tap(srv.span, B.TAP_Q_ROT, block, sess, -1, q0, nq, q, q.numel() * 2)
    B.span_debug_tap(srv.span, B.TAP_K_ROT, block, sess, -1, q0, nq, k, k.numel() * 2)
    B.span_debug_tap(srv.span, B.TAP_LOGITS, block, sess, head, q0, nq, lg, lg.numel() * 4)


def check_taps(shape, srv, sess, block, head, past, q0, nq, bufs, oracle_taps):
    """Logits of the kernel against the oracle's routine on the tapped operands; operands against the oracle's."""
    q_t, k_t, lg_t = (to_np(t) for t in bufs)
    hd, G = shape.head_dim, shape.n_q_heads // shape.n_kv_heads
    ld = lg_t.shape[1]
    k_cache, _ = srv.read_kv(sess, block, 0, ld)
    torch.cuda.synchronize()
    k_cache = to_np(k_cache)                                          # [ld, Hkv, hd]
    # the key tap is what the cache holds for the new tokens, bit for bit
    assert np.array_equal(k_t.reshape(nq, shape.n_kv_heads, hd), k_cache[past + q0:past + q0 + nq])
    slope = float(so.alibi_slopes(shape.n_q_heads)[head]) if shape.arch == "bloom" else 0.0
    worst = 0.0
    for i in range(nq):
        pos = past + q0 + i
        qv = q_t[i].reshape(shape.n_q_heads, hd)[head]
        ref = so.attention_logits(qv, k_cache[:pos + 1, head // G], hd, slope, pos)
        got = lg_t[i]
        assert np.all(np.isfinite(got[:pos + 1])) and np.all(np.isnan(got[pos + 1:])), (i, pos)
        worst = max(worst, float(np.max(np.abs(got[:pos + 1] - ref)) / np.max(np.abs(ref))))
    assert worst < LOGIT_TOL, worst
    # operands: one bf16 rounding away from the oracle's post-rotary q and k (new tokens q0 .. q0+nq of this call)
    q_ref = oracle_taps["q"][q0:q0 + nq].reshape(nq, -1)
    k_ref = oracle_taps["k"][q0:q0 + nq].reshape(nq, -1)
    eq = float(np.max(np.abs(q_t - q_ref)) / np.max(np.abs(q_ref)))
    ek = float(np.max(np.abs(k_t - k_ref)) / np.max(np.abs(k_ref)))
    assert eq < KV_TOL and ek < KV_TOL, (eq, ek)
    return worst


@pytest.mark.parametrize("name", list(SHAPES))
def test_multi_token_attention_logits_on_the_paths_own_operands(name):
    shape = SHAPES[name]
    srv, W = make(shape)
    xs = [draw_hidden(shape, 11, i, 200) for i in range(3)]
    osess = [so.Session(shape, W) for _ in range(3)]
    ids = [srv.open(320) for _ in range(3)]
    # pasts of 37 / 0 / 70 tokens (session 1 stays empty for now)
    srv.forward([ids[0], ids[2]], [37, 70], np.concatenate([xs[0][:37], xs[2][:70]]))
    osess[0].forward(xs[0][:37]); osess[2].forward(xs[2][:70])
    # ragged call: 50 new tokens on a 37-token cache, 19 on an empty one, a single token on 70
    cnt = [50, 19, 1]
    x_call = np.concatenate([xs[0][37:87], xs[1][:19], xs[2][70:71]])
    block, head = 1, shape.n_q_heads - 1
    q0, nq = 10, 36                                # tokens 10..45: crosses the 32-query tile boundary and the diagonal
    bufs = tap_buffers(shape, nq, 37 + 50)
    arm(srv, block, ids[0], head, q0, nq, bufs)
    y = srv.forward(ids, cnt, x_call)
    torch.cuda.synchronize()
    taps = [[], [], []]
    refs = [osess[0].forward(xs[0][37:87], taps[0]), osess[1].forward(xs[1][:19], taps[1]), osess[2].forward(xs[2][70:71], taps[2])]
    assert row_rel_err(to_np(y), np.concatenate(refs)) < HIDDEN_TOL
    w0 = check_taps(shape, srv, ids[0], block, head, 37, q0, nq, bufs, taps[0][block])

    # the same call on fresh sessions without taps gives the same outputs bit for bit (the tapped kernel differs
    # only in its extra stores), and taps are one-shot: nothing is written the second time
    for s in ids:
        srv.close(s)
    ids = [srv.open(320) for _ in range(3)]
    srv.forward([ids[0], ids[2]], [37, 70], np.concatenate([xs[0][:37], xs[2][:70]]))
    before = [t.clone() for t in bufs]
    y2 = srv.forward(ids, cnt, x_call)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    assert all(torch.equal(a.view(torch.int16), b.view(torch.int16)) if a.dtype == torch.bfloat16
               else torch.equal(a.view(torch.int32), b.view(torch.int32)) for a, b in zip(before, bufs))

    # second tapped call on top of the caches: the empty-past session's follow-up chunk, first block, head 0,
    # whole range; then a replay (Algorithm 3) of a fresh session with the tap on its last rows
    bufs = tap_buffers(shape, 23, 19 + 23)
    arm(srv, 0, ids[1], 0, 0, 23, bufs)
    srv.forward([ids[1]], [23], xs[1][19:42])
    torch.cuda.synchronize()
    t1 = []
    osess[1].forward(xs[1][19:42], t1)
    w1 = check_taps(shape, srv, ids[1], 0, 0, 19, 0, 23, bufs, t1[0])
    fresh = srv.open(320)
    bufs = tap_buffers(shape, 40, 150)
    arm(srv, block, fresh, head, 110, 40, bufs)
    srv.forward([fresh], [150], xs[2][:150], replay=True)
    torch.cuda.synchronize()
    t2 = []
    so.Session(shape, W).forward(xs[2][:150], t2)
    w2 = check_taps(shape, srv, fresh, block, head, 0, 110, 40, bufs, t2[block])
    print(f"{name}: worst logit error / max |logit|: ragged call {w0:.2e}, chunk on a cache {w1:.2e}, replay {w2:.2e}")
    srv.destroy()


def test_taps_that_do_not_fit_the_call_fail_it_and_change_nothing():
    shape = SHAPES["llama-hd64-gqa"]
    srv, W = make(shape)
    x = draw_hidden(shape, 11, 0, 64)
    a, b = srv.open(320), srv.open(320)
    srv.forward([a], [20], x[:20])
    free0 = B.span_debug_free_pages(srv.span)
    big = torch.zeros(1 << 16, dtype=torch.float32, device=DEV)

    def fails(what, sess, head, q0, nq, nbytes, ids, cnt, rows):
        B.span_debug_tap(srv.span, what, 0, sess, head, q0, nq, big, nbytes)
        with pytest.raises(B.SpanError) as e:
            srv.forward(ids, cnt, rows)
        assert e.value.code == B.SPAN_E_INVALID and "tap" in str(e.value)
        assert [B.span_session_length(srv.span, s) for s in (a, b)] == [20, 0]
        assert B.span_debug_free_pages(srv.span) == free0

    fails(B.TAP_Q_ROT, b, -1, 0, 1, 1 << 18, [a], [5], x[20:25])                 # tapped session not in the call
    fails(B.TAP_Q_ROT, a, -1, 3, 3, 1 << 18, [a], [5], x[20:25])                 # range beyond the new tokens
    fails(B.TAP_LOGITS, a, 0, 0, 5, 5 * 25 * 4 - 4, [a], [5], x[20:25])          # buffer too small
    fails(B.TAP_LOGITS, a, 0, 0, 1, 1 << 18, [a], [1], x[20:21])                 # decode step: no logits tap
    # the failed calls disarmed their taps: the next call goes through untouched
    y = srv.forward([a], [5], x[20:25])
    torch.cuda.synchronize()
    assert float(big.abs().max()) == 0.0 and B.span_session_length(srv.span, a) == 25
    ref = so.Session(shape, W).forward(x[:25])[20:]
    assert row_rel_err(to_np(y), ref) < HIDDEN_TOL
    with pytest.raises(B.SpanError):
        B.span_debug_tap(srv.span, 7, 0, a, 0, 0, 1, big, 64)
    with pytest.raises(B.SpanError):
        B.span_debug_tap(srv.span, B.TAP_LOGITS, 0, a, shape.n_q_heads, 0, 1, big, 64)
    with pytest.raises(B.SpanError):
        B.span_debug_tap(srv.span, B.TAP_K_ROT, 2, a, 0, 0, 1, big, 64)
    srv.destroy()

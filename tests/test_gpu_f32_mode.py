"""Single-precision mode (weight_bits = 32): configuration 1 as the configurations state it -- a tiny
Llama-style span with fp32 weights drawn from seed 0 (no bf16 rounding anywhere), 1 session, a 16-token
prefix, 8 decode steps, then a fresh session rebuilt by replaying the 24 stored inputs -- against the
fp64 oracle.  Without bf16 in the way the bar is 1e-5 (element error over the row's rms): fp32 sums of a
few hundred terms.  The same for the BLOOM-style tiny span, a ragged multi-session call with sub-spans,
cache reordering, and the integer state of the paged cache."""
import numpy as np
import pytest
import torch

from gpu_util import *  # noqa: F401,F403
from workloads import TINY, TINY_BLOOM, SpanShape

pytestmark = pytest.mark.gpu

F32_TOL = 1e-5


def make(shape, seed=0, **kw):
    W = SpanWeights(shape, seed=seed, bf16=False, cache=True)              # fp32 draws, not rounded to bf16
    cfg = config_for(shape, max_pages=kw.get("max_pages", 64), max_sessions=8, max_session_tokens=256,
                     max_batch_tokens=kw.get("max_batch_tokens", 256), io_f32=True, weight_bits=32)
    return SpanServer(cfg, W, DEV), W


def kv_err(srv, sess, osess, n_blocks):
    worst = 0.0
    for b in range(n_blocks):
        k, v = srv.read_kv(sess, b, 0, osess.length)
        torch.cuda.synchronize()
        assert k.dtype == torch.float32
        for got, ref in ((to_np(k), osess.k[b]), (to_np(v), osess.v[b])):
            worst = max(worst, float(np.max(np.abs(got - ref)) / np.max(np.abs(ref))))
    return worst


@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
def test_configuration_1_as_written(shape):
    srv, W = make(shape)
    assert not np.array_equal(W[0]["wq"], bf16_round(W[0]["wq"]))          # genuinely fp32 weights
    x = draw_hidden(shape, 0, 0, 24, bf16=False)
    osess = so.Session(shape, W)
    s = srv.open(64)
    ys, refs = [srv.forward([s], [16], x[:16])], [osess.forward(x[:16])]
    for n in range(16, 24):
        ys.append(srv.forward([s], [1], x[n:n + 1]))
        refs.append(osess.forward(x[n:n + 1]))
    torch.cuda.synchronize()
    got, ref = np.concatenate([to_np(y) for y in ys]), np.concatenate(refs)
    e_inc = row_rel_err(got, ref)
    assert e_inc < F32_TOL, e_inc
    assert B.span_session_length(srv.span, s) == 24 and B.span_debug_page_table(srv.span, s) == [0, 1]
    assert kv_err(srv, s, osess, shape.n_blocks) < F32_TOL
    # the server's session is lost: a fresh one replays the 24 stored inputs (Algorithm 3)
    srv.close(s)
    s2 = srv.open(64)
    y_all = to_np(srv.forward([s2], [24], x, replay=True))
    e_rep = row_rel_err(y_all, ref)
    assert e_rep < F32_TOL and row_rel_err(y_all, got) < F32_TOL
    assert kv_err(srv, s2, osess, shape.n_blocks) < F32_TOL
    # cached decode equals recomputing the whole sequence (Sections 2.1 / 3.2), now on the GPU's own numbers
    full = so.span_full(shape, W, x)
    assert row_rel_err(got, full) < F32_TOL
    print(f"{shape.arch}: element error / row rms: prefix + 8 steps {e_inc:.2e}, replay {e_rep:.2e}")
    srv.destroy()


def test_ragged_sessions_sub_spans_and_reordering_in_single_precision():
    shape = SpanShape("llama", 3, 128, 8, 2, 128, 352)                     # 128-wide heads, 4 query heads per kv head
    srv, W = make(shape, seed=5)
    xs = [draw_hidden(shape, 5, i, 80, bf16=False) for i in range(3)]
    ids = [srv.open(200) for _ in range(3)]
    osess = [so.Session(shape, W) for _ in range(3)]
    free0 = B.span_debug_free_pages(srv.span)
    done = [0, 0, 0]
    for cnt in ([17, 0, 33], [1, 20, 1], [1, 1, 0], [30, 1, 1]):
        rows = np.concatenate([xs[i][done[i]:done[i] + c] for i, c in enumerate(cnt)])
        y = to_np(srv.forward(ids, cnt, rows))
        ref = np.concatenate([osess[i].forward(xs[i][done[i]:done[i] + c]) for i, c in enumerate(cnt)])
        assert row_rel_err(y, ref) < F32_TOL, cnt
        done = [d + c for d, c in zip(done, cnt)]
    assert [B.span_session_length(srv.span, s) for s in ids] == done
    tables = [B.span_debug_page_table(srv.span, s) for s in ids]
    assert [len(t) for t in tables] == [(d + 15) // 16 for d in done] and len({p for t in tables for p in t}) == sum(len(t) for t in tables)
    # cache reordering (beam search): entry 0 and 2 continue from the cache of 1, entry 1 from 0
    srv.reorder(ids, [1, 0, 1])
    osess = so.reorder(osess, [1, 0, 1])
    nxt = draw_hidden(shape, 5, 9, 3, bf16=False)
    y = to_np(srv.forward(ids, [1, 1, 1], nxt))
    ref = np.concatenate([o.forward(nxt[i:i + 1]) for i, o in enumerate(osess)])
    assert row_rel_err(y, ref) < F32_TOL
    assert max(kv_err(srv, s, o, shape.n_blocks) for s, o in zip(ids, osess)) < F32_TOL
    # a sub-span chain: blocks [0, 1) on one session, [1, 3) on another, equals the whole span
    a, b = srv.open(200, 0, 1), srv.open(200, 1, 2)
    mid = srv.forward([a], [40], xs[0][:40])
    y = to_np(srv.forward([b], [40], mid))
    assert row_rel_err(y, so.span_full(shape, W, xs[0][:40])) < F32_TOL
    for s in ids + [a, b]:
        srv.close(s)
    assert B.span_debug_free_pages(srv.span) == free0
    srv.destroy()


def test_single_precision_mode_refuses_what_it_does_not_have():
    srv, _ = make(TINY)
    s = srv.open(64)
    buf = torch.zeros(1024, dtype=torch.float32, device=DEV)
    with pytest.raises(B.SpanError):
        B.span_debug_tap(srv.span, B.TAP_Q_ROT, 0, s, -1, 0, 1, buf, 4096)
    with pytest.raises(B.SpanError):
        B.span_train_sizes(srv.cfg, 16)
    with pytest.raises(B.SpanError):                                      # bf16 I/O cannot carry fp32 rows
        B.span_query_sizes(config_for(TINY, max_pages=8, max_sessions=2, max_session_tokens=64, max_batch_tokens=64,
                                      io_f32=False, weight_bits=32))
    srv.destroy()

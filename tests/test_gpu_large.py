"""Parity at the full shapes of the benchmark configurations (7B-, 70B- and BLOOM-176B-shaped
spans, and the ragged fail-over replay), in the launch configuration bench.py times.

The oracle cannot afford every session at these sizes, so it computes sampled sessions
completely (sessions are independent, so a per-session oracle is exact) and the rest is
covered by properties that hold at any size: a session fed the same inputs as a checked one
must give the same outputs, and a replay-rebuilt run must match the uninterrupted run.
The oracle runs the whole token sequence of a session through each block in one piece (the
cached form it is pinned against on small inputs gives the same result, Sections 2.1/3.2),
in fp32 at the 70B / 176B shapes to stay within minutes of host time.

Bars: every block on its own (sessions opened on one block, fed the oracle's input of that block)
meets the benchmark spec's 2e-2; whole spans of the 70B- and 176B-shaped configurations are held to 1.25 x
the floor of the bf16 precision contract itself (gpu_bars, from tests/golden/precision_floor.txt: a
numpy model of the contract against the oracle, no GPU involved): the largest row and element errors
within a quarter of it, the rms element error within 5 % of it.  The model's own output, computed
beside the oracle on the same inputs, is compared too: the GPU must lie closer to it than the oracle
does (two realisations of one contract; see gpu_util on why they cannot coincide).
"""
import time

import numpy as np
import pytest
import torch

import precision_model as pm
from conftest import progress
from gpu_util import *  # noqa: F401,F403
from workloads import WORKLOADS, SpanWeights, draw_hidden

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def oracle_block_by_block(shape, weights, x, dtype):
    """Whole sequence x [N, d] through all blocks, no cache; returns outputs of every position."""
    h = np.asarray(x, dtype=dtype)
    empty = np.zeros((0, shape.n_kv_heads, shape.head_dim), dtype)
    for b in range(shape.n_blocks):
        h = so.block_forward(shape, weights[b], h, empty, empty, dtype=dtype, matrix_attention=True)[0]
    return h.astype(np.float64)


def build(shape, wl, max_len, max_batch_tokens, n_sessions, seed=0, keep_canonical=False):
    t0 = time.time()
    W = SpanWeights(shape, seed=seed, bf16=True, cache=True, threads=16)
    pages = n_sessions * ((max_len + 15) // 16) + 4
    cfg = config_for(shape, max_pages=pages, max_sessions=n_sessions, max_session_tokens=max_len,
                     max_batch_tokens=max_batch_tokens, io_f32=True)
    srv = SpanServer(cfg, W, DEV, keep_canonical=keep_canonical)
    progress(f"  [{wl}] weights drawn, uploaded and packed in {time.time() - t0:.0f} s")
    return srv, W


def model_span(shape, weights, x):
    """The bf16 precision model of the whole span on one session's inputs (norms folded as the path folds them)."""
    return pm.Session(shape, weights).forward(np.asarray(x, np.float32)).astype(np.float64)


def test_llama7b_prefix_and_128_decode_steps():
    """Configuration 2 in full: 4 sessions x (512-token prefix + 128 batched decode steps); all checked
    against the oracle (2e-2 end to end) and against the precision model."""
    wl = WORKLOADS["llama7b"]
    shape = wl.shape
    srv, W = build(shape, "llama7b", 640, 2048, 4)
    xs = [draw_hidden(shape, wl.seed, i, 640) for i in range(4)]
    ids = [srv.open(640) for _ in range(4)]
    y_prefix = to_np(srv.forward(ids, [512] * 4, np.concatenate([x[:512] for x in xs])))
    y_dec = []
    for t in range(512, 640):
        y_dec.append(srv.forward(ids, [1] * 4, np.stack([x[t] for x in xs])))
    torch.cuda.synchronize()
    y_dec = np.stack([to_np(y) for y in y_dec])                  # [128, 4, d]
    (_, elem_p, rms_p), (_, elem_d, rms_d) = deep_span_bars("llama7b", rows="prefix"), deep_span_bars("llama7b", rows="decode")
    for i in range(4):
        ref = oracle_block_by_block(shape, W, xs[i], np.float64)
        mod = model_span(shape, W, xs[i])
        ep = check_hidden(y_prefix[i * 512:(i + 1) * 512], ref[:512], HIDDEN_TOL, elem_p, rms_p)
        ed = check_hidden(y_dec[:, i], ref[512:], HIDDEN_TOL, elem_d, rms_d)
        mp = check_hidden(y_prefix[i * 512:(i + 1) * 512], mod[:512], HIDDEN_TOL)
        md = check_hidden(y_dec[:, i], mod[512:], HIDDEN_TOL)
        progress(f"  [llama7b] session {i}: (row rel err, max elem err, rms err) prefix {ep[0]:.2e} {ep[1]:.2e} {ep[2]:.2e}"
                 f" | decode {ed[0]:.2e} {ed[1]:.2e} {ed[2]:.2e} | vs precision model: prefix {mp[0]:.2e} decode {md[0]:.2e}"
                 f" (model's own floor {row_l2_rel_err(mod, ref):.2e})")
    assert all(B.span_session_length(srv.span, s) == 640 for s in ids)
    srv.destroy()


@pytest.fixture(scope="module")
def server70b():
    wl = WORKLOADS["llama70b"]
    srv, W = build(wl.shape, "llama70b", 4096 + 64 + 16, 16384, 16, keep_canonical=True)
    yield srv, W
    srv.destroy()


N_70B = 2048 + 128          # configuration 3: 2048-token prefix + 128 decode steps
_ORACLE_70B = {}


def oracle_70b_session0(shape, weights):
    """Session 0 of the 70B workload (2048 + 128 tokens) through the fp32 oracle -- the inputs of every block
    and the span output -- and through the bf16 precision model of the whole span.  Computed once per test
    module run (a few minutes of host time) and shared by the tests that follow: attention is causal, so the
    first n rows are what a shorter run of n tokens gives."""
    if not _ORACLE_70B:
        wl = WORKLOADS["llama70b"]
        x = draw_hidden(shape, wl.seed, 0, N_70B)
        t0 = time.time()
        _ORACLE_70B["x"] = x
        _ORACLE_70B["hs"] = oracle_inputs_per_block(shape, weights, x)
        t1 = time.time()
        progress(f"  [llama70b] one session ({N_70B} tokens x 8 blocks): fp32 oracle {t1 - t0:.0f} s")
        _ORACLE_70B["model"] = model_span(shape, weights, x)
        progress(f"  [llama70b] the same through the bf16 precision model: {time.time() - t1:.0f} s; the model's own floor "
                 f"against the oracle: {row_l2_rel_err(_ORACLE_70B['model'], _ORACLE_70B['hs'][-1]):.2e}")
    return _ORACLE_70B


def oracle_inputs_per_block(shape, weights, x, dtype=np.float32):
    """Inputs of every block (and the span output) for one whole sequence x, from the oracle."""
    hs = [np.asarray(x, dtype=dtype)]
    empty = np.zeros((0, shape.n_kv_heads, shape.head_dim), dtype)
    for b in range(shape.n_blocks):
        hs.append(so.block_forward(shape, weights[b], hs[-1], empty, empty, dtype=dtype, matrix_attention=True)[0])
    return hs


def test_llama70b_replay_prefill_and_decode(server70b):
    """Configuration 3 at full shape and full length: 8 sessions x 2048-token prefix rebuilt by cache
    replay, then all 128 batched decode steps.  Session 0 is followed by the oracle at every position,
      (a) block by block: sessions opened on one block each (sub-segment requests) receive the
          oracle's own input of that block, so every block is held to HIDDEN_TOL (2e-2) at full shape
          without the error of earlier blocks in its input;
      (b) through the whole 8-block span: against the oracle under the bars derived from the floor of
          the bf16 contract (gpu_bars); the distance from the bf16 precision model itself stays under that floor.
    Session 7 is fed the same inputs as session 0 and must reproduce its outputs."""
    srv, W = server70b
    wl = WORKLOADS["llama70b"]
    shape = wl.shape
    n_dec = wl.decode_steps
    N = 2048 + n_dec
    assert N == N_70B and n_dec == 128
    o70 = oracle_70b_session0(shape, W)
    hs = o70["hs"]
    xs = [o70["x"]] + [draw_hidden(shape, wl.seed, i, N) for i in range(1, 7)] + [o70["x"]]

    def run(first_block, n_blocks, x0):
        """8 sessions on the given block range; sessions 0 and 7 get x0, the others their own draws."""
        inputs = [x0] + xs[1:7] + [x0]
        ids = [srv.open(N, first_block, n_blocks) for _ in range(8)]
        y_pre = srv.forward(ids, [2048] * 8, np.concatenate([x[:2048] for x in inputs]), replay=True)
        y_dec = [srv.forward(ids, [1] * 8, np.stack([x[2048 + t] for x in inputs])) for t in range(n_dec)]
        torch.cuda.synchronize()
        assert all(B.span_session_length(srv.span, s) == N for s in ids)
        for s in ids:
            srv.close(s)
        y_pre = y_pre.view(8, 2048, shape.d_model)
        y_dec = torch.stack(y_dec)                               # [n_dec, 8, d]
        # identical inputs -> identical outputs, wherever the rows sit in the batch
        same = max(float((y_pre[7] - y_pre[0]).abs().max()), float((y_dec[:, 7] - y_dec[:, 0]).abs().max()))
        assert same <= 1e-5 * float(y_pre[0].abs().max()), same
        return to_np(y_pre[0]), to_np(y_dec[:, 0])

    empty = np.zeros((0, shape.n_kv_heads, shape.head_dim), np.float32)
    for b in range(shape.n_blocks):
        y_pre, y_dec = run(b, 1, hs[b])
        ref = hs[b + 1].astype(np.float64)
        (_, elem_p, rms_p), (_, elem_d, rms_d) = alone_bars("llama70b", b + 1, "prefix"), alone_bars("llama70b", b + 1, "decode")
        ep, ed = check_hidden(y_pre, ref[:2048], HIDDEN_TOL, elem_p, rms_p), check_hidden(y_dec, ref[2048:], HIDDEN_TOL, elem_d, rms_d)
        # the same block through the precision model, fed the same rows: what the kernels add of their own
        mod = pm.block_forward(shape, W[b], hs[b], empty, empty, pm.ALL_POINTS, folded_norm1=False)[0].astype(np.float64)
        fl = floor_of("llama70b", "alone", b + 1)
        mp, md = check_hidden(y_pre, mod[:2048], fl), check_hidden(y_dec, mod[2048:], fl)
        progress(f"  [llama70b] block {b} alone (row rel err, max elem err, rms err): replay {ep[0]:.2e} {ep[1]:.2e} "
                 f"{ep[2]:.2e} | {n_dec} decode steps {ed[0]:.2e} {ed[1]:.2e} {ed[2]:.2e} | vs precision model: replay "
                 f"{mp[0]:.2e} decode {md[0]:.2e}")
    y_pre, y_dec = run(0, shape.n_blocks, xs[0])
    ref, mod = hs[-1].astype(np.float64), o70["model"]
    (row_bar, elem_bar, rms_p), (row_d, elem_d, rms_d) = deep_span_bars("llama70b", rows="prefix"), deep_span_bars("llama70b", rows="decode")
    ep, ed = check_hidden(y_pre, ref[:2048], row_bar, elem_bar, rms_p), check_hidden(y_dec, ref[2048:], row_d, elem_d, rms_d)
    fl = floor_of("llama70b", "span", shape.n_blocks)
    mp, md = check_hidden(y_pre, mod[:2048], fl), check_hidden(y_dec, mod[2048:], fl)
    progress(f"  [llama70b] whole span vs oracle (row rel err, max elem err, rms err; bars {row_bar:.2e}, {elem_bar:.2e}): "
             f"replay {ep[0]:.2e} {ep[1]:.2e} {ep[2]:.2e} | {n_dec} decode steps {ed[0]:.2e} {ed[1]:.2e} {ed[2]:.2e}")
    progress(f"  [llama70b] whole span vs bf16 precision model: replay {mp[0]:.2e} {mp[1]:.2e} {mp[2]:.2e}"
             f" | decode {md[0]:.2e} {md[1]:.2e} {md[2]:.2e}")


def test_llama70b_decode_sessions_and_a_replaying_session_in_one_call(server70b):
    """Continuous batching at full shape: seven sessions with 2048 cached tokens take a decode step
    in the same call in which an eighth, fresh session replays its 2048 stored inputs (a failed
    peer's client arriving while others generate).  Session 0 and the newcomer both carry the
    inputs the oracle followed: the decode row and all 2048 replayed rows are checked against it,
    then all eight decode together and the newcomer must agree with session 0 from then on."""
    srv, W = server70b
    wl = WORKLOADS["llama70b"]
    shape = wl.shape
    N = 2048 + 8
    o70 = oracle_70b_session0(shape, W)
    x0, ref = o70["x"][:N], o70["hs"][-1].astype(np.float64)
    row_bar, elem_bar, _ = deep_span_bars("llama70b")
    rms_p = deep_span_bars("llama70b", rows="prefix")[2]
    xs = [x0] + [draw_hidden(shape, wl.seed, i, N) for i in range(1, 7)]
    free0 = B.span_debug_free_pages(srv.span)
    ids = [srv.open(N) for _ in range(7)]
    srv.forward(ids, [2048] * 7, np.concatenate([x[:2048] for x in xs]), replay=True)
    new = srv.open(N)
    # the mixed call: 7 x 1 token + 1 x 2048 tokens
    y = srv.forward(ids + [new], [1] * 7 + [2048], np.concatenate([np.stack([x[2048] for x in xs]), x0[:2048]]))
    torch.cuda.synchronize()
    assert [B.span_session_length(srv.span, s) for s in ids + [new]] == [2049] * 7 + [2048]
    e_dec = check_hidden(to_np(y[0:1]), ref[2048:2049], row_bar, elem_bar)
    e_rep = check_hidden(to_np(y[7:]), ref[:2048], row_bar, elem_bar, rms_p)
    check_hidden(to_np(y[7:]), o70["model"][:2048], floor_of("llama70b", "span", shape.n_blocks))
    progress(f"  [llama70b] mixed call (row rel err, max elem err, rms err): decode row {e_dec[0]:.2e} | replayed rows "
             f"{e_rep[0]:.2e} {e_rep[1]:.2e} {e_rep[2]:.2e}")
    # the newcomer catches up (token 2048), then all eight decode in lock step
    y_new = srv.forward([new], [1], x0[2048:2049])
    e_new = check_hidden(to_np(y_new), ref[2048:2049], row_bar, elem_bar)
    worst = 0.0
    for t in range(2049, N):
        y = srv.forward(ids + [new], [1] * 8, np.stack([x[t] for x in xs] + [x0[t]]))
        check_hidden(to_np(y[0:1]), ref[t:t + 1], row_bar, elem_bar)
        check_hidden(to_np(y[7:8]), ref[t:t + 1], row_bar, elem_bar)
        worst = max(worst, row_l2_rel_err(to_np(y[7:8]), to_np(y[0:1])))
    progress(f"  [llama70b] newcomer's first decode row vs oracle {e_new[0]:.2e}; newcomer vs session 0 over "
             f"{N - 2049} joint steps (row rel err) {worst:.2e}")
    assert worst < HIDDEN_TOL          # two GPU runs of the same session: its cache built by different kernels
    tables = [B.span_debug_page_table(srv.span, s) for s in ids + [new]]
    flat = [p for t in tables for p in t]
    assert len(set(flat)) == len(flat) and [len(t) for t in tables] == [(N + 15) // 16] * 8
    for s in ids + [new]:
        srv.close(s)
    assert B.span_debug_free_pages(srv.span) == free0


def test_llama70b_short_calls_follow_the_oracle(server70b):
    """Prompt chunks of 100, 128, 160 and 192 tokens at full shape (the narrow projections of the first
    two run as skinny launches over 64-row chunks, the last two as tiles with a padded band of token
    tiles), each on top of the cache the earlier ones left: the outputs are the first 580 rows of the
    oracle's uninterrupted run."""
    srv, W = server70b
    wl = WORKLOADS["llama70b"]
    shape = wl.shape
    o70 = oracle_70b_session0(shape, W)
    x0, ref = o70["x"], o70["hs"][-1].astype(np.float64)
    row_bar, elem_bar, _ = deep_span_bars("llama70b")
    free0 = B.span_debug_free_pages(srv.span)
    sid = srv.open(1024)
    off, worst = 0, 0.0
    for n in (100, 128, 160, 192):
        y = srv.forward([sid], [n], x0[off:off + n])
        worst = max(worst, check_hidden(to_np(y), ref[off:off + n], row_bar, elem_bar)[0])
        off += n
    progress(f"  [llama70b] calls of 100, 128, 160, 192 tokens, whole span: worst row rel err {worst:.2e}")
    assert B.span_session_length(srv.span, sid) == off
    srv.close(sid)
    assert B.span_debug_free_pages(srv.span) == free0


def test_llama70b_beam_clones_continue_like_their_source(server70b):
    """Cache reordering at full shape: a 2050-token session (last page partly filled) is cloned
    into three empty sessions; the four then take the same decode steps.  Every clone must
    reproduce the source (same inputs, same outputs) and follow the oracle; only the partly
    filled page is copied, the 128 full pages are shared."""
    srv, W = server70b
    wl = WORKLOADS["llama70b"]
    shape = wl.shape
    N = 2048 + 8
    o70 = oracle_70b_session0(shape, W)
    x0, ref = o70["x"][:N], o70["hs"][-1].astype(np.float64)
    row_bar, elem_bar, _ = deep_span_bars("llama70b")
    free0 = B.span_debug_free_pages(srv.span)
    ids = [srv.open(N) for _ in range(4)]
    srv.forward(ids[:1], [2050], x0[:2050], replay=True)
    srv.reorder(ids, [0, 0, 0, 0])
    tables = [B.span_debug_page_table(srv.span, s) for s in ids]
    assert all(t[:128] == tables[0][:128] for t in tables) and len({t[128] for t in tables}) == 4
    assert B.span_debug_free_pages(srv.span) == free0 - 128 - 4
    worst = 0.0
    for t in range(2050, N):
        y = srv.forward(ids, [1] * 4, np.stack([x0[t]] * 4))
        check_hidden(to_np(y[0:1]), ref[t:t + 1], row_bar, elem_bar)
        worst = max(worst, float((y[1:] - y[0:1]).abs().max()) / float(y[0].abs().max()))
    progress(f"  [llama70b] three clones vs their source over {N - 2050} steps: max difference {worst:.1e} of the largest output")
    assert worst <= 1e-5
    # drop the source, keep one clone, move another: 128 shared pages stay alive until the last holder closes
    srv.reorder(ids, [1, 1, 3, 3])
    srv.close(ids[0]); srv.close(ids[2]); srv.close(ids[3])
    assert len(B.span_debug_page_table(srv.span, ids[1])) == (N + 15) // 16
    k, v = srv.read_kv(ids[1], 7, 2040, 16)
    torch.cuda.synchronize()
    assert torch.isfinite(k.float()).all() and float(k.float().abs().max()) > 0
    srv.close(ids[1])
    assert B.span_debug_free_pages(srv.span) == free0


def test_failover_ragged_replay_matches_uninterrupted_run(server70b):
    """Configuration 5: 16 sessions with ragged histories (128..4096 tokens).  Server A builds the
    caches incrementally (512-token requests), server B by one ragged cache replay of the stored
    inputs (Algorithm 3); both then run the same 64 decode steps with sessions of all lengths
    in one batch.  B must match A, and the shortest and the median-length session are checked against
    the oracle and the precision model (caches included: the 64 decode steps read them)."""
    srv, W = server70b
    wl = WORKLOADS["failover70b"]
    shape = wl.shape
    lens = list(wl.prefix_lens)
    n_dec = wl.decode_steps
    xs = [draw_hidden(shape, wl.seed, i, L + n_dec) for i, L in enumerate(lens)]
    x_dec = [np.stack([x[L + t] for x, L in zip(xs, lens)]) for t in range(n_dec)]
    free0 = B.span_debug_free_pages(srv.span)

    def decode(ids):
        out = [srv.forward(ids, [1] * 16, x_dec[t]) for t in range(n_dec)]
        torch.cuda.synchronize()
        return torch.stack(out)

    # --- server A: uninterrupted, caches built request by request
    t0 = time.time()
    ids = [srv.open(L + n_dec) for L in lens]
    ya_pre = [[] for _ in lens]
    done = [0] * 16
    while any(d < L for d, L in zip(done, lens)):
        cnt = [min(512, L - d) for d, L in zip(done, lens)]
        act = [i for i in range(16) if cnt[i] > 0]
        y = srv.forward([ids[i] for i in act], [cnt[i] for i in act],
                        np.concatenate([xs[i][done[i]:done[i] + cnt[i]] for i in act]))
        off = 0
        for i in act:
            ya_pre[i].append(y[off:off + cnt[i]])
            off += cnt[i]
            done[i] += cnt[i]
    ya_pre = [torch.cat(p) for p in ya_pre]
    ya_dec = decode(ids)
    pages_a = [B.span_debug_page_table(srv.span, s) for s in ids]
    assert len({p for pt in pages_a for p in pt}) == sum(len(pt) for pt in pages_a)      # pages are disjoint
    assert [len(pt) for pt in pages_a] == [(L + n_dec + 15) // 16 for L in lens]
    for s in ids:
        srv.close(s)
    assert B.span_debug_free_pages(srv.span) == free0
    progress(f"  [failover] server A (incremental, {sum(lens)} tokens + {n_dec} steps) took {time.time() - t0:.1f} s")

    # --- server B: every session lost; fresh sessions replay the client-side caches in one ragged request
    t0 = time.time()
    ids = [srv.open(L + n_dec) for L in lens]
    yb_all = srv.forward(ids, lens, np.concatenate([x[:L] for x, L in zip(xs, lens)]), replay=True)
    yb_dec = decode(ids)
    progress(f"  [failover] server B (ragged replay + {n_dec} steps) took {time.time() - t0:.1f} s")
    off, worst_pre = 0, 0.0
    for i, L in enumerate(lens):
        worst_pre = max(worst_pre, check_hidden_where_different(to_np(yb_all[off:off + L]), to_np(ya_pre[i]), HIDDEN_TOL))
        off += L
    worst_dec = check_hidden_where_different(to_np(yb_dec).reshape(-1, shape.d_model), to_np(ya_dec).reshape(-1, shape.d_model),
                                             HIDDEN_TOL)
    progress(f"  [failover] B vs A (row rel err): replay outputs {worst_pre:.2e}, continued decode {worst_dec:.2e}")
    assert [B.span_session_length(srv.span, s) for s in ids] == [L + n_dec for L in lens]

    # --- oracle and precision model on the shortest and on the median-length session
    row_bar, elem_bar, rms_bar = deep_span_bars("failover70b")
    fl = floor_of("failover70b", "span", shape.n_blocks)
    order = np.argsort(lens)
    for i in (int(order[0]), int(order[len(order) // 2])):
        t0 = time.time()
        ref = oracle_block_by_block(shape, W, xs[i], np.float32)
        mod = model_span(shape, W, xs[i])
        start, L = sum(lens[:i]), lens[i]
        e_b = check_hidden(to_np(yb_all[start:start + L]), ref[:L], row_bar, elem_bar, rms_bar)
        e_bd = check_hidden(to_np(yb_dec[:, i]), ref[L:], row_bar, elem_bar, rms_bar)
        e_a = check_hidden(to_np(ya_pre[i]), ref[:L], row_bar, elem_bar, rms_bar)
        e_ad = check_hidden(to_np(ya_dec[:, i]), ref[L:], row_bar, elem_bar, rms_bar)
        m_b = check_hidden(to_np(yb_all[start:start + L]), mod[:L], fl)
        m_bd = check_hidden(to_np(yb_dec[:, i]), mod[L:], fl)
        progress(f"  [failover] session {i} (L={L}) vs oracle (row rel err / max elem err; bars {row_bar:.2e} / {elem_bar:.2e}): "
                 f"replay {e_b[0]:.2e} / {e_b[1]:.2e}, decode after replay {e_bd[0]:.2e} / {e_bd[1]:.2e}, uninterrupted prefix "
                 f"{e_a[0]:.2e}, decode {e_ad[0]:.2e} | vs precision model: replay {m_b[0]:.2e}, decode {m_bd[0]:.2e} "
                 f"(oracle + model took {time.time() - t0:.0f} s)")
    for s in ids:
        srv.close(s)


def test_llama70b_training_passes(server70b):
    """Training-time passes (Section 3.3) at the 70B shape.  The oracle (fp64 reverse-mode through
    its own forward) can afford one and two blocks on a 203-token batch.  As for the forward path,
    a single block is held to the tight bar (GRAD_TOL) and the chain of two to that bar scaled by the
    growth the forward precision model shows over the same depth (stored floor after two blocks / after
    one): the error a block's backward pass receives is amplified by the blocks before it.  The 1227-token batch of 128-token sequences that takes the direct-to-LDS tiled
    kernel (the shape bench.py times) is then checked by a property that holds at any size: the
    sequences of a batch are independent, so each sequence's gradient must equal the one it gets
    in a small batch, through two blocks and through the whole 8-block span."""
    from oracle import backward_oracle as bo
    srv, W = server70b
    wl = WORKLOADS["llama70b"]
    shape = wl.shape
    srv.attach_training(1536)
    rng = np.random.default_rng(77)
    small = [128, 75]
    big = [128] * 4 + [75] + [128] * 4 + [128 + 128]               # 1227 tokens; sequences 0 and 4 are the small batch
    xs = [draw_hidden(shape, wl.seed, 100 + i, n) for i, n in enumerate(big)]
    gs = [bf16_round(rng.standard_normal((n, shape.d_model)).astype(np.float32)) for n in big]
    x_small, g_small = np.concatenate([xs[0], xs[4]]), np.concatenate([gs[0], gs[4]])
    x_big, g_big = np.concatenate(xs), np.concatenate(gs)
    off4 = sum(big[:4])

    t0 = time.time()
    _, gx_ref1 = bo.span_forward_backward(shape, W, x_small, g_small, small, first_block=1, n_blocks=1)
    y_ref, gx_ref = bo.span_forward_backward(shape, W, x_small, g_small, small, first_block=0, n_blocks=2)
    progress(f"  [llama70b] fp64 oracle forward + backward, 1 block and 2 blocks x 203 tokens: {time.time() - t0:.0f} s")
    gx1 = srv.backward(small, x_small, g_small, first_block=1, n_blocks=1)
    gx2, y2 = srv.backward(small, x_small, g_small, first_block=0, n_blocks=2, want_y=True)
    gx2_big = srv.backward(big, x_big, g_big, first_block=0, n_blocks=2)
    gx8 = srv.backward(small, x_small, g_small)
    gx8_big, y8_big = srv.backward(big, x_big, g_big, want_y=True)
    y8 = srv.train_forward(small, x_small)
    torch.cuda.synchronize()
    grad_chain_tol = GRAD_TOL * deep_span_bars("llama70b", 2)[0] / deep_span_bars("llama70b", 1)[0]
    e1 = check_hidden(to_np(gx1), gx_ref1, GRAD_TOL)
    ey = check_hidden(to_np(y2), y_ref)
    eg = check_hidden(to_np(gx2), gx_ref, grad_chain_tol)
    progress(f"  [llama70b] vs oracle (row rel err, max elem err, rms err): 1 block grad_x {e1[0]:.2e} {e1[1]:.2e} {e1[2]:.2e}"
             f" | 2 blocks y {ey[0]:.2e} {ey[1]:.2e} {ey[2]:.2e} grad_x {eg[0]:.2e} {eg[1]:.2e} {eg[2]:.2e}")

    def pick(t):
        a = to_np(t)
        return np.concatenate([a[:128], a[off4:off4 + 75]])
    e2 = check_hidden(pick(gx2_big), gx_ref, grad_chain_tol)
    e2g = row_l2_rel_err(pick(gx2_big), to_np(gx2))
    e8g = row_l2_rel_err(pick(gx8_big), to_np(gx8))
    e8y = row_l2_rel_err(pick(y8_big), to_np(y8))
    progress(f"  [llama70b] 1227-token batch: 2 blocks vs oracle {e2[0]:.2e}; vs the small batch on the GPU: 2 blocks "
             f"{e2g:.2e}, 8 blocks grad {e8g:.2e}, 8 blocks y {e8y:.2e}")
    assert e2g < HIDDEN_TOL and e8g < HIDDEN_TOL and e8y < HIDDEN_TOL      # GPU against GPU: another summation order only
    assert np.all(np.isfinite(to_np(gx8_big)))


def test_bloom176b_prefix_and_decode():
    """Configuration 4 at full shape and full length: 16 sessions x 128-token prefix, then all 64 batched
    decode steps.  The oracle and the bf16 precision model follow sessions 0 and 9 (fp32, block by block
    as the weights are drawn); like the 70B case, every block is checked on its own with the oracle's
    inputs (HIDDEN_TOL) and the whole 4-block span end to end (bars from the stored floor of the bf16
    contract; closer to the model than the oracle is).  Then one block's backward pass against the fp64 oracle."""
    wl = WORKLOADS["bloom176b"]
    shape = wl.shape
    n_dec = wl.decode_steps
    N = 128 + n_dec
    assert n_dec == 64
    W = SpanWeights(shape, seed=wl.seed, bf16=True, cache=False, threads=16)
    xs = [draw_hidden(shape, wl.seed, i, N) for i in range(16)]
    checked = [0, 9]
    hs = {i: [xs[i].astype(np.float32)] for i in checked}
    mod = {i: xs[i].astype(np.float32) for i in checked}
    carry = {i: {} for i in checked}
    empty = np.zeros((0, shape.n_kv_heads, shape.head_dim), np.float32)
    dev_w = []
    from oracle import backward_oracle as bo
    lens_t = [96, 37]
    x_t = np.concatenate([xs[3][:96], xs[5][:37]])
    g_t = bf16_round(np.random.default_rng(176).standard_normal(x_t.shape).astype(np.float32))
    t0 = time.time()
    for b in range(shape.n_blocks):
        w = W[b]
        dev_w.append({k: dev_bf16(v) for k, v in w.items()})
        for i in checked:
            hs[i].append(so.block_forward(shape, w, hs[i][-1], empty, empty, dtype=np.float32, matrix_attention=True)[0])
            mod[i] = pm.block_forward(shape, w, mod[i], empty, empty, pm.ALL_POINTS, folded_norm1=b > 0, carry=carry[i])[0]
        if b == 1:
            # training-time passes through this block (LayerNorm, GELU and ALiBi derivatives at full shape):
            # the fp64 oracle while the block's weights are in hand
            gx_ref_t = bo.span_forward_backward(shape, {1: w}, x_t, g_t, lens_t, first_block=1, n_blocks=1)[1]
        del w
        progress(f"  [bloom176b] block {b}: weights drawn + uploaded, oracle advanced ({time.time() - t0:.0f} s)")
    cfg = config_for(shape, max_pages=16 * ((N + 15) // 16) + 4, max_sessions=16, max_session_tokens=N,
                     max_batch_tokens=2048, io_f32=True)
    srv = SpanServer(cfg, dev_w, DEV, keep_canonical=True)
    del dev_w

    def run(first_block, n_blocks, level):
        inputs = [hs[i][level] if i in checked else xs[i] for i in range(16)]
        ids = [srv.open(N, first_block, n_blocks) for _ in range(16)]
        y_pre = srv.forward(ids, [128] * 16, np.concatenate([x[:128] for x in inputs])).view(16, 128, shape.d_model)
        y_dec = torch.stack([srv.forward(ids, [1] * 16, np.stack([x[128 + t] for x in inputs])) for t in range(n_dec)])
        torch.cuda.synchronize()
        for s in ids:
            srv.close(s)
        return y_pre, y_dec

    row_bar, elem_bar, rms_bar = deep_span_bars("bloom176b")
    fl = floor_of("bloom176b", "span", shape.n_blocks)
    for b in range(shape.n_blocks):
        y_pre, y_dec = run(b, 1, b)
        for i in checked:
            ref = hs[i][b + 1].astype(np.float64)
            _, elem_alone, rms_alone = alone_bars("bloom176b", b + 1)
            ep = check_hidden(to_np(y_pre[i]), ref[:128], HIDDEN_TOL, elem_alone, rms_alone)
            ed = check_hidden(to_np(y_dec[:, i]), ref[128:], HIDDEN_TOL, elem_alone, rms_alone)
            progress(f"  [bloom176b] block {b} alone, session {i} (row rel err, max elem err, rms err): prefix {ep[0]:.2e} "
                     f"{ep[1]:.2e} {ep[2]:.2e} | decode {ed[0]:.2e} {ed[1]:.2e} {ed[2]:.2e}")
    y_pre, y_dec = run(0, shape.n_blocks, 0)
    for i in checked:
        ref = hs[i][-1].astype(np.float64)
        ep = check_hidden(to_np(y_pre[i]), ref[:128], row_bar, elem_bar, rms_bar)
        ed = check_hidden(to_np(y_dec[:, i]), ref[128:], row_bar, elem_bar, rms_bar)
        m = mod[i].astype(np.float64)
        mp, md = check_hidden(to_np(y_pre[i]), m[:128], fl), check_hidden(to_np(y_dec[:, i]), m[128:], fl)
        progress(f"  [bloom176b] whole span, session {i} vs oracle (row rel err, max elem err, rms err; bars {row_bar:.2e}, "
                 f"{elem_bar:.2e}): prefix {ep[0]:.2e} {ep[1]:.2e} {ep[2]:.2e} | {n_dec} decode steps {ed[0]:.2e} {ed[1]:.2e} "
                 f"{ed[2]:.2e} | vs precision model: prefix {mp[0]:.2e} decode {md[0]:.2e} (model's own floor "
                 f"{row_l2_rel_err(m, ref):.2e})")
    srv.attach_training(256)
    gx = srv.backward(lens_t, x_t, g_t, first_block=1, n_blocks=1)
    torch.cuda.synchronize()
    eg = check_hidden(to_np(gx), gx_ref_t, GRAD_TOL)
    progress(f"  [bloom176b] block 1, backward w.r.t. the inputs of 96 + 37 tokens (row rel err, max elem err, rms err): "
             f"{eg[0]:.2e} {eg[1]:.2e} {eg[2]:.2e}")
    srv.destroy()

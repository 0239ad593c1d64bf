"""End-to-end parity of the span path against the oracle on the small configurations:
prefix + decode steps, replay on a fresh session, ragged multi-session batches, sub-spans,
and the integer state of the paged cache."""
import numpy as np
import pytest
import torch

from gpu_util import *  # noqa: F401,F403
from workloads import TINY, TINY_BLOOM, SpanShape

pytestmark = pytest.mark.gpu


def make_server(shape, *, max_pages=64, max_sessions=8, max_session_tokens=256, max_batch_tokens=512, seed=0,
                io_f32=True, weight_bits=0, levels=None):
    W = SpanWeights(shape, seed=seed, bf16=True, cache=True)
    cfg = config_for(shape, max_pages=max_pages, max_sessions=max_sessions, max_session_tokens=max_session_tokens,
                     max_batch_tokens=max_batch_tokens, io_f32=io_f32, weight_bits=weight_bits, levels=levels)
    return SpanServer(cfg, W, DEV), W


def check_kv(srv, sess, osess, n_blocks):
    worst = 0.0
    for b in range(n_blocks):
        k, v = srv.read_kv(sess, b, 0, osess.length)
        torch.cuda.synchronize()
        for got, ref in ((to_np(k), osess.k[b]), (to_np(v), osess.v[b])):
            scale = np.max(np.abs(ref)) + 1e-30
            worst = max(worst, float(np.max(np.abs(got - ref)) / scale))
    return worst


@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
def test_prefix_decode_then_replay(shape):
    """Configuration 1 protocol: 16-token prefix, 8 decode steps, then a fresh session
    rebuilt from the 24 stored inputs (Algorithm 3) must match the uninterrupted run."""
    srv, W = make_server(shape)
    x = draw_hidden(shape, 0, 0, 25)
    osess = so.Session(shape, W)
    s = srv.open(64)
    ys = [srv.forward([s], [16], x[:16])]
    refs = [osess.forward(x[:16])]
    for n in range(16, 24):
        ys.append(srv.forward([s], [1], x[n:n + 1]))
        refs.append(osess.forward(x[n:n + 1]))
    torch.cuda.synchronize()
    got, ref = np.concatenate([to_np(y) for y in ys]), np.concatenate(refs)
    assert row_rel_err(got, ref) < HIDDEN_TOL
    assert B.span_session_length(srv.span, s) == 24
    assert check_kv(srv, s, osess, shape.n_blocks) < KV_TOL

    # failure: the server's session is lost; a fresh one replays the client-side cache
    srv.close(s)
    s2 = srv.open(64)
    y_all = srv.forward([s2], [24], x[:24], replay=True)
    torch.cuda.synchronize()
    assert row_rel_err(to_np(y_all), ref) < HIDDEN_TOL
    assert row_rel_err(to_np(y_all), got) < HIDDEN_TOL            # GPU replay vs GPU incremental
    assert B.span_session_length(srv.span, s2) == 24
    assert check_kv(srv, s2, osess, shape.n_blocks) < KV_TOL
    # and generation continues identically after the replay
    y_next = srv.forward([s2], [1], x[24:25])
    ref_next = osess.forward(x[24:25])
    torch.cuda.synchronize()
    assert row_rel_err(to_np(y_next), ref_next) < HIDDEN_TOL


@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
def test_ragged_multi_session_batches(shape):
    """Several sessions with different histories in one call, mixed T (0, 1, many), chunked."""
    srv, W = make_server(shape)
    lens = [37, 5, 70, 16, 1]
    xs = [draw_hidden(shape, 1, i, n + 6) for i, n in enumerate(lens)]
    osess = [so.Session(shape, W) for _ in lens]
    ids = [srv.open(128) for _ in lens]
    # call 1: ragged prefixes in one request
    y = to_np(srv.forward(ids, lens, np.concatenate([x[:n] for x, n in zip(xs, lens)])))
    ref = np.concatenate([o.forward(x[:n]) for o, x, n in zip(osess, xs, lens)])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    # call 2: mixed token counts (0 = untouched, 1 = decode, 3 = chunk)
    T2 = [1, 0, 3, 1, 2]
    y = to_np(srv.forward(ids, T2, np.concatenate([x[n:n + t] for x, n, t in zip(xs, lens, T2)])))
    ref = np.concatenate([o.forward(x[n:n + t]) for o, x, n, t in zip(osess, xs, lens, T2)])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    cur = [n + t for n, t in zip(lens, T2)]
    # call 3: a pure decode step on a subset, in a different order
    order = [3, 0, 4]
    y = to_np(srv.forward([ids[i] for i in order], [1] * 3, np.concatenate([xs[i][cur[i]:cur[i] + 1] for i in order])))
    ref = np.concatenate([osess[i].forward(xs[i][cur[i]:cur[i] + 1]) for i in order])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    for i in order:
        cur[i] += 1
    for i, s in enumerate(ids):
        assert B.span_session_length(srv.span, s) == cur[i] == osess[i].length
        assert check_kv(srv, s, osess[i], shape.n_blocks) < KV_TOL


@pytest.mark.parametrize("shape", [SpanShape("llama", 1, 256, 8, 1, 64, 512), SpanShape("llama", 2, 256, 4, 1, 128, 512),
                                   SpanShape("llama", 1, 256, 12, 1, 64, 512), SpanShape("bloom", 1, 256, 8, 2, 64, 512),
                                   SpanShape("bloom", 1, 512, 4, 1, 128, 512)],
                         ids=["g8-hd64", "g4-hd128", "g12-hd64", "alibi-g4-hd64", "alibi-g4-hd128"])
def test_prefill_with_wide_query_groups(shape):
    """Four to twelve query heads per kv head (12 heads = a second, half-empty workgroup per query
    tile of the prefill attention kernel), 64- and 128-wide heads, with and without ALiBi: ragged
    prefixes, a second chunk on top of a cache, then decode steps."""
    srv, W = make_server(shape, max_session_tokens=256, max_batch_tokens=512)
    lens = [150, 33, 64, 1]
    xs = [draw_hidden(shape, 4, i, n + 45) for i, n in enumerate(lens)]
    osess = [so.Session(shape, W) for _ in lens]
    ids = [srv.open(256) for _ in lens]
    y = to_np(srv.forward(ids, lens, np.concatenate([x[:n] for x, n in zip(xs, lens)])))
    ref = np.concatenate([o.forward(x[:n]) for o, x, n in zip(osess, xs, lens)])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    T2 = [40, 17, 1, 43]                                                    # chunks on top of the cache
    y = to_np(srv.forward(ids, T2, np.concatenate([x[n:n + t] for x, n, t in zip(xs, lens, T2)])))
    ref = np.concatenate([o.forward(x[n:n + t]) for o, x, n, t in zip(osess, xs, lens, T2)])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    cur = [n + t for n, t in zip(lens, T2)]
    y = to_np(srv.forward(ids, [1] * 4, np.concatenate([x[n:n + 1] for x, n in zip(xs, cur)])))
    ref = np.concatenate([o.forward(x[n:n + 1]) for o, x, n in zip(osess, xs, cur)])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    for i, sid in enumerate(ids):
        assert check_kv(srv, sid, osess[i], shape.n_blocks) < KV_TOL


@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
@pytest.mark.parametrize("bits", [0, 8], ids=["bf16", "int8"])
def test_long_call_with_a_few_tail_rows(shape, bits):
    """A call of more than 1024 rows whose last 256-row tile holds only a few of them: those rows
    take the skinny projection kernel (three decoding sessions batched with one that replays 1030
    tokens; then a 1088-token chunk on top of that cache)."""
    from oracle import lowbit_oracle as lo
    from workloads import normal_levels16
    srv, W = make_server(shape, max_pages=256, max_sessions=5, max_session_tokens=2304, max_batch_tokens=1280,
                         weight_bits=bits, levels=normal_levels16() if bits else None)
    Wo = lo.quantized_weights([W[b] for b in range(shape.n_blocks)], bits, normal_levels16()) if bits else W
    lens = [20, 33, 5]
    xs = [draw_hidden(shape, 6, i, n + 1) for i, n in enumerate(lens)] + [draw_hidden(shape, 6, 3, 1030 + 1100)]
    osess = [so.Session(shape, Wo) for _ in range(4)]
    ids = [srv.open(2304) for _ in range(4)]
    y = to_np(srv.forward(ids[:3], lens, np.concatenate([x[:n] for x, n in zip(xs, lens)])))
    ref = np.concatenate([o.forward(x[:n]) for o, x, n in zip(osess, xs, lens)])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    # 3 single tokens + 1030 replayed tokens = 1033 rows: tiles cover 1024, the skinny kernel 9
    T = [1, 1, 1, 1030]
    x_call = np.concatenate([xs[0][20:21], xs[1][33:34], xs[2][5:6], xs[3][:1030]])
    y = to_np(srv.forward(ids, T, x_call))
    ref = np.concatenate([osess[0].forward(xs[0][20:21]), osess[1].forward(xs[1][33:34]), osess[2].forward(xs[2][5:6]),
                          osess[3].forward(xs[3][:1030])])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    # a 1088-token call (1024 + 64 -> skinny tail) on top of the cache
    y = to_np(srv.forward(ids[3:], [1088], xs[3][1030:2118]))
    ref = osess[3].forward(xs[3][1030:2118])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    for i, sid in enumerate(ids):
        assert B.span_session_length(srv.span, sid) == osess[i].length
        assert check_kv(srv, sid, osess[i], shape.n_blocks) < KV_TOL


@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
@pytest.mark.parametrize("bits", [0, 8], ids=["bf16", "int8"])
def test_long_all_tile_calls_fold_the_norms(shape, bits):
    """Calls that run every projection as tiles (no skinny tail rows, no 64-row chunks) fold every norm but
    the first into the projections: 300 rows (64-token tiles, a ragged last tile), then 1100 rows on top of
    that cache (1024 + 76: 256-token tiles), then three sessions of 129 + 200 + 70 rows in one call.  With
    8-bit weights only the RMSNorm span folds; the LayerNorm span keeps the stand-alone kernel."""
    from oracle import lowbit_oracle as lo
    from workloads import normal_levels16
    srv, W = make_server(shape, max_pages=192, max_sessions=4, max_session_tokens=1408, max_batch_tokens=1280,
                         weight_bits=bits, levels=normal_levels16() if bits else None)
    Wo = lo.quantized_weights([W[b] for b in range(shape.n_blocks)], bits, normal_levels16()) if bits else W
    x = draw_hidden(shape, 8, 0, 1400)
    o = so.Session(shape, Wo)
    sid = srv.open(1408)
    for a, b in ((0, 300), (300, 1400)):
        y = to_np(srv.forward([sid], [b - a], x[a:b]))
        ref = o.forward(x[a:b])
        assert row_rel_err(y, ref) < HIDDEN_TOL, (a, b)
    assert check_kv(srv, sid, o, shape.n_blocks) < KV_TOL
    lens = [129, 200, 70]
    xs = [draw_hidden(shape, 8, 1 + i, n) for i, n in enumerate(lens)]
    osess = [so.Session(shape, Wo) for _ in lens]
    ids = [srv.open(256) for _ in lens]
    y = to_np(srv.forward(ids, lens, np.concatenate(xs)))
    ref = np.concatenate([oo.forward(xx) for oo, xx in zip(osess, xs)])
    assert row_rel_err(y, ref) < HIDDEN_TOL


@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
@pytest.mark.parametrize("bits", [0, 8, 4], ids=["bf16", "int8", "4bit"])
def test_short_calls_around_the_chunking_limits(shape, bits):
    """Calls of 65 ... 193 rows: narrow projections of short calls run as skinny launches over chunks of
    64 rows (bf16 up to 128 rows, compressed weights up to 192), longer ones as tiles, and three
    leftover token tiles form one band of four.  One session takes chunk after chunk on top of its
    growing cache, two decoding sessions ride along in some of the calls."""
    from oracle import lowbit_oracle as lo
    from workloads import normal_levels16
    sizes = [65, 100, 128, 129, 160, 192, 193]
    total = sum(sizes)
    srv, W = make_server(shape, max_pages=96, max_sessions=3, max_session_tokens=total + 16, max_batch_tokens=256,
                         weight_bits=bits, levels=normal_levels16() if bits == 4 else None)
    Wo = lo.quantized_weights([W[b] for b in range(shape.n_blocks)], bits, normal_levels16()) if bits else W
    xs = [draw_hidden(shape, 12, 0, total), draw_hidden(shape, 12, 1, 16), draw_hidden(shape, 12, 2, 16)]
    osess = [so.Session(shape, Wo) for _ in range(3)]
    ids = [srv.open(total + 16) for _ in range(3)]
    for i in (1, 2):                                   # the two riders start with a short prefix
        y = to_np(srv.forward([ids[i]], [5], xs[i][:5]))
        assert row_rel_err(y, osess[i].forward(xs[i][:5])) < HIDDEN_TOL
    off, dec = 0, 5
    for c, n in enumerate(sizes):
        if c % 2 == 0:                                 # the chunk alone
            y = to_np(srv.forward([ids[0]], [n], xs[0][off:off + n]))
            ref = osess[0].forward(xs[0][off:off + n])
        else:                                          # the chunk (2 rows shorter) batched with two single tokens
            T = [1, n - 2, 1]
            x_call = np.concatenate([xs[1][dec:dec + 1], xs[0][off:off + n - 2], xs[2][dec:dec + 1]])
            y = to_np(srv.forward([ids[1], ids[0], ids[2]], T, x_call))
            ref = np.concatenate([osess[1].forward(xs[1][dec:dec + 1]), osess[0].forward(xs[0][off:off + n - 2]),
                                  osess[2].forward(xs[2][dec:dec + 1])])
            dec += 1
            n -= 2
        assert row_rel_err(y, ref) < HIDDEN_TOL, (c, n)
        off += n
    for i, sid in enumerate(ids):
        assert B.span_session_length(srv.span, sid) == osess[i].length
        assert check_kv(srv, sid, osess[i], shape.n_blocks) < KV_TOL


@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
def test_largest_call_of_64_sessions(shape):
    """The most sessions one call may carry: 64 ragged prefixes (one of them empty) in one request,
    then two decode steps of all 64 (the widest skinny projection, 64 sessions through the split
    attention kernel); a 65th session is refused without touching anything."""
    srv, W = make_server(shape, max_pages=80, max_sessions=65, max_session_tokens=16, max_batch_tokens=256)
    lens = [(3 * i) % 5 for i in range(64)]
    lens[0] = 4
    xs = [draw_hidden(shape, 8, i, n + 2) for i, n in enumerate(lens)]
    osess = [so.Session(shape, W) for _ in lens]
    ids = [srv.open(16) for _ in lens]
    y = to_np(srv.forward(ids, lens, np.concatenate([x[:n] for x, n in zip(xs, lens)])))
    ref = np.concatenate([o.forward(x[:n]) for o, x, n in zip(osess, xs, lens)])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    for step in range(2):
        y = to_np(srv.forward(ids, [1] * 64, np.concatenate([x[n + step:n + step + 1] for x, n in zip(xs, lens)])))
        ref = np.concatenate([o.forward(x[n + step:n + step + 1]) for o, x, n in zip(osess, xs, lens)])
        assert row_rel_err(y, ref) < HIDDEN_TOL
    extra = srv.open(16)
    free = B.span_debug_free_pages(srv.span)
    x65 = torch.zeros(65, shape.d_model, device=DEV)
    with pytest.raises(B.SpanError) as e:
        B.span_forward(srv.span, ids + [extra], [1] * 65, x65, torch.empty_like(x65), srv.stream)
    assert e.value.code == B.SPAN_E_INVALID
    assert B.span_debug_free_pages(srv.span) == free
    assert [B.span_session_length(srv.span, s) for s in ids] == [n + 2 for n in lens]


@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
def test_continuous_batching_with_churn(shape):
    """A server's life: in every call some sessions decode one token, some send a chunk, some
    sit out (0 tokens), a new session may join with its whole prefix in the same call, and
    sessions leave between calls.  Every call is checked against per-session oracles, and the
    integer state (lengths, page ownership, free-list size) is exact after every call."""
    srv, W = make_server(shape, max_pages=40, max_sessions=6, max_session_tokens=96, max_batch_tokens=128)
    rng = np.random.default_rng(2024)
    total_pages = B.span_debug_free_pages(srv.span)
    live = []                                    # dicts: id, oracle session, inputs, cursor
    n_drawn = 0

    def join():
        nonlocal n_drawn
        x = draw_hidden(shape, 3, n_drawn, 96)
        n_drawn += 1
        return {"id": srv.open(96), "o": so.Session(shape, W), "x": x, "cur": 0}

    for call in range(28):
        if len(live) < 6 and (call % 3 == 0 or not live):
            live.append(join())
        ids, counts, rows, refs = [], [], [], []
        for s in live:
            room = 96 - s["cur"]
            if s["cur"] == 0:
                t = int(rng.integers(5, 41))                     # a joining session sends its prefix
            else:
                t = int(rng.choice([0, 1, 1, 1, int(rng.integers(2, 10))]))
            t = min(t, room)
            ids.append(s["id"]); counts.append(t)
            rows.append(s["x"][s["cur"]:s["cur"] + t])
            refs.append(s["o"].forward(s["x"][s["cur"]:s["cur"] + t]))
            s["cur"] += t
        y = to_np(srv.forward(ids, counts, np.concatenate(rows)))
        if sum(counts):
            assert row_rel_err(y, np.concatenate(refs)) < HIDDEN_TOL, f"call {call}"
        # integer state
        tables = [B.span_debug_page_table(srv.span, s["id"]) for s in live]
        assert [B.span_session_length(srv.span, s["id"]) for s in live] == [s["cur"] for s in live]
        assert [len(t) for t in tables] == [(s["cur"] + 15) // 16 for s in live]
        flat = [p for t in tables for p in t]
        assert len(set(flat)) == len(flat)
        assert B.span_debug_free_pages(srv.span) == total_pages - len(flat)
        # sessions leave: the longest-lived full one, or a random one now and then
        for s in list(live):
            if s["cur"] >= 96 or rng.random() < 0.08:
                assert check_kv(srv, s["id"], s["o"], shape.n_blocks) < KV_TOL
                srv.close(s["id"])
                live.remove(s)
    for s in live:
        assert check_kv(srv, s["id"], s["o"], shape.n_blocks) < KV_TOL
        srv.close(s["id"])
    assert B.span_debug_free_pages(srv.span) == total_pages


@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
def test_beam_reorder_matches_oracle_gather(shape):
    """Cache reordering between steps (appendix on beam search): entries are cloned, moved and
    dropped; every entry then decodes with its own inputs and must follow the oracle, whose
    reorder is a plain copy of the source's cache.  Full pages end up shared, partial last
    pages private, and the pool accounting stays exact."""
    srv, W = make_server(shape, max_pages=40, max_sessions=5, max_session_tokens=96, max_batch_tokens=160)
    total_pages = B.span_debug_free_pages(srv.span)
    lens = [21, 35, 16, 9, 48]
    xs = [draw_hidden(shape, 4, i, n) for i, n in enumerate(lens)]
    osess = [so.Session(shape, W) for _ in lens]
    ids = [srv.open(96) for _ in lens]
    y = to_np(srv.forward(ids, lens, np.concatenate(xs)))
    ref = np.concatenate([o.forward(x) for o, x in zip(osess, xs)])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    step = 0
    for hypo in ([1, 1, 0, 1, 4], [0, 1, 2, 3, 4], [4, 2, 2, 0, 0], [3, 3, 3, 3, 3]):
        srv.reorder(ids, hypo)
        osess = so.reorder(osess, hypo)
        assert [B.span_session_length(srv.span, s) for s in ids] == [o.length for o in osess]
        tables = [B.span_debug_page_table(srv.span, s) for s in ids]
        assert [len(t) for t in tables] == [(o.length + 15) // 16 for o in osess]
        last_partial = [t[-1] for t, o in zip(tables, osess) if o.length % 16]
        assert len(set(last_partial)) == len(last_partial)               # nobody shares a page it will append to
        for i, t in enumerate(tables):                                   # and no other session lists such a page at all
            for j, u in enumerate(tables):
                if i != j and osess[i].length % 16:
                    assert t[-1] not in u
        assert B.span_debug_free_pages(srv.span) == total_pages - len({p for t in tables for p in t})
        for s, o in zip(ids, osess):
            assert check_kv(srv, s, o, shape.n_blocks) < KV_TOL
        for _ in range(3):                                               # the beam decodes, each entry its own token
            x = np.stack([draw_hidden(shape, 5, 100 * step + i, 1)[0] for i in range(len(ids))])
            y = to_np(srv.forward(ids, [1] * len(ids), x))
            ref = np.concatenate([o.forward(x[i:i + 1]) for i, o in enumerate(osess)])
            assert row_rel_err(y, ref) < HIDDEN_TOL
            step += 1
    for s, o in zip(ids, osess):
        assert check_kv(srv, s, o, shape.n_blocks) < KV_TOL
        srv.close(s)
    assert B.span_debug_free_pages(srv.span) == total_pages


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("shape", [TINY, TINY_BLOOM], ids=["llama", "bloom"])
def test_compressed_weight_span_follows_the_dequantised_oracle(shape, bits):
    """Section 3.1, "Compression": a server holding 8-bit or 4-bit weights computes the span of
    the dequantised matrices.  The oracle encodes and decodes the same weights on its own and
    runs its ordinary span on them; replay, decode steps, a ragged mixed call, a long request and
    the cache contents are compared as for the uncompressed span."""
    from oracle import lowbit_oracle as lo
    from workloads import normal_levels16
    levels = normal_levels16()
    srv, W = make_server(shape, weight_bits=bits, levels=levels)
    Wq = lo.quantized_weights(W, bits, levels)
    lens = [70, 23, 5]
    xs = [draw_hidden(shape, 6, i, n + 8) for i, n in enumerate(lens)]
    osess = [so.Session(shape, Wq) for _ in lens]
    ids = [srv.open(128) for _ in lens]
    y = to_np(srv.forward(ids, lens, np.concatenate([x[:n] for x, n in zip(xs, lens)]), replay=True))
    ref = np.concatenate([o.forward(x[:n]) for o, x, n in zip(osess, xs, lens)])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    # the compressed span must not simply equal the uncompressed one
    plain = np.concatenate([so.Session(shape, W).forward(x[:n]) for x, n in zip(xs, lens)])
    assert row_rel_err(ref, plain) > 2 * row_rel_err(y, ref)
    cur = list(lens)
    for t in range(4):                                           # decode steps
        y = to_np(srv.forward(ids, [1, 1, 1], np.stack([x[c] for x, c in zip(xs, cur)])))
        ref = np.concatenate([o.forward(x[c:c + 1]) for o, x, c in zip(osess, xs, cur)])
        assert row_rel_err(y, ref) < HIDDEN_TOL
        cur = [c + 1 for c in cur]
    T = [3, 0, 1]                                                # ragged mixed call
    y = to_np(srv.forward(ids, T, np.concatenate([x[c:c + t] for x, c, t in zip(xs, cur, T)])))
    ref = np.concatenate([o.forward(x[c:c + t]) for o, x, c, t in zip(osess, xs, cur, T)])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    for s, o in zip(ids, osess):
        assert B.span_session_length(srv.span, s) == o.length
        assert check_kv(srv, s, o, shape.n_blocks) < KV_TOL
    # a long request goes through the tiled kernels on a bf16 expansion of the compressed matrices
    fresh = srv.open(200)
    xl = draw_hidden(shape, 6, 9, 150)
    y = to_np(srv.forward([fresh], [150], xl))
    of = so.Session(shape, Wq)
    assert row_rel_err(y, of.forward(xl)) < HIDDEN_TOL
    y = to_np(srv.forward([fresh], [1], xl[:1]))                 # and decoding continues from that cache
    assert row_rel_err(y, of.forward(xl[:1])) < HIDDEN_TOL
    assert check_kv(srv, fresh, of, shape.n_blocks) < KV_TOL


def test_page_table_state_is_exact():
    shape = TINY
    srv, W = make_server(shape, max_pages=6, max_session_tokens=96)
    a, b = srv.open(96), srv.open(96)
    xa, xb = draw_hidden(shape, 2, 0, 60), draw_hidden(shape, 2, 1, 60)
    srv.forward([a, b], [17, 16], np.concatenate([xa[:17], xb[:16]]))
    pa, pb = B.span_debug_page_table(srv.span, a), B.span_debug_page_table(srv.span, b)
    assert len(pa) == 2 and len(pb) == 1 and len(set(pa + pb)) == 3
    assert B.span_debug_free_pages(srv.span) == 3
    srv.forward([b], [1], xb[16:17])                      # crosses into a new page
    assert len(B.span_debug_page_table(srv.span, b)) == 2
    # a request that does not fit leaves everything as it was
    with pytest.raises(B.SpanError) as e:
        srv.forward([a, b], [43, 43], np.concatenate([xa[17:60], xb[17:60]]))
    assert e.value.code == B.SPAN_E_CACHE_FULL
    assert B.span_session_length(srv.span, a) == 17 and B.span_session_length(srv.span, b) == 17
    assert B.span_debug_page_table(srv.span, a) == pa and B.span_debug_free_pages(srv.span) == 2
    # the sessions still work and still match the oracle afterwards
    oa = so.Session(shape, W); oa.forward(xa[:17])
    y = to_np(srv.forward([a], [3], xa[17:20]))
    assert row_rel_err(y, oa.forward(xa[17:20])) < HIDDEN_TOL
    srv.close(a); srv.close(b)
    assert B.span_debug_free_pages(srv.span) == 6


def test_sub_span_sessions_chain_to_whole_span():
    """A client may use a sub-segment of a server's blocks (Appendix D): block 0 then block 1
    as separate sessions equals one session on both."""
    shape = TINY
    srv, W = make_server(shape)
    x = draw_hidden(shape, 3, 0, 20)
    whole, first, second = srv.open(64), srv.open(64, 0, 1), srv.open(64, 1, 1)
    y_whole = to_np(srv.forward([whole], [20], x))
    y1 = srv.forward([first], [20], x)
    y2 = to_np(srv.forward([second], [20], y1))
    ref = so.Session(shape, W).forward(x)
    assert row_rel_err(y_whole, ref) < HIDDEN_TOL and row_rel_err(y2, ref) < HIDDEN_TOL
    with pytest.raises(B.SpanError) as e:
        srv.forward([whole, first], [1, 1], x[:2])
    assert e.value.code == B.SPAN_E_MIXED_SPANS


def test_chunked_replay_equals_single_request():
    """Replay longer than max_batch_tokens is processed in chunks that may split a session."""
    shape = TINY
    srv, W = make_server(shape, max_batch_tokens=48, max_session_tokens=128)
    lens = [50, 31, 60]
    xs = [draw_hidden(shape, 4, i, n) for i, n in enumerate(lens)]
    ids = [srv.open(128) for _ in lens]
    y = to_np(srv.forward(ids, lens, np.concatenate(xs), replay=True))
    ref = np.concatenate([so.Session(shape, W).forward(x) for x in xs])
    assert row_rel_err(y, ref) < HIDDEN_TOL
    with pytest.raises(B.SpanError) as e:       # replay needs empty sessions
        srv.forward(ids, lens, np.concatenate(xs), replay=True)
    assert e.value.code == B.SPAN_E_NOT_EMPTY


def test_bf16_io_mode():
    shape = TINY
    srv, W = make_server(shape, io_f32=False)
    x = draw_hidden(shape, 5, 0, 12)
    s = srv.open(32)
    y = to_np(srv.forward([s], [12], x))
    ref = so.Session(shape, W).forward(x)
    # output rounded to bf16: up to 2^-9 of the largest entry of a row on top of the path's error
    assert row_rel_err(y, ref) < HIDDEN_TOL


@pytest.mark.parametrize("offset", [6.0, -40.0])
def test_layernorm_rows_whose_mean_is_large_against_their_spread(offset):
    """BLOOM-style spans fold every LayerNorm but the first into the neighbouring projections (decode steps
    and long all-tile calls).  Hidden states with mean >> standard deviation must not lose precision there:
    the folded norms round and sum the rows shifted by the mean the previous norm found.  (Rounding x * gain
    itself to bf16 would cost |mean| / sigma times the usual error: 2e-1 at offset -40.)"""
    shape = SpanShape("bloom", 3, 512, 8, 8, 64, 1024)
    srv, W = make_server(shape, max_pages=64, max_session_tokens=400, max_batch_tokens=640, seed=12)
    n = 300 + 6
    xs = [bf16_round((offset + draw_hidden(shape, 12, i, n, bf16=False)).astype(np.float32)) for i in range(2)]
    ids = [srv.open(400) for _ in range(2)]
    osess = [so.Session(shape, W) for _ in range(2)]
    def spread_err(got, ref):
        """largest element error over the row's standard deviation (the mean would hide the error in a row norm)"""
        return float(np.max(np.abs(got - ref) / np.std(ref, axis=-1, keepdims=True)))

    y = to_np(srv.forward(ids, [300, 300], np.concatenate([x[:300] for x in xs])))           # tiles, norms folded
    ref = np.concatenate([o.forward(x[:300]) for o, x in zip(osess, xs)])
    e_long = spread_err(y, ref)
    assert e_long < HIDDEN_TOL, e_long
    worst = 0.0
    for t in range(300, n):                                                                  # decode steps, norms folded
        y = to_np(srv.forward(ids, [1, 1], np.stack([x[t] for x in xs])))
        ref = np.concatenate([o.forward(x[t:t + 1]) for o, x in zip(osess, xs)])
        worst = max(worst, spread_err(y, ref))
    assert worst < HIDDEN_TOL, worst
    assert max(check_kv(srv, s, o, shape.n_blocks) for s, o in zip(ids, osess)) < KV_TOL
    print(f"offset {offset}: long call {e_long:.2e}, decode steps {worst:.2e}")
    srv.destroy()

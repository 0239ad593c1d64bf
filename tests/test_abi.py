"""The C-ABI library loads without a GPU, exports every symbol include/span.h declares,
and its host-side logic (session table, page allocator, error handling, chunked replay
bookkeeping) behaves as the header says.  Uses dry-run spans: no device work."""
import os
import re

import pytest

from paper_2312_08361_amd import binding as B
from paper_2312_08361_amd.server import config_for
from workloads import LLAMA_70B, TINY, TINY_BLOOM, BLOOM_176B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "span.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(span_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_functions()
    assert len(names) >= 16
    for n in names:
        assert hasattr(B.lib, n), f"libspan.so does not export {n}"
        assert callable(getattr(B, n)), f"binding has no function {n}"
    assert sorted(B.EXPORTS) == names


def dry(shape=TINY, **kw):
    args = dict(max_pages=8, max_sessions=3, max_session_tokens=64, max_batch_tokens=40)
    args.update(kw)
    cfg = config_for(shape, dry_run=True, **args)
    return B.span_create(cfg, None, None, None, None), cfg


def code(fn, *a):
    with pytest.raises(B.SpanError) as e:
        fn(*a)
    return e.value.code


def test_sizes_scale_with_the_configuration():
    cfg = config_for(LLAMA_70B, max_pages=1100, max_sessions=8, max_session_tokens=2304, max_batch_tokens=16384)
    w, kv, ws = B.span_query_sizes(cfg)
    assert abs(w / 1e9 - 13.69) < 0.05                           # packed bf16 weights of 8 blocks
    assert kv == 8 * 1100 * 2 * 8 * 16 * 128 * 2                 # blocks x pages x (K,V) x heads x 16 x hd x 2 B
    cfgb = config_for(BLOOM_176B, max_pages=200, max_sessions=16, max_session_tokens=256, max_batch_tokens=2048)
    wb, _, _ = B.span_query_sizes(cfgb)
    assert abs(wb / 1e9 - 19.73) < 0.06


def test_bad_configurations_are_rejected():
    for kw in (dict(head_dim=96), dict(n_kv_heads=3), dict(d_model=100), dict(page_tokens=8), dict(max_pages=0)):
        cfg = config_for(TINY, max_pages=8, max_sessions=2, max_session_tokens=64, max_batch_tokens=16, dry_run=True)
        for k, v in kw.items():
            setattr(cfg, k, v)
        assert code(B.span_query_sizes, cfg) == B.SPAN_E_INVALID
    assert "head_dim" in B.span_last_error() or B.span_last_error()


def test_compute_without_gpu_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    cfg = config_for(TINY, max_pages=8, max_sessions=2, max_session_tokens=64, max_batch_tokens=16)
    dummy = torch.zeros(16, dtype=torch.uint8)
    weights = [{n: dummy for n in B.WEIGHT_FIELDS}, {n: dummy for n in B.WEIGHT_FIELDS}]
    assert code(B.span_create, cfg, weights, dummy, dummy, dummy) == B.SPAN_E_HIP


def test_session_lifecycle_and_page_accounting():
    sp, _ = dry()
    a = B.span_session_open(sp, 0, 2, 64)
    b = B.span_session_open(sp, 0, 2, 40)
    assert a != b and B.span_session_length(sp, a) == 0
    B.span_forward(sp, [a, b], [16, 3], None, None)
    assert B.span_session_length(sp, a) == 16 and B.span_session_length(sp, b) == 3
    pa, pb = B.span_debug_page_table(sp, a), B.span_debug_page_table(sp, b)
    assert len(pa) == 1 and len(pb) == 1 and pa != pb and B.span_debug_free_pages(sp) == 6
    B.span_forward(sp, [a], [1], None, None)                     # position 16 starts page 2
    assert len(B.span_debug_page_table(sp, a)) == 2 and B.span_debug_page_table(sp, a)[0] == pa[0]
    B.span_forward(sp, [a, b], [0, 0], None, None)               # empty request: nothing happens
    assert B.span_session_length(sp, a) == 17
    B.span_session_close(sp, a)
    assert B.span_debug_free_pages(sp) == 7
    assert code(B.span_session_length, sp, a) == B.SPAN_E_BAD_SESSION
    c = B.span_session_open(sp, 0, 2, 64)
    assert c not in (a, b)                                       # handles are not reused
    B.span_destroy(sp)


def test_failed_calls_change_nothing():
    sp, _ = dry()
    a = B.span_session_open(sp, 0, 2, 64)
    b = B.span_session_open(sp, 0, 2, 20)
    sub = B.span_session_open(sp, 1, 1, 64)
    B.span_forward(sp, [a, b], [10, 10], None, None)
    state = lambda: (B.span_session_length(sp, a), B.span_session_length(sp, b), B.span_debug_page_table(sp, a),
                     B.span_debug_page_table(sp, b), B.span_debug_free_pages(sp))
    before = state()
    assert code(B.span_forward, sp, [a, b], [5, 11], None, None) == B.SPAN_E_TOO_LONG
    assert code(B.span_forward, sp, [a, a], [1, 1], None, None) == B.SPAN_E_DUPLICATE
    assert code(B.span_forward, sp, [a, sub], [1, 1], None, None) == B.SPAN_E_MIXED_SPANS
    assert code(B.span_forward, sp, [a, 999], [1, 1], None, None) == B.SPAN_E_BAD_SESSION
    assert code(B.span_forward, sp, [a, b], [38, 3], None, None) == B.SPAN_E_TOO_MANY_TOKENS
    assert code(B.span_forward, sp, [a], [-1], None, None) == B.SPAN_E_INVALID
    assert code(B.span_forward, sp, [a] * 65, [1] * 65, None, None) == B.SPAN_E_INVALID
    assert state() == before
    assert code(B.span_session_open, sp, 0, 2, 64) == B.SPAN_E_NO_SLOT
    assert code(B.span_session_open, sp, 1, 2, 64) == B.SPAN_E_INVALID
    assert code(B.span_session_open, sp, 0, 1, 65) == B.SPAN_E_INVALID
    B.span_destroy(sp)


def test_cache_full_is_all_or_nothing():
    sp, _ = dry(max_pages=4)
    a = B.span_session_open(sp, 0, 2, 64)
    b = B.span_session_open(sp, 0, 2, 64)
    B.span_forward(sp, [a, b], [16, 16], None, None)             # 2 pages used, 2 free
    assert code(B.span_forward, sp, [a, b], [17, 17], None, None) == B.SPAN_E_CACHE_FULL   # needs 4
    assert B.span_debug_free_pages(sp) == 2 and B.span_session_length(sp, a) == 16
    B.span_forward(sp, [a, b], [16, 16], None, None)             # exactly fits
    assert B.span_debug_free_pages(sp) == 0
    assert code(B.span_forward, sp, [a], [1], None, None) == B.SPAN_E_CACHE_FULL
    B.span_session_close(sp, b)
    B.span_forward(sp, [a], [1], None, None)
    B.span_destroy(sp)


def test_replay_bookkeeping_and_rollback():
    sp, _ = dry(max_pages=8, max_batch_tokens=24, max_session_tokens=64)
    a = B.span_session_open(sp, 0, 2, 64)
    b = B.span_session_open(sp, 0, 2, 64)
    B.span_replay(sp, [a, b], [50, 31], None, None)              # 81 tokens in chunks of 24, splitting sessions
    assert B.span_session_length(sp, a) == 50 and B.span_session_length(sp, b) == 31
    assert len(B.span_debug_page_table(sp, a)) == 4 and len(B.span_debug_page_table(sp, b)) == 2
    assert code(B.span_replay, sp, [a], [1], None, None) == B.SPAN_E_NOT_EMPTY
    B.span_session_close(sp, a); B.span_session_close(sp, b)
    # a replay that runs out of pages midway leaves the sessions empty and the pool whole
    a = B.span_session_open(sp, 0, 2, 64)
    b = B.span_session_open(sp, 0, 2, 64)
    c = B.span_session_open(sp, 0, 2, 64)
    assert code(B.span_replay, sp, [a, b, c], [60, 60, 60], None, None) == B.SPAN_E_CACHE_FULL
    assert [B.span_session_length(sp, s) for s in (a, b, c)] == [0, 0, 0]
    assert B.span_debug_free_pages(sp) == 8
    B.span_replay(sp, [a, b, c], [0, 7, 0], None, None)          # empty histories are legal
    assert B.span_session_length(sp, b) == 7
    B.span_destroy(sp)


def test_reorder_shares_full_pages_and_copies_partial_ones():
    """Cache reordering (appendix on beam search) on the paged cache: bookkeeping only."""
    sp, _ = dry(max_pages=12, max_sessions=4, max_session_tokens=64, max_batch_tokens=96)
    a, b, c = (B.span_session_open(sp, 0, 2, 64) for _ in range(3))
    B.span_forward(sp, [a, b, c], [20, 33, 16], None, None)      # 2 + 3 + 1 pages; a and b end in partial pages
    pa, pb, pc = (B.span_debug_page_table(sp, s) for s in (a, b, c))
    assert B.span_debug_free_pages(sp) == 6
    # the paper's shape of call: one entry named three times, one kept, one dropped
    B.span_reorder(sp, [a, b, c], [1, 1, 1])
    na, nb, nc = (B.span_debug_page_table(sp, s) for s in (a, b, c))
    assert [B.span_session_length(sp, s) for s in (a, b, c)] == [33, 33, 33]
    assert na[:2] == nb[:2] == nc[:2] == pb[:2]                  # full pages shared by reference
    assert nb[2] == pb[2]                                        # the entry that names itself keeps its partial page
    assert len({na[2], nb[2], nc[2]}) == 3 and not {na[2], nc[2]} & set(pb)   # copies live in pages nobody else lists
    assert B.span_debug_free_pages(sp) == 12 - len(set(na + nb + nc)) == 12 - 5
    # each continues on its own: appending never touches a shared page
    B.span_forward(sp, [a, b, c], [1, 20, 0], None, None)
    assert B.span_debug_page_table(sp, a)[:3] == na and B.span_debug_page_table(sp, c) == nc
    assert len(B.span_debug_page_table(sp, b)) == 4
    # closing one sharer keeps the shared pages alive for the others
    B.span_session_close(sp, b)
    assert B.span_debug_free_pages(sp) == 12 - len(set(na + nc))
    B.span_session_close(sp, a); B.span_session_close(sp, c)
    assert B.span_debug_free_pages(sp) == 12
    B.span_destroy(sp)


def test_reorder_errors_change_nothing():
    sp, _ = dry(max_pages=4, max_sessions=4, max_session_tokens=64, max_batch_tokens=64)
    a, b = B.span_session_open(sp, 0, 2, 64), B.span_session_open(sp, 0, 2, 16)
    c = B.span_session_open(sp, 0, 1, 64)
    B.span_forward(sp, [a, b], [40, 8], None, None)              # 3 + 1 pages: pool exhausted
    before = [B.span_debug_page_table(sp, s) for s in (a, b)]
    assert code(B.span_reorder, sp, [a, b], [0, 0]) == B.SPAN_E_TOO_LONG          # b was opened for 16 tokens
    assert code(B.span_reorder, sp, [a, b], [0, 2]) == B.SPAN_E_INVALID
    assert code(B.span_reorder, sp, [a, a], [0, 0]) == B.SPAN_E_DUPLICATE
    assert code(B.span_reorder, sp, [a, c], [0, 0]) == B.SPAN_E_MIXED_SPANS
    assert code(B.span_reorder, sp, [a, 12345], [0, 0]) == B.SPAN_E_BAD_SESSION
    assert [B.span_debug_page_table(sp, s) for s in (a, b)] == before
    assert [B.span_session_length(sp, s) for s in (a, b)] == [40, 8]
    B.span_session_close(sp, b)
    d = B.span_session_open(sp, 0, 2, 64)
    B.span_forward(sp, [d], [3], None, None)                     # takes the freed page: pool exhausted again
    # cloning a (partial last page) needs one fresh page; d's own page comes back first, so it fits
    B.span_reorder(sp, [a, d], [0, 0])
    assert B.span_session_length(sp, d) == 40 and B.span_debug_free_pages(sp) == 0
    e = B.span_session_open(sp, 0, 2, 64)
    assert code(B.span_reorder, sp, [a, d, e], [0, 1, 0]) == B.SPAN_E_CACHE_FULL   # a third partial page does not fit
    assert B.span_session_length(sp, e) == 0 and B.span_debug_free_pages(sp) == 0
    B.span_reorder(sp, [a, d, e], [2, 2, 2])                     # everybody continues from the empty cache
    assert [B.span_session_length(sp, s) for s in (a, d, e)] == [0, 0, 0] and B.span_debug_free_pages(sp) == 4
    B.span_destroy(sp)


def test_bloom_dry_run_shapes():
    sp, _ = dry(TINY_BLOOM)
    a = B.span_session_open(sp, 0, 2, 64)
    B.span_forward(sp, [a], [33], None, None)
    assert len(B.span_debug_page_table(sp, a)) == 3
    B.span_destroy(sp)


def test_training_sizes_and_host_errors():
    """Arena sizes of the training-time passes: one transposed copy of the projection weights
    (a little more than the forward packs: other paddings), scratch that grows with the token
    capacity; and the errors that need no device."""
    cfg = config_for(LLAMA_70B, max_pages=1100, max_sessions=8, max_session_tokens=2304, max_batch_tokens=16384)
    wb, _, _ = B.span_query_sizes(cfg)
    wt, sc = B.span_train_sizes(cfg, 4096)
    params = LLAMA_70B.n_blocks * 2 * (8192 * 10240 + 8192 * 8192 + 3 * 8192 * 28672)
    assert params <= wt <= 1.01 * params and abs(wt - wb) < 0.01 * wb
    wt2, sc2 = B.span_train_sizes(cfg, 1024)
    assert wt2 == wt and sc2 < sc
    # every kept row of every block fits: x, x1 (fp32), q (bf16), o (fp32), gate | up (fp32) per token
    per_token = 4 * (2 * 8192 + 8192 + 2 * 28672) + 2 * 8192
    assert sc >= LLAMA_70B.n_blocks * 4096 * per_token
    assert code(B.span_train_sizes, cfg, 0) == B.SPAN_E_INVALID
    assert code(B.span_train_sizes, cfg, 16385) == B.SPAN_E_INVALID
    span, _ = dry()
    assert code(B.span_train_forward, span, 0, 2, [4], None, None) == B.SPAN_E_INVALID       # not attached
    assert code(B.span_backward, span, 0, 2, [4], None, None, None) == B.SPAN_E_INVALID
    B.span_destroy(span)

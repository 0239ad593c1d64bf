"""The allocation-free decode attention (span_op_attn_decode_static: scratch in an array the library's
code object holds on the GPU) against the entry point it is a variant of (span_op_attn_decode with
caller-provided scratch): same kernels, so outputs and logits must be identical, on two calls in a
row, the second with a smaller input (it finds the first call's leftovers in the shared array).
Collected last on purpose: a failure here must not hide the parity tests."""
import numpy as np
import pytest
import torch

from gpu_util import *  # noqa: F401,F403

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]

CASES = [
    # (Hq, Hkv, hd, alibi, lens)          first call large, second smaller in every dimension
    (16, 4, 128, 0, [1000, 517, 33, 1]),
    (8, 4, 64, 1, [300, 17]),
]


def run_pair(Hq, Hkv, hd, alibi, lens, seed):
    Bn, L = len(lens), max(lens)
    rng = np.random.default_rng([77, seed, Hq, Hkv, hd, L])
    q = dev_bf16(bf16_round(1.8 * rng.standard_normal((Bn, Hq, hd), dtype=np.float32)))
    k = dev_bf16(bf16_round(1.8 * rng.standard_normal((Bn, L, Hkv, hd), dtype=np.float32)))
    v = dev_bf16(bf16_round(1.8 * rng.standard_normal((Bn, L, Hkv, hd), dtype=np.float32)))
    st = torch.cuda.current_stream().cuda_stream
    outs = []
    for static in (False, True):
        out = torch.full((Bn, Hq, hd), float("nan"), dtype=torch.float32, device=DEV)
        logits = torch.full((Bn, Hq, L), float("nan"), dtype=torch.float32, device=DEV)
        if static:
            before = torch.cuda.memory_allocated()
            B.span_op_attn_decode_static(q, k, v, lens, Bn, L, Hq, Hkv, hd, alibi, out, logits, st)
            assert torch.cuda.memory_allocated() == before
        else:
            scratch = torch.empty(B.span_op_attn_decode_scratch(Bn, L, Hq, Hkv, hd), dtype=torch.uint8, device=DEV)
            B.span_op_attn_decode(q, k, v, lens, Bn, L, Hq, Hkv, hd, alibi, out, logits, scratch, st)
        torch.cuda.synchronize()
        outs.append((out, logits))
    (o_ref, l_ref), (o_st, l_st) = outs
    assert torch.isfinite(o_ref).all() and torch.isfinite(o_st).all()
    assert torch.equal(o_ref, o_st), float((o_ref - o_st).abs().max())
    for b, n in enumerate(lens):
        assert torch.equal(l_ref[b, :, :n], l_st[b, :, :n])
    # and against the oracle.  The softmax weights enter the P.V product rounded to bf16 (relative 2^-9 each),
    # so an output element is off by at most 2^-9 * sum_j p_j |v_j| <= 2^-9 * max|v| (here 1.8 * ~4.5 sigma),
    # i.e. 1e-2 of the row's rms (~1.8 when one key dominates) in the worst case; typical rows lie at 1e-3.
    slopes = so.alibi_slopes(Hq) if alibi else None
    qn, kn, vn = to_np(q), to_np(k), to_np(v)
    worst = 0.0
    for b, n in enumerate(lens):
        ref = so.attention_with_cache(qn[b:b + 1], kn[b, :n], vn[b, :n], n - 1, slopes)
        worst = max(worst, row_rel_err(to_np(o_st[b]), ref[0]))
    assert worst < 1e-2, worst


def test_static_scratch_decode_attention_matches_the_workspace_variant_twice_in_a_row():
    for i, (Hq, Hkv, hd, alibi, lens) in enumerate(CASES):
        run_pair(Hq, Hkv, hd, alibi, lens, i)
    # the second call of each shape family again, smaller still, after everything above has used the array
    run_pair(8, 4, 64, 0, [40], 9)


def test_static_scratch_rejects_shapes_beyond_its_size():
    Hq, Hkv, hd, L, Bn = 64, 8, 128, 4096, 8                 # 8 x 4096 tokens of K and V: 128 MiB of pages
    assert B.span_op_attn_decode_scratch(Bn, L, Hq, Hkv, hd) > 64 << 20
    q = torch.zeros((Bn, Hq, hd), dtype=torch.bfloat16, device=DEV)
    kv = torch.zeros((1,), dtype=torch.bfloat16, device=DEV)   # never read: the call must fail before any launch
    out = torch.zeros((Bn, Hq, hd), dtype=torch.float32, device=DEV)
    with pytest.raises(B.SpanError) as e:
        B.span_op_attn_decode_static(q, kv, kv, [L] * Bn, Bn, L, Hq, Hkv, hd, 0, out, None, 0)
    assert "built-in scratch" in str(e.value)
    torch.cuda.synchronize()

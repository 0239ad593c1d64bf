"""Parity of the training-time passes (Section 3.3: forward over whole sequences without a cache,
backward returning the gradient with respect to the input activations, weights frozen) against
the fp64 oracle, on the small configurations: ragged batches that take the skinny kernel, the
two register-staged tiled kernels and the direct-to-LDS tiled kernel; sub-spans; both block
styles; and the error paths of the entry points."""
import numpy as np
import pytest
import torch

from gpu_util import *  # noqa: F401,F403
from oracle import backward_oracle as bo
from workloads import TINY, TINY_BLOOM, SpanShape

pytestmark = pytest.mark.gpu

SHAPES = {"llama": TINY, "bloom": TINY_BLOOM}


def make_train_server(shape, max_tokens, seed=0, io_f32=True, max_session_tokens=1024):
    W = SpanWeights(shape, seed=seed, bf16=True, cache=True)
    cfg = config_for(shape, max_pages=32, max_sessions=4, max_session_tokens=max_session_tokens,
                     max_batch_tokens=max(max_tokens, 64), io_f32=io_f32)
    srv = SpanServer(cfg, W, DEV, keep_canonical=True)
    srv.attach_training(max_tokens)
    return srv, W


def draw_batch(shape, lens, seed):
    n = sum(lens)
    x = draw_hidden(shape, seed, 0, n)
    gy = bf16_round(np.random.default_rng(seed + 50).standard_normal((n, shape.d_model)).astype(np.float32))
    return x, gy


@pytest.mark.parametrize("arch", ["llama", "bloom"])
@pytest.mark.parametrize("lens", [[7, 12, 1, 30], [40, 70, 0, 33], [150, 130, 20], [600, 500],
                                  [(7 * i) % 6 for i in range(64)]],
                         ids=["50tok", "143tok", "300tok", "1100tok", "64seqs"])
def test_backward_matches_oracle(arch, lens):
    shape = SHAPES[arch]
    n = sum(lens)
    srv, W = make_train_server(shape, max_tokens=n)
    x, gy = draw_batch(shape, lens, seed=3)
    gx, y = srv.backward(lens, x, gy, want_y=True)
    y2 = srv.train_forward(lens, x)
    torch.cuda.synchronize()
    y_ref, gx_ref = bo.span_forward_backward(shape, W, x, gy, lens)
    assert row_rel_err(to_np(y), y_ref) < HIDDEN_TOL
    assert np.array_equal(to_np(y2), to_np(y))                    # same kernels, same order
    assert row_l2_rel_err(to_np(gx), gx_ref) < GRAD_TOL
    assert row_rel_err(to_np(gx), gx_ref) < 2 * GRAD_TOL          # element-wise, against the row's rms
    # a second call on the same span (stale scratch) gives the same bits
    gx2 = srv.backward(lens, x, gy)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(gx2), to_np(gx))


@pytest.mark.parametrize("shape", [SpanShape("llama", 1, 256, 16, 1, 64, 512), SpanShape("llama", 2, 256, 4, 2, 128, 512),
                                   SpanShape("bloom", 1, 256, 2, 2, 128, 512), SpanShape("llama", 1, 512, 12, 4, 64, 688),
                                   SpanShape("llama", 1, 64, 1, 1, 64, 8208)],
                         ids=["group16", "llama-hd128", "bloom-hd128", "group3", "long-k"])
def test_backward_head_layouts(shape):
    """Query groups wider than one workgroup of the attention kernels (16 heads per kv head), odd
    group sizes, 128-wide heads with and without the ALiBi bias, and an MLP wide enough that the
    transposed gate/up projection is split along k into several launches."""
    lens = [37, 90, 16] if shape.d_ff < 8192 else [500, 400, 190]     # the split applies above 1024 tokens
    srv, W = make_train_server(shape, max_tokens=sum(lens))
    x, gy = draw_batch(shape, lens, seed=11)
    gx, y = srv.backward(lens, x, gy, want_y=True)
    torch.cuda.synchronize()
    y_ref, gx_ref = bo.span_forward_backward(shape, W, x, gy, lens)
    assert row_rel_err(to_np(y), y_ref) < HIDDEN_TOL
    assert row_l2_rel_err(to_np(gx), gx_ref) < GRAD_TOL


@pytest.mark.parametrize("arch", ["llama", "bloom"])
def test_backward_sub_span_and_chain(arch):
    """A chain of two servers (one block each) hands the gradient back block by block."""
    shape = SHAPES[arch]
    lens = [9, 23]
    srv, W = make_train_server(shape, max_tokens=64)
    x, gy = draw_batch(shape, lens, seed=5)
    mid = srv.train_forward(lens, x, first_block=0, n_blocks=1)
    g_mid = srv.backward(lens, mid, gy, first_block=1, n_blocks=1)
    g_in = srv.backward(lens, x, g_mid, first_block=0, n_blocks=1)
    torch.cuda.synchronize()
    _, g_mid_ref = bo.span_forward_backward(shape, W, to_np(mid), gy, lens, first_block=1, n_blocks=1)
    assert row_l2_rel_err(to_np(g_mid), g_mid_ref) < GRAD_TOL
    _, whole = bo.span_forward_backward(shape, W, x, gy, lens)
    assert row_l2_rel_err(to_np(g_in), whole) < GRAD_TOL


def test_backward_bf16_io():
    shape = TINY
    lens = [20, 44]
    srv, W = make_train_server(shape, max_tokens=64, io_f32=False)
    x, gy = draw_batch(shape, lens, seed=7)
    gx = srv.backward(lens, x, gy)
    torch.cuda.synchronize()
    assert gx.dtype == torch.bfloat16
    _, gx_ref = bo.span_forward_backward(shape, W, x, gy, lens)
    assert row_l2_rel_err(to_np(gx), gx_ref) < GRAD_TOL


def test_training_passes_leave_sessions_alone():
    """Inference sessions of the same span keep decoding correctly around a backward call."""
    shape = TINY
    srv, W = make_train_server(shape, max_tokens=64)
    xs = draw_hidden(shape, 0, 1, 21)
    osess = so.Session(shape, W)
    s = srv.open(64)
    ys = [srv.forward([s], [12], xs[:12])]
    refs = [osess.forward(xs[:12])]
    free_before = B.span_debug_free_pages(srv.span)
    x, gy = draw_batch(shape, [30, 5], seed=9)
    for n in range(12, 21):
        if n % 3 == 0:
            srv.backward([30, 5], x, gy)
        ys.append(srv.forward([s], [1], xs[n:n + 1]))
        refs.append(osess.forward(xs[n:n + 1]))
    torch.cuda.synchronize()
    assert row_rel_err(np.concatenate([to_np(y) for y in ys]), np.concatenate(refs)) < HIDDEN_TOL
    assert B.span_session_length(srv.span, s) == 21
    assert B.span_debug_free_pages(srv.span) == free_before - 1          # 21 tokens: one more page, none for training


def test_training_errors():
    shape = TINY
    W = SpanWeights(shape, seed=0, bf16=True, cache=True)
    cfg = config_for(shape, max_pages=8, max_sessions=2, max_session_tokens=48, max_batch_tokens=64)
    srv = SpanServer(cfg, W, DEV, keep_canonical=True)
    x = torch.zeros(64, shape.d_model, device=DEV)
    g = torch.zeros_like(x)
    with pytest.raises(B.SpanError) as e:
        B.span_backward(srv.span, 0, 2, [4], x, x, g)
    assert e.value.code == B.SPAN_E_INVALID and "span_train_attach" in str(e.value)
    with pytest.raises(B.SpanError):
        B.span_train_sizes(cfg, 65)                                       # beyond max_batch_tokens
    srv.attach_training(32)
    for bad, code in [(dict(lens=[20, 13]), B.SPAN_E_TOO_MANY_TOKENS), (dict(lens=[-1]), B.SPAN_E_INVALID),
                      (dict(lens=[4], fb=1, nb=2), B.SPAN_E_INVALID), (dict(lens=[4], nb=0), B.SPAN_E_INVALID)]:
        with pytest.raises(B.SpanError) as e:
            B.span_backward(srv.span, bad.get("fb", 0), bad.get("nb", 2), bad["lens"], x, x, g)
        assert e.value.code == code, bad
    srv2 = SpanServer(config_for(shape, max_pages=8, max_sessions=2, max_session_tokens=16, max_batch_tokens=64), W, DEV,
                      keep_canonical=True)
    srv2.attach_training(64)
    with pytest.raises(B.SpanError) as e:
        B.span_backward(srv2.span, 0, 2, [17], x, x, g)                   # longer than the position table
    assert e.value.code == B.SPAN_E_TOO_LONG
    with pytest.raises(B.SpanError) as e:
        B.span_backward(srv.span, 0, 2, [4], x, None, g)
    assert e.value.code == B.SPAN_E_INVALID
    B.span_backward(srv.span, 0, 2, [], x, x, g)                          # an empty batch is a no-op
    B.span_backward(srv.span, 0, 2, [0, 0], x, x, g)
    torch.cuda.synchronize()


@pytest.mark.parametrize("arch", ["llama", "bloom"])
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("lens", [[9, 30], [100, 61, 16]], ids=["39tok", "177tok"])
def test_backward_through_compressed_weights(arch, bits, lens):
    """Fine-tuning through quantised servers (Sections 3.1 and 3.3): forward and backward passes of a
    span with 8-bit / 4-bit block-quantised weights follow the oracle run on the dequantised matrices."""
    from oracle import lowbit_oracle as lo
    from workloads import normal_levels16
    shape = SHAPES[arch]
    levels = normal_levels16()
    W = SpanWeights(shape, seed=2, bf16=True, cache=True)
    cfg = config_for(shape, max_pages=32, max_sessions=4, max_session_tokens=256, max_batch_tokens=256,
                     weight_bits=bits, levels=levels)
    srv = SpanServer(cfg, W, DEV)
    srv.attach_training(sum(lens))
    assert srv.train_sizes[0] == 0
    x, gy = draw_batch(shape, lens, seed=13)
    gx, y = srv.backward(lens, x, gy, want_y=True)
    torch.cuda.synchronize()
    Wq = lo.quantized_weights([W[b] for b in range(shape.n_blocks)], bits, levels)
    y_ref, gx_ref = bo.span_forward_backward(shape, Wq, x, gy, lens)
    assert row_rel_err(to_np(y), y_ref) < HIDDEN_TOL
    assert row_l2_rel_err(to_np(gx), gx_ref) < GRAD_TOL
    # the sessions of a compressed span are untouched as well
    assert B.span_debug_free_pages(srv.span) == 32

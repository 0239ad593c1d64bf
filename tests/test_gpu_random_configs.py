"""Seeded random small configurations through the whole boundary: a random block shape (both styles,
head widths, group sizes, compressed or bf16 weights, bf16 or fp32 I/O), a few calls with random token
counts per session (prefix, chunks, single tokens, idle sessions), a cache reordering in between, then
one training-time backward call with random sequence lengths -- every output against the oracles."""
import numpy as np
import pytest
import torch

from gpu_util import *  # noqa: F401,F403
from oracle import backward_oracle as bo
from oracle import lowbit_oracle as lo
from workloads import SpanShape, normal_levels16

pytestmark = pytest.mark.gpu

# Element-wise form of the output bar, max |gpu - oracle| / rms(oracle row).  These spans are at most three
# blocks deep and at most 512 wide; the same 2e-2 as the row form holds.
ELEM_TOL = HIDDEN_TOL


def random_shape(rng):
    arch = str(rng.choice(["llama", "bloom"]))
    hd = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 3, 4]))
    hq = hkv * int(rng.choice([1, 2, 3, 4, 5, 8, 16]))
    if hq * hd > 2048:
        hq = hkv
    d = int(rng.choice([32, 96, 256, 320, 512]))
    f = int(rng.choice([16, 48, 688, 512, 1040])) if arch == "llama" else int(rng.choice([32, 96, 512, 1056]))
    return SpanShape(arch, int(rng.choice([1, 2, 3])), d, hq, hkv, hd, f)


@pytest.mark.parametrize("seed", range(300, 324))
def test_random_configuration(seed):
    rng = np.random.default_rng(seed)
    shape = random_shape(rng)
    mbt = int(rng.choice([64, 130, 300, 1100]))
    bits = int(rng.choice([0, 0, 8, 4]))
    levels = normal_levels16()
    W = SpanWeights(shape, seed=seed, bf16=True, cache=True)
    cfg = config_for(shape, max_pages=200, max_sessions=6, max_session_tokens=1300, max_batch_tokens=mbt,
                     io_f32=bool(rng.integers(2)), weight_bits=bits, levels=levels if bits == 4 else None)
    srv = SpanServer(cfg, W, DEV, keep_canonical=True)
    Wo = lo.quantized_weights([W[b] for b in range(shape.n_blocks)], bits, levels) if bits else W
    n_sess = int(rng.integers(1, 5))
    ids = [srv.open(1300) for _ in range(n_sess)]
    osess = [so.Session(shape, Wo) for _ in range(n_sess)]
    for call in range(4):
        T = [int(rng.choice([0, 1, 1, 2, 17, 40])) for _ in range(n_sess)]
        if call == 0:
            T = [int(rng.integers(1, max(2, mbt // n_sess))) for _ in range(n_sess)]
        while sum(T) > mbt:
            T[int(np.argmax(T))] //= 2
        if sum(T) == 0:
            continue
        xs = [draw_hidden(shape, seed, 10 * call + i, t) for i, t in enumerate(T)]
        y = to_np(srv.forward(ids, T, np.concatenate(xs)))
        ref = np.concatenate([o.forward(x) for o, x in zip(osess, xs)])
        assert row_l2_rel_err(y, ref) < HIDDEN_TOL, (shape, bits, call, T)
        assert row_rel_err(y, ref) < ELEM_TOL, (shape, bits, call, T, row_rel_err(y, ref))      # element-wise form
        if call == 1 and n_sess > 1:
            hypo = [int(rng.integers(0, n_sess)) for _ in range(n_sess)]
            srv.reorder(ids, hypo)
            osess = so.reorder(osess, hypo)
    assert [B.span_session_length(srv.span, s) for s in ids] == [o.length for o in osess]

    mt = min(mbt, 400)
    srv.attach_training(mt)
    n_seq = int(rng.integers(1, 5))
    lens = [int(rng.integers(0, mt // n_seq + 1)) for _ in range(n_seq)]
    if sum(lens) == 0:
        lens[0] = 5
    n = sum(lens)
    x = draw_hidden(shape, seed, 99, n)
    gy = bf16_round(rng.standard_normal((n, shape.d_model)).astype(np.float32))
    gx, yy = srv.backward(lens, x, gy, want_y=True)
    torch.cuda.synchronize()
    y_ref, gx_ref = bo.span_forward_backward(shape, Wo, x, gy, lens)
    assert row_l2_rel_err(to_np(yy), y_ref) < HIDDEN_TOL, (shape, bits, lens)
    assert row_rel_err(to_np(yy), y_ref) < ELEM_TOL, (shape, bits, lens, row_rel_err(to_np(yy), y_ref))
    assert row_l2_rel_err(to_np(gx), gx_ref) < GRAD_TOL, (shape, bits, lens)
    srv.destroy()

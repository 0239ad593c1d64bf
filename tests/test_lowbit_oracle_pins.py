"""Pins for the low-bit weight oracle (Section 3.1, "Compression": 8-bit and 4-bit weights).

The paper names the formats and prints no numbers for them, so the encoder is pinned by what
an absmax block format fixes mathematically: the error bound of rounding to the nearest level,
exactness on representable inputs, idempotence, behaviour under exact rescaling, brute-force
nearest-level search, and the block boundaries (a mistake in the block size, the block axis,
the scale or the rounding rule fails at least one of these).
"""
import numpy as np
import pytest

from oracle import lowbit_oracle as lo
from oracle import span_oracle as so
from workloads import TINY, SpanWeights, draw_hidden, normal_levels16

LEVELS = normal_levels16()


def draw(n, k, seed=0, scale=0.02):
    return (scale * np.random.default_rng(seed).standard_normal((n, k))).astype(np.float32)


@pytest.mark.parametrize("k", [64, 256, 688, 100])
def test_int8_error_bound_and_extremes(k):
    w = draw(24, k, 1)
    codes, absmax = lo.quantize_int8(w)
    assert codes.dtype == np.int8 and codes.shape == w.shape and absmax.shape == (24, -(-k // 64))
    deq = lo.dequantize_int8(codes, absmax)
    step = np.repeat(absmax.astype(np.float64), 64, axis=1)[:, :k] / 127
    assert np.all(np.abs(deq - w) <= 0.5 * step * (1 + 1e-6))            # nearest of 255 evenly spaced levels
    assert np.max(np.abs(deq - w) / step) > 0.45                          # ... and no tighter grid than that
    # the largest element of every block maps to +-127 and comes back exactly
    for b in range(absmax.shape[1]):
        blk = w[:, b * 64:(b + 1) * 64]
        j = np.argmax(np.abs(blk), axis=1)
        rows = np.arange(24)
        assert np.all(np.abs(codes[rows, b * 64 + j]) == 127)
        assert np.all(absmax[:, b] == np.abs(blk[rows, j]))
        assert np.allclose(deq[rows, b * 64 + j], blk[rows, j], rtol=1e-7, atol=0)


def test_int8_is_exact_on_its_own_grid_and_idempotent():
    rng = np.random.default_rng(2)
    codes0 = rng.integers(-127, 128, size=(8, 192)).astype(np.int8)
    codes0[:, ::64] = 127                                                 # every block holds its absmax
    absmax0 = (2.0 ** rng.integers(-8, 3, size=(8, 3))).astype(np.float32)
    w = lo.dequantize_int8(codes0, absmax0, dtype=np.float64).astype(np.float32)
    codes, absmax = lo.quantize_int8(w)
    assert np.array_equal(codes, codes0) and np.array_equal(absmax, absmax0)
    # scaling a matrix by a power of two scales absmax and leaves the codes alone
    c2, a2 = lo.quantize_int8(draw(8, 192, 3) * np.float32(8))
    c1, a1 = lo.quantize_int8(draw(8, 192, 3))
    assert np.array_equal(c1, c2) and np.array_equal(a2, a1 * 8)


def test_blocks_run_along_the_input_features_of_each_row():
    w = np.full((3, 128), 0.001, np.float32)
    w[1, 70] = 1.0                                                        # row 1, second block only
    codes, absmax = lo.quantize_int8(w)
    assert absmax[1, 1] == 1.0 and np.all(absmax[[0, 2]] == np.float32(0.001)) and absmax[1, 0] == np.float32(0.001)
    assert np.all(codes[1, 64:70] == 0) and codes[1, 70] == 127 and np.all(codes[1, :64] == 127)
    c4, a4 = lo.quantize_codebook(w, LEVELS)
    assert np.array_equal(a4, absmax) and c4[1, 70] == 15 and np.all(c4[1, 64:70] == 7) and np.all(c4[0] == 15)


def test_zero_blocks_and_signs():
    w = np.zeros((2, 64), np.float32)
    w[1, 5] = -0.5
    codes, absmax = lo.quantize_int8(w)
    assert np.all(codes[0] == 0) and absmax[0, 0] == 0 and codes[1, 5] == -127 and absmax[1, 0] == 0.5
    assert np.all(lo.dequantize_int8(codes, absmax)[0] == 0)
    c4, a4 = lo.quantize_codebook(w, LEVELS)
    assert np.all(c4[0] == 7) and c4[1, 5] == 0 and LEVELS[7] == 0
    assert np.all(lo.dequantize_codebook(c4, a4, LEVELS)[0] == 0)
    assert lo.dequantize_codebook(c4, a4, LEVELS)[1, 5] == -0.5


@pytest.mark.parametrize("k", [64, 688])
def test_codebook_picks_the_nearest_level(k):
    w = draw(16, k, 4)
    codes, absmax = lo.quantize_codebook(w, LEVELS)
    assert codes.dtype == np.uint8 and codes.max() <= 15
    scale = np.repeat(absmax.astype(np.float64), 64, axis=1)[:, :k]
    r = w.astype(np.float64) / scale
    brute = np.argmin(np.abs(r[:, :, None] - LEVELS.astype(np.float64)[None, None, :]), axis=2)
    d = np.sort(np.abs(r[:, :, None] - LEVELS.astype(np.float64)[None, None, :]), axis=2)
    clear = (d[:, :, 1] - d[:, :, 0]) > 1e-6                              # away from fp32-sized ties
    assert clear.mean() > 0.999 and np.array_equal(codes[clear], brute[clear].astype(np.uint8))
    deq = lo.dequantize_codebook(codes, absmax, LEVELS)
    half_gap = 0.5 * np.max(np.diff(LEVELS.astype(np.float64)))
    assert np.all(np.abs(deq - w) <= half_gap * scale * (1 + 1e-6))
    # every level is reproduced exactly, ties go to the lower level
    grid = (LEVELS[None, :].repeat(4, 0) * np.float32(0.25)).astype(np.float32)
    grid = np.concatenate([grid, np.full((4, 48), 0.25, np.float32)], axis=1)   # block absmax 0.25, from the level 1.0
    cg, ag = lo.quantize_codebook(grid, LEVELS)
    assert np.array_equal(cg[:, :16], np.arange(16, dtype=np.uint8)[None].repeat(4, 0)) and np.all(ag == 0.25)
    mids = lo.codebook_midpoints(LEVELS)
    tie = np.concatenate([mids, [1.0]]).astype(np.float32)[None]
    ct, _ = lo.quantize_codebook(np.concatenate([tie, np.zeros((1, 48), np.float32)], axis=1), LEVELS)
    assert np.array_equal(ct[0, :15], np.arange(15, dtype=np.uint8))
    with pytest.raises(ValueError):
        lo.codebook_midpoints(LEVELS[::-1])


def test_quantized_span_is_the_span_of_the_dequantised_weights():
    """The meaning of a compressed server: the same span arithmetic on dequantised matrices; norm
    gains are left alone; the error against the uncompressed span shrinks with the bit width."""
    W = SpanWeights(TINY, seed=0, bf16=True, cache=True)
    x = draw_hidden(TINY, 0, 0, 12)
    y16 = so.span_full(TINY, W, x)
    errs = {}
    for bits in (8, 4):
        Wq = lo.quantized_weights(W, bits, LEVELS)
        assert all(np.array_equal(Wq[b]["norm1_g"], W[b]["norm1_g"]) for b in range(TINY.n_blocks))
        assert not np.array_equal(Wq[0]["wq"], W[0]["wq"]) and Wq[0]["wq"].shape == W[0]["wq"].shape
        yq = so.span_full(TINY, Wq, x)
        s = so.Session(TINY, Wq)
        assert np.max(np.abs(s.forward(x) - yq)) < 1e-9
        errs[bits] = float(np.sqrt(np.mean((yq - y16) ** 2) / np.mean(y16 ** 2)))
    assert errs[8] < 2e-2 and errs[8] < errs[4] < 0.3


# ----------------------------------------------------------------------------- hidden-state codec

from workloads import dynamic_levels256

DYN = dynamic_levels256()


@pytest.mark.parametrize("block", [64, 256])
def test_hidden_codec_picks_the_nearest_level_per_block(block):
    x = np.random.default_rng(8).standard_normal((6, 700)).astype(np.float32) * np.float32(3)
    x[2, 64:128] = 0.0                                                    # an all-zero block (for block 64)
    codes, absmax = lo.encode_hidden(x, DYN, block)
    assert codes.dtype == np.uint8 and codes.shape == x.shape and absmax.shape == (6, -(-700 // block))
    scale = np.repeat(absmax.astype(np.float64), block, axis=1)[:, :700]
    safe = np.where(scale > 0, scale, 1.0)
    r = x.astype(np.float64) / safe
    dist = np.abs(r[:, :, None] - DYN.astype(np.float64)[None, None, :])
    brute = np.argmin(dist, axis=2)
    d2 = np.sort(dist, axis=2)
    clear = (d2[:, :, 1] - d2[:, :, 0]) > 1e-6
    assert clear.mean() > 0.98 and np.array_equal(codes[clear], brute[clear].astype(np.uint8))   # (the zero block ties by design)
    deq = lo.decode_hidden(codes, absmax, DYN, block)
    assert np.all(np.abs(deq - x) <= 0.5 * np.max(np.diff(DYN.astype(np.float64))) * scale * (1 + 1e-6))
    # a block's largest element comes back exactly, with the code of +-1
    for b in range(absmax.shape[1]):
        blk = x[:, b * block:(b + 1) * block]
        j = np.argmax(np.abs(blk), axis=1)
        rows = np.arange(6)
        nz = absmax[:, b] > 0
        assert np.all(np.isin(codes[rows, b * block + j][nz], [0, 255]))
        assert np.allclose(deq[rows, b * block + j], blk[rows, j], rtol=1e-7, atol=0)
    if block == 64:
        assert np.all(codes[2, 64:128] == 127) and DYN[127] == 0 and np.all(deq[2, 64:128] == 0)


def test_hidden_codec_is_exact_on_its_grid_and_scale_free():
    rng = np.random.default_rng(9)
    codes0 = rng.integers(0, 256, size=(4, 128)).astype(np.uint8)
    codes0[:, ::64] = 255
    absmax0 = (2.0 ** rng.integers(-3, 4, size=(4, 2))).astype(np.float32)
    x = lo.decode_hidden(codes0, absmax0, DYN).astype(np.float32)
    codes, absmax = lo.encode_hidden(x, DYN)
    assert np.array_equal(absmax, absmax0)
    # levels this close to each other (1e-7 apart near zero) survive fp32 only when the block scale is 1;
    # away from the tiny levels the round trip is exact
    big = np.abs(DYN[codes0]) > 1e-4
    assert np.array_equal(codes[big], codes0[big])
    y = rng.standard_normal((4, 128)).astype(np.float32)
    c1, a1 = lo.encode_hidden(y, DYN)
    c2, a2 = lo.encode_hidden(y * np.float32(4), DYN)
    assert np.array_equal(c1, c2) and np.array_equal(a2, a1 * 4)
    # the relative error of a typical hidden row is about one percent (8 bits, non-uniform levels)
    rel = np.linalg.norm(lo.decode_hidden(c1, a1, DYN) - y) / np.linalg.norm(y)
    assert rel < 0.03
    with pytest.raises(ValueError):
        lo.encode_hidden(y, DYN[:255])

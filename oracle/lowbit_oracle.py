"""Block-wise low-bit weight formats: plain CPU reference (test infrastructure only).

The paper stores the servers' weights compressed (Section 3.1, "Compression": 8-bit weights
for BLOOM, the 4-bit NormalFloat format for Llama 2) so that a server holds more blocks and a
generation step streams fewer bytes.  What the hot path needs from such a format is

  * the encoder: weights -> (integer codes, one scale per block), and
  * the meaning of an encoded matrix: the dequantised matrix, used in y = x W^T as before.

Both formats here are *absmax block formats*: a row of a weight matrix [out, in] is cut into
blocks of 64 consecutive input features; a block is stored as its largest magnitude ("absmax",
fp32) and one code per element:

  int8      code = round(w / absmax * 127)            in [-127, 127];  w' = code * absmax / 127
  codebook  code = index of the level nearest to w / absmax, levels = 16 ascending numbers in
            [-1, 1] (a 4-bit format; the NormalFloat levels are one such table);
            w' = level[code] * absmax

Readings (the paper only names the formats): weights only are quantised, hidden states stay in
the working precision (no outlier decomposition: it concerns the hidden states); a row's last
block may be shorter than 64; an all-zero block has absmax 0 and codes 0 (int8) / the code of
the level nearest 0 (codebook); ties go to the lower level; every decision that yields an
integer is taken in fp32 with the operations written below, so that another implementation
using the same fp32 operations gets the same codes bit for bit.

Nothing outside tests/, the smoke check and the benchmark's CPU leg may import this module.
"""
from typing import Tuple

import numpy as np

BLOCK = 64


def _blocks(w: np.ndarray) -> Tuple[np.ndarray, int]:
    """fp32 [N, K] -> [N, nb, 64] zero-padded along K, and nb."""
    w = np.asarray(w, dtype=np.float32)
    n, k = w.shape
    nb = -(-k // BLOCK)
    pad = np.zeros((n, nb * BLOCK), np.float32)
    pad[:, :k] = w
    return pad.reshape(n, nb, BLOCK), nb


def quantize_int8(w: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (codes int8 [N, K], absmax fp32 [N, ceil(K/64)])."""
    k = w.shape[1]
    b, _ = _blocks(w)
    absmax = np.max(np.abs(b), axis=2).astype(np.float32)
    safe = np.where(absmax > 0, absmax, np.float32(1)).astype(np.float32)
    r = (b / safe[:, :, None]).astype(np.float32)            # fp32 division
    r = (r * np.float32(127)).astype(np.float32)             # fp32 product
    codes = np.rint(r).astype(np.int8)                       # round half to even
    return codes.reshape(w.shape[0], -1)[:, :k], absmax


def dequantize_int8(codes: np.ndarray, absmax: np.ndarray, dtype=np.float64) -> np.ndarray:
    n, k = codes.shape
    scale = np.repeat(absmax.astype(dtype), BLOCK, axis=1)[:, :k] / dtype(127)
    return codes.astype(dtype) * scale


def codebook_midpoints(levels: np.ndarray) -> np.ndarray:
    lv = np.asarray(levels, dtype=np.float32)
    if lv.shape != (16,) or not np.all(np.diff(lv) > 0):
        raise ValueError("a codebook is 16 strictly ascending levels")
    return ((lv[:-1] + lv[1:]) * np.float32(0.5)).astype(np.float32)


def quantize_codebook(w: np.ndarray, levels: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (codes uint8 [N, K] in 0..15, absmax fp32 [N, ceil(K/64)])."""
    k = w.shape[1]
    mids = codebook_midpoints(levels)
    b, _ = _blocks(w)
    absmax = np.max(np.abs(b), axis=2).astype(np.float32)
    safe = np.where(absmax > 0, absmax, np.float32(1)).astype(np.float32)
    r = (b / safe[:, :, None]).astype(np.float32)
    # nearest level = number of midpoints strictly below the value (a tie stays on the lower level)
    codes = np.zeros(r.shape, np.uint8)
    for m in mids:
        codes += (r > m).astype(np.uint8)
    return codes.reshape(w.shape[0], -1)[:, :k], absmax


def dequantize_codebook(codes: np.ndarray, absmax: np.ndarray, levels: np.ndarray, dtype=np.float64) -> np.ndarray:
    n, k = codes.shape
    lv = np.asarray(levels, dtype=np.float32).astype(dtype)
    scale = np.repeat(absmax.astype(dtype), BLOCK, axis=1)[:, :k]
    return lv[codes] * scale


def quantized_weights(weights, bits: int, levels=None, dtype=np.float64):
    """Block weight dicts with every projection matrix replaced by its dequantised form;
    vectors (norm gains, biases) are kept.  `weights` is a sequence of dicts name -> array."""
    out = []
    for w in weights:
        d = {}
        for name, a in w.items():
            a = np.asarray(a)
            if a.ndim == 2:
                if bits == 8:
                    d[name] = dequantize_int8(*quantize_int8(a), dtype=dtype)
                elif bits == 4:
                    c, s = quantize_codebook(a, levels)
                    d[name] = dequantize_codebook(c, s, levels, dtype=dtype)
                else:
                    raise ValueError("bits must be 8 or 4")
            else:
                d[name] = a
        out.append(d)
    return out


# --------------------------------------------------------------------------- hidden states on the wire

def encode_hidden(x: np.ndarray, levels: np.ndarray, block: int = 64) -> Tuple[np.ndarray, np.ndarray]:
    """Dynamic block-wise 8-bit quantisation of hidden states (Section 3.1, "Compression", last
    paragraph: applied before hidden states travel between pipeline stages, halving the bytes).
    Each row [d] is cut into blocks of `block` consecutive features; a block is stored as its
    absmax (fp32) and one byte per element: the index of the level nearest to x / absmax among
    256 ascending levels in [-1, 1] (the "dynamic" non-uniform 8-bit data type is one such table;
    ties go to the lower level; an all-zero block gets the code of the level nearest 0).
    Decisions in fp32 as in the weight formats.  Returns (codes uint8 [M, d], absmax fp32
    [M, ceil(d/block)])."""
    lv = np.asarray(levels, dtype=np.float32)
    if lv.shape != (256,) or not np.all(np.diff(lv) > 0):
        raise ValueError("the table is 256 strictly ascending levels")
    mids = ((lv[:-1] + lv[1:]) * np.float32(0.5)).astype(np.float32)
    x = np.asarray(x, dtype=np.float32)
    m, d = x.shape
    nb = -(-d // block)
    pad = np.zeros((m, nb * block), np.float32)
    pad[:, :d] = x
    b = pad.reshape(m, nb, block)
    absmax = np.max(np.abs(b), axis=2).astype(np.float32)
    safe = np.where(absmax > 0, absmax, np.float32(1)).astype(np.float32)
    r = (b / safe[:, :, None]).astype(np.float32)
    codes = np.searchsorted(mids, r.reshape(-1), side="left").astype(np.uint8)     # midpoints strictly below
    return codes.reshape(m, -1)[:, :d], absmax


def decode_hidden(codes: np.ndarray, absmax: np.ndarray, levels: np.ndarray, block: int = 64,
                  dtype=np.float64) -> np.ndarray:
    m, d = codes.shape
    lv = np.asarray(levels, dtype=np.float32).astype(dtype)
    scale = np.repeat(absmax.astype(dtype), block, axis=1)[:, :d]
    return lv[codes] * scale

"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

from oracle import span_oracle as so
from paper_2312_08361_amd import binding as B
from paper_2312_08361_amd.server import SpanServer, bf16_tensor_from_bits, config_for
from workloads import SpanWeights, bf16_bits, bf16_round, bf16_widen, draw_hidden
from gpu_bars import alone_bars, deep_span_bars, floor_of

DEV = "cuda:0"

# Tolerances of the bf16 path (bf16 operands and cache, fp32 accumulation) against the fp32 / fp64 oracle.
HIDDEN_TOL = 2e-2      # output hidden states (the benchmark spec's bar): max over token rows of the relative error of the
                       # row, ||gpu_t - oracle_t||_2 / ||oracle_t||_2 (row_l2_rel_err); the small-shape tests also
                       # hold the element-wise form max |gpu - oracle| / rms(oracle row) (row_rel_err) under the
                       # same number.  Held by every block on its own at every shape and by whole spans of the
                       # small and the 7B-shaped configurations.
# Whole spans of the 70B- and BLOOM-176B-shaped configurations cannot meet 2e-2 end to end, whatever the
# kernels do: the precision contract itself (every contraction operand and the cache rounded to bf16) puts a
# numpy model of the span 3.6e-2 (70B shape, 8 blocks) / 2.1e-2 (BLOOM shape, 4 blocks) from the oracle on these
# synthetic inputs (tests/precision_model.py, tests/test_precision_model.py; full-shape figures in
# tests/golden/precision_floor.txt).  The bars of those tests come from that stored floor (gpu_bars): 1.25 x for
# the largest row error and the largest element error, 1.05 x for the rms element error -- the GPU's error must
# have the size of the contract's own, and nothing on top.  The GPU's distance from the model itself is reported
# and held under the floor; it is not small, and cannot be: a value that differs by a fraction of a bf16 step
# (fp32 sums taken in another order flip one q / k / v rounding in 700) draws every later rounding afresh, so two
# faithful realisations of the contract part by about half the floor within one block (measured on block 0 of
# the 70B shape: identical inputs, q / k / v equal but for 0.15 % of the elements -> outputs 3.5e-3 apart; the
# numpy model run on the GPU's own q, k, v still 3.2e-3 from it).  Kernel arithmetic is held tightly where that
# is possible: operator by operator on identical operands (tests/test_gpu_ops.py, tests/test_gpu_taps.py).
GRAD_TOL = 3e-2        # input gradients of the training-time backward pass, same row metric as HIDDEN_TOL: the
                       # backward chain runs about twice as many bf16-input contractions as the forward pass
LOGIT_TOL = 1e-3       # same metric, normalised by max |logit| of the row, on attention logits
KV_TOL = 1.2e-2        # cached K/V entries: one bf16 rounding (2^-9 of the largest entry) + upstream


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True)) + 1e-30
    return float(np.max(np.abs(got - ref) / rms))


def row_l2_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.sqrt(np.sum((got - ref) ** 2, axis=-1))
    den = np.sqrt(np.sum(ref * ref, axis=-1)) + 1e-30
    return float(np.max(num / den))


def check_hidden(got: np.ndarray, ref: np.ndarray, tol: float = HIDDEN_TOL, elem_tol: float = None, rms_tol: float = None):
    """Returns (row relative error, largest element error / rms of its row, rms element error) and asserts the
    row bar and, when given, the fixed element bar and the bar on the rms element error."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms_ref = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True)) + 1e-30
    rel = (got - ref) / rms_ref
    l2, mx, rms = row_l2_rel_err(got, ref), float(np.max(np.abs(rel))), float(np.sqrt(np.mean(rel * rel)))
    assert l2 < tol, f"row relative error {l2:.3e} exceeds {tol:.3e}"
    if elem_tol is not None:
        assert mx < elem_tol, f"element error {mx:.3e} (of the row's rms) exceeds {elem_tol:.3e}"
    if rms_tol is not None:
        assert rms < rms_tol, f"rms element error {rms:.3e} exceeds {rms_tol:.3e}"
    return l2, mx, rms


def check_hidden_where_different(got: np.ndarray, ref: np.ndarray, tol: float = HIDDEN_TOL, elem_tol: float = None) -> float:
    """GPU against GPU: most rows of two runs are bit-identical (same kernels, same summation order) and
    only the rows that took another kernel in one of the runs differ; the bars are applied to those.
    Returns the row relative error (0.0 if all rows agree)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rows = np.any(got != ref, axis=-1)
    if not rows.any():
        return 0.0
    return check_hidden(got[rows], ref[rows], tol, elem_tol)[0]


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def dev_bf16(a: np.ndarray) -> torch.Tensor:
    """fp32 numpy holding bf16-representable values -> device bf16 tensor."""
    return bf16_tensor_from_bits(bf16_bits(a), DEV)

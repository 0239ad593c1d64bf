"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

from oracle import span_oracle as so
from paper_2312_08361_amd import binding as B
from paper_2312_08361_amd.server import SpanServer, bf16_tensor_from_bits, config_for
from workloads import SpanWeights, bf16_bits, bf16_round, bf16_widen, draw_hidden

DEV = "cuda:0"

# Tolerances of the bf16 path, fp32 accumulation:
HIDDEN_TOL = 2e-2      # output hidden states: max over token rows of the relative error of the row,
                       # ||gpu_t - oracle_t||_2 / ||oracle_t||_2 (row_l2_rel_err).  The small-shape tests
                       # also hold the stricter element-wise form (row_rel_err) under the same number.
DEEP_SPAN_TOL = 6e-2   # whole 8-block spans of the random-weight 70B shape with 2048+ token contexts: the
                       # rounding error of the first blocks (bf16 q/k in front of a peaked softmax alone gives
                       # 5e-3..2.5e-2 per row) is amplified by every later block; each block on its own
                       # still meets HIDDEN_TOL (checked separately with the oracle's inputs).
OUTLIER_SIGMAS = 8.0   # large shapes: no element may be further out than this many times the rms error
                       # (rounding noise over 1e7..1e8 elements peaks near 6 sigma; a wrong element is far beyond)
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


def check_hidden(got: np.ndarray, ref: np.ndarray, tol: float = HIDDEN_TOL):
    """Large-shape criterion: (row relative error, element-wise max error, rms error); asserts both bars."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms_ref = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True)) + 1e-30
    rel = (got - ref) / rms_ref
    l2, mx, rms = row_l2_rel_err(got, ref), float(np.max(np.abs(rel))), float(np.sqrt(np.mean(rel * rel)))
    assert l2 < tol, f"row relative error {l2:.3e} exceeds {tol}"
    assert mx <= OUTLIER_SIGMAS * rms, f"outlier: element error {mx:.3e} vs rms error {rms:.3e}"
    return l2, mx, rms


def check_hidden_where_different(got: np.ndarray, ref: np.ndarray, tol: float = HIDDEN_TOL) -> float:
    """GPU against GPU: most rows of two runs are bit-identical (same kernels, same summation order) and
    only the rows that took another kernel in one of the runs differ.  The outlier bar of check_hidden
    compares the largest element error with the rms error, so it is applied to the rows that differ at
    all (identical rows would dilute the rms).  Returns the row relative error (0.0 if all rows agree)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rows = np.any(got != ref, axis=-1)
    if not rows.any():
        return 0.0
    return check_hidden(got[rows], ref[rows], tol)[0]


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def dev_bf16(a: np.ndarray) -> torch.Tensor:
    """fp32 numpy holding bf16-representable values -> device bf16 tensor."""
    return bf16_tensor_from_bits(bf16_bits(a), DEV)

"""Seeded synthetic workloads for the block-span forward path.

This module only *draws numbers and describes shapes*; it contains none of the
transformer arithmetic.  Both the CPU oracle's tests and the HIP path's tests
take their inputs from here so that the two sides see identical bits.

Recipe (one independent numpy Generator per tensor, so tensors can be drawn in
any order and in parallel):

    rng = numpy.random.default_rng([seed, block, tensor_id])
    matrices      W = 0.02 * N(0,1)                (std 0.02)
    norm gains    g = 1 + 0.02 * N(0,1)
    biases        b = 0.02 * N(0,1)
    hidden states x = N(0,1),  rng = default_rng([seed, 1000 + session])

bf16 workloads round every drawn value to the nearest bf16 (ties to even); the
rounded value is what both sides consume (the oracle widened to fp64, the GPU as
the raw 16-bit pattern).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Sequence

import numpy as np

ARCH_LLAMA = "llama"
ARCH_BLOOM = "bloom"


@dataclass(frozen=True)
class SpanShape:
    """Shape of one server's span of transformer blocks."""
    arch: str
    n_blocks: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    norm_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def with_blocks(self, n: int) -> "SpanShape":
        return replace(self, n_blocks=n)


# tensor names and (rows, cols) builders; a vector has cols == 0
def tensor_shapes(s: SpanShape) -> Dict[str, tuple]:
    d, qd, kd, f = s.d_model, s.q_dim, s.kv_dim, s.d_ff
    if s.arch == ARCH_LLAMA:
        return {
            "norm1_g": (d,), "wq": (qd, d), "wk": (kd, d), "wv": (kd, d), "wo": (d, qd),
            "norm2_g": (d,), "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
        }
    if s.arch == ARCH_BLOOM:
        return {
            "norm1_g": (d,), "norm1_b": (d,),
            "wq": (qd, d), "bq": (qd,), "wk": (kd, d), "bk": (kd,), "wv": (kd, d), "bv": (kd,),
            "wo": (d, qd), "bo": (d,),
            "norm2_g": (d,), "norm2_b": (d,),
            "w_up": (f, d), "b_up": (f,), "w_down": (d, f), "b_down": (d,),
        }
    raise ValueError(f"unknown arch {s.arch!r}")


_TENSOR_IDS = ["norm1_g", "norm1_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo",
               "norm2_g", "norm2_b", "w_gate", "w_up", "b_up", "w_down", "b_down"]


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns, round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_widen(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> fp32 values (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """fp32 -> nearest bf16 value, returned as fp32."""
    return bf16_widen(bf16_bits(a))


def draw_tensor(shape: SpanShape, seed: int, block: int, name: str, bf16: bool = True) -> np.ndarray:
    """One weight tensor of one block as fp32 (bf16-representable when bf16=True)."""
    dims = tensor_shapes(shape)[name]
    rng = np.random.default_rng([seed, block, _TENSOR_IDS.index(name)])
    a = rng.standard_normal(dims, dtype=np.float32)
    a *= np.float32(0.02)
    if name.endswith("_g"):
        a += np.float32(1.0)
    return bf16_round(a) if bf16 else a


class SpanWeights(Sequence):
    """Lazy, indexable-by-block view of a span's seeded weights.

    ``weights[b]`` returns ``{name: fp32 ndarray}`` for block ``b``.  Blocks are
    regenerated on every access unless ``cache=True`` (large shapes do not fit
    host memory all at once as fp32).
    """

    def __init__(self, shape: SpanShape, seed: int = 0, bf16: bool = True, cache: bool = False,
                 threads: int = 8):
        self.shape, self.seed, self.bf16 = shape, seed, bf16
        self._cache: Optional[dict] = {} if cache else None
        self._threads = threads

    def __len__(self) -> int:
        return self.shape.n_blocks

    def tensor(self, block: int, name: str) -> np.ndarray:
        return draw_tensor(self.shape, self.seed, block, name, self.bf16)

    def __getitem__(self, block: int) -> Dict[str, np.ndarray]:
        if not 0 <= block < self.shape.n_blocks:
            raise IndexError(block)
        if self._cache is not None and block in self._cache:
            return self._cache[block]
        names = list(tensor_shapes(self.shape))
        with ThreadPoolExecutor(self._threads) as ex:
            arrs = list(ex.map(lambda n: self.tensor(block, n), names))
        out = dict(zip(names, arrs))
        if self._cache is not None:
            self._cache[block] = out
        return out


def draw_hidden(shape: SpanShape, seed: int, session: int, n_tokens: int, bf16: bool = True) -> np.ndarray:
    """Pre-drawn open-loop hidden states for one session: [n_tokens, d_model] fp32, N(0,1)."""
    rng = np.random.default_rng([seed, 1000 + session])
    x = rng.standard_normal((n_tokens, shape.d_model), dtype=np.float32)
    return bf16_round(x) if bf16 else x



def dynamic_levels256() -> np.ndarray:
    """A 256-level table for the 8-bit hidden-state codec (input data): 127 magnitudes built like a
    sign / unary-exponent / linear-fraction code (exponent e = 0..6 decades, 2^(6-e) evenly spaced
    fractions in each decade, so resolution is spent where values are large), mirrored, plus zero
    and one extra tiny level, scaled to [-1, 1].  It has the structure of the published dynamic
    8-bit data type without claiming its digits; the library takes any ascending table."""
    mags = []
    for e in range(7):
        n = 2 ** (6 - e)
        for j in range(n):
            mags.append(10.0 ** (-e) * (0.1 + 0.9 * (j + 1) / n))
    mags = np.array(sorted(set(mags)), dtype=np.float64)
    assert mags.size == 127 and mags[-1] == 1.0
    lv = np.concatenate([-mags[::-1], [0.0, mags[0] * 0.1], mags])
    assert lv.size == 256 and np.all(np.diff(lv) > 0)
    return lv.astype(np.float32)


def normal_levels16() -> np.ndarray:
    """A 16-level table for the 4-bit codebook format (input data, like the weights): an exact
    zero, seven negative and eight positive levels placed at evenly spaced quantiles of a
    standard normal distribution (the outermost at the 1/32 tail), scaled to [-1, 1].  It has
    the structure of the published 4-bit NormalFloat table without claiming its digits; the
    library takes any ascending table, so the published one can be passed in its place."""
    from statistics import NormalDist
    inv = NormalDist().inv_cdf
    tail = 1.0 - 1.0 / 32.0
    pos = [inv(0.5 + (tail - 0.5) * i / 8.0) for i in range(1, 9)]
    neg = [-inv(0.5 + (tail - 0.5) * i / 7.0) for i in range(7, 0, -1)]
    lv = np.array(neg + [0.0] + pos, dtype=np.float64)
    return bf16_round((lv / np.max(np.abs(lv))).astype(np.float32))   # levels meet the hidden states in bf16


@dataclass(frozen=True)
class Workload:
    """One of the benchmark / parity configurations."""
    name: str
    shape: SpanShape
    n_sessions: int
    prefix_lens: tuple          # per session
    decode_steps: int
    page_tokens: int = 16
    bf16: bool = True
    seed: int = 0

    @property
    def total_prefix(self) -> int:
        return int(sum(self.prefix_lens))


def _failover_lengths(n: int = 16, lo: int = 128, hi: int = 4096, seed: int = 5) -> tuple:
    rng = np.random.default_rng(seed)
    return tuple(int(v) for v in rng.integers(lo, hi + 1, size=n))


TINY = SpanShape(ARCH_LLAMA, 2, 256, 4, 2, 64, 688)
TINY_BLOOM = SpanShape(ARCH_BLOOM, 2, 256, 4, 4, 64, 1024)
LLAMA_7B = SpanShape(ARCH_LLAMA, 4, 4096, 32, 32, 128, 11008)
LLAMA_70B = SpanShape(ARCH_LLAMA, 8, 8192, 64, 8, 128, 28672)
BLOOM_176B = SpanShape(ARCH_BLOOM, 4, 14336, 112, 112, 128, 57344)

WORKLOADS = {
    "tiny": Workload("tiny", TINY, 1, (16,), 8, bf16=False),
    "tiny_bloom": Workload("tiny_bloom", TINY_BLOOM, 1, (16,), 8, bf16=False),
    "llama7b": Workload("llama7b", LLAMA_7B, 4, (512,) * 4, 128),
    "llama70b": Workload("llama70b", LLAMA_70B, 8, (2048,) * 8, 128),
    "bloom176b": Workload("bloom176b", BLOOM_176B, 16, (128,) * 16, 64),
    "failover70b": Workload("failover70b", LLAMA_70B, 16, _failover_lengths(), 64),
}

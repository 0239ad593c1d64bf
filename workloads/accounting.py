"""Byte / flop / parameter accounting used by the roofline figures.

Pure integer and float bookkeeping (no transformer arithmetic).  The formulas
follow the paper's own weight-streaming arithmetic: one generated token must
touch every parameter once (Section 2.1 and Appendix B), and an attention cache
holds one key and one value vector per layer per past token (Section 3.1).
"""
from __future__ import annotations

from . import SpanShape, ARCH_LLAMA


def params_per_block(s: SpanShape, with_vectors: bool = True) -> int:
    d, qd, kd, f = s.d_model, s.q_dim, s.kv_dim, s.d_ff
    if s.arch == ARCH_LLAMA:
        n = d * qd + 2 * d * kd + qd * d + 3 * d * f
        if with_vectors:
            n += 2 * d
    else:
        n = d * qd + 2 * d * kd + qd * d + 2 * d * f
        if with_vectors:
            n += (qd + 2 * kd) + d + f + d + 4 * d
    return n


def weight_bytes(s: SpanShape, bytes_per_param: float = 2) -> float:
    return s.n_blocks * params_per_block(s) * bytes_per_param


def kv_bytes_per_token_per_block(s: SpanShape, bytes_per_elem: int = 2) -> int:
    return 2 * s.kv_dim * bytes_per_elem


def kv_cache_bytes(n_layers: int, kv_dim: int, n_tokens: int, bytes_per_elem: int = 2) -> int:
    """Keys + values for n_tokens past tokens over n_layers layers."""
    return 2 * n_layers * kv_dim * n_tokens * bytes_per_elem


def activation_bytes(d_model: int, n_tokens: int = 1, bytes_per_elem: int = 2) -> int:
    return d_model * n_tokens * bytes_per_elem


def streaming_seconds(n_bytes: float, bytes_per_second: float) -> float:
    """Time to move n_bytes once over a link / memory system of the given rate."""
    return n_bytes / bytes_per_second


def compressed_weight_bytes(s: SpanShape, bits: int) -> float:
    """Bytes of a span whose projection matrices are stored as `bits`-bit codes plus one fp32
    absmax per 64 input features; vectors (norm gains, biases) stay bf16."""
    mat = params_per_block(s, with_vectors=False)
    vec = params_per_block(s) - mat
    return s.n_blocks * (mat * bits / 8.0 + mat / 64.0 * 4.0 + vec * 2.0)


def decode_step_bytes(s: SpanShape, past_lens, weight_bits: int = 16) -> float:
    """Algorithmic bytes of one decode step: every weight once + every cached K/V once."""
    wb = weight_bytes(s) if weight_bits == 16 else compressed_weight_bytes(s, weight_bits)
    return wb + sum(int(l) for l in past_lens) * kv_bytes_per_token_per_block(s) * s.n_blocks


def prefill_flops(s: SpanShape, new_lens, past_lens=None) -> float:
    """Algorithmic flops of a prefill: 2 flop per parameter per token + causal attention."""
    past_lens = past_lens or [0] * len(new_lens)
    total = 2.0 * s.n_blocks * params_per_block(s, with_vectors=False) * sum(int(t) for t in new_lens)
    for t, l in zip(new_lens, past_lens):
        # QK^T and PV, 2 flop per MAC, causal half of T x T plus the full T x L past rectangle
        total += s.n_blocks * s.n_q_heads * s.head_dim * (2.0 * t * t + 4.0 * t * l)
    return total

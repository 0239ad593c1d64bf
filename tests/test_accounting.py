"""Accounting functions against the closed-form figures the paper prints."""
import math

from workloads import BLOOM_176B, LLAMA_70B, LLAMA_7B, TINY, WORKLOADS
from workloads import accounting as acc


def test_kv_cache_gpt3_sized_sequence():
    # Section 2.1: 96 layers x 12288 units, 2048 tokens, half precision -> 9.6 GB per sequence
    b = acc.kv_cache_bytes(n_layers=96, kv_dim=12288, n_tokens=2048, bytes_per_elem=2)
    assert b == 2 * 96 * 12288 * 2048 * 2
    assert abs(b / 1e9 - 9.6) < 0.1


def test_one_token_activation_is_24_kib():
    # Section 3.2 footnote: one 12288-dim token in 16-bit precision = 24 KiB
    assert acc.activation_bytes(12288, 1, 2) == 24 * 1024


def test_offloading_streaming_times():
    # Section 2.1 + footnote: 175B params in 16 bit over PCIe 4 at 31.5 GB/s -> ~11 s per token
    assert abs(acc.streaming_seconds(175e9 * 2, 31.5e9) - 11.1) < 0.1
    # Appendix B: 176 GB (8-bit) over 256 Gbit/s -> 5.5 s -> 0.18 tokens/s
    t = acc.streaming_seconds(176e9, 256e9 / 8)
    assert abs(t - 5.5) < 0.01 and abs(1 / t - 0.18) < 0.005


def test_bloom_176b_parameter_count():
    # Section 4.2 / Appendix G: 70 blocks, hidden 14336, vocab 250880, embeddings < 3 %
    per_block = acc.params_per_block(BLOOM_176B)
    assert per_block == 2_466_437_120
    total_blocks = 70 * per_block
    emb = 250880 * 14336
    assert abs((total_blocks + emb) / 1e9 - 176.2) < 0.2
    assert emb / (total_blocks + emb) < 0.03


def test_block_parameter_counts():
    assert acc.params_per_block(LLAMA_70B) == 855_654_400
    assert acc.params_per_block(LLAMA_7B) == 202_383_360
    assert acc.params_per_block(TINY) == 725_504


def test_decode_bytes_and_prefill_flops_llama70b():
    wl = WORKLOADS["llama70b"]
    assert acc.kv_bytes_per_token_per_block(wl.shape) == 4096
    b = acc.decode_step_bytes(wl.shape, [2048] * 8)
    assert abs(b / 1e9 - (13.690 + 0.537)) < 0.01
    f = acc.prefill_flops(wl.shape, [2048] * 8)
    assert abs(f / 1e12 - 228.7) < 0.5


def test_failover_lengths_are_seeded_and_in_range():
    lens = WORKLOADS["failover70b"].prefix_lens
    assert len(lens) == 16 and all(128 <= l <= 4096 for l in lens)
    assert lens == WORKLOADS["failover70b"].prefix_lens

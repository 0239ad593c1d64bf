"""Kernel-level parity: projection kernels and decode attention against the oracle's
textbook definitions on seeded inputs, through the C ABI."""
import numpy as np
import pytest
import torch

from gpu_util import *  # noqa: F401,F403

pytestmark = pytest.mark.gpu


def _linear_case(M, N, K, path, seed):
    rng = np.random.default_rng([seed, M, N, K])
    x = bf16_round(rng.standard_normal((M, K), dtype=np.float32))
    w = bf16_round(0.02 * rng.standard_normal((N, K), dtype=np.float32))
    xd, wd = dev_bf16(x), dev_bf16(w)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    scratch = torch.empty(B.span_op_linear_scratch(M, N, K), dtype=torch.uint8, device=DEV)
    B.span_op_linear(xd, wd, y, M, N, K, path, scratch, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    ref = so.linear(x, w)                      # fp64 x W^T
    return row_rel_err(to_np(y), ref)


@pytest.mark.parametrize("M,N,K", [(1, 32, 64), (8, 512, 256), (16, 1376, 256), (5, 256, 688), (13, 48, 8),
                                   (40, 1024, 512), (64, 256, 2048), (8, 8192, 8192), (8, 1024, 28672),
                                   (8, 10240, 8192), (20, 10752, 1024), (64, 12320, 96), (3, 9600, 2048)])
def test_skinny_linear_matches_textbook(M, N, K):
    # fp32 accumulation of exact bf16 products: error ~ sqrt(K) * 2^-24 relative.  The last
    # shapes have pair counts that are no multiple of the CU count, so neighbouring
    # workgroups share tile pairs and combine their pieces through memory.
    assert _linear_case(M, N, K, 0, 11) < 2e-5


def test_skinny_linear_shared_pairs_are_repeatable():
    # the combination order of shared pairs is fixed, and the pair counters return to zero:
    # repeated launches on the same scratch give the same bits
    M, N, K = 24, 10240, 4096
    rng = np.random.default_rng(5)
    x = bf16_round(rng.standard_normal((M, K), dtype=np.float32))
    w = bf16_round(0.02 * rng.standard_normal((N, K), dtype=np.float32))
    xd, wd = dev_bf16(x), dev_bf16(w)
    scratch = torch.empty(B.span_op_linear_scratch(M, N, K), dtype=torch.uint8, device=DEV)
    st = torch.cuda.current_stream().cuda_stream
    outs = []
    for _ in range(4):
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        B.span_op_linear(xd, wd, y, M, N, K, 0, scratch, st)
        torch.cuda.synchronize()
        outs.append(to_np(y))
    assert row_rel_err(outs[0], so.linear(x, w)) < 2e-5
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])


@pytest.mark.parametrize("M,N,K", [(1, 32, 64), (70, 512, 256), (300, 1376, 256), (257, 256, 688), (1100, 784, 320),
                                   (2048, 4096, 4096), (1300, 10240, 1024), (1000, 65552, 128),
                                   # weight rows cut into 256-row tiles and narrower ones (192, 128 and 64 rows)
                                   (2048, 14336, 256), (2048, 12288, 128), (2048, 43008, 64), (2048, 10240, 96),
                                   (1900, 14080, 160),           # ... whose last 192-row tile holds 128 rows of the matrix
                                   (2048, 4096, 512), (700, 2048, 256)])   # less than one round of 256-row tiles: 128- and 64-row tiles only
def test_tiled_linear_matches_textbook(M, N, K):
    assert _linear_case(M, N, K, 1, 12) < 2e-5


@pytest.mark.parametrize("Hq,Hkv,hd,alibi,lens", [
    (8, 2, 128, 0, [1, 17, 300, 32, 33]),
    (4, 4, 64, 1, [5, 64, 129]),
    (64, 8, 128, 0, [2048, 2175, 1]),
    (16, 1, 128, 1, [700]),
])
def test_decode_attention_logits_and_output(Hq, Hkv, hd, alibi, lens):
    Bn, L = len(lens), max(lens)
    rng = np.random.default_rng([21, Hq, Hkv, hd, L])
    q = bf16_round(1.8 * rng.standard_normal((Bn, Hq, hd), dtype=np.float32))
    k = bf16_round(1.8 * rng.standard_normal((Bn, L, Hkv, hd), dtype=np.float32))
    v = bf16_round(1.8 * rng.standard_normal((Bn, L, Hkv, hd), dtype=np.float32))
    out = torch.full((Bn, Hq, hd), float("nan"), dtype=torch.float32, device=DEV)
    logits = torch.full((Bn, Hq, L), float("nan"), dtype=torch.float32, device=DEV)
    scratch = torch.empty(B.span_op_attn_decode_scratch(Bn, L, Hq, Hkv, hd), dtype=torch.uint8, device=DEV)
    B.span_op_attn_decode(dev_bf16(q), dev_bf16(k), dev_bf16(v), lens, Bn, L, Hq, Hkv, hd, alibi, out, logits,
                          scratch, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    out_np, logit_np = to_np(out), to_np(logits)
    slopes = so.alibi_slopes(Hq) if alibi else None
    G = Hq // Hkv
    worst_logit = worst_out = 0.0
    for b, n in enumerate(lens):
        ref = so.attention_with_cache(q[b:b + 1].astype(np.float64), k[b, :n].astype(np.float64),
                                      v[b, :n].astype(np.float64), n - 1, slopes)
        worst_out = max(worst_out, row_rel_err(out_np[b], ref[0]))
        for h in range(Hq):
            s_ref = so.attention_logits(q[b, h], k[b, :n, h // G], hd, slopes[h] if alibi else 0.0, n - 1)
            err = np.max(np.abs(logit_np[b, h, :n] - s_ref)) / (np.max(np.abs(s_ref)) + 1e-30)
            worst_logit = max(worst_logit, float(err))
    assert worst_logit < LOGIT_TOL, worst_logit
    # probabilities are rounded to bf16 before the P.V product: 2^-9 relative per term
    assert worst_out < 5e-3, worst_out


# ----------------------------------------------------------------------------- compressed weights

from oracle import lowbit_oracle as lo
from workloads import normal_levels16

LEVELS = normal_levels16()


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("N,K", [(16, 64), (48, 256), (1376, 688), (8192, 1024), (272, 8192)])
def test_weight_encoder_codes_are_bit_exact(bits, N, K):
    """Integer work: codes and block maxima must equal the oracle's bit for bit (both sides take
    the rounding decisions in fp32 with the same operations)."""
    rng = np.random.default_rng([21, N, K])
    w = bf16_round(0.02 * rng.standard_normal((N, K), dtype=np.float32))
    w[0, :64] = 0.0                                               # an all-zero block
    w[N // 2, K - 1] = 0.5                                        # a block dominated by one element
    wd = dev_bf16(w)
    codes = torch.full((N, K), 99, dtype=torch.uint8, device=DEV)
    absmax = torch.full((N, (K + 63) // 64), float("nan"), dtype=torch.float32, device=DEV)
    scratch = torch.empty(B.span_op_lowbit_scratch(1, N, K), dtype=torch.uint8, device=DEV)
    B.span_op_quantize(wd, N, K, bits, LEVELS, codes, absmax, scratch, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    if bits == 8:
        ref_c, ref_a = lo.quantize_int8(w)
        ref_c = ref_c.view(np.uint8)
    else:
        ref_c, ref_a = lo.quantize_codebook(w, LEVELS)
    assert np.array_equal(absmax.cpu().numpy(), ref_a)
    assert np.array_equal(codes.cpu().numpy(), ref_c)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,N,K", [(1, 32, 64), (8, 512, 256), (16, 1376, 688), (40, 1024, 512), (64, 256, 2048),
                                   (8, 10240, 8192), (3, 9600, 2048)])
def test_lowbit_linear_matches_dequantised_textbook(bits, M, N, K):
    rng = np.random.default_rng([22, M, N, K])
    x = bf16_round(rng.standard_normal((M, K), dtype=np.float32))
    w = bf16_round(0.02 * rng.standard_normal((N, K), dtype=np.float32))
    xd, wd = dev_bf16(x), dev_bf16(w)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    scratch = torch.empty(B.span_op_lowbit_scratch(M, N, K), dtype=torch.uint8, device=DEV)
    B.span_op_linear_lowbit(xd, wd, y, M, N, K, bits, LEVELS, scratch, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    if bits == 8:
        wq = lo.dequantize_int8(*lo.quantize_int8(w))
    else:
        c, a = lo.quantize_codebook(w, LEVELS)
        wq = lo.dequantize_codebook(c, a, LEVELS)
    # exact products, fp32 accumulation inside a block, one fp32 multiply-add per block
    assert row_rel_err(to_np(y), so.linear(x, wq)) < 2e-5


# ----------------------------------------------------------------------------- hidden states on the wire

from workloads import dynamic_levels256

DYN = dynamic_levels256()


@pytest.mark.parametrize("f32_io", [True, False])
@pytest.mark.parametrize("M,d,block", [(1, 64, 64), (8, 8192, 64), (5, 700, 128), (33, 14336, 4096), (2048, 256, 64)])
def test_hidden_codec_codes_bit_exact_and_roundtrip(M, d, block, f32_io):
    """Section 3.1, "Compression": hidden states are block-quantised to 8 bits between stages.
    Codes and block maxima equal the oracle's bit for bit; decoding gives the oracle's values."""
    rng = np.random.default_rng([31, M, d, block])
    x = (rng.standard_normal((M, d)) * rng.choice([0.1, 1.0, 30.0], size=(M, 1))).astype(np.float32)
    if d >= 128:
        x[0, 64:128] = 0.0
    if not f32_io:
        x = bf16_round(x)
    xd = torch.from_numpy(x).to(DEV) if f32_io else dev_bf16(x)
    nb = (d + block - 1) // block
    codes = torch.full((M, d), 77, dtype=torch.uint8, device=DEV)
    absmax = torch.full((M, nb), float("nan"), dtype=torch.float32, device=DEV)
    st = torch.cuda.current_stream().cuda_stream
    B.span_hidden_encode(xd, int(f32_io), M, d, block, DYN, codes, absmax, st)
    y = torch.full((M, d), float("nan"), dtype=torch.float32 if f32_io else torch.bfloat16, device=DEV)
    B.span_hidden_decode(codes, absmax, M, d, block, DYN, int(f32_io), y, st)
    torch.cuda.synchronize()
    ref_c, ref_a = lo.encode_hidden(x, DYN, block)
    assert np.array_equal(absmax.cpu().numpy(), ref_a)
    assert np.array_equal(codes.cpu().numpy(), ref_c)
    ref_y = lo.decode_hidden(ref_c, ref_a, DYN, block)
    got = to_np(y)
    tol = 1e-6 if f32_io else 2.0 ** -8
    assert np.max(np.abs(got - ref_y) / (np.abs(ref_y) + 1e-30)) <= tol
    # the codec's own error on these rows: about a percent
    assert np.linalg.norm(ref_y - x) / np.linalg.norm(x) < 0.03

"""Oracle pieces against library routines (torch CPU ops and, when importable, the
transformers library's own Llama / BLOOM block modules with our weights loaded).

These are independent implementations of the textbook operators the oracle spells
out, so they pin the conventions listed in the oracle's header (half-split rotary,
grouped heads, tanh GELU, ALiBi slopes incl. the 112-head extension, residual
placement).  They run on CPU in fp64.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import span_oracle as so
from workloads import SpanShape, SpanWeights, TINY, TINY_BLOOM, draw_hidden

torch.set_grad_enabled(False)


def t64(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def test_norms_and_activations_match_torch():
    rng = np.random.default_rng(0)
    x, g, b = rng.standard_normal((5, 48)), rng.standard_normal(48), rng.standard_normal(48)
    assert np.allclose(so.layer_norm(x, g, b, 1e-5), F.layer_norm(t64(x), (48,), t64(g), t64(b), 1e-5).numpy(), atol=1e-12)
    assert np.allclose(so.rms_norm(x, g, 1e-5), F.rms_norm(t64(x), (48,), t64(g), 1e-5).numpy(), atol=1e-12)
    z = rng.standard_normal(100) * 3
    assert np.allclose(so.silu(z), F.silu(t64(z)).numpy(), atol=1e-14)
    assert np.allclose(so.gelu_tanh(z), F.gelu(t64(z), approximate="tanh").numpy(), atol=1e-14)


@pytest.mark.parametrize("n_past", [0, 5])
def test_attention_matches_torch_sdpa(n_past):
    rng = np.random.default_rng(1)
    T, Hq, Hkv, hd = 7, 4, 2, 16
    q = rng.standard_normal((T, Hq, hd))
    k = rng.standard_normal((n_past + T, Hkv, hd))
    v = rng.standard_normal((n_past + T, Hkv, hd))
    ours = so.attention_with_cache(q, k, v, n_past)
    kk = t64(k).repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)[None]
    vv = t64(v).repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)[None]
    qq = t64(q).permute(1, 0, 2)[None]
    mask = torch.arange(n_past + T)[None, :] <= (n_past + torch.arange(T))[:, None]
    ref = F.scaled_dot_product_attention(qq, kk, vv, attn_mask=mask)[0].permute(1, 0, 2).numpy()
    assert np.allclose(ours, ref, atol=1e-12)
    assert np.allclose(so.attention_full_masked(q, k, v, None, n_past), ref, atol=1e-12)


def _hf():
    return pytest.importorskip("transformers")


def test_llama_block_matches_transformers_module():
    _hf()
    from transformers.models.llama.modeling_llama import LlamaConfig, LlamaDecoderLayer, LlamaRotaryEmbedding
    s = TINY
    cfg = LlamaConfig(hidden_size=s.d_model, intermediate_size=s.d_ff, num_attention_heads=s.n_q_heads,
                      num_key_value_heads=s.n_kv_heads, head_dim=s.head_dim, rms_norm_eps=s.norm_eps,
                      rope_theta=s.rope_base, num_hidden_layers=1, vocab_size=8, attention_bias=False,
                      mlp_bias=False, hidden_act="silu", max_position_embeddings=64)
    cfg._attn_implementation = "eager"
    layer = LlamaDecoderLayer(cfg, 0).double().eval()
    w = SpanWeights(s, seed=3, bf16=False)[0]
    sd = {"input_layernorm.weight": w["norm1_g"], "self_attn.q_proj.weight": w["wq"],
          "self_attn.k_proj.weight": w["wk"], "self_attn.v_proj.weight": w["wv"],
          "self_attn.o_proj.weight": w["wo"], "post_attention_layernorm.weight": w["norm2_g"],
          "mlp.gate_proj.weight": w["w_gate"], "mlp.up_proj.weight": w["w_up"], "mlp.down_proj.weight": w["w_down"]}
    layer.load_state_dict({k: t64(v) for k, v in sd.items()}, strict=True)
    N = 11
    x = draw_hidden(s, 3, 0, N, bf16=False).astype(np.float64)
    pos = torch.arange(N)[None]
    cos, sin = LlamaRotaryEmbedding(cfg)(t64(x)[None], pos)
    mask = torch.full((N, N), -float("inf"), dtype=torch.float64).triu(1)[None, None]
    out = layer(t64(x)[None], attention_mask=mask, position_ids=pos,
                position_embeddings=(cos.double(), sin.double()))
    out = out[0] if isinstance(out, tuple) else out
    ref = out[0].numpy() if out.dim() == 3 else out.numpy()
    e = np.zeros((0, s.n_kv_heads, s.head_dim))
    ours = so.block_forward(s, w, x, e, e)[0]
    # HF builds cos/sin in fp32, so agreement is to fp32 rounding of the angles
    assert np.max(np.abs(ours - ref)) / np.sqrt(np.mean(ref ** 2)) < 1e-5
    # and the cached path: prefix 6 then 5 single steps
    sess = so.Session(s.with_blocks(1), [w])
    inc = np.concatenate([sess.forward(x[:6])] + [sess.forward(x[i:i + 1]) for i in range(6, N)])
    assert np.max(np.abs(inc - ref)) / np.sqrt(np.mean(ref ** 2)) < 1e-5


@pytest.mark.parametrize("n_heads", [4, 7])     # 7 exercises the non-power-of-two slope rule
def test_bloom_block_matches_transformers_module(n_heads):
    _hf()
    from transformers.models.bloom.modeling_bloom import BloomBlock, BloomConfig, build_alibi_tensor
    hd = 64
    s = SpanShape("bloom", 1, n_heads * hd, n_heads, n_heads, hd, 4 * n_heads * hd)
    cfg = BloomConfig(hidden_size=s.d_model, n_head=n_heads, n_layer=1, layer_norm_epsilon=s.norm_eps,
                      hidden_dropout=0.0, attention_dropout=0.0, vocab_size=8,
                      apply_residual_connection_post_layernorm=False, pretraining_tp=1, slow_but_exact=False)
    cfg._attn_implementation = "eager"
    block = BloomBlock(cfg, 0).double().eval()
    w = SpanWeights(s, seed=4, bf16=False)[0]
    # the library stores q,k,v interleaved per head: rows ordered [head][q|k|v][head_dim]
    def fuse(q, k, v):
        parts = [np.stack([q.reshape(n_heads, hd, -1)[h], k.reshape(n_heads, hd, -1)[h], v.reshape(n_heads, hd, -1)[h]])
                 for h in range(n_heads)]
        return np.concatenate([p.reshape(3 * hd, -1) for p in parts])
    wqkv = fuse(w["wq"], w["wk"], w["wv"])
    bqkv = fuse(w["bq"][:, None], w["bk"][:, None], w["bv"][:, None])[:, 0]
    sd = {"input_layernorm.weight": w["norm1_g"], "input_layernorm.bias": w["norm1_b"],
          "self_attention.query_key_value.weight": wqkv, "self_attention.query_key_value.bias": bqkv,
          "self_attention.dense.weight": w["wo"], "self_attention.dense.bias": w["bo"],
          "post_attention_layernorm.weight": w["norm2_g"], "post_attention_layernorm.bias": w["norm2_b"],
          "mlp.dense_h_to_4h.weight": w["w_up"], "mlp.dense_h_to_4h.bias": w["b_up"],
          "mlp.dense_4h_to_h.weight": w["w_down"], "mlp.dense_4h_to_h.bias": w["b_down"]}
    block.load_state_dict({k: t64(v) for k, v in sd.items()}, strict=True)
    N = 9
    x = draw_hidden(s, 4, 0, N, bf16=False).astype(np.float64)
    alibi = build_alibi_tensor(torch.ones(1, N), n_heads, torch.float64)
    # library slopes == oracle slopes
    assert np.allclose(alibi.reshape(n_heads, N)[:, 1].numpy(), so.alibi_slopes(n_heads), rtol=1e-6)
    causal = torch.full((N, N), -float("inf"), dtype=torch.float64).triu(1)[None, None]
    out = block(t64(x)[None], alibi=alibi, attention_mask=causal)
    out = out[0] if isinstance(out, tuple) else out
    ref = out[0].numpy() if out.dim() == 3 else out.numpy()
    e = np.zeros((0, n_heads, hd))
    ours = so.block_forward(s, w, x, e, e)[0]
    assert np.max(np.abs(ours - ref)) / np.sqrt(np.mean(ref ** 2)) < 1e-5

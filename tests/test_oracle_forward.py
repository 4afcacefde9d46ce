"""Pins for the oracle's decoder forward.

The paper leaves the target model a black box; the oracle's arithmetic is the
standard pre-norm rotary GQA SwiGLU decoder.  It is pinned against closed
forms, structural properties, torch's scaled_dot_product_attention, and --
end to end -- the Hugging Face Llama implementation evaluated in fp64 on a
tiny randomly initialised model with a pre-filled KV cache.
"""
import math

import numpy as np
import pytest
import torch

import synth
from oracle import fly_oracle as O
from tests import helpers

F64 = torch.float64


def test_round_to_bf16_matches_definition_and_torch():
    # hand values: 1 + 2^-8 is a tie -> even mantissa (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    x = torch.tensor([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20,
                      -2.5, 3.0e38 * 0 + 65504.0, 1e-3], dtype=F64)
    r = O.round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2 ** -6 and r[3] == 1.0 + 2 ** -7
    g = torch.Generator().manual_seed(0)
    y = torch.randn(100000, generator=g, dtype=F64) * 10
    ref = y.to(torch.float32).to(torch.bfloat16).to(F64)   # library conversion
    assert torch.equal(O.round_to_bf16(y), ref)


def test_rmsnorm_closed_forms():
    x = torch.full((3, 8), 2.0, dtype=F64)
    g = torch.arange(8, dtype=F64)
    y = O.rmsnorm(x, g, 0.0)
    assert torch.allclose(y, g.expand(3, 8))            # constant vector -> gain itself
    x = torch.randn(4, 64, dtype=F64)
    y = O.rmsnorm(x, torch.ones(64, dtype=F64), 0.0)
    assert torch.allclose((y * y).mean(-1), torch.ones(4, dtype=F64))
    assert torch.allclose(O.rmsnorm(3 * x, torch.ones(64, dtype=F64), 0.0), y)
    # eps enters under the square root, added to the mean square
    x = torch.zeros(1, 4, dtype=F64); x[0, 0] = 2.0     # mean square = 1
    assert abs(O.rmsnorm(x, torch.ones(4, dtype=F64), 3.0)[0, 0].item() - 1.0) < 1e-15


def test_silu():
    x = torch.tensor([0.0, 1.0, -1.0, 30.0], dtype=F64)
    y = O.silu(x)
    assert y[0] == 0.0
    assert abs(y[1].item() - 1 / (1 + math.exp(-1))) < 1e-15
    assert abs(y[2].item() + 1 / (1 + math.exp(1))) < 1e-15
    assert abs(y[3].item() - 30.0) < 1e-10


def test_rope_properties():
    hd, th = 64, 500000.0
    x = torch.randn(5, 3, hd, dtype=F64)
    c0, s0 = O.rope_tables(torch.zeros(5, dtype=torch.int64), hd, th)
    assert torch.equal(O.apply_rope(x, c0, s0), x)                     # position 0 = identity
    pos = torch.tensor([0, 1, 17, 4096, 32768])
    c, s = O.rope_tables(pos, hd, th)
    y = O.apply_rope(x, c, s)
    assert torch.allclose(y.norm(dim=-1), x.norm(dim=-1))              # a rotation
    # frequency i is theta^(-2i/hd): pair (0, hd/2) turns by exactly `pos` radians
    assert abs(c[1, 0].item() - math.cos(1.0)) < 1e-15
    assert abs(s[2, 0].item() - math.sin(17.0)) < 1e-15
    assert abs(c[2, hd // 2 - 1].item() - math.cos(17.0 * th ** (-(hd - 2) / hd))) < 1e-15
    # direction of rotation: (1, 0) in pair (0, hd/2) at angle a -> (cos a, sin a)
    e = torch.zeros(1, 1, hd, dtype=F64); e[0, 0, 0] = 1.0
    c1, s1 = O.rope_tables(torch.tensor([1]), hd, th)
    r = O.apply_rope(e, c1, s1)
    assert abs(r[0, 0, 0].item() - math.cos(1.0)) < 1e-15
    assert abs(r[0, 0, hd // 2].item() - math.sin(1.0)) < 1e-15
    # relative-position property: <rope(q, m), rope(k, n)> depends on m - n only
    q = torch.randn(1, 1, hd, dtype=F64); k = torch.randn(1, 1, hd, dtype=F64)

    def dot(m, n):
        cm, sm = O.rope_tables(torch.tensor([m]), hd, th)
        cn, sn = O.rope_tables(torch.tensor([n]), hd, th)
        return (O.apply_rope(q, cm, sm) * O.apply_rope(k, cn, sn)).sum().item()

    assert abs(dot(10, 3) - dot(1007, 1000)) < 1e-9
    assert abs(dot(10, 3) - dot(3, 10)) > 1e-6


def test_attention_closed_forms():
    num = O.Numerics("f32")
    hd = 16
    # one visible key: the output is that key's value
    q = torch.randn(1, 2, hd, dtype=F64)
    k = torch.randn(1, 1, hd, dtype=F64); v = torch.randn(1, 1, hd, dtype=F64)
    o = O.attention_one_sequence(q, k, v, 0, num)
    assert torch.allclose(o[0, 0], v[0, 0]) and torch.allclose(o[0, 1], v[0, 0])
    # all keys equal: the output is the mean of the visible values
    T = 9
    k = torch.ones(T, 1, hd, dtype=F64); v = torch.randn(T, 1, hd, dtype=F64)
    q = torch.randn(3, 2, hd, dtype=F64)
    o = O.attention_one_sequence(q, k, v, T - 3, num)
    for i in range(3):
        assert torch.allclose(o[i, 0], v[: T - 3 + i + 1, 0].mean(0))


def test_attention_against_torch_sdpa_with_gqa_and_prefix():
    torch.manual_seed(0)
    R, Hq, Hkv, hd, L = 5, 6, 2, 32, 11
    q = torch.randn(R, Hq, hd, dtype=F64)
    k = torch.randn(L + R, Hkv, hd, dtype=F64)
    v = torch.randn(L + R, Hkv, hd, dtype=F64)
    o = O.attention_one_sequence(q, k, v, L, O.Numerics("f32"))
    G = Hq // Hkv
    kk = k.repeat_interleave(G, dim=1).permute(1, 0, 2)[None]       # [1,Hq,T,hd]
    vv = v.repeat_interleave(G, dim=1).permute(1, 0, 2)[None]
    mask = torch.arange(L + R)[None, :] <= (L + torch.arange(R))[:, None]
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.permute(1, 0, 2)[None], kk, vv, attn_mask=mask)[0].permute(1, 0, 2)
    assert torch.allclose(o, ref, atol=1e-12)


TINY = synth.CONFIGS["c1_tiny"].replace(d=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn=48,
                                        vocab=96, kv_len=7, K=4, batch=2, weight_std=0.3)


def _hf_reference(cfg, model, tokens, scale):
    """Logits of the Hugging Face Llama implementation on the same weights."""
    from transformers import LlamaConfig, LlamaForCausalLM
    from transformers.cache_utils import DynamicCache
    hc = LlamaConfig(vocab_size=cfg.vocab, hidden_size=cfg.d, intermediate_size=cfg.ffn,
                     num_hidden_layers=cfg.n_layers, num_attention_heads=cfg.n_q_heads,
                     num_key_value_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                     rms_norm_eps=cfg.rms_eps, rope_theta=cfg.rope_theta,
                     rope_parameters={"rope_type": "default", "rope_theta": cfg.rope_theta},
                     attention_bias=False, mlp_bias=False, tie_word_embeddings=False,
                     max_position_embeddings=4096, attn_implementation="eager")
    hf = LlamaForCausalLM(hc).to(F64).eval()
    sd = {"model.embed_tokens.weight": model["embed"], "model.norm.weight": model["g_final"],
          "lm_head.weight": model["w_lm"].T.contiguous()}
    for i, w in enumerate(model["layers"]):
        p = f"model.layers.{i}."
        sd.update({p + "self_attn.q_proj.weight": w.wq.T, p + "self_attn.k_proj.weight": w.wk.T,
                   p + "self_attn.v_proj.weight": w.wv.T, p + "self_attn.o_proj.weight": w.wo.T,
                   p + "mlp.gate_proj.weight": w.wg.T, p + "mlp.up_proj.weight": w.wu.T,
                   p + "mlp.down_proj.weight": w.wd.T, p + "input_layernorm.weight": w.g_attn,
                   p + "post_attention_layernorm.weight": w.g_ffn})
    missing, unexpected = hf.load_state_dict({k: v.contiguous() for k, v in sd.items()}, strict=False)
    assert not unexpected and all("rotary" in m or "inv_freq" in m for m in missing), (missing, unexpected)
    B, R = tokens.shape
    L = cfg.kv_len
    cache = DynamicCache(config=hc)
    for li, (k, v) in enumerate(model["kv_prefix"]):
        cache.update(k.permute(0, 2, 1, 3).contiguous(), v.permute(0, 2, 1, 3).contiguous(), li)
    pos = torch.arange(L, L + R)[None].expand(B, R)
    with torch.no_grad():
        out = hf(input_ids=torch.from_numpy(tokens.astype(np.int64)), past_key_values=cache,
                 position_ids=pos, use_cache=True)
    return out.logits.numpy() * scale.reshape(B, R, 1).numpy().astype(np.float64)


def test_full_forward_against_hf_llama_fp64():
    cfg = TINY.replace(rms_eps=1e-2)
    model = helpers.oracle_model(cfg)
    # the workload's norm gains are all ones; use distinct random gains here so
    # that a misplaced or swapped gain would show
    gg = torch.Generator().manual_seed(5)
    model["g_final"] = torch.rand(cfg.d, generator=gg, dtype=F64) + 0.5
    for w in model["layers"]:
        w.g_attn = torch.rand(cfg.d, generator=gg, dtype=F64) + 0.5
        w.g_ffn = torch.rand(cfg.d, generator=gg, dtype=F64) + 0.5
    rng = np.random.default_rng(0)
    tokens = rng.integers(0, cfg.vocab, size=(cfg.batch, cfg.K + 1)).astype(np.int32)
    out = helpers.oracle_verify(cfg, model, tokens, return_logits=True)
    ref = _hf_reference(cfg, model, tokens, helpers.row_scale(cfg))
    assert out["logits"].shape == ref.shape
    # The library builds its rotary tables in float32, so agreement stops near
    # float32 resolution; any structural slip (pairing, sign, head mapping,
    # mask, eps placement with eps = 1e-2) is orders of magnitude larger.
    assert np.abs(out["logits"] - ref).max() < 2e-6 * max(1.0, np.abs(ref).max())
    # and the statistics are those of the logits
    assert np.array_equal(out["argmax"], ref.argmax(-1))


def test_causality_and_sequence_independence():
    cfg = TINY
    model = helpers.oracle_model(cfg)
    rng = np.random.default_rng(1)
    tokens = rng.integers(0, cfg.vocab, size=(cfg.batch, cfg.K + 1)).astype(np.int32)
    a = helpers.oracle_verify(cfg, model, tokens, return_logits=True)["logits"]
    t2 = tokens.copy()
    t2[:, 3:] = (t2[:, 3:] + 1) % cfg.vocab
    b = helpers.oracle_verify(cfg, model, t2, return_logits=True)["logits"]
    assert np.array_equal(a[:, :3], b[:, :3])       # rows before the change are untouched
    assert not np.allclose(a[:, 3:], b[:, 3:])
    t3 = tokens.copy()
    t3[1] = (t3[1] + 5) % cfg.vocab
    c = helpers.oracle_verify(cfg, model, t3, return_logits=True)["logits"]
    assert np.array_equal(a[0], c[0])               # sequences do not interact


def test_bf16_mode_rounds_where_declared():
    cfg = TINY.replace(dtype="bf16", batch=1)
    model = helpers.oracle_model(cfg)
    rng = np.random.default_rng(2)
    tokens = rng.integers(0, cfg.vocab, size=(1, cfg.K + 1)).astype(np.int32)
    out16 = helpers.oracle_verify(cfg, model, tokens, return_logits=True)
    out64 = helpers.oracle_verify(cfg.replace(dtype="f32"), model, tokens, return_logits=True)
    diff = np.abs(out16["logits"] - out64["logits"]).max()
    assert 0 < diff < 0.25 * np.abs(out64["logits"]).max()
    # appended keys and values are bf16-representable in bf16 mode
    k_new, v_new = out16["new_kv"][0][0]
    assert torch.equal(O.round_to_bf16(k_new), k_new) and torch.equal(O.round_to_bf16(v_new), v_new)


def test_draft_chain_and_end_to_end_accept():
    cfg = TINY.replace(batch=3, K=6, logit_gain=4.0, window=2)
    model = helpers.oracle_model(cfg)
    tokens = helpers.draft_chain(cfg, model)
    out = helpers.oracle_verify(cfg, model, tokens)
    u, alt, _ = synth.make_draft_draws(cfg)
    want_match = (u.numpy() < cfg.p_match)
    got_match = tokens[:, 1:] == out["argmax"][:, :-1]
    # chosen matches match; chosen mismatches differ unless the alt token hits the argmax
    assert np.array_equal(got_match | (alt.numpy() == out["argmax"][:, :-1]), want_match | got_match)
    assert np.all(got_match[want_match])
    # the accept outputs are the rule applied to this block's statistics
    ref = O.accept_block(tokens[:, 1:], out["argmax"], out["h"], cfg.theta, cfg.window)
    for k in ("accept_len", "next_token", "n_loose"):
        assert np.array_equal(out[k], ref[k])
    assert np.all(out["h"] >= 0) and np.all(out["h"] <= 1 + 1e-12)

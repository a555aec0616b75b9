"""Pins for the oracle's transformer and verifier (CPU only): textbook special
cases, library routines (torch.nn.functional, Hugging Face GPT-2 / LLaMA modules
with the same weights) and the cached-vs-uncached identity."""
import math
import numpy as np
import pytest
import torch
import workloads as W
from oracle import model as om


def test_norms_have_unit_statistics_and_match_torch():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(5, 48)) * 3 + 1.5
    y = om.layer_norm(x, np.ones(48), np.zeros(48), 0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-12) and np.allclose(y.var(-1), 1, atol=1e-12)
    z = om.rms_norm(x, np.ones(48), 0.0)
    assert np.allclose((z ** 2).mean(-1), 1, atol=1e-12)
    g, b = rng.normal(size=48), rng.normal(size=48)
    ref = torch.nn.functional.layer_norm(torch.tensor(x), (48,), torch.tensor(g), torch.tensor(b), 1e-5)
    assert np.allclose(om.layer_norm(x, g, b, 1e-5), ref.numpy(), atol=1e-12)
    ref = torch.nn.functional.rms_norm(torch.tensor(x), (48,), torch.tensor(g), 1e-5)
    assert np.allclose(om.rms_norm(x, g, 1e-5), ref.numpy(), atol=1e-12)


def test_activations_match_library():
    x = np.linspace(-6, 6, 101)
    assert np.allclose(om.gelu_tanh(x), torch.nn.functional.gelu(torch.tensor(x), approximate="tanh").numpy(), atol=1e-12)
    assert np.allclose(om.silu(x), torch.nn.functional.silu(torch.tensor(x)).numpy(), atol=1e-12)
    assert abs(om.gelu_tanh(np.array([1.0]))[0] - 0.8411919906082768) < 1e-12


def test_attention_special_cases():
    rng = np.random.default_rng(1)
    q = rng.normal(size=(4, 16))
    V1 = rng.normal(size=(1, 2, 16))
    out = om.attend(q, rng.normal(size=(1, 2, 16)), V1)       # one key: returns its value
    assert np.allclose(out[0], V1[0, 0]) and np.allclose(out[3], V1[0, 1])
    K = np.repeat(rng.normal(size=(1, 2, 16)), 7, axis=0)     # equal keys: uniform weights
    V = rng.normal(size=(7, 2, 16))
    out = om.attend(q, K, V)
    assert np.allclose(out[1], V[:, 0].mean(0)) and np.allclose(out[2], V[:, 1].mean(0))
    # against the library routine, MHA
    K, V = rng.normal(size=(9, 4, 16)), rng.normal(size=(9, 4, 16))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.tensor(q)[None, :, None, :], torch.tensor(K).permute(1, 0, 2)[None],
        torch.tensor(V).permute(1, 0, 2)[None])[0, :, 0].numpy()
    assert np.allclose(om.attend(q, K, V), ref, atol=1e-12)
    # GQA equals MHA on repeated KV heads
    K2, V2 = rng.normal(size=(9, 2, 16)), rng.normal(size=(9, 2, 16))
    assert np.allclose(om.attend(q, K2, V2), om.attend(q, np.repeat(K2, 2, 1), np.repeat(V2, 2, 1)))


def test_rope_properties():
    rng = np.random.default_rng(2)
    x, y = rng.normal(size=(3, 64)), rng.normal(size=(3, 64))
    assert np.allclose(om.rope(x, 0, 10000.0), x)
    assert np.allclose(np.linalg.norm(om.rope(x, 37, 10000.0), axis=-1), np.linalg.norm(x, axis=-1))
    # inner products depend on the position difference only
    a = (om.rope(x, 11, 1e4) * om.rope(y, 5, 1e4)).sum(-1)
    b = (om.rope(x, 106, 1e4) * om.rope(y, 100, 1e4)).sum(-1)
    assert np.allclose(a, b, atol=1e-9)
    # explicit 2-D rotation of the pair (i, i + d/2) by pos * theta^(-2i/d)
    i, pos, th = 5, 9, 5e5
    ang = pos * th ** (-2 * i / 64)
    r = om.rope(x[0], pos, th)
    assert math.isclose(r[i], x[0, i] * math.cos(ang) - x[0, i + 32] * math.sin(ang), rel_tol=1e-12)
    assert math.isclose(r[i + 32], x[0, i + 32] * math.cos(ang) + x[0, i] * math.sin(ang), rel_tol=1e-12)


def _hf_gpt2(cfg, w):
    from transformers import GPT2Config, GPT2LMHeadModel
    c = GPT2Config(vocab_size=cfg.vocab, n_positions=cfg.max_pos, n_embd=cfg.d_model, n_layer=cfg.n_layer,
                   n_head=cfg.n_head, n_inner=cfg.d_ff, activation_function="gelu_new",
                   layer_norm_epsilon=cfg.norm_eps, resid_pdrop=0.0, embd_pdrop=0.0, attn_pdrop=0.0,
                   bos_token_id=None, eos_token_id=None)
    m = GPT2LMHeadModel(c).double().eval()
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    sd = {"transformer.wte.weight": t(w["tok_emb"]), "transformer.wpe.weight": t(w["pos_emb"]),
          "transformer.ln_f.weight": t(w["normf.g"]), "transformer.ln_f.bias": t(w["normf.b"]),
          "lm_head.weight": t(w["tok_emb"])}
    for i in range(cfg.n_layer):
        p, h = f"l{i}.", f"transformer.h.{i}."
        sd.update({h + "ln_1.weight": t(w[p + "norm1.g"]), h + "ln_1.bias": t(w[p + "norm1.b"]),
                   h + "attn.c_attn.weight": t(w[p + "wqkv"]).T.contiguous(), h + "attn.c_attn.bias": t(w[p + "bqkv"]),
                   h + "attn.c_proj.weight": t(w[p + "wo"]).T.contiguous(), h + "attn.c_proj.bias": t(w[p + "bo"]),
                   h + "ln_2.weight": t(w[p + "norm2.g"]), h + "ln_2.bias": t(w[p + "norm2.b"]),
                   h + "mlp.c_fc.weight": t(w[p + "w1"]).T.contiguous(), h + "mlp.c_fc.bias": t(w[p + "b1"]),
                   h + "mlp.c_proj.weight": t(w[p + "w2"]).T.contiguous(), h + "mlp.c_proj.bias": t(w[p + "b2"])})
    missing = m.load_state_dict(sd, strict=False)
    assert not [k for k in missing.missing_keys if "attn.bias" not in k and "masked_bias" not in k]
    return m


def _hf_llama(cfg, w):
    from transformers import LlamaConfig, LlamaForCausalLM
    try:
        c = LlamaConfig(vocab_size=cfg.vocab, hidden_size=cfg.d_model, intermediate_size=cfg.d_ff,
                        num_hidden_layers=cfg.n_layer, num_attention_heads=cfg.n_head,
                        num_key_value_heads=cfg.n_kv_head, max_position_embeddings=cfg.max_pos,
                        rms_norm_eps=cfg.norm_eps, rope_theta=cfg.rope_theta, attention_bias=False,
                        tie_word_embeddings=False, hidden_act="silu", head_dim=cfg.d_head)
    except TypeError:
        pytest.skip("LlamaConfig signature differs")
    if getattr(c, "rope_parameters", None) is not None:
        c.rope_parameters["rope_theta"] = cfg.rope_theta
    m = LlamaForCausalLM(c).double().eval()
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    H, KVH, dh = cfg.n_head, cfg.n_kv_head, cfg.d_head
    sd = {"model.embed_tokens.weight": t(w["tok_emb"]), "model.norm.weight": t(w["normf.g"]),
          "lm_head.weight": t(w["lm_head"])}
    for i in range(cfg.n_layer):
        p, h = f"l{i}.", f"model.layers.{i}."
        qkv = w[p + "wqkv"]
        sd.update({h + "self_attn.q_proj.weight": t(qkv[:H * dh]),
                   h + "self_attn.k_proj.weight": t(qkv[H * dh:(H + KVH) * dh]),
                   h + "self_attn.v_proj.weight": t(qkv[(H + KVH) * dh:]),
                   h + "self_attn.o_proj.weight": t(w[p + "wo"]),
                   h + "mlp.gate_proj.weight": t(w[p + "wg"]), h + "mlp.up_proj.weight": t(w[p + "wu"]),
                   h + "mlp.down_proj.weight": t(w[p + "w2"]),
                   h + "input_layernorm.weight": t(w[p + "norm1.g"]),
                   h + "post_attention_layernorm.weight": t(w[p + "norm2.g"])})
    missing = m.load_state_dict(sd, strict=False)
    assert not [k for k in missing.missing_keys if "rotary" not in k]
    return m


@pytest.mark.parametrize("theta", [10000.0, 500000.0])
def test_llama_matches_library_module(theta):
    cfg = W.ModelCfg(W.ARCH_LLAMA, 2, 64, 4, 2, 96, 83, 64, 1e-5, theta)
    w = {k: v * 5 if v.ndim == 2 else v for k, v in W.make_model_weights(cfg, 3, False).items()}
    tokens = np.random.default_rng(0).integers(0, cfg.vocab, size=13)
    hf, logits = om.Decoder(cfg, w).forward_full(tokens)
    m = _hf_llama(cfg, w)
    with torch.no_grad():
        out = m(torch.tensor(tokens)[None], output_hidden_states=True)
    # the library keeps its rotary cos/sin tables in float32, hence 5e-6 and not 1e-10
    assert np.abs(out.logits[0].numpy() - logits).max() < 5e-6
    assert np.abs(out.hidden_states[-1][0].numpy() - hf).max() < 5e-6   # post-norm final state


def test_gpt_matches_library_module():
    cfg = W.ModelCfg(W.ARCH_GPT, 2, 48, 3, 3, 80, 71, 32)
    w = {k: v * 5 if v.ndim == 2 else v for k, v in W.make_model_weights(cfg, 4, False).items()}
    tokens = np.random.default_rng(1).integers(0, cfg.vocab, size=11)
    hf, logits = om.Decoder(cfg, w).forward_full(tokens)
    m = _hf_gpt2(cfg, w)
    with torch.no_grad():
        out = m(torch.tensor(tokens)[None], output_hidden_states=True)
    assert np.abs(out.logits[0].numpy() - logits).max() < 1e-10
    assert np.abs(out.hidden_states[-1][0].numpy() - hf).max() < 1e-10


@pytest.mark.parametrize("kind", ["gpt", "llama"])
def test_cached_route_equals_uncached_route(kind):
    cfg = W.mini_config(kind, W.DT_F32)
    for mc, seed in ((cfg.draft, 1), (cfg.target, 2)):
        w = W.make_model_weights(mc, seed, False)
        dec = om.Decoder(mc, w)
        rng = np.random.default_rng(seed)
        tokens = rng.integers(0, mc.vocab, size=10)
        # contiguous positions, then positions with gaps (a target cache in the own-history reading)
        for pos in (np.arange(10), np.array([0, 1, 2, 5, 6, 9, 13, 14, 20, 31])):
            hf_full, lg_full = dec.forward_full(tokens, pos)
            cache = dec.new_cache()
            for j in range(10):
                hf, lg = dec.step([tokens[j]], [pos[j]], [cache])
                assert np.abs(hf[0] - hf_full[j]).max() < 1e-9
                assert np.abs(lg[0] - lg_full[j]).max() < 1e-9
            assert cache.positions == list(pos) and len(cache.K[0]) == 10
        # rows in one step call do not interact
        c1, c2 = dec.new_cache(), dec.new_cache()
        a, _ = dec.step([tokens[0], tokens[1]], [0, 0], [c1, c2])
        b, _ = dec.step([tokens[1]], [0], [dec.new_cache()])
        assert np.abs(a[1] - b[0]).max() < 1e-12


def test_verifier_definition():
    rng = np.random.default_rng(3)
    w = W.make_verifier_weights(16, 8, 5)
    w = {k: v * 30 for k, v in w.items()}
    hf = rng.normal(size=(4, 16))
    v = om.Verifier(w)
    for r in range(4):                                   # scalar re-evaluation
        z = float(w["v.b2"][0])
        for j in range(8):
            a = float(w["v.b1"][j]) + sum(float(w["v.w1"][j, i]) * hf[r, i] for i in range(16))
            z += float(w["v.w2"][j]) * max(a, 0.0)
        assert math.isclose(v(hf)[r], 1 / (1 + math.exp(-z)), rel_tol=1e-6)
    lin = {"v.w2": w["v.w2"][:8].repeat(2), "v.b2": w["v.b2"]}     # single layer (the paper's)
    assert np.allclose(om.Verifier(lin)(hf), 1 / (1 + np.exp(-(hf @ lin["v.w2"] + lin["v.b2"][0]))), atol=1e-7)
    assert om.Verifier(lin)(hf).dtype == np.float32

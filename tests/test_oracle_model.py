"""Pins for the oracle's EE transformer: an independent library model, brute force, caches."""
import numpy as np
import pytest
import torch

import synth
from oracle import ee_oracle as eo


def _small_cfg(**kw):
    base = dict(n_layers=4, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96,
                vocab=61, exit_draft=1, exit_inter=2, rope_theta=10000.0, sigma=0.08)
    base.update(kw)
    return synth.EEConfig(**base)


def _model(cfg, seed=3, round_mode=None):
    W = synth.WeightStore(cfg, seed)
    return eo.EEModel(eo.ModelSpec.from_config(cfg, round_mode), W), W


def _hf_model(cfg, W):
    from transformers import LlamaConfig, LlamaForCausalLM
    hc = LlamaConfig(hidden_size=cfg.d_model, intermediate_size=cfg.d_ffn, num_hidden_layers=cfg.n_layers,
                     num_attention_heads=cfg.n_q_heads, num_key_value_heads=cfg.n_kv_heads,
                     head_dim=cfg.head_dim, rms_norm_eps=cfg.rms_eps, vocab_size=cfg.vocab,
                     tie_word_embeddings=False, attention_bias=False, mlp_bias=False,
                     rope_theta=cfg.rope_theta, max_position_embeddings=512, attn_implementation="eager")
    hf = LlamaForCausalLM(hc).double().eval()
    sd = {"model.embed_tokens.weight": W.get("emb"), "model.norm.weight": W.get("gfinal"),
          "lm_head.weight": W.get("head")}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "wgate": "mlp.gate_proj", "wup": "mlp.up_proj",
             "wdown": "mlp.down_proj", "g1": "input_layernorm", "g2": "post_attention_layernorm"}
    for l in range(cfg.n_layers):
        for k, v in names.items():
            sd[f"model.layers.{l}.{v}.weight"] = W.get(k, l)
    hf.load_state_dict({k: torch.from_numpy(np.asarray(v, np.float64)) for k, v in sd.items()}, strict=True)
    return hf


def test_forward_matches_hf_llama_at_every_exit():
    """The whole architecture (pre-norm, GQA, half-split RoPE, SwiGLU, untied shared head) against
    the transformers library's Llama in float64, at the draft, intermediate and final exits."""
    cfg = _small_cfg()
    m, W = _model(cfg)
    hf = _hf_model(cfg, W)
    toks = synth.gen_prompt(cfg.vocab, 23, 5)
    with torch.no_grad():
        out = hf(torch.from_numpy(toks.astype(np.int64))[None], output_hidden_states=True)
    for L in (cfg.exit_draft, cfg.exit_inter, 3):
        hid, logits = m.forward_nocache(toks, L)
        np.testing.assert_allclose(hid, out.hidden_states[L][0].numpy(), rtol=1e-5, atol=1e-6)
        want = hf.lm_head(hf.model.norm(out.hidden_states[L]))[0].detach().numpy()
        np.testing.assert_allclose(logits, want, rtol=1e-5, atol=1e-6)
    _, logits = m.forward_nocache(toks, cfg.n_layers)
    # (the library evaluates its rotary cos/sin table in float32, hence 1e-6 and not 1e-12)
    np.testing.assert_allclose(logits, out.logits[0].numpy(), rtol=1e-5, atol=1e-6)


def test_hf_greedy_generation_equals_oracle_ar():
    cfg = _small_cfg()
    m, W = _model(cfg)
    hf = _hf_model(cfg, W)
    prompt = synth.gen_prompt(cfg.vocab, 9, 6)
    with torch.no_grad():
        out = hf.generate(torch.from_numpy(prompt.astype(np.int64))[None], max_new_tokens=12, do_sample=False,
                          pad_token_id=0, eos_token_id=None)
    assert eo.ar_generate(m, prompt, 12) == out[0, len(prompt):].tolist()


@pytest.mark.parametrize("round_mode", ["none", "bf16"])
def test_cached_decoding_equals_cacheless_recompute(round_mode):
    cfg = _small_cfg(dtype="bf16" if round_mode == "bf16" else "f32")
    m, _ = _model(cfg, round_mode=round_mode)
    prompt = synth.gen_prompt(cfg.vocab, 7, 1)
    for L in (None, cfg.exit_inter):
        assert eo.ar_generate(m, prompt, 10, L) == eo.ar_generate_nocache(m, prompt, 10, L)
    # block-parallel pass over new rows == the same positions of a from-scratch pass
    toks = synth.gen_prompt(cfg.vocab, 15, 2)
    cache = eo.KVCache(m.spec, 15)
    x1 = m.run_layers(range(3), m.embed(toks[:10]), np.arange(10), cache)
    x2 = m.run_layers(range(3), m.embed(toks[10:]), np.arange(10, 15), cache)
    full, _ = m.forward_nocache(toks, 3)
    tol = 1e-11 if round_mode == "none" else 0.0
    np.testing.assert_allclose(np.concatenate([x1, x2]), full, rtol=tol, atol=tol)


def test_zero_gate_kills_the_ffn_branch_and_zero_wo_kills_attention():
    cfg = _small_cfg()
    m, W = _model(cfg)
    toks = synth.gen_prompt(cfg.vocab, 6, 3)
    for l in range(cfg.n_layers):
        W.override("wgate", l, np.zeros(synth.tensor_shape(cfg, "wgate")))
        W.override("wo", l, np.zeros(synth.tensor_shape(cfg, "wo")))
    hid, _ = m.forward_nocache(toks, cfg.n_layers)
    np.testing.assert_array_equal(hid, m.embed(toks))       # silu(0) = 0: both branches vanish


def test_damping_makes_exits_identical():
    """gamma_3 = 0 zeroes every residual write of G3, so the L_i and L_f hidden states coincide."""
    cfg = _small_cfg(gamma=(1.0, 1.0, 0.0))
    m, _ = _model(cfg)
    toks = synth.gen_prompt(cfg.vocab, 8, 4)
    hi, li = m.forward_nocache(toks, cfg.exit_inter)
    hf_, lf = m.forward_nocache(toks, cfg.n_layers)
    np.testing.assert_array_equal(hi, hf_)
    np.testing.assert_array_equal(li, lf)


# --- auxiliary low-rank exit heads (App. I) -------------------------------------------------------

def _aux_cfg(**kw):
    return _small_cfg(head_rank=8, rms_eps=1e-12, **kw)


def test_low_rank_head_with_zero_up_projection_is_the_shared_head():
    cfg = _aux_cfg()
    m, W = _model(cfg)
    for e in (0, 1):
        W.override("aux_b", e, np.zeros(synth.tensor_shape(cfg, "aux_b")))
    x = np.random.default_rng(0).standard_normal((5, cfg.d_model))
    for e in (0, 1):
        np.testing.assert_array_equal(m.exit_logits(x, e), m.exit_logits(x, 2))


def test_low_rank_head_leaves_the_final_exit_alone_and_changes_the_early_ones():
    cfg = _aux_cfg()
    m, _ = _model(cfg)
    m0, _ = _model(_small_cfg(rms_eps=1e-12))
    x = np.random.default_rng(1).standard_normal((4, cfg.d_model))
    np.testing.assert_array_equal(m.exit_logits(x, 2), m0.exit_logits(x, 2))
    assert np.max(np.abs(m.exit_logits(x, 0) - m0.exit_logits(x, 0))) > 1e-3
    assert np.max(np.abs(m.exit_logits(x, 0) - m.exit_logits(x, 1))) > 1e-3      # each exit has its own adapter


def test_full_rank_identity_adapter_only_rescales_the_hidden_state():
    """A = I, B = c I, unit gain: z = x (1 + c / rms(x)) is a positive multiple of x, which the
    shared RMSNorm removes again, so the logits are those of the shared head."""
    cfg = _small_cfg(head_rank=64, rms_eps=1e-12)
    m, W = _model(cfg)
    d = cfg.d_model
    W.override("aux_g", 0, np.ones(d))
    W.override("aux_a", 0, np.eye(d))
    W.override("aux_b", 0, 0.37 * np.eye(d))
    x = np.random.default_rng(2).standard_normal((6, d))
    np.testing.assert_allclose(m.exit_logits(x, 0), m.exit_logits(x, 2), rtol=1e-9, atol=1e-9)


def test_single_entry_adapter_moves_one_coordinate_by_one_normalised_feature():
    """A = e_i e_j^T, B = e_k e_i^T  =>  z = x + e_k * RMSNorm(x; g)_j: pins which index of each
    factor is the input and which the output."""
    cfg = _aux_cfg()
    m, W = _model(cfg)
    d, r = cfg.d_model, cfg.head_rank
    i, j, k = 5, 17, 40
    A = np.zeros((r, d)); A[i, j] = 1.0
    B = np.zeros((d, r)); B[k, i] = 1.0
    W.override("aux_a", 1, A)
    W.override("aux_b", 1, B)
    x = np.random.default_rng(3).standard_normal((3, d))
    g = np.asarray(W.get("aux_g", 1), np.float64)
    z = x.copy()
    z[:, k] += x[:, j] * g[j] / np.sqrt(np.mean(x * x, axis=1))
    np.testing.assert_allclose(m.exit_logits(x, 1), m.exit_logits(z, 2), rtol=1e-9, atol=1e-9)


def test_low_rank_head_rounds_its_matrix_operands_in_bf16_mode():
    cfg = _small_cfg(head_rank=32, dtype="bf16")
    m, W = _model(cfg)
    x = np.random.default_rng(4).standard_normal((2, cfg.d_model))
    n = eo.round_bf16(eo.rmsnorm(x, np.asarray(W.get("aux_g", 0), np.float64), cfg.rms_eps))
    t = eo.round_bf16(n @ np.asarray(W.get("aux_a", 0), np.float64).T)
    z = x + t @ np.asarray(W.get("aux_b", 0), np.float64).T
    np.testing.assert_array_equal(m.exit_logits(x, 0), m.exit_logits(z, 2))

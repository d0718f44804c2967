"""Pins for the oracle's decoding state machine (Algorithms 1 and 2, Sec. 3.2 cache handling)."""
import itertools

import numpy as np
import pytest

import synth
from oracle import ee_oracle as eo


def _cfg(**kw):
    base = dict(n_layers=5, d_model=48, n_q_heads=4, n_kv_heads=2, head_dim=12, d_ffn=80,
                vocab=97, exit_draft=1, exit_inter=3, rope_theta=10000.0, sigma=0.08,
                gamma=(1.0, 0.15, 0.15))
    base.update(kw)
    return synth.EEConfig(**base)


def _model(cfg, seed=11, round_mode=None):
    return eo.EEModel(eo.ModelSpec.from_config(cfg, round_mode), synth.WeightStore(cfg, seed))


# --- lossless guarantee: HiSpec == greedy AR of the full model ---------------------------------

CASES = [
    # (exit_draft, exit_inter, k, trigger, bonus_inter, bonus_full, gamma)
    (1, 3, 4, dict(every=2), True, True, (1.0, 0.15, 0.15)),
    (1, 3, 4, dict(every=2), False, False, (1.0, 0.15, 0.15)),
    (2, 4, 2, dict(n_i=4), True, True, (1.0, 0.15, 0.15)),       # the paper's default N_d=2, N_i=4
    (2, 4, 2, dict(n_i=4), True, False, (1.0, 0.3, 0.05)),
    (1, 2, 6, dict(n_i=3), False, True, (1.0, 0.05, 0.3)),
    (3, 4, 3, dict(every=1), True, True, (1.0, 1.0, 1.0)),
    (1, 4, 5, dict(every=4), True, True, (1.0, 0.02, 0.02)),
    (1, 3, 1, dict(n_i=1), True, True, (1.0, 0.15, 0.15)),
]


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("round_mode", ["none", "bf16"])
def test_hispec_stream_equals_ar(case, round_mode):
    ld, li, k, trig, bi, bf, gamma = case
    cfg = _cfg(exit_draft=ld, exit_inter=li, gamma=gamma, dtype="bf16" if round_mode == "bf16" else "f32")
    m = _model(cfg, round_mode=round_mode)
    prompt = synth.gen_prompt(cfg.vocab, 11, 100 + k)
    want = eo.ar_generate(m, prompt, 40)
    log = []
    got = eo.HiSpecOracle(m, bi, bf).generate(prompt, 40, k, log=log, **trig)
    assert got == want
    if gamma[1] < 0.5 and k > 1:
        # the damped models must actually exercise partial acceptance, not just a = 0
        assert len({e[1] for e in log if e[0] == "inter"}) >= 2


def test_self_speculative_equals_ar_and_is_hispec_without_the_middle():
    cfg = _cfg()
    m = _model(cfg)
    prompt = synth.gen_prompt(cfg.vocab, 9, 5)
    want = eo.ar_generate(m, prompt, 24)
    log = []
    assert eo.self_speculative_generate(m, prompt, 24, 3, log=log) == want
    assert len({a for a, _ in log}) >= 2
    # gamma_2 = 0 makes L_i == L_d: the intermediate verifier accepts every draft block in full
    cfg0 = _cfg(gamma=(1.0, 0.0, 0.4))
    m0 = _model(cfg0)
    hlog = []
    eo.HiSpecOracle(m0).generate(prompt, 24, 3, every=1, log=hlog)
    assert all(e[1] == 3 for e in hlog if e[0] == "inter")
    # ... and then each macro step is exactly Algorithm 1 on blocks of 3 draft tokens + L_d's bonus,
    # so the committed stream is still the AR stream of that model
    assert eo.HiSpecOracle(m0).generate(prompt, 24, 3, every=1) == eo.ar_generate(m0, prompt, 24)
    # gamma_3 = 0 makes L_f == L_i: full verification accepts the whole tentative buffer
    cfg1 = _cfg(gamma=(1.0, 0.4, 0.0))
    m1 = _model(cfg1)
    flog = []
    eo.HiSpecOracle(m1).generate(prompt, 24, 3, every=2, log=flog)
    fulls = [e for e in flog if e[0] == "full"]
    assert fulls and all(e[1] == len(e[3]) - 1 for e in fulls)


# --- LeadingSubstringVerify through the model ---------------------------------------------------

def _fresh(m, prompt, k=4, **kw):
    o = eo.HiSpecOracle(m, **kw)
    seq = eo.Sequence_(m.spec, len(prompt) + 64)
    o.prefill(seq, prompt)
    return o, seq


@pytest.mark.parametrize("wrong_at", [0, 1, 3, None])
def test_accept_length_follows_first_wrong_token(wrong_at):
    cfg = _cfg()
    m = _model(cfg)
    prompt = synth.gen_prompt(cfg.vocab, 10, 8)
    o, seq = _fresh(m, prompt)
    k = 4
    # the intermediate verifier's own greedy continuation of T (teacher forced), by brute force
    greedy = eo.ar_generate_nocache(m, seq.T, k + 1, cfg.exit_inter)
    S = list(greedy[:k])
    if wrong_at is not None:
        S[wrong_at] = (S[wrong_at] + 1) % cfg.vocab
    o.draft_inject(seq, S)
    a, nxt = o.verify_intermediate(seq)
    if wrong_at is None:
        assert (a, nxt) == (k, greedy[k])                 # everything accepted + bonus token
        assert seq.V == greedy[:k + 1]
    else:
        assert (a, nxt) == (wrong_at, greedy[wrong_at])   # refilled with the verifier's token
        assert seq.V == greedy[:wrong_at + 1]


def test_block_verify_equals_token_by_token_verify():
    """v_j from the single block-parallel pass == v_j from feeding x||S_{1:j-1} one prefix at a time."""
    cfg = _cfg()
    m = _model(cfg)
    prompt = synth.gen_prompt(cfg.vocab, 10, 9)
    o, seq = _fresh(m, prompt)
    S = o.draft(seq, 5)
    T = list(seq.T)
    o.verify_intermediate(seq)
    v_block = eo.argmax_rows(o.last_logits)
    for j in range(6):
        _, lg = m.forward_nocache(T + S[:j], cfg.exit_inter)
        assert int(eo.argmax_rows(lg[-1:])[0]) == int(v_block[j])
        np.testing.assert_allclose(o.last_logits[j], lg[-1], rtol=1e-9, atol=1e-11)


def test_sequential_draft_equals_block_inject():
    cfg = _cfg()
    m = _model(cfg)
    prompt = synth.gen_prompt(cfg.vocab, 10, 10)
    o1, s1 = _fresh(m, prompt)
    S = o1.draft(s1, 4)
    o2, s2 = _fresh(m, prompt)
    o2.draft_inject(s2, S)
    np.testing.assert_allclose(np.stack(s1.H_d), np.stack(s2.H_d), rtol=1e-10, atol=1e-12)
    assert o1.verify_intermediate(s1) == o2.verify_intermediate(s2)


# --- cache alignment (Sec. 3.2: a misaligned cache corrupts everything downstream) --------------

def _reference_cache(m, tokens, layers):
    c = eo.KVCache(m.spec, len(tokens))
    m.run_layers(range(max(layers) + 1), m.embed(tokens), np.arange(len(tokens)), c)
    return c


@pytest.mark.parametrize("bonus", [(True, True), (False, False), (True, False)])
def test_rollback_restores_the_exact_prefix(bonus):
    cfg = _cfg()
    m = _model(cfg)
    prompt = synth.gen_prompt(cfg.vocab, 12, 13)
    o, seq = _fresh(m, prompt, bonus_inter=bonus[0], bonus_full=bonus[1])
    for step in range(6):
        snapK = seq.cache.K.copy()
        old_len = list(seq.len)
        o.draft(seq, 3)
        o.verify_intermediate(seq)
        if step % 2 == 1:
            o.verify_full(seq)
        # invariant between calls
        nT, nC = len(seq.T), len(seq.C)
        assert seq.len == [nT - 1, nT - 1, nC - 1]
        assert len(seq.H_i) == len(seq.V) and not seq.H_d
        for g in range(3):
            for l in cfg.group_layers(g):
                # entries that were valid before and are still inside the new length are untouched
                keep = min(old_len[g], seq.len[g])
                np.testing.assert_array_equal(seq.cache.K[l, :keep], snapK[l, :keep])
                # everything beyond the length is poisoned, everything inside is finite
                assert np.isnan(seq.cache.K[l, seq.len[g]:]).all()
                assert np.isfinite(seq.cache.K[l, :seq.len[g]]).all()
                assert np.isfinite(seq.cache.V[l, :seq.len[g]]).all()
    # and the surviving cache equals a from-scratch pass over the surviving tokens
    ref = _reference_cache(m, seq.T[:-1], range(cfg.n_layers))
    for g in range(3):
        for l in cfg.group_layers(g):
            n = seq.len[g]
            np.testing.assert_allclose(seq.cache.K[l, :n], ref.K[l, :n], rtol=1e-9, atol=1e-11)
            np.testing.assert_allclose(seq.cache.V[l, :n], ref.V[l, :n], rtol=1e-9, atol=1e-11)
    # buffered L_i hidden rows equal the from-scratch L_i hidden states of their positions
    if seq.V:
        hid, _ = m.forward_nocache(seq.T[:-1], cfg.exit_inter)
        np.testing.assert_allclose(np.stack(seq.H_i), hid[len(seq.C) - 1:], rtol=1e-9, atol=1e-11)


def test_explicit_rollback_then_continue_equals_ar_from_the_cut():
    cfg = _cfg()
    m = _model(cfg)
    prompt = synth.gen_prompt(cfg.vocab, 12, 14)
    o, seq = _fresh(m, prompt)
    for _ in range(3):
        o.draft(seq, 3); o.verify_intermediate(seq); o.verify_full(seq)
    cut = len(prompt) + 2                       # keep prompt + 3 committed tokens, last one pending
    o.rollback(seq, 0b111, cut)
    assert seq.len == [cut, cut, cut] and len(seq.C) == cut + 1 and not seq.V
    kept = list(seq.C)
    while len(seq.C) < cut + 1 + 12:
        o.draft(seq, 3); o.verify_intermediate(seq); o.verify_full(seq)
    assert seq.C[cut + 1:cut + 13] == eo.ar_generate(m, kept, 12)
    # tentative-only cut: V shrinks, G3 stays
    o.draft(seq, 3); o.verify_intermediate(seq)
    o.draft(seq, 3); o.verify_intermediate(seq)
    nv, l3 = len(seq.V), seq.len[2]
    assert nv >= 2
    o.rollback(seq, 0b011, seq.len[0] - 1)
    assert len(seq.V) == nv - 1 and len(seq.H_i) == nv - 1 and seq.len[2] == l3
    with pytest.raises(ValueError):
        o.rollback(seq, 0b011, len(seq.C) - 3)   # reaches committed tokens without G3
    with pytest.raises(ValueError):
        o.rollback(seq, 0b100, 1)
    with pytest.raises(ValueError):
        o.rollback(seq, 0b111, seq.len[0] + 1)   # growing is not a rollback


def test_generate_truncates_to_requested_length():
    cfg = _cfg()
    m = _model(cfg)
    prompt = synth.gen_prompt(cfg.vocab, 8, 2)
    for n in (1, 2, 7):
        out = eo.HiSpecOracle(m).generate(prompt, n, 4, n_i=4)
        assert len(out) == n and out == eo.ar_generate(m, prompt, n)


@pytest.mark.parametrize("round_mode", ["none", "bf16"])
def test_hispec_stream_equals_ar_with_low_rank_exit_heads(round_mode):
    """The early exits' own heads change what is drafted and what survives L_i, never the output."""
    cfg = _cfg(exit_draft=2, exit_inter=4, head_rank=32, dtype="bf16" if round_mode == "bf16" else "f32")
    m = _model(cfg, round_mode=round_mode)
    plain = _model(_cfg(exit_draft=2, exit_inter=4, dtype=cfg.dtype), round_mode=round_mode)
    prompt = synth.gen_prompt(cfg.vocab, 11, 7)
    want = eo.ar_generate(m, prompt, 40)
    assert want == eo.ar_generate(plain, prompt, 40)            # the final exit has no adapter
    log = []
    assert eo.HiSpecOracle(m, True, True).generate(prompt, 40, 3, n_i=4, log=log) == want
    assert eo.ar_generate(m, prompt, 12, cfg.exit_draft) != eo.ar_generate(plain, prompt, 12, cfg.exit_draft)

"""Pins for the oracle's chain of intermediate verifiers (the extension sketched in the paper's Future Work):
it is Alg. 2 when the chain has one link, it never changes the output, and its caches and buffered hidden
rows are those of a from-scratch recomputation."""
import numpy as np
import pytest

import synth
from oracle import ee_oracle as eo


def _cfg(**kw):
    base = dict(n_layers=8, d_model=48, n_q_heads=4, n_kv_heads=2, head_dim=12, d_ffn=80, vocab=97,
                exit_draft=2, exit_inter=4, exit_extra=(6,), rope_theta=10000.0, sigma=0.08, gamma=(1.0, 0.15, 0.15))
    base.update(kw)
    return synth.EEConfig(**base)


def _model(cfg, seed=11, round_mode=None):
    return eo.EEModel(eo.ModelSpec.from_config(cfg, round_mode), synth.WeightStore(cfg, seed))


@pytest.mark.parametrize("extra,windows,k", [((6,), [4, 6], 3), ((5, 7), [2, 3, 4], 4), ((3,), [1, 1], 2), ((), [5], 3)])
@pytest.mark.parametrize("round_mode", ["none", "bf16"])
def test_stream_equals_ar(extra, windows, k, round_mode):
    cfg = _cfg(exit_draft=1, exit_inter=2, exit_extra=extra, dtype="bf16" if round_mode == "bf16" else "f32")
    m = _model(cfg, round_mode=round_mode)
    prompt = synth.gen_prompt(cfg.vocab, 9, 40 + k)
    log = []
    assert eo.MultiLevelOracle(m).generate(prompt, 36, k, windows, log=log) == eo.ar_generate(m, prompt, 36)
    levels = {lv for lv, _ in log}
    assert levels == set(range(1, len(extra) + 3))                      # every level did run
    assert any(a > 0 for lv, a in log if lv == 1) and any(a == 0 for lv, a in log if lv == 1)


def test_one_intermediate_verifier_is_algorithm_2_step_by_step():
    cfg = _cfg(exit_extra=())
    m = _model(cfg)
    prompt = synth.gen_prompt(cfg.vocab, 10, 3)
    H, M = eo.HiSpecOracle(m, True, True), eo.MultiLevelOracle(m)
    sh, sm = eo.Sequence_(m.spec, 200), eo.MultiSequence(m.spec, 200)
    assert H.prefill(sh, prompt) == M.prefill(sm, prompt)
    rng = np.random.default_rng(0)
    for rnd in range(8):
        k = int(rng.integers(1, 5))
        greedy = eo.ar_generate(m, sh.T, k, cfg.exit_inter)
        S = synth.make_draft_block(greedy, k, 0.6, cfg.vocab, rng)
        H.draft_inject(sh, S); M.draft_inject(sm, S)
        a, nxt = H.verify_intermediate(sh)
        a2, nxt2, _ = M.verify_level(sm, 1)
        assert (a, nxt) == (a2, nxt2) and sh.V == sm.V[1] and sh.len == sm.len
        np.testing.assert_array_equal(np.stack(sh.H_i), np.stack(sm.H[1]))
        if rnd % 3 == 2:
            f, nf, F = H.verify_full(sh)
            f2, nf2, F2 = M.verify_level(sm, 2)
            assert (f, nf, list(F)) == (f2, nf2, F2) and sh.C == sm.C and sh.len == sm.len and not sm.V[1]
    np.testing.assert_array_equal(np.nan_to_num(sh.cache.K[:, :sh.len[2]]), np.nan_to_num(sm.cache.K[:, :sm.len[2]]))


def test_caches_and_buffered_rows_equal_a_recomputation_from_scratch():
    """After any mix of levels: group g holds exactly the KV of T[:len[g]] and H[j] the e_j hidden rows of
    the positions just before each token of V[j], as a cacheless forward pass over T gives them."""
    cfg = _cfg(exit_draft=1, exit_inter=3, exit_extra=(5, 6))
    m = _model(cfg)
    M = eo.MultiLevelOracle(m)
    n = M.n
    seq = eo.MultiSequence(m.spec, 160)
    M.prefill(seq, synth.gen_prompt(cfg.vocab, 12, 5))
    rng = np.random.default_rng(4)
    plan = [1, 1, 2, 1, 2, 3, 1, 1, 2, 1, 2, 3, 4, 1, 2, 3, 1]
    ran = set()
    for lv in plan:
        if lv == 1:
            greedy = eo.ar_generate(m, seq.T, 3, cfg.exit_inter)
            M.draft_inject(seq, synth.make_draft_block(greedy, 3, 0.7, cfg.vocab, rng))
        elif not seq.V[lv - 1] or any(seq.V[i] for i in range(1, lv - 1)):
            continue
        M.verify_level(seq, lv)
        ran.add(lv)
        T = seq.T
        # length invariants
        assert seq.len[0] == seq.len[1] == len(T) - 1
        for g in range(2, n + 1):
            assert seq.len[g] == len(seq.C) + sum(len(seq.V[i]) for i in range(g, n)) - 1
        for j in range(1, n):
            assert len(seq.H[j]) == len(seq.V[j])
        # brute force over the whole text
        scratch = eo.KVCache(m.spec, len(T))
        x = m.embed(T)
        hid = {}
        for g in range(n + 1):
            x = m.run_layers(M.group(g), x, np.arange(len(T)), scratch)
            hid[g] = x
            L = seq.len[g]
            for l in M.group(g):
                np.testing.assert_allclose(seq.cache.K[l, :L], scratch.K[l, :L], rtol=1e-9, atol=1e-11)
                np.testing.assert_allclose(seq.cache.V[l, :L], scratch.V[l, :L], rtol=1e-9, atol=1e-11)
        for j in range(1, n):
            if seq.V[j]:
                first = len(seq.C) + sum(len(seq.V[i]) for i in range(j + 1, n)) - 1      # the token just before V[j]
                np.testing.assert_allclose(np.stack(seq.H[j]), hid[j][first:first + len(seq.V[j])], rtol=1e-9, atol=1e-11)
    assert ran == {1, 2, 3, 4}


def test_a_deeper_verifier_rejects_what_a_shallower_one_let_through():
    """Each level compares against its own exit: a buffer that level 1 accepted in full is cut by level 2
    exactly where exit e_2's greedy continuation first differs."""
    cfg = _cfg(exit_draft=1, exit_inter=2, exit_extra=(5,), gamma=(1.0, 1.0, 1.0))   # undamped: the exits disagree early
    m = _model(cfg)
    M = eo.MultiLevelOracle(m)
    seq = eo.MultiSequence(m.spec, 120)
    M.prefill(seq, synth.gen_prompt(cfg.vocab, 10, 2))
    e1 = eo.ar_generate(m, seq.T, 6, cfg.exit_inter)
    M.draft_inject(seq, e1[:5])
    a, nxt, _ = M.verify_level(seq, 1)
    assert (a, nxt) == (5, e1[5]) and seq.V[1] == e1
    e2 = eo.ar_generate(m, seq.T[:len(seq.C)], 7, 5)
    want = next((i for i in range(6) if e1[i] != e2[i]), 6)
    a2, nxt2, moved = M.verify_level(seq, 2)
    assert (a2, nxt2) == (want, e2[want]) and seq.V[2] == e2[:want + 1] == moved and not seq.V[1]


def _check_against_recomputation(m, M, seq):
    n, T = M.n, seq.T
    assert seq.len[0] == seq.len[1] == len(T) - 1
    for g in range(2, n + 1):
        assert seq.len[g] == len(seq.C) + sum(len(seq.V[i]) for i in range(g, n)) - 1
    scratch = eo.KVCache(m.spec, len(T))
    x = m.embed(T)
    for g in range(n + 1):
        x = m.run_layers(M.group(g), x, np.arange(len(T)), scratch)
        L = seq.len[g]
        for l in M.group(g):
            np.testing.assert_allclose(seq.cache.K[l, :L], scratch.K[l, :L], rtol=1e-9, atol=1e-11)
        if 1 <= g < n and seq.V[g]:
            first = len(seq.C) + sum(len(seq.V[i]) for i in range(g + 1, n)) - 1
            np.testing.assert_allclose(np.stack(seq.H[g]), x[first:first + len(seq.V[g])], rtol=1e-9, atol=1e-11)


@pytest.mark.parametrize("cut_in", ["V1", "V2", "C"])
def test_rollback_through_the_buffers_then_continue(cut_in):
    """A prune that ends inside the level-1 buffer, inside the level-2 buffer or inside the committed tokens
    leaves a state that a recomputation from scratch confirms, and decoding from it is still lossless."""
    cfg = _cfg(exit_draft=1, exit_inter=3, exit_extra=(5,))
    m = _model(cfg)
    M = eo.MultiLevelOracle(m)
    seq = eo.MultiSequence(m.spec, 200)
    prompt = synth.gen_prompt(cfg.vocab, 12, 5)
    M.prefill(seq, prompt)
    rng = np.random.default_rng(3)
    for lv in [1, 2, 1, 2, 3, 1, 2, 1, 2, 1]:           # ends with tokens in C, V[2] and V[1]
        if lv == 1:
            greedy = eo.ar_generate(m, seq.T, 3, cfg.exit_inter)
            M.draft_inject(seq, synth.make_draft_block(greedy, 3, 0.8, cfg.vocab, rng))
        M.verify_level(seq, lv)
    assert seq.V[1] and seq.V[2] and len(seq.C) > len(prompt) + 1
    M.draft_inject(seq, [1, 2, 3])                        # a pending block is dropped by the prune as well
    nC, n2, n1 = len(seq.C), len(seq.V[2]), len(seq.V[1])
    keep = {"V1": nC + n2 + max(1, n1 - 1), "V2": nC + max(1, n2 - 1), "C": nC - 1}[cut_in]
    before = seq.T[:keep]
    M.rollback(seq, keep - 1)
    assert seq.T == before and not seq.S
    if cut_in == "C":
        assert not seq.V[1] and not seq.V[2] and seq.len == [keep - 1] * 4
    elif cut_in == "V2":
        assert not seq.V[1] and len(seq.V[2]) == max(1, n2 - 1)
    _check_against_recomputation(m, M, seq)
    # go on: bottom-up through whatever still waits, then a few more rounds; the committed stream stays the AR stream
    for rnd in range(6):
        M.draft(seq, 3)
        M.verify_level(seq, 1)
        M.verify_level(seq, 2)
        if rnd % 2:
            M.verify_level(seq, 3)
    M.draft(seq, 2); M.verify_level(seq, 1); M.verify_level(seq, 2); M.verify_level(seq, 3)
    # the committed tokens that survived the cut stay; what follows them is the full model's greedy continuation
    surv = before[:min(nC, keep)]
    assert seq.C[:len(surv)] == surv
    assert seq.C[len(surv):] == eo.ar_generate(m, surv, len(seq.C) - len(surv))
    _check_against_recomputation(m, M, seq)


def test_chain_with_low_rank_heads_at_every_early_exit():
    """head_rank gives every exit but the last its own adapter (the final exit decides the output, so the
    stream stays the greedy stream of the plain model)."""
    cfg = _cfg(exit_draft=1, exit_inter=3, exit_extra=(5,), head_rank=16)
    m = _model(cfg)
    plain = _model(_cfg(exit_draft=1, exit_inter=3, exit_extra=(5,)))
    x = np.random.default_rng(0).standard_normal((3, cfg.d_model))
    for e in range(3):
        assert np.max(np.abs(m.exit_logits(x, e) - plain.exit_logits(x, e))) > 1e-3       # exits 0, 1, 2 have adapters
    np.testing.assert_array_equal(m.exit_logits(x, 3), plain.exit_logits(x, 3))
    np.testing.assert_array_equal(m.exit_logits(x), plain.exit_logits(x))                # default: the final exit
    assert m.spec.exit_index(5) == 2 and m.spec.exit_index(8) == 3 and m.spec.exit_index(2) == 3
    prompt = synth.gen_prompt(cfg.vocab, 9, 1)
    assert eo.MultiLevelOracle(m).generate(prompt, 30, 3, [3, 4]) == eo.ar_generate(plain, prompt, 30)

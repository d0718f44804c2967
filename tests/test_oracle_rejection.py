"""Pins of the oracle's rejection-sampling acceptance (App. G): the sampling primitive against brute force,
the acceptance rule against the cases that have closed forms, and the lemma it rests on -- the emitted token
is distributed as the target distribution whatever the draft distribution -- by a chi-square test, for one
stage and for the two stages composed (draft -> intermediate -> full)."""
import numpy as np
import pytest

from oracle import ee_oracle as eo


def _dist(rng, n, zeros=0):
    p = rng.random(n) ** 2
    if zeros:
        p[rng.choice(n, zeros, replace=False)] = 0.0
    return p / p.sum()


def test_inverse_cdf_against_brute_force():
    rng = np.random.default_rng(0)
    for _ in range(200):
        w = _dist(rng, 11, zeros=3) * rng.uniform(0.1, 7.0)       # unnormalised, with empty bins
        u = rng.random()
        acc, want = 0.0, None
        for i, x in enumerate(w):                                  # first bin whose running sum passes u * total
            acc += x
            if acc > u * w.sum():
                want = i
                break
        got, margin = eo.sample_inverse_cdf(w, u)
        assert got == want and w[got] > 0 and margin >= 0
    # the ends of the unit interval
    w = np.array([0.0, 0.25, 0.0, 0.75, 0.0])
    assert eo.sample_inverse_cdf(w, 0.0)[0] == 1
    assert eo.sample_inverse_cdf(w, 0.2499)[0] == 1 and eo.sample_inverse_cdf(w, 0.2501)[0] == 3
    assert eo.sample_inverse_cdf(w, 1.0 - 1e-12)[0] == 3            # never an empty trailing bin


def test_softmax_rows_closed_forms():
    lg = np.array([[0.0, 0.0, 0.0, 0.0], [np.log(1.0), np.log(2.0), np.log(3.0), np.log(4.0)], [1000.0, 0.0, -1000.0, 1000.0]])
    p = eo.softmax_rows(lg)
    assert np.allclose(p[0], 0.25) and np.allclose(p[1], [0.1, 0.2, 0.3, 0.4]) and np.allclose(p[2], [0.5, 0, 0, 0.5])
    assert np.allclose(eo.softmax_rows(lg + 123.0), p)              # shift invariance


def test_identical_distributions_accept_everything():
    rng = np.random.default_rng(1)
    k, n = 5, 9
    P = np.stack([_dist(rng, n) for _ in range(k + 1)])
    S = [int(rng.choice(n, p=P[j])) for j in range(k)]
    for _ in range(50):
        a, out, _ = eo.rejection_verify(S, P[:k], P, rng.random(k), 0.37)
        assert a == k and out[:k] == S and len(out) == k + 1
        assert out[k] == eo.sample_inverse_cdf(P[k], 0.37)[0]       # the next token comes from the target's extra row
    a, out, _ = eo.rejection_verify(S, P[:k], P[:k], rng.random(k), 0.37)
    assert a == k and out == S                                      # no extra row: nothing is added


def test_disjoint_supports_reject_at_once_and_resample_from_target():
    rng = np.random.default_rng(2)
    n = 10
    pd = np.zeros(n); pd[:5] = _dist(rng, 5)
    pt = np.zeros(n); pt[5:] = _dist(rng, 5)
    for _ in range(50):
        u = rng.random()
        a, out, _ = eo.rejection_verify([2, 3], np.stack([pd, pd]), np.stack([pt, pt, pt]), [rng.random(), rng.random()], u)
        assert a == 0 and out == [eo.sample_inverse_cdf(pt, u)[0]]  # residual max(0, pt - pd) = pt


def test_accept_probability_and_cut_position():
    # ratio 0.5 at position 1: accepted exactly when u < 0.5; everything after the cut is dropped
    pd = np.array([[0.5, 0.5, 0.0], [0.8, 0.2, 0.0], [0.3, 0.3, 0.4]])
    pt = np.array([[0.5, 0.5, 0.0], [0.4, 0.1, 0.5], [0.3, 0.3, 0.4], [0.2, 0.2, 0.6]])
    S = [1, 0, 2]
    a, out, m = eo.rejection_verify(S, pd, pt, [0.9, 0.49, 0.9], 0.1)
    assert a == 3 and out[:3] == S and abs(m - 0.01) < 1e-12
    a, out, _ = eo.rejection_verify(S, pd, pt, [0.9, 0.51, 0.0], 0.999)
    assert a == 1 and out == [1, 2]                                # residual at position 1 is all on token 2


def _chi2_ok(counts, p, n):
    exp = p * n
    keep = exp > 0
    if counts[~keep].sum() != 0:                                    # mass where the target has none
        return False
    chi2 = float(((counts[keep] - exp[keep]) ** 2 / exp[keep]).sum())
    dof = int(keep.sum()) - 1
    return chi2 < dof + 5.0 * np.sqrt(2.0 * dof)                    # mean + 5 sigma of the chi-square law


def test_lemma_one_stage_output_follows_target():
    rng = np.random.default_rng(3)
    n, trials = 12, 40000
    pd, pt = _dist(rng, n, zeros=2), _dist(rng, n, zeros=3)
    counts = np.zeros(n)
    for _ in range(trials):
        s = eo.sample_inverse_cdf(pd, rng.random())[0]
        _, out, _ = eo.rejection_verify([s], pd[None], pt[None], [rng.random()], rng.random())
        counts[out[0]] += 1
    assert _chi2_ok(counts, pt, trials)


def test_lemma_two_stages_composed_output_follows_final_target():
    """draft ~ p_d -> kept or replaced against p_i -> kept or replaced against p_f: the emitted token ~ p_f."""
    rng = np.random.default_rng(4)
    n, trials = 10, 40000
    pd, pi, pf = _dist(rng, n, zeros=1), _dist(rng, n, zeros=2), _dist(rng, n, zeros=2)
    counts = np.zeros(n)
    for _ in range(trials):
        s = eo.sample_inverse_cdf(pd, rng.random())[0]
        _, v, _ = eo.rejection_verify([s], pd[None], pi[None], [rng.random()], rng.random())
        _, f, _ = eo.rejection_verify(v, pi[None], pf[None], [rng.random()], rng.random())
        counts[f[0]] += 1
    assert _chi2_ok(counts, pf, trials)
    # a planted mistake is seen: testing against the intermediate distribution instead must fail
    assert not _chi2_ok(counts, pi, trials)


def test_lemma_three_stages_composed_output_follows_final_target():
    """A chain of verifiers (the hierarchy of the Future Work section under App. G's rule): draft ~ p_0, then three
    accept-or-replace stages against p_1, p_2, p_3, each using the previous stage's law as its draft law: the emitted
    token ~ p_3, and not ~ p_2."""
    rng = np.random.default_rng(6)
    n, trials = 9, 40000
    p = [_dist(rng, n, zeros=z) for z in (1, 2, 1, 2)]
    counts = np.zeros(n)
    for _ in range(trials):
        tok = [eo.sample_inverse_cdf(p[0], rng.random())[0]]
        for j in (1, 2, 3):
            _, tok, _ = eo.rejection_verify(tok, p[j - 1][None], p[j][None], [rng.random()], rng.random())
        counts[tok[0]] += 1
    assert _chi2_ok(counts, p[3], trials)
    assert not _chi2_ok(counts, p[2], trials)


def _chain_model(exit_extra, seed=5):
    import synth
    cfg = synth.tiny_config(n_layers=6, exit_draft=1, exit_inter=2, exit_extra=exit_extra, gamma=(1.0, 0.3, 0.3), vocab=64,
                            d_model=64, n_q_heads=2, n_kv_heads=2, head_dim=32, d_ffn=96)
    return cfg, eo.EEModel(eo.ModelSpec.from_config(cfg), synth.WeightStore(cfg, seed))


def test_chain_sampling_with_one_verifier_is_alg2_sampling_call_for_call():
    """MultiLevelOracle under App. G's rule with exits (L_d, L_i, L_f) takes, on the same uniform numbers, exactly
    the steps of HiSpecOracle's sampling calls: tokens, accept counts, committed streams, lengths, decision margins."""
    import synth
    cfg, model = _chain_model(())
    H, M = eo.HiSpecOracle(model), eo.MultiLevelOracle(model)
    prompt = synth.gen_prompt(cfg.vocab, 12, 3)
    hs_, ms = eo.Sequence_(model.spec, 200), eo.MultiSequence(model.spec, 200)
    assert H.prefill(hs_, prompt) == M.prefill(ms, prompt)
    rng = np.random.default_rng(8)
    k = 3
    for rnd in range(6):
        u_d, u_a, u_r = rng.random(k), rng.random(k), float(rng.random())
        assert H.draft(hs_, k, u_d) == M.draft(ms, k, u_d)
        a, nxt = H.verify_intermediate(hs_, (u_a, u_r))
        a2, nxt2, moved = M.verify_level(ms, 1, (u_a, u_r))
        assert (a, nxt) == (a2, nxt2) and H.last_margin == M.last_margin
        if rnd % 2:
            uf_a, uf_r = rng.random(len(hs_.V)), float(rng.random())
            f, fn, F = H.verify_full(hs_, (uf_a, uf_r))
            f2, fn2, F2 = M.verify_level(ms, 2, (uf_a, uf_r))
            assert (f, fn, F) == (f2, fn2, F2)
        assert hs_.T == ms.T and hs_.len == ms.len
    assert len(ms.C) > 13


def test_chain_sampling_keeps_the_law_of_each_level():
    """Two intermediate verifiers under App. G's rule: every buffer holds as many stored distributions as tokens,
    the stored rows are the level's own softmax of the rows that predicted those tokens, an explicit prune cuts
    tokens, rows and distributions alike, and a level refuses a buffer that the arg max calls produced."""
    import synth
    cfg, model = _chain_model((4,))
    M = eo.MultiLevelOracle(model)
    s = eo.MultiSequence(model.spec, 200)
    M.prefill(s, synth.gen_prompt(cfg.vocab, 10, 4))
    rng = np.random.default_rng(2)
    k = 4
    for rnd in range(5):
        M.draft(s, k, rng.random(k))
        assert len(s.P[0]) == k and all(abs(p.sum() - 1) < 1e-12 for p in s.P[0])
        M.verify_level(s, 1, (rng.random(k), float(rng.random())))
        assert len(s.P[1]) == len(s.V[1]) and not s.P[0]
        if rnd % 2:
            n1 = len(s.V[1])
            a, nxt, moved = M.verify_level(s, 2, (rng.random(n1), float(rng.random())))
            assert len(s.P[2]) == len(s.V[2]) == len(s.H[2]) and not s.P[1] and not s.V[1]
            # the stored law of the last moved token is the level's softmax of the row that predicted it
            assert np.allclose(s.P[2][-1], eo.softmax_rows(M.last_logits)[len(moved) - 1])
    assert len(s.V[2]) >= 2
    M.rollback(s, len(s.C) + len(s.V[2]) - 2)
    assert len(s.P[2]) == len(s.V[2]) == len(s.H[2])
    n2 = len(s.V[2])
    M.verify_level(s, 3, (rng.random(n2), float(rng.random())))
    assert not s.V[2] and not s.P[2] and s.len == [len(s.C) - 1] * 4
    M.draft(s, k)                                   # an arg max block has no distributions to test against
    with pytest.raises(AssertionError):
        M.verify_level(s, 1, (rng.random(k), 0.5))

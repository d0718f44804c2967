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

"""The host policy of the decoding loops (paper_2510_01336_amd/loop.py) driven by a session that the oracle
backs: whatever the trigger, the window sizes or the adaptive rule, the loops must call the levels in a legal
order and return the greedy stream of the full model (Alg. 2 changes the speed, not the output)."""
import numpy as np
import pytest

import synth
from oracle import ee_oracle as eo


class OracleSession:
    """The calls the loops use, answered by the oracle (one sequence at a time, batch-wide signatures)."""

    def __init__(self, cfg, seed, prompts):
        self.model = eo.EEModel(eo.ModelSpec.from_config(cfg), synth.WeightStore(cfg, seed))
        self.M = eo.MultiLevelOracle(self.model)
        self.seqs = []
        for p in prompts:
            s = eo.MultiSequence(self.model.spec, len(p) + 400)
            self.M.prefill(s, p)
            self.seqs.append(s)
        self.batch = len(prompts)
        self.calls = []

    def n_levels(self):
        return self.M.n

    def draft(self, k):
        self.calls.append(("draft", k))
        return np.array([self.M.draft(s, k) for s in self.seqs], np.int32)

    def verify_intermediate(self):
        self.calls.append(("level", 1))
        res = [self.M.verify_level(s, 1) for s in self.seqs]
        return np.array([r[0] for r in res]), np.array([r[1] for r in res])

    def verify_level(self, level, active=None):
        self.calls.append(("level", level))
        a, nxt, moved = [], [], []
        for b, s in enumerate(self.seqs):
            src = s.V[level - 1]
            if (active is not None and not active[b]) or not src:
                a.append(-1); nxt.append(-1); moved.append([])
                continue
            r = self.M.verify_level(s, level)          # asserts the bottom-up order itself
            a.append(r[0]); nxt.append(r[1]); moved.append(r[2])
        return np.array(a), np.array(nxt), moved

    def verify_full(self, active=None):
        return self.verify_level(self.M.n, active)

    # ---- the same calls under the acceptance rule of App. G (uniform numbers supplied by the loop)
    max_rows = 64

    def draft_sample(self, k, u):
        self.calls.append(("draft", k))
        return np.array([self.M.draft(s, k, u[b]) for b, s in enumerate(self.seqs)], np.int32)

    def verify_intermediate_rs(self, u_acc, u_res):
        self.calls.append(("level", 1))
        res = [self.M.verify_level(s, 1, (u_acc[b], float(u_res[b]))) for b, s in enumerate(self.seqs)]
        return np.array([r[0] for r in res]), np.array([r[1] for r in res])

    def verify_level_rs(self, level, u_acc, u_res, active=None):
        self.calls.append(("level", level))
        a, nxt, moved = [], [], []
        for b, s in enumerate(self.seqs):
            if (active is not None and not active[b]) or not s.V[level - 1]:
                a.append(-1); nxt.append(-1); moved.append([])
                continue
            r = self.M.verify_level(s, level, (u_acc[b], float(u_res[b])))
            a.append(r[0]); nxt.append(r[1]); moved.append(r[2])
        return np.array(a), np.array(nxt), moved

    def verify_full_rs(self, u_acc, u_res, active=None):
        return self.verify_level_rs(self.M.n, u_acc, u_res, active)

    def counts(self):
        return (np.array([len(s.C) for s in self.seqs]), np.array([len(s.T) - len(s.C) for s in self.seqs]))

    def lengths(self):
        return np.array([s.len for s in self.seqs])


def _cfg(**kw):
    base = dict(n_layers=6, d_model=48, n_q_heads=4, n_kv_heads=2, head_dim=12, d_ffn=80, vocab=97,
                exit_draft=1, exit_inter=3, rope_theta=10000.0, sigma=0.08, gamma=(1.0, 0.15, 0.15))
    base.update(kw)
    return synth.EEConfig(**base)


def _ar(sess, prompts, n):
    return np.array([eo.ar_generate(sess.model, p, n + 1)[1:] for p in prompts])


@pytest.mark.parametrize("policy", [dict(n_i=5), dict(n_i=3, trigger="any"), dict(every=2), "adaptive"],
                         ids=["n_i5_all", "n_i3_any", "every2", "adaptive"])
def test_three_exit_loop_returns_the_greedy_stream(policy):
    from paper_2510_01336_amd.loop import AdaptivePolicy, hispec_generate
    if policy == "adaptive":
        policy = dict(n_i=4, adaptive=AdaptivePolicy(nd_max=4))
    cfg = _cfg()
    prompts = [synth.gen_prompt(cfg.vocab, n, 20 + i) for i, n in enumerate([9, 14, 6])]
    sess = OracleSession(cfg, 11, prompts)
    toks, st = hispec_generate(sess, 30, 3, **policy)
    assert np.array_equal(toks, _ar(sess, prompts, 30))
    assert st.full_verifies >= 2 and 0 < st.accepted_inter < st.drafted
    # every full verification comes after at least one intermediate one since the last
    kinds = [c for c in sess.calls if c[0] == "level"]
    assert all(kinds[i - 1][1] == 1 for i in range(len(kinds)) if kinds[i][1] == 2)


@pytest.mark.parametrize("extra,windows", [((4,), [3, 4]), ((4, 5), [2, 2, 3])], ids=["3_levels", "4_levels"])
def test_chain_loop_returns_the_greedy_stream(extra, windows):
    from paper_2510_01336_amd.loop import hispec_generate_levels
    cfg = _cfg(exit_extra=extra)
    prompts = [synth.gen_prompt(cfg.vocab, n, 40 + i) for i, n in enumerate([8, 12])]
    sess = OracleSession(cfg, 11, prompts)
    toks, stats = hispec_generate_levels(sess, 28, 3, windows)
    assert np.array_equal(toks, _ar(sess, prompts, 28))
    assert all(c > 0 for c in stats["calls"][1:])
    assert all(0 <= a <= c for a, c in zip(stats["accepted"][1:], stats["checked"][1:]))


def test_chain_loop_under_the_sampling_rule_is_legal_and_repeatable():
    """The chain loop with App. G's acceptance at every exit: the levels are called bottom-up (the oracle asserts it),
    every sequence gets its tokens, what the loop returns is what the last level committed, and the same uniform
    numbers give the same stream."""
    from paper_2510_01336_amd.loop import hispec_generate_levels
    cfg = _cfg(exit_extra=(4,))
    prompts = [synth.gen_prompt(cfg.vocab, n, 60 + i) for i, n in enumerate([8, 12])]
    runs = []
    for rep in range(2):
        sess = OracleSession(cfg, 11, prompts)
        toks, stats = hispec_generate_levels(sess, 24, 3, [3, 4], rng=np.random.default_rng(5))
        assert toks.shape == (2, 24) and all(c > 0 for c in stats["calls"][1:])
        assert all(0 <= a <= c for a, c in zip(stats["accepted"][1:], stats["checked"][1:]))
        for b, s in enumerate(sess.seqs):
            committed = s.C[len(prompts[b]) + 1:]              # behind the prompt and the token the prompt predicts
            assert committed[:24] == toks[b].tolist()
        runs.append(toks)
    assert np.array_equal(runs[0], runs[1])
    other = hispec_generate_levels(OracleSession(cfg, 11, prompts), 24, 3, [3, 4], rng=np.random.default_rng(6))[0]
    assert not np.array_equal(other, runs[0])


def test_chain_loop_under_the_sampling_rule_keeps_the_target_law():
    """Lossless in distribution (App. G, applied at every exit of the chain): over many runs of the whole loop the
    first token it commits is distributed as the full model's next-token distribution -- chi-square against the
    distribution computed directly at L_f, with a control that the draft exit's distribution would be refused."""
    from scipy import stats as sps
    from paper_2510_01336_amd.loop import hispec_generate_levels
    cfg = _cfg(exit_extra=(4,), vocab=11, gamma=(1.0, 0.5, 0.5))
    prompt = synth.gen_prompt(cfg.vocab, 7, 3)
    base = OracleSession(cfg, 11, [prompt])
    model = base.model
    ctx = list(base.seqs[0].C)                                # prompt + the token it predicts
    _, lg_f = model.forward_nocache(ctx, cfg.n_layers)
    _, lg_d = model.forward_nocache(ctx, cfg.exit_draft)
    p_f, p_d = eo.softmax_rows(lg_f[-1:])[0], eo.softmax_rows(lg_d[-1:])[0]
    N = 600
    counts = np.zeros(cfg.vocab)
    rng = np.random.default_rng(17)
    import copy
    for _ in range(N):
        sess = copy.copy(base)
        sess.seqs = copy.deepcopy(base.seqs)
        sess.calls = []
        toks, _ = hispec_generate_levels(sess, 1, 3, [2, 2], rng=rng)
        counts[toks[0, 0]] += 1

    def pvalue(p):
        keep = p * N >= 5                                      # pool the rare tokens
        obs = np.append(counts[keep], counts[~keep].sum())
        exp = np.append(p[keep], p[~keep].sum()) * N
        if exp[-1] == 0:
            obs, exp = obs[:-1], exp[:-1]
        return sps.chisquare(obs, exp * obs.sum() / exp.sum()).pvalue

    assert pvalue(p_f) > 1e-3
    assert pvalue(p_d) < 1e-6                                  # the test can tell the two exits apart

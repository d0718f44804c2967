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

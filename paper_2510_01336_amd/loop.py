"""Host policy around the library calls: the decoding loop of Algorithm 2 (hierarchical speculative decoding).

Everything that computes runs in the library (ee_draft, ee_verify_intermediate, ee_verify_full); this
module only decides when the full verification fires -- when the tentative buffer holds at least N_i
tokens (Sec. 3.4) or after a fixed number of intermediate rounds -- and collects acceptance statistics
(draft tokens accepted by L_i per round, tentative tokens accepted by L_f per full verification).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np


@dataclass
class LoopStats:
    rounds: int = 0                 # draft + intermediate-verify rounds
    full_verifies: int = 0
    drafted: int = 0                # draft tokens proposed (per sequence summed)
    accepted_inter: int = 0         # of those, accepted by the intermediate verifier
    tentative: int = 0              # tentative tokens put to the full model
    accepted_full: int = 0          # of those, accepted by the full model
    committed: int = 0              # tokens committed (incl. the full model's own)
    per_round_accept: List[int] = field(default_factory=list)


def adapt_step(value: int, rate: float, tau_low: float, tau_high: float, lo: int, hi: int) -> int:
    """One update of the adaptive hyper-parameter rule (App. J, the N_d and N_i update equations, which
    differ only in their thresholds and bounds): one up at an acceptance rate of tau_high or more, one down
    below tau_low, unchanged in between, clamped to [lo, hi]."""
    if rate >= tau_high:
        return min(hi, value + 1)
    if rate < tau_low:
        return max(lo, value - 1)
    return value


@dataclass
class AdaptivePolicy:
    """App. J: N_d follows the intermediate verifier's acceptance rate of the last round (thresholds 0.5 / 0.8),
    N_i the full model's acceptance rate of the last full verification (0.3 / 0.8)."""
    nd_min: int = 1
    nd_max: int = 3
    ni_min: int = 3
    ni_max: int = 8
    nd_tau: tuple = (0.5, 0.8)
    ni_tau: tuple = (0.3, 0.8)


def hispec_generate(sess, n_new: int, k: int, *, n_i: Optional[int] = None, every: Optional[int] = None,
                    adaptive: Optional[AdaptivePolicy] = None, trigger: str = "all"):
    """Generate n_new tokens per sequence after the session's current context (ee_prefill done, nothing pending).

    Exactly one of n_i (fire the full verification when every sequence's -- trigger="any": any sequence's -- tentative buffer holds >= n_i
    tokens) and every (fire after that many intermediate rounds) is given.  With `adaptive` (needs n_i), k
    and n_i are the starting values of N_d and N_i and move by the rule of App. J.  Returns (tokens
    [batch, n_new], LoopStats).  The committed stream may run a few tokens past n_new inside the session;
    the returned rows are cut to n_new.
    """
    assert (n_i is None) != (every is None)
    assert adaptive is None or n_i is not None
    B = sess.batch
    out: List[List[int]] = [[] for _ in range(B)]
    st = LoopStats()
    while min(len(o) for o in out) < n_new:
        rounds = 0
        while True:
            sess.draft(k)
            a, _ = sess.verify_intermediate()
            rounds += 1
            st.rounds += 1
            st.drafted += B * k
            st.accepted_inter += int(a.sum())
            st.per_round_accept.append(int(a.sum()))
            if adaptive is not None:
                k_used = k
                k = adapt_step(k, float(a.sum()) / (B * k_used), *adaptive.nd_tau, adaptive.nd_min, adaptive.nd_max)
            _, nv = sess.counts()
            full = int(nv.min()) if trigger == "all" else int(nv.max())     # batch: every / any sequence holds N_i tokens
            if (n_i is not None and full >= n_i) or (every is not None and rounds >= every):
                break
            if min(len(o) + int(v) for o, v in zip(out, nv)) >= n_new + k + 2:
                break
        _, nv = sess.counts()
        f, _, com = sess.verify_full()
        st.full_verifies += 1
        st.tentative += int(nv.sum())
        st.accepted_full += int(np.minimum(f, nv).sum())
        if adaptive is not None:
            n_i = adapt_step(n_i, float(np.minimum(f, nv).sum()) / max(1, int(nv.sum())), *adaptive.ni_tau,
                             adaptive.ni_min, adaptive.ni_max)
        for b in range(B):
            out[b].extend(int(t) for t in com[b])
            st.committed += len(com[b])
    return np.array([o[:n_new] for o in out], np.int32), st


def hispec_generate_levels(sess, n_new: int, k: int, windows: Sequence[int], rng: Optional[np.random.Generator] = None):
    """The decoding loop over a chain of verifier exits (models with extra exits; ee_verify_level).

    Every iteration drafts k tokens and checks them at level 1 (L_i).  A sequence then climbs: level j runs
    for it when level j-1 has just run for it and the tokens waiting below level j number at least
    windows[j-2] (the per-stage windows N_{i,1}, N_{i,2}, ... of the paper's Future Work section), or when the
    sequence already holds enough tokens and is being flushed.  The last level commits.  With rng the calls are the
    ones of the rejection-sampling acceptance of App. G (ee_draft_sample, ee_verify_intermediate_rs,
    ee_verify_level_rs, ee_verify_full_rs; the session's sampling buffers must be attached) and rng supplies their
    uniform numbers; without it the greedy ones.  Returns (tokens [batch, n_new], {"calls", "checked", "accepted"}:
    per level, index 0 unused).
    """
    n = sess.n_levels()
    assert len(windows) == n - 1 and all(w >= 1 for w in windows)
    B = sess.batch
    out: List[List[int]] = [[] for _ in range(B)]
    stats = {"calls": [0] * (n + 1), "checked": [0] * (n + 1), "accepted": [0] * (n + 1)}

    def uniforms():
        return rng.random((B, sess.max_rows), np.float32), rng.random(B, np.float32)

    while min(len(o) for o in out) < n_new:
        if rng is None:
            sess.draft(k)
            a, _ = sess.verify_intermediate()
        else:
            sess.draft_sample(k, rng.random((B, k), np.float32))
            a, _ = sess.verify_intermediate_rs(rng.random((B, k), np.float32), rng.random(B, np.float32))
        stats["calls"][1] += 1
        stats["checked"][1] += B * k
        stats["accepted"][1] += int(a.sum())
        lens = sess.lengths()
        flush = np.array([len(out[b]) + int(lens[b, 1] - lens[b, n]) >= n_new + k + 2 for b in range(B)])
        ran = np.ones(B, bool)
        for j in range(2, n + 1):
            waiting = lens[:, j - 1] - lens[:, j]             # tokens accepted at level j-1 that level j has not seen
            act = ran & (waiting > 0) & ((waiting >= windows[j - 2]) | flush)
            if not act.any():
                break
            mask = act.astype(np.uint8)
            if rng is None:
                f, _, moved = sess.verify_level(j, mask) if j < n else sess.verify_full(mask)
            else:
                f, _, moved = sess.verify_level_rs(j, *uniforms(), mask) if j < n else sess.verify_full_rs(*uniforms(), mask)
            stats["calls"][j] += 1
            stats["checked"][j] += int(waiting[act].sum())
            stats["accepted"][j] += int(np.minimum(f, waiting)[act].sum())
            if j == n:
                for b in np.flatnonzero(act):
                    out[b].extend(int(t) for t in moved[b])
            ran = act
            lens = sess.lengths()
    return np.array([o[:n_new] for o in out], np.int32), stats


def hispec_generate_sampling(sess, n_new: int, k: int, n_i: int, rng: np.random.Generator):
    """The same loop with the rejection-sampling acceptance of App. G (ee_draft_sample, ee_verify_intermediate_rs,
    ee_verify_full_rs; the session's sampling buffers must be attached).  rng supplies the uniform numbers.
    Returns (tokens [batch, n_new], LoopStats)."""
    B = sess.batch
    out: List[List[int]] = [[] for _ in range(B)]
    st = LoopStats()
    while min(len(o) for o in out) < n_new:
        while True:
            sess.draft_sample(k, rng.random((B, k), np.float32))
            a, _ = sess.verify_intermediate_rs(rng.random((B, k), np.float32), rng.random(B, np.float32))
            st.rounds += 1
            st.drafted += B * k
            st.accepted_inter += int(a.sum())
            st.per_round_accept.append(int(a.sum()))
            _, nv = sess.counts()
            if int(nv.min()) >= n_i or min(len(o) + int(v) for o, v in zip(out, nv)) >= n_new + k + 2:
                break
        _, nv = sess.counts()
        f, _, com = sess.verify_full_rs(rng.random((B, sess.max_rows), np.float32), rng.random(B, np.float32))
        st.full_verifies += 1
        st.tentative += int(nv.sum())
        st.accepted_full += int(np.minimum(f, nv).sum())
        for b in range(B):
            out[b].extend(int(t) for t in com[b])
            st.committed += len(com[b])
    return np.array([o[:n_new] for o in out], np.int32), st

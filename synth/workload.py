"""Seeded synthetic workloads: prompts, ragged context lengths, draft blocks.

The paper measures on public benchmark prompts with trained models
(its Evaluation Methodology and benchmark-description appendix); uniform-random
token prompts and teacher-forced draft blocks with a chosen per-position
agreement probability stand in for them.  Nothing here runs a model: the
verifier's greedy continuation, where needed, is passed in as an array.
"""
from __future__ import annotations

from typing import Optional

import numpy as np


def gen_prompt(vocab: int, length: int, seed: int) -> np.ndarray:
    """i.i.d. uniform token ids in [0, vocab)."""
    rng = np.random.default_rng([seed, 0x50524F4D])
    return rng.integers(0, vocab, size=length, dtype=np.int64).astype(np.int32)


def gen_context_lengths(batch: int, seed: int, median: float = 1024.0, sigma: float = 0.7,
                        lo: int = 128, hi: int = 4096) -> np.ndarray:
    """Per-sequence KV context lengths: lognormal(ln median, sigma), clipped to [lo, hi]."""
    rng = np.random.default_rng([seed, 0x4C454E53])
    x = np.exp(rng.normal(np.log(median), sigma, size=batch))
    return np.clip(np.rint(x), lo, hi).astype(np.int32)


def draw_first_mismatch(k: int, p: float, rng: np.random.Generator) -> int:
    """Index of the first disagreeing draft position, k if all k agree.

    Each position agrees independently with probability p, so the index is
    min(Geometric(1-p) - 1, k).
    """
    if p >= 1.0:
        return k
    return int(min(rng.geometric(1.0 - p) - 1, k))


def make_draft_block(greedy: np.ndarray, k: int, p: float, vocab: int,
                     rng: np.random.Generator, first_mismatch: Optional[int] = None) -> np.ndarray:
    """Draft block S[0..k-1] agreeing with a verifier's greedy continuation.

    `greedy[j]` is the verifier's own greedy token at block position j given
    that positions < j held greedy tokens (teacher forced).  S copies it up to
    the drawn first-mismatch index a*, puts a uniformly drawn *different* token
    at a*, and uniform tokens after it (those are never looked at by a
    leading-prefix verifier).
    """
    a = draw_first_mismatch(k, p, rng) if first_mismatch is None else first_mismatch
    S = rng.integers(0, vocab, size=k, dtype=np.int64).astype(np.int32)
    S[:a] = np.asarray(greedy[:a], dtype=np.int32)
    if a < k:
        wrong = int(rng.integers(0, vocab - 1))
        if wrong >= int(greedy[a]):
            wrong += 1
        S[a] = wrong
    return S


def expected_accept_len(k: int, p: float) -> float:
    """E[min(Geometric(1-p)-1, k)] = p (1 - p^k) / (1 - p)."""
    return float(k) if p >= 1.0 else p * (1.0 - p ** k) / (1.0 - p)

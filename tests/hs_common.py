"""Shared helpers of the GPU parity tests: an oracle and a library session on the same seeded inputs."""
from __future__ import annotations

import numpy as np

import synth
from oracle import ee_oracle as eo

MARGIN = 1e-2      # top-1/top-2 logit margin every compared row must clear in the oracle
TOL = {"f32": 1e-4, "bf16": 2e-2}   # max|gpu - ref| / max|ref| for logits and hidden states


def max_rel(got: np.ndarray, ref: np.ndarray) -> float:
    return float(np.max(np.abs(np.asarray(got, np.float64) - ref)) / np.max(np.abs(ref)))


# Which oracle gates which check.  The paper states no numeric precision, so the model is the real-valued one:
# the PLAIN oracle (round_mode="none", float64, no operand rounding) is the reference of the 2e-2 bound on logits,
# hidden rows and KV entries of a bf16 model, and of its token / accept-length decisions on inputs whose deciding
# rows clear the margin in it.  The ROUNDING oracle (round_mode="bf16": operands rounded where a bf16 model stores
# or multiplies them) is a second, tighter check of the same quantities (measured maxima are several times
# smaller against it) and takes the same decisions on the compared inputs: candidates on which the two oracles
# decide differently although both clear the margin are counted (STATS["oracles_disagree"]) and not used.
STATS = {}    # name -> largest value seen in this test session (printed by conftest at the end of the run)


def note(name, value):
    STATS[name] = max(STATS.get(name, 0.0), float(value))


def count(name, n=1):
    STATS[name] = STATS.get(name, 0) + n


class OracleSide:
    """The oracle of a test: `o` / `seqs` follow the model's own rounding mode (the rounding oracle for a bf16
    configuration); with plain_twin a second OracleSide `P` holds the unrounded model in lockstep."""

    def __init__(self, cfg, seed, bonus_inter=True, bonus_full=True, round_mode=None, plain_twin=False, weights=None):
        self.cfg = cfg
        self.W = weights if weights is not None else synth.WeightStore(cfg, seed)
        self.model = eo.EEModel(eo.ModelSpec.from_config(cfg, round_mode=round_mode), self.W)
        self.o = eo.HiSpecOracle(self.model, bonus_inter, bonus_full)
        self.seqs = []
        twin = plain_twin and cfg.dtype == "bf16" and round_mode != "none"
        self.P = OracleSide(cfg, seed, bonus_inter, bonus_full, round_mode="none", weights=self.W) if twin else None

    def sides(self):
        return [self] + ([self.P] if self.P else [])

    def prefill(self, prompts, capacity):
        self.seqs, first, margins = [], [], []
        for p in prompts:
            s = eo.Sequence_(self.model.spec, capacity)
            first.append(self.o.prefill(s, p))
            margins.append(float(eo.top2_margin(self.o.last_logits)[0]))
            self.seqs.append(s)
        if self.P:
            pfirst, pmargins = self.P.prefill(prompts, capacity)
            margins = [min(a, b) if f == g else 0.0 for a, b, f, g in zip(margins, pmargins, first, pfirst)]
        return np.array(first), margins

    def greedy(self, seq, n, exit_layer):
        """Teacher-forced greedy continuation of T at an exit (fresh cache, state untouched)."""
        return eo.ar_generate(self.model, seq.T, n, exit_layer)


def gpu_side(cfg, seed, batch, max_ctx, max_rows, bonus_inter=True, bonus_full=True):
    import paper_2510_01336_amd as hs
    model = hs.Model(cfg, seed, int(bonus_inter), int(bonus_full))
    sess = hs.Session(model, batch, max_ctx, max_rows)
    return model, sess


def bf16_small(**kw):
    """A bf16 model whose GEMM shapes span several MFMA tiles with ragged tails: K = 688 is not a
    multiple of 32, vocab = 1000 not a multiple of 16, 4 query heads per KV head."""
    base = dict(n_layers=6, d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=688, vocab=1000,
                exit_draft=2, exit_inter=4, rope_theta=10000.0, dtype="bf16", sigma=0.05,
                gamma=(1.0, 0.2, 0.2))
    base.update(kw)
    return synth.EEConfig(**base)


def bf16_d128(**kw):
    base = dict(n_layers=5, d_model=512, n_q_heads=8, n_kv_heads=1, head_dim=128, d_ffn=1024, vocab=2048,
                exit_draft=1, exit_inter=3, rope_theta=500000.0, dtype="bf16", sigma=0.04,
                gamma=(1.0, 0.2, 0.2))
    base.update(kw)
    return synth.EEConfig(**base)

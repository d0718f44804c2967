"""CPU oracle for HiSpec's verification path (TEST INFRASTRUCTURE, not product code).

A plain, slow, numpy implementation of an early-exit (EE) transformer and of
the paper's decoding algorithms, written from the paper:

* auto-regressive decoding                     -- Sec. 3.1, "Vanilla generation"
* self-speculative decoding                    -- Algorithm 1
* hierarchical speculative decoding (HiSpec)   -- Algorithm 2
* LeadingSubstringVerify                       -- last function of Algorithms 1/2
* KV-cache / hidden-state reuse with pruning   -- Sec. 3.2
* per-sequence acceptance in a batch           -- Sec. "HiSpec Supports Batched Inference"
* rejection-sampling acceptance                -- App. G (rejection_verify and the rs arguments)
* low-rank exit heads                          -- App. I (EEModel.exit_logits, ModelSpec.head_rank)
* a chain of intermediate verifiers            -- Future Work section (MultiLevelOracle; with App. G's rule: its rs arguments)

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module; the product path never does.  It shares no code with the HIP
path and does not import the input generators either: weights arrive through
any object with `get(name, layer) -> ndarray` in the logical
[out_features, in_features] layout.

Arithmetic is float64 throughout.  The paper never states a numeric precision,
so the model's *operand rounding* is a parameter: `round_mode="none"` is the
exact real-valued model; `round_mode="bf16"` rounds (to nearest even) exactly
the values a bf16 model stores or feeds to a matrix product -- normalised
activations, rotated Q and K, V, the attention output, the SwiGLU product -- so
that the argmax decisions are taken in the same precision as a bf16 kernel
path.  Accumulation, softmax, norms and the residual stream stay float64.

Architecture (pre-norm decoder, one layer l, rows x at positions pos):
    n1 = RMSNorm(x; g1_l);  q,k,v = Wq n1, Wk n1, Wv n1;  q,k <- RoPE(., pos)
    x += Wo * Attn(q, K[0..pos], V[0..pos])        (grouped-query, causal)
    n2 = RMSNorm(x; g2_l);  x += Wdown (silu(Wgate n2) * (Wup n2))
    exit at layer L:  logits_L = Whead RMSNorm(x_L; gfinal)   (shared head)
Parity status: every function here is pinned by tests/test_oracle_*.py (library
routines, closed forms, brute force, the lossless invariant); the paper prints
no worked numeric example, so no value is pinned to a printed number.
"""
from __future__ import annotations

import dataclasses
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------
# numerics
# ----------------------------------------------------------------------------

def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bf16 (ties to even), returned as float64.

    Done through float32 bit patterns: float64 -> float32 (nearest even) is
    itself a rounding, so values are first snapped to float32 and then the low
    16 bits are rounded away.  NaN is passed through.
    """
    a = np.asarray(x, dtype=F64)
    f = a.astype(np.float32)
    u = f.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)) << np.uint32(16)
    out = r.view(np.float32).astype(F64)
    return np.where(np.isnan(a), a, out)


def _identity(x: np.ndarray) -> np.ndarray:
    return np.asarray(x, dtype=F64)


def rounding(mode: str) -> Callable[[np.ndarray], np.ndarray]:
    return {"none": _identity, "bf16": round_bf16}[mode]


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """y = x * rsqrt(mean(x^2) + eps) * g, row-wise."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, F64)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, half-split pairing: element i pairs with i + D/2.

    x: [m, H, D]; pos: [m].  Pair (x_i, x_{i+D/2}) is rotated by the angle
    pos * theta**(-2i/D).
    """
    x = np.asarray(x, F64)
    m, H, D = x.shape
    half = D // 2
    inv = theta ** (-2.0 * np.arange(half, dtype=F64) / D)
    ang = np.asarray(pos, F64)[:, None] * inv[None, :]            # [m, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, qpos: np.ndarray) -> np.ndarray:
    """Grouped-query causal attention of m query rows over n cached positions.

    q: [m, Hq, D]; K, V: [n, Hkv, D] (cache position j at index j); query row r
    sits at position qpos[r] and sees cache positions 0..qpos[r].  Scale 1/sqrt(D).
    Returns [m, Hq, D].
    """
    m, Hq, D = q.shape
    n, Hkv, _ = K.shape
    rep = Hq // Hkv
    allowed = np.arange(n)[None, :] <= np.asarray(qpos)[:, None]      # [m, n]
    out = np.empty((m, Hq, D), F64)
    for h in range(Hq):
        kv = h // rep
        s = (q[:, h, :] @ K[:, kv, :].T) / np.sqrt(float(D))          # [m, n]
        s = np.where(allowed, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ V[:, kv, :]
    return out


# ----------------------------------------------------------------------------
# model
# ----------------------------------------------------------------------------

@dataclasses.dataclass
class ModelSpec:
    """Architecture numbers the oracle needs (mirrors, but does not import, the input config)."""
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    exit_draft: int
    exit_inter: int
    rope_theta: float
    rms_eps: float
    round_mode: str = "none"
    head_rank: int = 0       # > 0: low-rank adapters in front of the shared head at L_d and L_i (App. I)
    exit_extra: Tuple[int, ...] = ()   # further intermediate verifiers L_{i,2} < L_{i,3} < ... (the paper's Future Work)

    @classmethod
    def from_config(cls, cfg, round_mode: Optional[str] = None) -> "ModelSpec":
        rm = round_mode if round_mode is not None else ("bf16" if getattr(cfg, "dtype", "f32") == "bf16" else "none")
        return cls(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                   cfg.d_ffn, cfg.vocab, cfg.exit_draft, cfg.exit_inter,
                   float(cfg.rope_theta), float(cfg.rms_eps), rm, int(getattr(cfg, "head_rank", 0)),
                   tuple(int(e) for e in getattr(cfg, "exit_extra", ())))

    @property
    def exits(self) -> Tuple[int, ...]:
        """L_d < L_{i,1} < L_{i,2} < ... < L_f."""
        return (self.exit_draft, self.exit_inter) + tuple(self.exit_extra) + (self.n_layers,)

    def exit_index(self, exit_layer: int) -> int:
        """Position of a layer in the exit list; any other depth counts as the final exit (the shared head alone)."""
        ex = self.exits
        return ex.index(exit_layer) if exit_layer in ex else len(ex) - 1

    def group_layers(self, g: int) -> range:
        b = (0, self.exit_draft, self.exit_inter, self.n_layers)
        return range(b[g], b[g + 1])


class KVCache:
    """Per-sequence K/V for every layer; index = token position.  Pruning = lowering a length."""

    def __init__(self, spec: ModelSpec, capacity: int):
        shape = (spec.n_layers, capacity, spec.n_kv_heads, spec.head_dim)
        self.K = np.full(shape, np.nan, F64)
        self.V = np.full(shape, np.nan, F64)
        self.capacity = capacity


class EEModel:
    def __init__(self, spec: ModelSpec, weights):
        self.spec, self.W = spec, weights
        self.rnd = rounding(spec.round_mode)

    def _w(self, name: str, layer: int = 0) -> np.ndarray:
        return np.asarray(self.W.get(name, layer), F64)

    def embed(self, tokens: Sequence[int]) -> np.ndarray:
        return np.asarray(self.W.get("emb", 0))[np.asarray(tokens, dtype=np.int64)].astype(F64)

    def layer(self, l: int, x: np.ndarray, pos: np.ndarray, cache: KVCache) -> np.ndarray:
        """Run 0-based layer l on rows x [m, d] at positions pos, writing K/V at those positions
        and attending over cache positions 0..pos[r]."""
        sp, rnd = self.spec, self.rnd
        m = x.shape[0]
        n1 = rnd(rmsnorm(x, self._w("g1", l), sp.rms_eps))
        q = (n1 @ self._w("wq", l).T).reshape(m, sp.n_q_heads, sp.head_dim)
        k = (n1 @ self._w("wk", l).T).reshape(m, sp.n_kv_heads, sp.head_dim)
        v = (n1 @ self._w("wv", l).T).reshape(m, sp.n_kv_heads, sp.head_dim)
        q = rnd(rope(q, pos, sp.rope_theta))
        k = rnd(rope(k, pos, sp.rope_theta))
        v = rnd(v)
        cache.K[l, pos] = k
        cache.V[l, pos] = v
        n = int(np.max(pos)) + 1
        o = attention(q, cache.K[l, :n], cache.V[l, :n], pos)
        o = rnd(o.reshape(m, sp.n_q_heads * sp.head_dim))
        x = x + o @ self._w("wo", l).T
        n2 = rnd(rmsnorm(x, self._w("g2", l), sp.rms_eps))
        h = rnd(silu(n2 @ self._w("wgate", l).T) * (n2 @ self._w("wup", l).T))
        return x + h @ self._w("wdown", l).T

    def run_layers(self, layers: range, x: np.ndarray, pos: np.ndarray, cache: KVCache) -> np.ndarray:
        for l in layers:
            x = self.layer(l, x, pos, cache)
        return x

    def exit_logits(self, x: np.ndarray, which: Optional[int] = None) -> np.ndarray:
        """Prediction head of exit number `which` in spec.exits (0 = L_d, 1 = L_i, ..., last = L_f, the
        default) on hidden rows x.

        The final layer, and every exit of a model without auxiliary heads, uses the shared final
        norm + shared LM head.  With head_rank = r > 0 (the post-training conversion of App. I,
        "low-rank prediction heads") every early exit first passes the hidden state through its own
        rank-r residual adapter,  z = x + B_e (A_e RMSNorm(x; g_e)),  and feeds z to the shared norm
        and head: the reading that fits the appendix's bound on added parameters."""
        last = len(self.spec.exits) - 1
        which = last if which is None else which
        if self.spec.head_rank > 0 and which < last:
            n = self.rnd(rmsnorm(x, self._w("aux_g", which), self.spec.rms_eps))
            t = self.rnd(n @ self._w("aux_a", which).T)
            x = x + t @ self._w("aux_b", which).T
        n = self.rnd(rmsnorm(x, self._w("gfinal"), self.spec.rms_eps))
        return n @ self._w("head").T

    def forward_nocache(self, tokens: Sequence[int], n_layers: int) -> Tuple[np.ndarray, np.ndarray]:
        """Brute force: recompute layers 1..n_layers for the whole sequence from scratch.
        Returns (hidden [t, d], logits [t, vocab]) at exit n_layers."""
        t = len(tokens)
        scratch = KVCache(self.spec, t)
        pos = np.arange(t)
        x = self.run_layers(range(n_layers), self.embed(tokens), pos, scratch)
        return x, self.exit_logits(x, self.spec.exit_index(n_layers))


def argmax_rows(logits: np.ndarray) -> np.ndarray:
    """Row-wise argmax; the lowest token id wins a tie."""
    return np.argmax(logits, axis=-1).astype(np.int64)


def top2_margin(logits: np.ndarray) -> np.ndarray:
    """Row-wise gap between the largest and second-largest logit."""
    part = np.partition(logits, -2, axis=-1)
    return part[..., -1] - part[..., -2]


def leading_substring_verify(S: Sequence[int], v: Sequence[int]) -> Tuple[int, List[int]]:
    """LeadingSubstringVerify of Algorithms 1/2, given the verifier's argmaxes.

    v[j] is the verifier's greedy token for the slot S[j] occupies (computed
    with S[0..j-1] in context); v may hold len(S)+1 entries (bonus available) or
    len(S).  Returns (a, out): a = number of leading matches, out = S[:a] plus
    the verifier's own token v[a] when it exists.
    """
    a = 0
    while a < len(S) and int(S[a]) == int(v[a]):
        a += 1
    out = [int(t) for t in S[:a]]
    if a < len(v):
        out.append(int(v[a]))
    return a, out


# ----------------------------------------------------------------------------
# decoding state machine (Algorithm 2 with the cache management of Sec. 3.2)
# ----------------------------------------------------------------------------

def softmax_rows(logits: np.ndarray) -> np.ndarray:
    """p = softmax(logits) per row (the exit distributions p_L of Sec. 3.1)."""
    x = np.asarray(logits, F64)
    e = np.exp(x - x.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def sample_inverse_cdf(w: np.ndarray, u: float) -> Tuple[int, float]:
    """Token drawn from the distribution proportional to the non-negative weights w with the uniform
    number u in [0, 1): the first index whose cumulative weight exceeds u * sum(w).  Also returns how far
    u * sum(w) is from the nearest boundary of that index's interval, relative to sum(w) (a margin for
    comparisons against implementations that add in another order)."""
    c = np.cumsum(np.asarray(w, F64))
    total = c[-1]
    assert total > 0
    t = u * total
    idx = int(np.searchsorted(c, t, side="right"))
    last = int(np.nonzero(w)[0][-1])
    idx = min(idx, last)
    lo = c[idx - 1] if idx > 0 else 0.0
    return idx, float(min(t - lo, c[idx] - t) / total)


def rejection_verify(S: Sequence[int], P_draft: np.ndarray, P_target: np.ndarray, u_acc: Sequence[float],
                     u_res: float) -> Tuple[int, List[int], float]:
    """The acceptance rule of App. G for one block: draft token S[j], drawn from row j of P_draft, is accepted
    when u_acc[j] < min(1, P_target[j, S[j]] / P_draft[j, S[j]]); at the first rejection the block is cut and
    a replacement is drawn (with u_res) from the residual distribution max(0, P_target[j] - P_draft[j])
    normalised.  When every token is accepted and P_target has one more row, the next token is drawn from that
    row (the target's own token after a fully accepted block).  Returns (number accepted, accepted tokens plus
    the drawn one, smallest margin of the decisions taken: |u - ratio| of the accept tests and the interval
    margin of the draw)."""
    k = len(S)
    margin = np.inf
    for j in range(k):
        s = int(S[j])
        ratio = min(1.0, float(P_target[j, s] / P_draft[j, s]))
        margin = min(margin, abs(float(u_acc[j]) - ratio) if ratio < 1.0 else np.inf)
        if float(u_acc[j]) < ratio:
            continue
        tok, mg = sample_inverse_cdf(np.maximum(0.0, P_target[j] - P_draft[j]), u_res)
        return j, [int(t) for t in S[:j]] + [tok], float(min(margin, mg))
    if len(P_target) > k:
        tok, mg = sample_inverse_cdf(P_target[k], u_res)
        return k, [int(t) for t in S] + [tok], float(min(margin, mg))
    return k, [int(t) for t in S], float(margin)


class Sequence_:
    """One sequence: committed tokens C, tentative buffer V, shared KV cache with three
    group lengths, and the buffered exit hidden states H_d (draft) and H_i (intermediate).

    Invariant between calls (the pending token T[-1], T = C||V, has no KV anywhere):
        len[0] = len[1] = |T| - 1,  len[2] = |C| - 1,
        H_i holds the L_i hidden rows of positions |C|-1 .. |T|-2,  H_d is empty.
    """

    def __init__(self, spec: ModelSpec, capacity: int):
        self.cache = KVCache(spec, capacity)
        self.C: List[int] = []
        self.V: List[int] = []
        self.S: List[int] = []
        self.len = [0, 0, 0]
        self.H_d: List[np.ndarray] = []
        self.H_i: List[np.ndarray] = []
        self.P_d: List[np.ndarray] = []      # rejection sampling only: the distributions the draft tokens were drawn from
        self.P_i: List[np.ndarray] = []      # ... and the L_i distributions of the tokens in V
        self.prompt_len = 0

    @property
    def T(self) -> List[int]:
        return self.C + self.V


class HiSpecOracle:
    """Step-by-step HiSpec on one model.  Sequences are independent (per-sequence acceptance),
    so a batch is a list of Sequence_ objects stepped one at a time."""

    def __init__(self, model: EEModel, bonus_inter: bool = True, bonus_full: bool = True,
                 poison: bool = True):
        self.m, self.spec = model, model.spec
        self.bonus_inter, self.bonus_full, self.poison = bonus_inter, bonus_full, poison
        self.last_logits: Optional[np.ndarray] = None
        self.last_hidden: Optional[np.ndarray] = None
        self.last_margin: float = np.inf     # rejection sampling: smallest decision margin of the last call

    # -- cache pruning -------------------------------------------------------
    def _set_len(self, seq: Sequence_, g: int, new_len: int) -> None:
        assert 0 <= new_len
        if self.poison and new_len < seq.len[g]:
            for l in self.spec.group_layers(g):
                seq.cache.K[l, new_len:seq.len[g]] = np.nan
                seq.cache.V[l, new_len:seq.len[g]] = np.nan
        seq.len[g] = new_len

    def rollback(self, seq: Sequence_, group_mask: int, new_len: int) -> None:
        """Cut a sequence back so that `new_len` positions keep their KV (shrink only).

        An unverified draft block is dropped first.  Groups G1 and G2 always move
        together (bits 0 and 1): the stream T = C||V is cut to new_len + 1 tokens, the last of
        which becomes the pending token, and the buffered L_i hidden rows follow V.  If the cut
        reaches into the committed tokens, V is emptied and G3 (bit 2) must be cut to the same
        length.  G3 alone can never shrink: its KV for committed positions could not be rebuilt.
        """
        seq.H_d, seq.S, seq.P_d = [], [], []
        self._set_len(seq, 0, seq.len[1])
        m12 = group_mask & 0b011
        if m12 not in (0, 0b011):
            raise ValueError("G1 and G2 roll back together")
        if m12 == 0:
            if (group_mask & 0b100) and new_len != seq.len[2]:
                raise ValueError("G3 cannot roll back alone")
            return
        if not (0 <= new_len <= seq.len[1]):
            raise ValueError("rollback can only shrink")
        n_t = new_len + 1
        if n_t <= len(seq.C):
            if new_len < seq.len[2] and not (group_mask & 0b100):
                raise ValueError("cut reaches committed tokens: G3 must roll back too")
            seq.C, seq.V, seq.H_i, seq.P_i = seq.C[:n_t], [], [], []
            self._set_len(seq, 2, new_len)
            seq.prompt_len = min(seq.prompt_len, new_len)
        else:
            seq.V = seq.V[:n_t - len(seq.C)]
            seq.H_i = seq.H_i[:len(seq.V)]
            seq.P_i = seq.P_i[:len(seq.V)]
        self._set_len(seq, 0, new_len)
        self._set_len(seq, 1, new_len)

    # -- prefill -------------------------------------------------------------
    def prefill(self, seq: Sequence_, prompt: Sequence[int]) -> int:
        t = len(prompt)
        pos = np.arange(t)
        x = self.m.run_layers(range(self.spec.n_layers), self.m.embed(prompt), pos, seq.cache)
        logits = self.m.exit_logits(x[-1:])
        c0 = int(argmax_rows(logits)[0])
        seq.C, seq.V, seq.H_d, seq.H_i, seq.S = [int(p) for p in prompt] + [c0], [], [], [], []
        seq.len = [t, t, t]
        seq.prompt_len = t
        self.last_logits, self.last_hidden = logits, x[-1:]
        return c0

    # -- drafting at exit L_d ------------------------------------------------
    def draft(self, seq: Sequence_, k: int, u: Optional[Sequence[float]] = None) -> List[int]:
        """Generate(L_d, x||V, k): k sequential shallow passes (plus, in bonus mode, one more
        G1-only pass so the last draft token also owns an L_d hidden row).  With uniform numbers u[0..k-1]
        the tokens are drawn from p_{L_d} (App. G) instead of taken as its arg max, and the
        distributions are kept for the acceptance tests."""
        assert not seq.H_d
        seq.P_d = []
        G1 = self.spec.group_layers(0)
        p0 = len(seq.T) - 1
        assert seq.len[0] == p0
        tok, S, logs = seq.T[-1], [], []
        rows = k + (1 if self.bonus_inter else 0)
        for j in range(rows):
            x = self.m.run_layers(G1, self.m.embed([tok]), np.array([p0 + j]), seq.cache)
            seq.H_d.append(x[0])
            if j < k:
                lg = self.m.exit_logits(x, 0)
                logs.append(lg[0])
                if u is None:
                    tok = int(argmax_rows(lg)[0])
                else:
                    pd = softmax_rows(lg)[0]
                    tok, mg = sample_inverse_cdf(pd, float(u[j]))
                    seq.P_d.append(pd)
                    self.last_margin = min(self.last_margin, mg) if j else mg
                S.append(tok)
        seq.len[0] = p0 + rows
        seq.S = S
        self.last_logits = np.stack(logs)
        self.last_hidden = np.stack(seq.H_d)
        return S

    def draft_inject(self, seq: Sequence_, S: Sequence[int]) -> None:
        """Take an externally supplied draft block: G1 runs block-parallel on [pending, S...]."""
        assert not seq.H_d
        G1 = self.spec.group_layers(0)
        p0 = len(seq.T) - 1
        assert seq.len[0] == p0
        k = len(S)
        rows = k + (1 if self.bonus_inter else 0)
        toks = ([seq.T[-1]] + [int(s) for s in S])[:rows]
        x = self.m.run_layers(G1, self.m.embed(toks), p0 + np.arange(rows), seq.cache)
        seq.H_d = [x[r] for r in range(rows)]
        seq.len[0] = p0 + rows
        seq.S = [int(s) for s in S]
        self.last_hidden = x

    # -- intermediate verification at exit L_i ---------------------------------
    def verify_intermediate(self, seq: Sequence_, rs: Optional[Tuple[Sequence[float], float]] = None) -> Tuple[int, int]:
        """LeadingSubstringVerify(S, L_i, x||V); appends the result to V, keeps the hidden rows of
        surviving positions in H_i and prunes G1/G2 KV.  Returns (a, next_token); next_token is
        -1 when everything matched and no bonus row exists."""
        G2 = self.spec.group_layers(1)
        rows = len(seq.H_d)
        assert rows > 0
        p0 = len(seq.T) - 1
        assert seq.len[1] == p0 and seq.len[0] == p0 + rows
        Y = self.m.run_layers(G2, np.stack(seq.H_d), p0 + np.arange(rows), seq.cache)
        seq.len[1] = p0 + rows
        logits = self.m.exit_logits(Y, 1)
        if rs is None:
            v = argmax_rows(logits)
            a, vhat = leading_substring_verify(seq.S, v)
        else:       # App. G: rs = (u_acc[k], u_res); the tokens kept are distributed as p_{L_i}
            P = softmax_rows(logits)
            a, vhat, self.last_margin = rejection_verify(seq.S, np.stack(seq.P_d), P, rs[0], rs[1])
            seq.P_i = seq.P_i + [P[r] for r in range(len(vhat))]
            seq.P_d = []
        keep = len(vhat)                       # rows whose input token is now in T
        seq.V = seq.V + vhat
        seq.H_i = seq.H_i + [Y[r] for r in range(keep)]
        self._set_len(seq, 0, p0 + keep)
        self._set_len(seq, 1, p0 + keep)
        seq.H_d, seq.S = [], []
        self.last_logits, self.last_hidden = logits, Y
        return a, (vhat[-1] if len(vhat) > a else -1)

    # -- full verification at L_f ----------------------------------------------
    def verify_full(self, seq: Sequence_, rs: Optional[Tuple[Sequence[float], float]] = None) -> Tuple[int, int, List[int]]:
        """LeadingSubstringVerify(V, L_f, x): consumes the buffered L_i hidden rows, commits the
        accepted prefix (+ the target's own token) and prunes all three groups.
        Returns (f, next_token, committed_tokens)."""
        sp = self.spec
        nv, nc = len(seq.V), len(seq.C)
        assert nv > 0 and not seq.H_d
        assert len(seq.H_i) == nv and seq.len[2] == nc - 1
        rows_h = list(seq.H_i)
        if self.bonus_full:
            # the pending token V[-1] owns no hidden state yet: catch it up through G1 and G2
            p = nc + nv - 1
            x = self.m.embed([seq.V[-1]])
            x = self.m.run_layers(sp.group_layers(0), x, np.array([p]), seq.cache)
            x = self.m.run_layers(sp.group_layers(1), x, np.array([p]), seq.cache)
            seq.len[0] = seq.len[1] = p + 1
            rows_h.append(x[0])
        rows = len(rows_h)
        Z = self.m.run_layers(sp.group_layers(2), np.stack(rows_h), (nc - 1) + np.arange(rows), seq.cache)
        seq.len[2] = nc - 1 + rows
        logits = self.m.exit_logits(Z)
        if rs is None:
            w = argmax_rows(logits)
            f, F = leading_substring_verify(seq.V, w)
        else:       # App. G, second stage: V (distributed as p_{L_i}) is the draft, p_{L_f} the target
            assert len(seq.P_i) == nv
            f, F, self.last_margin = rejection_verify(seq.V, np.stack(seq.P_i), softmax_rows(logits), rs[0], rs[1])
        seq.C = seq.C + F
        seq.V, seq.H_i, seq.P_i = [], [], []
        for g in range(3):
            self._set_len(seq, g, len(seq.C) - 1)
        self.last_logits, self.last_hidden = logits, Z
        return f, (F[-1] if len(F) > f else -1), F

    # -- Algorithm 2 ---------------------------------------------------------
    def generate(self, prompt: Sequence[int], n_new: int, k: int, *, n_i: Optional[int] = None,
                 every: Optional[int] = None, capacity: Optional[int] = None,
                 draft_fn: Optional[Callable[[Sequence_, int], Sequence[int]]] = None,
                 log: Optional[list] = None) -> List[int]:
        """HiSpec decoding of n_new tokens after the prompt.

        Full verification fires when |V| >= n_i (the paper's dynamic policy) or
        after `every` intermediate rounds (fixed-period variant); exactly one of
        the two is given.  `draft_fn(seq, k)` may supply external draft tokens.
        """
        assert (n_i is None) != (every is None)
        cap = capacity or (len(prompt) + n_new + (k + 2) * ((every or n_i) + 3) + 8)
        seq = Sequence_(self.spec, cap)
        self.prefill(seq, prompt)
        while len(seq.C) - seq.prompt_len < n_new:
            rounds = 0
            while True:
                if draft_fn is None:
                    self.draft(seq, k)
                else:
                    self.draft_inject(seq, draft_fn(seq, k))
                a, nxt = self.verify_intermediate(seq)
                rounds += 1
                if log is not None:
                    log.append(("inter", a, nxt))
                if (n_i is not None and len(seq.V) >= n_i) or (every is not None and rounds >= every):
                    break
                if len(seq.T) - seq.prompt_len >= n_new + k + 2:
                    break
            f, nxt, F = self.verify_full(seq)
            if log is not None:
                log.append(("full", f, nxt, list(F)))
        return seq.C[seq.prompt_len:seq.prompt_len + n_new]


# ----------------------------------------------------------------------------
# several intermediate verifiers
# ----------------------------------------------------------------------------

class MultiSequence:
    """One sequence under a hierarchy of verifiers at the exits e_0 = L_d < e_1 < ... < e_n = L_f.

    V[j] (j = 1..n-1) holds the tokens accepted at exit e_j that still wait for exit e_{j+1}; the
    text so far is  T = C || V[n-1] || ... || V[1],  deepest verdict first.  H[j] holds, for buffer
    V[j], the e_j hidden rows of the tokens [the token just before V[j], V[j][0], ..., V[j][-2]]:
    row r is the state that predicts V[j][r] one level up.  H[0] are the draft block's L_d rows.
    len[g] is the KV length of layer group g (layers e_{g-1}..e_g, e_{-1} = 0)."""

    def __init__(self, spec: ModelSpec, capacity: int):
        n = len(spec.exits) - 1
        self.n = n
        self.cache = KVCache(spec, capacity)
        self.C: List[int] = []
        self.V: List[List[int]] = [[] for _ in range(n)]         # V[0] unused
        self.S: List[int] = []
        self.H: List[List[np.ndarray]] = [[] for _ in range(n)]
        # rejection sampling only: P[0] the distributions the draft tokens were drawn from, P[j] the exit-e_j
        # distributions of the tokens in V[j] (the law they follow, by the lemma of App. G applied level by level)
        self.P: List[List[np.ndarray]] = [[] for _ in range(n)]
        self.len = [0] * (n + 1)
        self.prompt_len = 0

    @property
    def T(self) -> List[int]:
        out = list(self.C)
        for j in range(self.n - 1, 0, -1):
            out += self.V[j]
        return out


class MultiLevelOracle:
    """Alg. 2 with the single intermediate verifier replaced by a chain of them (the extension the
    paper's Future Work section sketches; with exits (L_d, L_i, L_f) it is Alg. 2 itself).

    Level 1 checks a draft block S exactly as L_i does in Alg. 2.  Level j >= 2 treats the buffer
    V[j-1] as its draft: the buffered e_{j-1} rows, plus one row for the buffer's last token (which
    has no state yet: it runs through the groups below first), pass through layer group j, and
    LeadingSubstringVerify against exit e_j's arg max keeps the matching prefix and e_j's own next
    token.  What is kept moves to V[j] (to C at the last level); everything below is dropped and
    the KV lengths of the groups up to j are pruned to the kept prefix (Sec. 3.2).  A level runs
    only when every buffer below the one it checks is empty.

    With uniform numbers (the `u` / `rs` arguments) the same chain runs under the acceptance rule of App. G instead
    of arg max comparison: draft tokens are drawn from p_{L_d}; level j accepts a token of the buffer below with
    probability min(1, p_{e_j} / p_{e_{j-1}}), replaces the first rejected one from the normalised positive part of
    p_{e_j} - p_{e_{j-1}}, and after a fully accepted buffer draws the next token from its extra row.  By the
    appendix's lemma the tokens a level keeps follow that level's distribution, which makes them a valid draft for
    the next level: applied n times, what is committed follows p_{L_f}."""

    def __init__(self, model: EEModel):
        self.m, self.spec = model, model.spec
        self.exits = model.spec.exits
        self.n = len(self.exits) - 1
        self.last_logits: Optional[np.ndarray] = None
        self.last_margin: float = np.inf     # rejection sampling: smallest decision margin of the last call

    def group(self, g: int) -> range:
        return range(self.exits[g - 1] if g else 0, self.exits[g])

    def _head(self, x: np.ndarray, level: int) -> np.ndarray:
        return self.m.exit_logits(x, level)

    def prefill(self, seq: MultiSequence, prompt: Sequence[int]) -> int:
        t = len(prompt)
        x = self.m.run_layers(range(self.spec.n_layers), self.m.embed(prompt), np.arange(t), seq.cache)
        self.last_logits = self.m.exit_logits(x[-1:])
        c0 = int(argmax_rows(self.last_logits)[0])
        seq.C = [int(p) for p in prompt] + [c0]
        seq.len = [t] * (self.n + 1)
        seq.prompt_len = t
        return c0

    def _draft_rows(self, seq: MultiSequence, tokens: Sequence[int]) -> None:
        p0 = len(seq.T) - 1
        x = self.m.run_layers(self.group(0), self.m.embed(tokens), p0 + np.arange(len(tokens)), seq.cache)
        seq.H[0] = [r for r in x]
        seq.len[0] = p0 + len(tokens)

    def draft_inject(self, seq: MultiSequence, S: Sequence[int]) -> None:
        """A given draft block: the pending token and S through the draft layers in one pass."""
        assert not seq.S and not seq.H[0]
        seq.S = [int(t) for t in S]
        self._draft_rows(seq, [seq.T[-1]] + seq.S)

    def draft(self, seq: MultiSequence, k: int, u: Optional[Sequence[float]] = None) -> List[int]:
        """Generate(L_d, T, k): k sequential shallow passes, then the last draft token's own row.  With uniform
        numbers u[0..k-1] the tokens are drawn from p_{L_d} and the distributions kept (App. G)."""
        assert not seq.S and not seq.H[0]
        p0 = len(seq.T) - 1
        tok, rows, S = seq.T[-1], [], []
        seq.P[0] = []
        for j in range(k + 1):
            x = self.m.run_layers(self.group(0), self.m.embed([tok]), np.array([p0 + j]), seq.cache)
            rows.append(x[0])
            if j < k:
                lg = self._head(x, 0)
                if u is None:
                    tok = int(argmax_rows(lg)[0])
                else:
                    pd = softmax_rows(lg)[0]
                    tok, mg = sample_inverse_cdf(pd, float(u[j]))
                    seq.P[0].append(pd)
                    self.last_margin = min(self.last_margin, mg) if j else mg
                S.append(tok)
        seq.S, seq.H[0], seq.len[0] = S, rows, p0 + k + 1
        return S

    def verify_level(self, seq: MultiSequence, j: int,
                     rs: Optional[Tuple[Sequence[float], float]] = None) -> Tuple[int, int, List[int]]:
        """Returns (a, next token, the tokens that moved up: accepted prefix + next token).  rs = (u_acc, u_res):
        the acceptance rule of App. G with the stored distributions of the buffer below as the draft law."""
        n = self.n
        assert 1 <= j <= n
        src = seq.S if j == 1 else seq.V[j - 1]
        assert src, "nothing to verify at this level"
        assert j == 1 or (not seq.S and all(not seq.V[i] for i in range(1, j - 1)))
        above = len(seq.C) + sum(len(seq.V[i]) for i in range(j, n))     # tokens already past level j
        p0 = above - 1
        rows = list(seq.H[j - 1])
        if j >= 2:      # the buffer's last token has no state anywhere yet
            p = p0 + len(src)
            x = self.m.embed([src[-1]])
            for g in range(j):
                x = self.m.run_layers(self.group(g), x, np.array([p]), seq.cache)
            rows.append(x[0])
        assert len(rows) == len(src) + 1
        Y = self.m.run_layers(self.group(j), np.stack(rows), p0 + np.arange(len(rows)), seq.cache)
        self.last_logits = self._head(Y, j)
        if rs is None:
            a, out = leading_substring_verify(src, argmax_rows(self.last_logits))
        else:
            assert len(seq.P[j - 1]) == len(src), "the buffer below was not produced by the sampling calls"
            Pt = softmax_rows(self.last_logits)
            a, out, self.last_margin = rejection_verify(src, np.stack(seq.P[j - 1]), Pt, rs[0], rs[1])
        moved = [int(t) for t in out]                 # accepted prefix and the verifier's own next token
        keep = len(moved)
        if j == n:
            seq.C += moved
        else:
            seq.V[j] += moved
            seq.H[j] += [r for r in Y[:keep]]
            if rs is not None:
                seq.P[j] += [Pt[r] for r in range(keep)]
        seq.S = []
        for i in range(j):
            seq.H[i] = []
            seq.P[i] = []
            if i >= 1:
                seq.V[i] = []
        for g in range(j + 1):
            seq.len[g] = p0 + keep
        if j == n:
            seq.len = [len(seq.C) - 1] * (n + 1)
        return a, moved[-1], moved

    def rollback(self, seq: MultiSequence, new_len: int) -> None:
        """Explicit prune to new_len positions in every group that is longer (Sec. 3.2: only lengths
        change).  new_len + 1 tokens of T remain, the last of them pending again; a pending draft block is
        dropped; every buffer keeps the tokens (and the hidden rows) that lie before the cut."""
        n = self.n
        assert 0 <= new_len <= seq.len[1]
        keep = new_len + 1
        room = keep
        take = min(room, len(seq.C)); seq.C = seq.C[:take]; room -= take
        for j in range(n - 1, 0, -1):
            take = min(room, len(seq.V[j]))
            seq.V[j] = seq.V[j][:take]
            seq.H[j] = seq.H[j][:take]
            seq.P[j] = seq.P[j][:take]
            room -= take
        seq.S, seq.H[0], seq.P[0] = [], [], []
        seq.len[0] = seq.len[1] = new_len
        for g in range(2, n + 1):
            seq.len[g] = min(seq.len[g], new_len)
        seq.cache.K[:, new_len:] = np.nan       # dead entries must never be read again
        seq.cache.V[:, new_len:] = np.nan

    def generate(self, prompt: Sequence[int], n_new: int, k: int, windows: Sequence[int],
                 log: Optional[list] = None) -> List[int]:
        """Decoding loop: draft + level 1 until |V[1]| >= windows[0]; then level 2, and so on up as long
        as the buffer a level has just filled reaches its window (windows[j-1] for V[j]); a
        generation that has enough tokens flushes every level in order."""
        n = self.n
        assert len(windows) == n - 1
        seq = MultiSequence(self.spec, len(prompt) + n_new + (k + 2) * (sum(windows) + 4) + 8)
        self.prefill(seq, prompt)
        while len(seq.C) - seq.prompt_len < n_new:
            flush = len(seq.T) - seq.prompt_len >= n_new + k + 2
            self.draft(seq, k)
            a, _, _ = self.verify_level(seq, 1)
            if log is not None:
                log.append((1, a))
            for j in range(2, n + 1):
                if not seq.V[j - 1] or not (flush or len(seq.V[j - 1]) >= windows[j - 2]):
                    break
                a, _, _ = self.verify_level(seq, j)
                if log is not None:
                    log.append((j, a))
        return seq.C[seq.prompt_len:seq.prompt_len + n_new]


# ----------------------------------------------------------------------------
# reference decoders
# ----------------------------------------------------------------------------

def ar_generate(model: EEModel, prompt: Sequence[int], n_new: int, exit_layer: Optional[int] = None) -> List[int]:
    """Greedy auto-regressive decoding at `exit_layer` (default: the full model) with a KV cache."""
    L = exit_layer or model.spec.n_layers
    cache = KVCache(model.spec, len(prompt) + n_new)
    x = model.run_layers(range(L), model.embed(prompt), np.arange(len(prompt)), cache)
    which = model.spec.exit_index(L)
    out = [int(argmax_rows(model.exit_logits(x[-1:], which))[0])]
    while len(out) < n_new:
        p = len(prompt) + len(out) - 1
        x = model.run_layers(range(L), model.embed([out[-1]]), np.array([p]), cache)
        out.append(int(argmax_rows(model.exit_logits(x, which))[0]))
    return out


def ar_generate_nocache(model: EEModel, prompt: Sequence[int], n_new: int,
                        exit_layer: Optional[int] = None) -> List[int]:
    """Greedy decoding that recomputes the whole prefix for every token (brute force)."""
    L = exit_layer or model.spec.n_layers
    toks = [int(t) for t in prompt]
    for _ in range(n_new):
        _, logits = model.forward_nocache(toks, L)
        toks.append(int(argmax_rows(logits[-1:])[0]))
    return toks[len(prompt):]


def self_speculative_generate(model: EEModel, prompt: Sequence[int], n_new: int, k: int,
                              log: Optional[list] = None) -> List[int]:
    """Algorithm 1: draft k tokens at L_d, verify them at L_f in one pass, accept the leading
    prefix plus the target's token.  Written without any cache so it is independent of the
    state machine above."""
    sp = model.spec
    toks = [int(t) for t in prompt]
    _, lg = model.forward_nocache(toks, sp.n_layers)
    toks.append(int(argmax_rows(lg[-1:])[0]))
    while len(toks) - len(prompt) < n_new:
        ctx = list(toks)
        S: List[int] = []
        for _ in range(k):
            _, lg = model.forward_nocache(ctx + S, sp.exit_draft)
            S.append(int(argmax_rows(lg[-1:])[0]))
        _, lg = model.forward_nocache(ctx + S, sp.n_layers)
        v = argmax_rows(lg[len(ctx) - 1:])          # k+1 predictions
        a, F = leading_substring_verify(S, v)
        if log is not None:
            log.append((a, list(F)))
        toks += F
    return toks[len(prompt):len(prompt) + n_new]

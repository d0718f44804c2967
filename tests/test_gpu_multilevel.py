"""GPU: a chain of intermediate verifiers (ee_verify_level; the extension of the paper's Future Work section)
in lockstep with the oracle's MultiLevelOracle, and the lossless invariant of the whole loop on the GPU."""
import copy

import numpy as np
import pytest

import synth
from oracle import ee_oracle as eo
from hs_common import MARGIN, TOL, max_rel

pytestmark = pytest.mark.gpu


def f32_chain(**kw):
    base = dict(n_layers=8, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=688, vocab=1024,
                exit_draft=2, exit_inter=4, exit_extra=(6,), rope_theta=10000.0, dtype="f32", gamma=(1.0, 0.3, 0.3))
    base.update(kw)
    return synth.EEConfig(**base)


def bf16_chain(**kw):
    base = dict(n_layers=8, d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=688, vocab=1000,
                exit_draft=1, exit_inter=3, exit_extra=(5, 6), rope_theta=10000.0, dtype="bf16", sigma=0.05,
                gamma=(1.0, 0.2, 0.2))
    base.update(kw)
    return synth.EEConfig(**base)


# (model, weight seed, context lengths, k, rounds): a round is a draft block checked at level 1 and then at the
# listed higher levels, bottom-up.  The seeds are ones for which every row that decides an output clears the
# margin in the oracle (run_plan checks it and picks draft blocks accordingly).
PLANS = [
    ("f32_3_levels", f32_chain(), 3, [40, 9, 70], 4, [[1], [1, 2], [1, 2, 3], [1, 2], [1, 2, 3]]),
    ("bf16_4_levels", bf16_chain(), 8, [90, 33], 6, [[1, 2], [1], [1, 2, 3], [1, 2, 3, 4], [1, 2, 3, 4]]),
    # low-rank heads at every early exit (L_d, L_i and the extra one), the shared head alone at L_f
    ("f32_3_levels_low_rank_heads", f32_chain(head_rank=24), 1, [40, 9], 4, [[1], [1, 2], [1, 2, 3], [1, 2, 3]]),
    # an explicit prune through the buffers in the middle, then on
    ("f32_3_levels_rollback", f32_chain(), 1, [40, 9], 4, [[1, 2], [1, 2], [1], "cut", [1, 2], [1, 2, 3], "cut", [1, 2, 3]]),
]


def margin_of(cfg):
    return MARGIN if cfg.dtype == "bf16" else 1e-3         # fp32 rounding is far below either


def run_plan(cfg, seed, ctx, k, plan, sess=None, p=0.7):
    """The rounds on the oracle and, when a session is given, on the GPU in lockstep.  Returns the smallest
    margin among the deciding rows (-1 if no draft block could be found for some round)."""
    W = synth.WeightStore(cfg, seed)
    model = eo.EEModel(eo.ModelSpec.from_config(cfg), W)
    M = eo.MultiLevelOracle(model)
    n, B = M.n, len(ctx)
    tol, need = TOL[cfg.dtype], margin_of(cfg)
    cap = max(ctx) + 16 * (k + 2)
    prompts = [synth.gen_prompt(cfg.vocab, int(c), 300 + b) for b, c in enumerate(ctx)]
    seqs, worst = [], np.inf
    for pr in prompts:
        s = eo.MultiSequence(model.spec, cap)
        M.prefill(s, pr)
        worst = min(worst, float(eo.top2_margin(M.last_logits)[0]))
        seqs.append(s)
    if sess is not None:
        assert sess.n_levels() == n
        assert sess.prefill(prompts).tolist() == [s.C[-1] for s in seqs]
    rng = np.random.default_rng(1)

    def trial(s, S, levels):
        t, w = copy.deepcopy(s), np.inf
        M.draft_inject(t, S)
        for lv in levels:
            a, _, _ = M.verify_level(t, lv)
            w = min(w, float(eo.top2_margin(M.last_logits)[:a + 1].min()))
        return w

    for levels in plan:
        if levels == "cut":
            # prune one token short of the end of the level-2 buffer (of the committed tokens if it is empty):
            # the level-1 buffer goes, deeper state stays; all groups roll back together
            for b, s in enumerate(seqs):
                keep = len(s.C) + (max(1, len(s.V[2]) - 1) if s.V[2] else -1)
                M.rollback(s, keep - 1)
                if sess is not None:
                    sess.rollback(b, (1 << (n + 1)) - 1, keep - 1)
            if sess is not None:
                lens = sess.lengths()
                nc, nv = sess.counts()
                for b, s in enumerate(seqs):
                    assert list(lens[b]) == s.len and sess.tokens(b).tolist() == s.T
                    assert (nc[b], nv[b]) == (len(s.C), len(s.T) - len(s.C))
            continue
        drafts = []
        for s in seqs:
            greedy = eo.ar_generate(model, s.T, k, cfg.exit_inter)
            for _ in range(40):
                S = synth.make_draft_block(greedy, k, p, cfg.vocab, rng, first_mismatch=synth.draw_first_mismatch(k, p, rng))
                if trial(s, S, levels) > need:
                    break
            else:
                return -1.0
            drafts.append(S)
        drafts = np.stack(drafts)
        for lv in levels:
            if sess is not None:
                if lv == 1:
                    sess.draft_inject(drafts)
                    ga, gn = sess.verify_intermediate()
                else:
                    ga, gn, gmoved = sess.verify_level(lv) if lv < n else sess.verify_full()
                glog = sess.last_logits()
            r0 = 0
            for b, s in enumerate(seqs):
                if lv == 1:
                    M.draft_inject(s, drafts[b])
                a, nxt, moved = M.verify_level(s, lv)
                rows = len(M.last_logits)
                worst = min(worst, float(eo.top2_margin(M.last_logits)[:a + 1].min()))
                if sess is not None:
                    assert (int(ga[b]), int(gn[b])) == (a, nxt), (lv, b)
                    if lv > 1:
                        assert gmoved[b] == moved
                    assert max_rel(glog[r0:r0 + rows], M.last_logits) <= tol
                r0 += rows
            if sess is not None:
                lens = sess.lengths()
                nc, nv = sess.counts()
                for b, s in enumerate(seqs):
                    assert list(lens[b]) == s.len, (lv, b)
                    assert sess.tokens(b).tolist() == s.T
                    assert (nc[b], nv[b]) == (len(s.C), len(s.T) - len(s.C))
    return worst


@pytest.mark.parametrize("name,cfg,seed,ctx,k,plan", PLANS, ids=[p[0] for p in PLANS])
def test_levels_match_oracle(name, cfg, seed, ctx, k, plan):
    import paper_2510_01336_amd as hs
    model = hs.Model(cfg, seed)
    sess = hs.Session(model, len(ctx), max(ctx) + 16 * (k + 2), 4 * (k + 2))
    sess.enable_logits(True)
    assert run_plan(cfg, seed, ctx, k, plan, sess) > margin_of(cfg)
    # order and range of the levels
    with pytest.raises(hs.EEError):
        sess.verify_level(1)
    with pytest.raises(hs.EEError):
        sess.verify_level(sess.n_levels() + 1)
    sess.close(); model.close()


def test_levels_must_run_bottom_up():
    import paper_2510_01336_amd as hs
    cfg, seed, k = f32_chain(), 5, 4
    model = hs.Model(cfg, seed)
    sess = hs.Session(model, 1, 200, 4 * (k + 2))
    sess.prefill([synth.gen_prompt(cfg.vocab, 30, 1)])
    rng = np.random.default_rng(0)
    sess.draft_inject(rng.integers(0, cfg.vocab, (1, k)).astype(np.int32))
    sess.verify_intermediate()
    sess.verify_level(2)                                   # V[1] -> V[2]
    sess.draft_inject(rng.integers(0, cfg.vocab, (1, k)).astype(np.int32))
    sess.verify_intermediate()                             # V[1] is filled again
    before = (sess.lengths().tolist(), sess.tokens(0).tolist())
    with pytest.raises(hs.EEError):
        sess.verify_full()                                 # level 3 while level 1's buffer waits
    with pytest.raises(hs.EEError):
        sess.decode_ar(1)                                  # vanilla steps need everything committed
    assert (sess.lengths().tolist(), sess.tokens(0).tolist()) == before
    sess.verify_level(2); sess.verify_full()
    nc, nv = sess.counts()
    assert nv[0] == 0 and len(set(sess.lengths()[0].tolist())) == 1
    assert sess.decode_ar(2).shape == (1, 2)
    sess.close(); model.close()


@pytest.mark.parametrize("cfg,windows", [(f32_chain(gamma=(1.0, 0.1, 0.1)), [2, 3]),
                                         (bf16_chain(dtype="f32", gamma=(1.0, 0.1, 0.1)), [2, 3, 5])], ids=["3_levels", "4_levels"])
def test_multilevel_stream_equals_vanilla_stream_on_gpu(cfg, windows):
    import paper_2510_01336_amd as hs
    from paper_2510_01336_amd.loop import hispec_generate_levels
    n_new, k, ctx = 48, 4, [32, 19]
    prompts = [synth.gen_prompt(cfg.vocab, c, 11 + i) for i, c in enumerate(ctx)]
    rows = 6 * (k + 2)
    model = hs.Model(cfg, 4242)
    sess = hs.Session(model, len(ctx), max(ctx) + 16 * n_new, max(rows, n_new))      # a slow sequence keeps the fast one drafting
    first = sess.prefill(prompts)
    ar = np.concatenate([first[:, None], sess.decode_ar(n_new - 1)], axis=1)
    sess.prefill(prompts)
    toks, stats = hispec_generate_levels(sess, n_new - 1, k, windows)
    assert np.array_equal(np.concatenate([first[:, None], toks], axis=1), ar)
    assert all(c > 0 for c in stats["calls"][1:]) and 0 < stats["accepted"][1] < stats["checked"][1]
    sess.close(); model.close()


def _limit_case(sess=None):
    """Two sequences whose level-2 buffers grow by six tokens per round (every draft block is the L_i verifier's own
    continuation and exit 6 agrees with it): with max_rows = 14 sequence 0 reaches the most a buffer below a
    catch-up row may hold (max_rows - 1 = 13 tokens: 1, 7, 13), sequence 1 (6, 12) would pass it and is refused.
    Level 3 then consumes sequence 0's thirteen rows plus the catch-up row (14 = max_rows rows), and afterwards
    sequence 1's buffer, which must have stayed intact next to the full one.  With a session the GPU runs in
    lockstep; returns the smallest margin of the deciding rows."""
    import paper_2510_01336_amd as hs
    cfg, seed, k, ctx, max_rows = f32_chain(gamma=(1.0, 0.1, 0.1)), 3, 4, [40, 9], 14
    W = synth.WeightStore(cfg, seed)
    model = eo.EEModel(eo.ModelSpec.from_config(cfg), W)
    M = eo.MultiLevelOracle(model)
    tol = TOL["f32"]
    prompts = [synth.gen_prompt(cfg.vocab, c, 300 + b) for b, c in enumerate(ctx)]
    seqs, worst = [], np.inf
    for pr in prompts:
        s = eo.MultiSequence(model.spec, 300)
        M.prefill(s, pr)
        seqs.append(s)
    if sess is not None:
        assert sess.prefill(prompts).tolist() == [s.C[-1] for s in seqs]

    def level(lv, active):
        """Level lv for the active sequences on both sides; compares decisions, moved tokens, logits and state."""
        nonlocal worst
        if sess is not None:
            if lv == 1:
                ga, gn = sess.verify_intermediate()
            else:
                act = np.array(active, np.uint8)
                ga, gn, gmoved = sess.verify_level(lv, act) if lv < M.n else sess.verify_full(act)
            glog, r0 = sess.last_logits(), 0
        for b, s in enumerate(seqs):
            if not active[b]:
                continue
            a, nxt, moved = M.verify_level(s, lv)
            rows = len(M.last_logits)
            worst = min(worst, float(eo.top2_margin(M.last_logits)[:a + 1].min()))
            if sess is not None:
                assert (int(ga[b]), int(gn[b])) == (a, nxt), (lv, b)
                if lv > 1:
                    assert gmoved[b] == moved
                assert max_rel(glog[r0:r0 + rows], M.last_logits) <= tol
                r0 += rows
        if sess is not None:
            lens = sess.lengths()
            for b, s in enumerate(seqs):
                assert list(lens[b]) == s.len and sess.tokens(b).tolist() == s.T, (lv, b)

    def inject():
        drafts = np.stack([np.array(eo.ar_generate(model, s.T, k, cfg.exit_inter), np.int32) for s in seqs])
        for b, s in enumerate(seqs):
            M.draft_inject(s, drafts[b])
        if sess is not None:
            sess.draft_inject(drafts)

    for rnd in range(2):
        inject(); level(1, [1, 1]); level(2, [1, 1])
    assert [len(s.V[2]) for s in seqs] == [7, 12]
    inject(); level(1, [1, 1]); level(2, [1, 0])
    assert len(seqs[0].V[2]) == max_rows - 1
    if sess is not None:
        before = (sess.lengths().tolist(), sess.tokens(1).tolist())
        with pytest.raises(hs.EEError) as e:                 # 12 + 5 + 1 tokens would not leave room for a catch-up row
            sess.verify_level(2, np.array([0, 1], np.uint8))
        assert e.value.code == -3
        assert (sess.lengths().tolist(), sess.tokens(1).tolist()) == before
    level(3, [1, 0])                                          # 13 buffered rows + the catch-up row = max_rows rows
    # sequence 1: drop its level-1 buffer (and the last token of the level-2 buffer), then level 3 over the rest
    s = seqs[1]
    keep = len(s.C) + len(s.V[2]) - 1
    M.rollback(s, keep - 1)
    if sess is not None:
        sess.rollback(1, (1 << (M.n + 1)) - 1, keep - 1)
    level(3, [0, 1])
    return worst


def test_level_buffer_filled_to_its_limit_in_a_batch():
    import paper_2510_01336_amd as hs
    cfg = f32_chain(gamma=(1.0, 0.1, 0.1))
    model = hs.Model(cfg, 3)
    sess = hs.Session(model, 2, 300, 14)
    sess.enable_logits(True)
    assert _limit_case(sess) > margin_of(cfg)
    sess.close(); model.close()

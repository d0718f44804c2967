"""GPU: rejection-sampling acceptance (App. G) through the C ABI against the oracle, with the same uniform numbers
on both sides.  Decisions (accept counts, drawn tokens) must be equal whenever the oracle's decision margin --
the distance of a uniform number from the accept threshold or from the edge of the drawn token's interval of
the CDF -- exceeds what fp32 summation order can move; rounds below the margin are redrawn."""
import copy

import numpy as np
import pytest

import synth
from oracle import ee_oracle as eo
from hs_common import OracleSide, bf16_small, gpu_side

pytestmark = pytest.mark.gpu

RS_MARGIN = {"f32": 2e-5}


def _trial(O, seq, k, u_d, u_a, u_r, full, uf_a=None, uf_r=None):
    t = copy.deepcopy(seq)
    O.o.draft(t, k, u_d)
    m = O.o.last_margin
    O.o.verify_intermediate(t, (u_a, u_r))
    m = min(m, O.o.last_margin)
    if full:
        O.o.verify_full(t, (uf_a, uf_r))
        m = min(m, O.o.last_margin)
    return m


def test_rejection_sampling_rounds_match_oracle():
    cfg = synth.tiny_config(gamma=(1.0, 0.3, 0.3))
    k, ctxs = 4, [40, 23]
    B = len(ctxs)
    rows = 3 * (k + 1) + 2
    margin = RS_MARGIN["f32"]
    O = OracleSide(cfg, 77)
    prompts = [synth.gen_prompt(cfg.vocab, n, 300 + b) for b, n in enumerate(ctxs)]
    model, sess = gpu_side(cfg, 77, B, max(ctxs) + 8 * rows, rows)
    sess.enable_sampling()
    first = sess.prefill(prompts)
    for p in prompts:
        s = eo.Sequence_(O.model.spec, max(ctxs) + 8 * rows)
        O.o.prefill(s, p)
        O.seqs.append(s)
    for b, s in enumerate(O.seqs):
        s.C[-1] = int(first[b])
    rng = np.random.default_rng(5)
    compared = accepted = rejected = 0
    for rnd in range(8):
        full = rnd % 2 == 1
        for _ in range(40):      # redraw the round's uniform numbers until every decision clears the margin
            u_d, u_a, u_r = rng.random((B, k), np.float32), rng.random((B, k), np.float32), rng.random(B, np.float32)
            uf_a, uf_r = rng.random((B, rows), np.float32), rng.random(B, np.float32)
            if all(_trial(O, s, k, u_d[b], u_a[b], float(u_r[b]), full, uf_a[b], float(uf_r[b])) > margin
                   for b, s in enumerate(O.seqs)):
                break
        else:
            pytest.fail("no draw cleared the margin")
        gS = sess.draft_sample(k, u_d)
        ga, gn = sess.verify_intermediate_rs(u_a, u_r)
        for b, s in enumerate(O.seqs):
            assert gS[b].tolist() == O.o.draft(s, k, u_d[b]), (rnd, b)
            a, nxt = O.o.verify_intermediate(s, (u_a[b], float(u_r[b])))
            assert (int(ga[b]), int(gn[b])) == (a, nxt), (rnd, b)
            accepted += a; rejected += k - a
        if full:
            gf, gfn, gcom = sess.verify_full_rs(uf_a, uf_r)
            for b, s in enumerate(O.seqs):
                f, nxt, F = O.o.verify_full(s, (uf_a[b], float(uf_r[b])))
                assert (int(gf[b]), int(gfn[b]), gcom[b]) == (f, nxt, F), (rnd, b)
        lens = sess.lengths()
        for b, s in enumerate(O.seqs):
            assert list(lens[b]) == s.len and sess.tokens(b).tolist() == s.T
        compared += 1
    assert compared == 8 and accepted > 0 and rejected > 0      # both outcomes of the accept test were exercised
    # the two acceptance rules may not be mixed within a round
    import paper_2510_01336_amd as hs
    sess.draft(k)
    with pytest.raises(hs.EEError):
        sess.verify_intermediate_rs(rng.random((B, k), np.float32), rng.random(B, np.float32))
    with pytest.raises(hs.EEError):
        sess.draft_sample(k, np.full((B, k), 1.0, np.float32))  # (also: a block is pending)
    sess.close(); model.close()


def test_sampling_needs_attached_buffers_and_valid_uniforms():
    import paper_2510_01336_amd as hs
    cfg = synth.tiny_config()
    model, sess = gpu_side(cfg, 3, 1, 96, 12)
    sess.prefill([synth.gen_prompt(cfg.vocab, 16, 1)])
    with pytest.raises(hs.EEError):
        sess.draft_sample(4, np.zeros((1, 4), np.float32))       # nothing attached
    sess.enable_sampling()
    with pytest.raises(hs.EEError):
        sess.draft_sample(4, np.array([[0.1, 0.2, 1.0, 0.3]], np.float32))   # 1.0 is outside [0, 1)
    assert sess.lengths().tolist() == [[16, 16, 16]]
    S = sess.draft_sample(4, np.array([[0.1, 0.2, 0.9, 0.3]], np.float32))
    assert S.shape == (1, 4) and (S >= 0).all() and (S < cfg.vocab).all()
    # fewer uniform numbers than draft tokens: refused, the block stays pending and verifies with enough of them
    with pytest.raises(hs.EEError) as e:
        sess.verify_intermediate_rs(np.full((1, 3), 0.5, np.float32), np.array([0.5], np.float32))
    assert e.value.code == -1
    a, n = sess.verify_intermediate_rs(np.full((1, 4), 0.5, np.float32), np.array([0.5], np.float32))
    assert 0 <= int(a[0]) <= 4
    sess.close(); model.close()


def test_bf16_distributions_and_decisions():
    """bf16 model: token probabilities carry the model's ~1e-2 relative error, more than the width of a token's
    interval of the CDF, so drawn tokens cannot be compared with the oracle's directly.  Checked instead: (1) the
    distributions the GPU forms (p_{L_d} per drafted position, p_{L_i} per verified row) against the oracle's on the
    same tokens, within the bf16 tolerance; (2) every decision of the GPU against the oracle's acceptance rule
    applied to the GPU's own distributions with the same uniform numbers (same inputs, so only the summation
    order differs: fp32 margin)."""
    from hs_common import TOL
    cfg = bf16_small()
    k, ctxs = 5, [37, 70]
    B, rows = len(ctxs), 3 * (k + 1) + 2
    O = OracleSide(cfg, 78)
    prompts = [synth.gen_prompt(cfg.vocab, n, 400 + b) for b, n in enumerate(ctxs)]
    model, sess = gpu_side(cfg, 78, B, max(ctxs) + 8 * rows, rows)
    sess.enable_sampling()
    sess.enable_logits(True)
    first = sess.prefill(prompts)
    for b, p in enumerate(prompts):
        s = eo.Sequence_(O.model.spec, max(ctxs) + 8 * rows)
        O.o.prefill(s, p)
        s.C[-1] = int(first[b])
        O.seqs.append(s)
    rng = np.random.default_rng(9)
    checked = skipped = 0
    for rnd in range(6):
        u_d, u_a, u_r = rng.random((B, k), np.float32), rng.random((B, k), np.float32), rng.random(B, np.float32)
        nv = sess.counts()[1]
        S = sess.draft_sample(k, u_d)
        Pd = [sess.read_dist(0, b, 0, k).astype(np.float64) for b in range(B)]
        ga, gn = sess.verify_intermediate_rs(u_a, u_r)
        Pt = sess.last_logits().astype(np.float64)                # this call's p_{L_i}, rows packed sequence by sequence
        for b in range(B):
            assert np.allclose(Pd[b].sum(axis=1), 1.0, atol=1e-4) and (Pd[b] >= 0).all()
            for j in range(k):                                    # the drafted tokens, from the GPU's own p_{L_d}
                tok, mg = eo.sample_inverse_cdf(Pd[b][j], float(u_d[b, j]))
                if mg > RS_MARGIN["f32"]:
                    assert int(S[b, j]) == tok, (rnd, b, j)
                    checked += 1
                else:
                    skipped += 1
            pt = Pt[b * (k + 1):(b + 1) * (k + 1)]
            a, out, mg = eo.rejection_verify(S[b].tolist(), Pd[b], pt, u_a[b], float(u_r[b]))
            if mg > RS_MARGIN["f32"]:
                assert (int(ga[b]), int(gn[b])) == (a, out[-1]), (rnd, b)
                checked += 1
            else:
                skipped += 1
            # the stored p_{L_i} rows of the tokens now in V are the rows of this call
            keep = int(ga[b]) + 1
            Pi = sess.read_dist(1, b, int(nv[b]), keep)
            assert np.array_equal(Pi, pt[:keep].astype(np.float32))
        if rnd == 0:      # distributions against the oracle on the same tokens (fresh from the context build)
            for b, s in enumerate(O.seqs):
                O.o.draft_inject(s, S[b])
                pd_ref = eo.softmax_rows(O.model.exit_logits(np.stack(s.H_d[:k]), 0))
                s.P_d = list(pd_ref)
                assert np.max(np.abs(Pd[b] - pd_ref)) / np.max(pd_ref) <= TOL["bf16"]
                O.o.verify_intermediate(s, (u_a[b], float(u_r[b])))
                pi_ref = eo.softmax_rows(O.o.last_logits)
                assert np.max(np.abs(Pt[b * (k + 1):(b + 1) * (k + 1)] - pi_ref)) / np.max(pi_ref) <= TOL["bf16"]
        if rnd % 2 == 1:
            nv = sess.counts()[1]
            Pi = [sess.read_dist(1, b, 0, int(nv[b])).astype(np.float64) for b in range(B)]
            V = [sess.tokens(b)[-int(nv[b]):].tolist() for b in range(B)]
            uf_a, uf_r = rng.random((B, rows), np.float32), rng.random(B, np.float32)
            gf, gfn, gcom = sess.verify_full_rs(uf_a, uf_r)
            Pf = sess.last_logits().astype(np.float64)
            r0 = 0
            for b in range(B):
                n = int(nv[b]) + 1
                f, out, mg = eo.rejection_verify(V[b], Pi[b], Pf[r0:r0 + n], uf_a[b], float(uf_r[b]))
                if mg > RS_MARGIN["f32"]:
                    assert (int(gf[b]), int(gfn[b]), gcom[b]) == (f, out[-1], out), (rnd, b)
                    checked += 1
                else:
                    skipped += 1
                r0 += n
    assert checked > 10 * max(1, skipped)
    sess.close(); model.close()


def test_chain_of_verifiers_under_the_sampling_rule_matches_oracle():
    """App. G's acceptance at every exit of a chain (L_d, L_i, one further verifier, L_f): drafting by sampling, then
    levels 1, 2 and 3 with the stochastic rule, in lockstep with the oracle's MultiLevelOracle on the same uniform
    numbers; decisions equal wherever the oracle's decision margin clears what fp32 summation order can move."""
    import paper_2510_01336_amd as hs
    cfg = synth.EEConfig(n_layers=8, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=688, vocab=1024,
                         exit_draft=2, exit_inter=4, exit_extra=(6,), rope_theta=10000.0, dtype="f32", gamma=(1.0, 0.3, 0.3))
    k, ctxs = 4, [40, 23]
    B, rows, margin = len(ctxs), 4 * (k + 2), RS_MARGIN["f32"]
    W = synth.WeightStore(cfg, 77)
    M = eo.MultiLevelOracle(eo.EEModel(eo.ModelSpec.from_config(cfg), W))
    prompts = [synth.gen_prompt(cfg.vocab, n, 300 + b) for b, n in enumerate(ctxs)]
    model, sess = gpu_side(cfg, 77, B, max(ctxs) + 16 * rows, rows)
    assert sess.n_levels() == 3
    sess.enable_sampling()
    first = sess.prefill(prompts)
    seqs = []
    for b, p in enumerate(prompts):
        s = eo.MultiSequence(M.spec, max(ctxs) + 16 * rows)
        M.prefill(s, p)
        s.C[-1] = int(first[b])
        seqs.append(s)
    rng = np.random.default_rng(9)
    plan = [[1], [1, 2], [1, 2, 3], [1, 2], [1], [1, 2, 3]]

    def trial(s, levels, u):
        t, worst = copy.deepcopy(s), np.inf
        M.draft(t, k, u["d"])
        worst = min(worst, M.last_margin)
        for lv in levels:
            M.verify_level(t, lv, (u[lv][0], u[lv][1]))
            worst = min(worst, M.last_margin)
        return worst

    accepted = rejected = 0
    for levels in plan:
        for _ in range(60):      # redraw the round's uniform numbers until every decision clears the margin
            us = [{"d": rng.random(k, np.float32), **{lv: (rng.random(rows, np.float32), float(rng.random(dtype=np.float32))) for lv in levels}}
                  for _b in range(B)]
            if all(trial(s, levels, us[b]) > margin for b, s in enumerate(seqs)):
                break
        else:
            pytest.fail("no draw cleared the margin")
        gS = sess.draft_sample(k, np.stack([u["d"] for u in us]))
        for b, s in enumerate(seqs):
            assert gS[b].tolist() == M.draft(s, k, us[b]["d"])
        for lv in levels:
            u_a = np.stack([us[b][lv][0] for b in range(B)])
            u_r = np.array([us[b][lv][1] for b in range(B)], np.float32)
            if lv == 1:
                ga, gn = sess.verify_intermediate_rs(u_a[:, :k], u_r)
            elif lv < 3:
                ga, gn, gm = sess.verify_level_rs(lv, u_a, u_r)
            else:
                ga, gn, gm = sess.verify_full_rs(u_a, u_r)
            for b, s in enumerate(seqs):
                n_src = len(s.S) if lv == 1 else len(s.V[lv - 1])
                a, nxt, moved = M.verify_level(s, lv, (us[b][lv][0], us[b][lv][1]))
                assert (int(ga[b]), int(gn[b])) == (a, nxt), (levels, lv, b)
                if lv > 1:
                    assert gm[b] == moved
                accepted += a; rejected += n_src - a
            lens = sess.lengths()
            for b, s in enumerate(seqs):
                assert list(lens[b]) == s.len and sess.tokens(b).tolist() == s.T
    assert accepted > 0 and rejected > 0
    # a buffer filled by the arg max calls has no stored law: the sampling call of the level above refuses it
    sess.draft(k); sess.verify_intermediate(); sess.verify_level(2)
    with pytest.raises(hs.EEError) as e:
        sess.verify_full_rs(rng.random((B, rows), np.float32), rng.random(B, np.float32))
    assert e.value.code == -2
    sess.verify_full()
    sess.close(); model.close()


@pytest.mark.gpu
def test_chain_loop_under_the_sampling_rule_runs_on_the_gpu():
    """The host loop over a chain of exits with App. G's acceptance at each (loop.hispec_generate_levels with rng):
    every call succeeds, each sequence gets its tokens, what the loop returns is what the session committed, and the
    same uniform numbers give the same stream again."""
    from paper_2510_01336_amd.loop import hispec_generate_levels
    cfg = synth.EEConfig(n_layers=8, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=688, vocab=1024,
                         exit_draft=2, exit_inter=4, exit_extra=(6,), rope_theta=10000.0, dtype="f32", gamma=(1.0, 0.3, 0.3))
    k, n_new, ctxs = 4, 20, [40, 23]
    prompts = [synth.gen_prompt(cfg.vocab, n, 300 + b) for b, n in enumerate(ctxs)]
    streams = []
    for rep in range(2):
        model, sess = gpu_side(cfg, 77, len(ctxs), max(ctxs) + n_new + 16 * (k + 2), 4 * (k + 2))
        sess.enable_sampling()
        sess.prefill(prompts)
        toks, stats = hispec_generate_levels(sess, n_new, k, [3, 4], rng=np.random.default_rng(21))
        assert toks.shape == (len(ctxs), n_new) and all(c > 0 for c in stats["calls"][1:])
        assert all(0 <= a <= c for a, c in zip(stats["accepted"][1:], stats["checked"][1:]))
        nc, _ = sess.counts()
        for b in range(len(ctxs)):
            committed = sess.tokens(b)[ctxs[b] + 1:int(nc[b])].tolist()
            assert committed[:n_new] == toks[b].tolist()
        streams.append(toks)
        sess.close(); model.close()
    assert np.array_equal(streams[0], streams[1])

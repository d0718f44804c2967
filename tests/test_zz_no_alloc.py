"""GPU: the verify call that allocates nothing (ee_verify_intermediate_static: all scratch of the call in the
library's static device array) against ee_verify_intermediate, through the C ABI, on two calls in a row, the
second with a smaller input; and its size limit."""
import numpy as np
import pytest

import synth
from hs_common import bf16_small, gpu_side

pytestmark = pytest.mark.gpu


def _both_ways(sess, drafts, starts):
    """The same pending block verified by the existing call and, after pruning back, by the static-scratch call."""
    out = []
    for static in (False, True):
        sess.draft_inject(drafts)
        a, n = sess.verify_intermediate_static() if static else sess.verify_intermediate()
        out.append((a.copy(), n.copy(), sess.last_logits().copy(), sess.last_hidden().copy(), sess.lengths().copy()))
        for b, n0 in enumerate(starts):
            sess.rollback(b, 0b011, n0)
    return out


def test_static_scratch_call_equals_the_arena_call():
    cfg = bf16_small()
    model, sess = gpu_side(cfg, 777, 2, 400, 20)
    sess.enable_logits(True)
    ctx = [150, 70]
    sess.prefill([synth.gen_prompt(cfg.vocab, n, 100 + b) for b, n in enumerate(ctx)])
    rng = np.random.default_rng(0)
    for k in (8, 3):                       # two calls in a row share the array; the second is the smaller one
        drafts = rng.integers(0, cfg.vocab, (2, k)).astype(np.int32)
        ref, got = _both_ways(sess, drafts, ctx)
        assert np.array_equal(ref[0], got[0]) and np.array_equal(ref[1], got[1])        # accept lengths, next tokens
        assert np.array_equal(ref[2], got[2]) and np.array_equal(ref[3], got[3])        # logits, hidden rows: same kernels
        assert np.array_equal(ref[4], got[4])
        assert ref[2].shape[0] >= 2 * (k + 1) and np.isfinite(ref[2]).all()
    # the session goes on as usual after a static-scratch call: a full verification of what it accepted
    drafts = rng.integers(0, cfg.vocab, (2, 4)).astype(np.int32)
    sess.draft_inject(drafts)
    a, n = sess.verify_intermediate_static()
    f, fn, com = sess.verify_full()
    assert all(len(c) >= 1 for c in com)
    sess.close(); model.close()


def test_static_scratch_at_the_8b_width_and_its_limit():
    """9 block rows at the 8B width (the benchmark's call shape) fit the 32 MiB array and give the arena call's
    results bit for bit; 16 x 9 rows need the row-tiled GEMM's K-share partials, which do not fit: refused, session
    unchanged, and the ordinary call then serves the same block."""
    import paper_2510_01336_amd as hs
    cfg = synth.llama8b_config(n_layers=3, exit_draft=1, exit_inter=2, gamma=(1.0, 0.3, 0.3))
    k = 8
    model = hs.Model(cfg, 20251001)
    sess = hs.Session(model, 1, 400, 2 * (k + 1) + 2)
    sess.enable_logits(True)
    sess.prefill([synth.gen_prompt(cfg.vocab, 300, 1)])
    rng = np.random.default_rng(1)
    drafts = rng.integers(0, cfg.vocab, (1, k)).astype(np.int32)
    ref, got = _both_ways(sess, drafts, [300])
    for r, g in zip(ref, got):
        assert np.array_equal(r, g)
    sess.close()
    B = 16
    sess = hs.Session(model, B, 128, 2 * (k + 1) + 2)
    sess.prefill([synth.gen_prompt(cfg.vocab, 20 + b, 50 + b) for b in range(B)])
    drafts = rng.integers(0, cfg.vocab, (B, k)).astype(np.int32)
    sess.draft_inject(drafts)
    before = (sess.lengths().tolist(), [sess.tokens(b).tolist() for b in range(B)])
    with pytest.raises(hs.EEError) as e:
        sess.verify_intermediate_static()
    assert e.value.code == -3
    assert (sess.lengths().tolist(), [sess.tokens(b).tolist() for b in range(B)]) == before
    a, n = sess.verify_intermediate()
    assert ((0 <= a) & (a <= k)).all()
    sess.close(); model.close()

"""Pins for the oracle's building blocks: library routines, closed forms, invariants.

None of these re-type the oracle's own formulas: each compares against a
torch library routine, a closed form, or a property the mathematics fixes.
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

from oracle import ee_oracle as eo

RNG = np.random.default_rng(1234)


def test_round_bf16_matches_library_rounding():
    x = np.concatenate([RNG.normal(size=4096), RNG.normal(size=256) * 1e-3, [0.0, 1.0, -1.0, 1.00390625, 1.001953125]])
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(eo.round_bf16(x), want)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert eo.round_bf16(np.array([1 + 2.0 ** -8]))[0] == 1.0
    assert eo.round_bf16(np.array([1 + 3 * 2.0 ** -8]))[0] == 1 + 2.0 ** -6


def test_rmsnorm_library_and_closed_form():
    x = RNG.normal(size=(5, 96))
    g = 1 + 0.1 * RNG.normal(size=96)
    want = Fn.rms_norm(torch.from_numpy(x), (96,), torch.from_numpy(g), 1e-5).numpy()
    np.testing.assert_allclose(eo.rmsnorm(x, g, 1e-5), want, rtol=1e-12, atol=1e-14)
    # constant vector c  ->  g * sign(c)  (up to eps)
    c = np.full((1, 96), -3.0)
    np.testing.assert_allclose(eo.rmsnorm(c, g, 1e-12), -g[None, :], rtol=1e-9)
    # scale invariance
    np.testing.assert_allclose(eo.rmsnorm(7.0 * x, g, 0.0), eo.rmsnorm(x, g, 0.0), rtol=1e-12)


def test_silu_library():
    x = RNG.normal(size=1000) * 4
    np.testing.assert_allclose(eo.silu(x), Fn.silu(torch.from_numpy(x)).numpy(), rtol=1e-12, atol=1e-15)
    assert eo.silu(np.array([0.0]))[0] == 0.0


def test_rope_properties():
    m, H, D, theta = 6, 3, 32, 10000.0
    x = RNG.normal(size=(m, H, D))
    # position 0 is the identity
    np.testing.assert_allclose(eo.rope(x, np.zeros(m), theta), x, atol=1e-15)
    pos = np.array([0, 1, 5, 17, 300, 40000])
    y = eo.rope(x, pos, theta)
    # rotations preserve the norm of every pair, hence of every head vector
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    # relative property: <R_p q, R_s k> = <R_{p-s} q, k>
    q, k = RNG.normal(size=(1, 1, D)), RNG.normal(size=(1, 1, D))
    for p, s in [(9, 4), (100, 99), (5, 5)]:
        lhs = np.sum(eo.rope(q, [p], theta) * eo.rope(k, [s], theta))
        rhs = np.sum(eo.rope(q, [p - s], theta) * k)
        np.testing.assert_allclose(lhs, rhs, rtol=1e-10, atol=1e-12)
    # the slowest pair (i = D/2-1 with i+D/2) turns by pos * theta^(-(D-2)/D); the fastest by pos
    e = np.zeros((1, 1, D)); e[0, 0, 0] = 1.0
    r = eo.rope(e, [1], theta)[0, 0]
    np.testing.assert_allclose([r[0], r[D // 2]], [np.cos(1.0), np.sin(1.0)], rtol=1e-12)
    e = np.zeros((1, 1, D)); e[0, 0, D // 2 - 1] = 1.0
    r = eo.rope(e, [3], theta)[0, 0]
    ang = 3 * theta ** (-(D - 2) / D)
    np.testing.assert_allclose([r[D // 2 - 1], r[D - 1]], [np.cos(ang), np.sin(ang)], rtol=1e-12)


def test_rope_matches_hf_library():
    from transformers import LlamaConfig
    from transformers.models.llama.modeling_llama import LlamaRotaryEmbedding, apply_rotary_pos_emb
    D, H, theta = 16, 2, 500000.0
    cfg = LlamaConfig(hidden_size=H * D, num_attention_heads=H, head_dim=D, rope_theta=theta,
                      max_position_embeddings=4096)
    rot = LlamaRotaryEmbedding(cfg).double()
    pos = np.array([0, 3, 77, 2047])
    x = RNG.normal(size=(len(pos), H, D))
    xt = torch.from_numpy(x).permute(1, 0, 2)[None]                     # [1, H, m, D]
    cos, sin = rot(xt, torch.from_numpy(pos)[None])
    got_hf, _ = apply_rotary_pos_emb(xt, xt, cos.double(), sin.double())
    got, want = eo.rope(x, pos, theta), got_hf[0].permute(1, 0, 2).numpy()
    # the library builds its angle table in float32: error grows like pos * 2^-24
    np.testing.assert_allclose(got[:3], want[:3], rtol=0, atol=2e-5)
    np.testing.assert_allclose(got[3], want[3], rtol=0, atol=5e-4)


def _sdpa(q, K, V, qpos):
    m, Hq, D = q.shape
    n, Hkv, _ = K.shape
    rep = Hq // Hkv
    qt = torch.from_numpy(q).permute(1, 0, 2)[None]
    kt = torch.from_numpy(K).permute(1, 0, 2)[None].repeat_interleave(rep, dim=1)
    vt = torch.from_numpy(V).permute(1, 0, 2)[None].repeat_interleave(rep, dim=1)
    mask = torch.from_numpy(np.arange(n)[None, :] <= np.asarray(qpos)[:, None])
    o = Fn.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask)
    return o[0].permute(1, 0, 2).numpy()


def test_attention_matches_library_sdpa():
    m, Hq, Hkv, D, n = 5, 8, 2, 16, 37
    q, K, V = RNG.normal(size=(m, Hq, D)), RNG.normal(size=(n, Hkv, D)), RNG.normal(size=(n, Hkv, D))
    qpos = np.arange(n - m, n)            # a block of m new rows at the end of the cache
    np.testing.assert_allclose(eo.attention(q, K, V, qpos), _sdpa(q, K, V, qpos), rtol=1e-10, atol=1e-12)


def test_attention_closed_forms():
    Hq, Hkv, D = 4, 2, 8
    # a single cached position: the output is that V row, whatever q is
    q, K, V = RNG.normal(size=(1, Hq, D)), RNG.normal(size=(1, Hkv, D)), RNG.normal(size=(1, Hkv, D))
    out = eo.attention(q, K, V, np.array([0]))
    for h in range(Hq):
        np.testing.assert_allclose(out[0, h], V[0, h // 2], rtol=1e-12)
    # zero query: uniform weights -> mean of the allowed V rows
    n = 9
    K, V = RNG.normal(size=(n, Hkv, D)), RNG.normal(size=(n, Hkv, D))
    out = eo.attention(np.zeros((2, Hq, D)), K, V, np.array([5, 8]))
    np.testing.assert_allclose(out[0, 3], V[:6, 1].mean(axis=0), rtol=1e-12)
    np.testing.assert_allclose(out[1, 0], V[:9, 0].mean(axis=0), rtol=1e-12)


def test_attention_is_causal_inside_the_block():
    m, Hq, Hkv, D, n = 4, 4, 4, 8, 12
    q, K, V = RNG.normal(size=(m, Hq, D)), RNG.normal(size=(n, Hkv, D)), RNG.normal(size=(n, Hkv, D))
    qpos = np.arange(n - m, n)
    base = eo.attention(q, K, V, qpos)
    K2, V2 = K.copy(), V.copy()
    K2[-1] += 5.0; V2[-1] -= 3.0          # only the last row may see the last position
    out = eo.attention(q, K2, V2, qpos)
    np.testing.assert_array_equal(out[:-1], base[:-1])
    assert np.abs(out[-1] - base[-1]).max() > 1e-3


def _cases(golden_dir):
    path = os.path.join(golden_dir, "leading_substring_cases.txt")
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        S, v, a, out = [[int(t) for t in part.split()] for part in line.split("|")]
        yield S, v, a[0], out


def test_leading_substring_verify_golden(golden_dir):
    n = 0
    for S, v, a, out in _cases(golden_dir):
        assert eo.leading_substring_verify(S, v) == (a, out)
        n += 1
    assert n == 5


def test_leading_substring_verify_bruteforce():
    """Against the definition: k* = min{k : S_k != v_k} else |S|+1, searched exhaustively."""
    import itertools
    for n in range(0, 4):
        for S in itertools.product(range(2), repeat=n):
            for v in itertools.product(range(2), repeat=n + 1):
                mism = [k for k in range(1, n + 1) if S[k - 1] != v[k - 1]]
                kstar = min(mism) if mism else n + 1
                want = list(S[:kstar - 1]) + [v[kstar - 1]]
                a, out = eo.leading_substring_verify(S, v)
                assert a == kstar - 1 and out == want


def test_argmax_tie_goes_to_lowest_id():
    lg = np.array([[0.0, 2.0, 2.0, 1.0], [3.0, 3.0, 3.0, 3.0]])
    assert list(eo.argmax_rows(lg)) == [1, 0]
    np.testing.assert_allclose(eo.top2_margin(np.array([[0.0, 2.5, 2.0, 1.0]])), [0.5])

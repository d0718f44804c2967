"""The seeded input generators: determinism, slicing, distribution, closed forms."""
import numpy as np
import pytest

import synth
from synth import model as sm


def test_generator_is_deterministic_and_sliceable():
    cfg = synth.tiny_config()
    a = synth.gen_tensor(cfg, 5, "wgate", 2)
    b = synth.gen_tensor(cfg, 5, "wgate", 2)
    assert np.array_equal(a, b)
    rows = synth.gen_tensor_rows(cfg, 5, "wgate", 2, 100, 7)
    assert np.array_equal(rows, a[100:107])
    assert not np.array_equal(a, synth.gen_tensor(cfg, 6, "wgate", 2))
    assert not np.array_equal(a, synth.gen_tensor(cfg, 5, "wup", 2))
    assert not np.array_equal(a, synth.gen_tensor(cfg, 5, "wgate", 1))


def test_generator_matches_scalar_restatement():
    """One element recomputed with Python integers (independent of the vectorised uint64 code)."""
    cfg = synth.tiny_config()
    seed, name, layer, e = 77, "wo", 3, 12345
    key = sm.stream_key(seed, sm.TENSOR_IDS[name], layer)
    mask = (1 << 64) - 1
    s = 0
    for j in range(3):
        w = sm._mix64_scalar((key + (3 * e + j + 1) * 0x9E3779B97F4A7C15) & mask)
        s += sum((w >> (16 * i)) & 0xFFFF for i in range(4))
    want = np.float32(s - 393210) * (np.float32(0.02) * np.float32(1.0) * np.float32(2.0 ** -16))
    got = sm.gen_flat(cfg, seed, name, layer, e, 1)[0]
    assert got == np.float32(want)


def test_distribution_moments():
    cfg = synth.tiny_config()
    w = synth.gen_tensor(cfg, 1, "head").ravel()
    assert abs(w.mean()) < 2e-4
    assert abs(w.std() / 0.02 - 1) < 0.01
    # Irwin-Hall(12): excess kurtosis -0.1
    k = ((w - w.mean()) ** 4).mean() / w.var() ** 2 - 3
    assert abs(k + 0.1) < 0.05
    g = synth.gen_tensor(cfg, 1, "g1", 0)
    assert abs(g.mean() - 1) < 0.01 and abs(g.std() / 0.02 - 1) < 0.2


def test_gamma_scales_only_residual_writers():
    c1 = synth.tiny_config()
    c2 = synth.tiny_config(gamma=(1.0, 0.5, 0.25))
    for name in ("wq", "wgate", "g1"):
        assert np.array_equal(synth.gen_tensor(c1, 3, name, 3), synth.gen_tensor(c2, 3, name, 3))
    assert np.array_equal(synth.gen_tensor(c1, 3, "wo", 0), synth.gen_tensor(c2, 3, "wo", 0))
    np.testing.assert_allclose(synth.gen_tensor(c2, 3, "wo", 1), 0.5 * synth.gen_tensor(c1, 3, "wo", 1), rtol=1e-6)
    np.testing.assert_allclose(synth.gen_tensor(c2, 3, "wdown", 3), 0.25 * synth.gen_tensor(c1, 3, "wdown", 3), rtol=1e-6)


def test_bf16_values_are_representable_and_rne():
    import torch
    cfg = synth.tiny_config(dtype="bf16")
    w = synth.gen_tensor(cfg, 9, "wq", 1)
    assert np.array_equal(w.view(np.uint32) & 0xFFFF, np.zeros_like(w, dtype=np.uint32))
    raw = synth.gen_tensor(synth.tiny_config(), 9, "wq", 1)
    want = torch.from_numpy(raw).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(w, want)
    bits = synth.f32_to_bf16_bits(raw)
    assert np.array_equal(synth.bf16_bits_to_f32(bits), want)


def test_shapes_of_paper_sized_models():
    c8, c70 = synth.llama8b_config(), synth.llama70b_config()
    per_layer = lambda c: sum(int(np.prod(synth.tensor_shape(c, n))) for n in sm.LAYER_TENSORS if n not in ("g1", "g2"))
    assert per_layer(c8) == 218_103_808
    assert per_layer(c70) == 855_638_016
    assert synth.tensor_shape(c8, "head") == (128256, 4096)


def test_prompt_and_lengths():
    p = synth.gen_prompt(1024, 32, 7)
    assert p.shape == (32,) and p.min() >= 0 and p.max() < 1024
    assert np.array_equal(p, synth.gen_prompt(1024, 32, 7))
    L = synth.gen_context_lengths(4096, 3)
    assert L.min() >= 128 and L.max() <= 4096
    assert abs(np.median(L) / 1024 - 1) < 0.08


@pytest.mark.parametrize("k,p", [(8, 0.8), (16, 0.9), (8, 0.5)])
def test_draft_block_agreement_law(k, p):
    """Mean accepted length of generated blocks -> p (1 - p^k) / (1 - p)."""
    rng = np.random.default_rng(11)
    greedy = np.arange(100, 100 + k)
    acc = []
    for _ in range(20000):
        S = synth.make_draft_block(greedy, k, p, 1000, rng)
        a = 0
        while a < k and S[a] == greedy[a]:
            a += 1
        acc.append(a)
    want = synth.expected_accept_len(k, p)
    assert abs(np.mean(acc) - want) < 0.05
    assert abs(synth.expected_accept_len(8, 0.8) - 3.3289) < 1e-3
    assert abs(synth.expected_accept_len(16, 0.9) - 7.332) < 1e-2


def test_draft_block_forced_mismatch():
    rng = np.random.default_rng(1)
    greedy = np.array([4, 4, 4, 4])
    for a in range(5):
        S = synth.make_draft_block(greedy, 4, 0.5, 8, rng, first_mismatch=a)
        assert list(S[:a]) == [4] * a
        if a < 4:
            assert S[a] != 4 and 0 <= S[a] < 8


def test_compiled_generator_equals_numpy_generator():
    """synth/gen_fast.c (built by the build entry point) restates the recipe of synth/model.py: same bits for
    fp32 and bf16 models, plain matrices, damped ones, gains and adapter tensors, at offsets inside a tensor."""
    import pytest
    from synth import model as sm
    if not sm._fast_lib():
        pytest.skip("synth/libsynthgen.so has not been built")
    for cfg in (synth.tiny_config(gamma=(1.0, 0.5, 0.25), head_rank=24),
                synth.llama8b_config(n_layers=3, exit_draft=1, exit_inter=2, gamma=(1.0, 0.3, 0.1), head_rank=64)):
        for name, layer in (("emb", 0), ("head", 0), ("gfinal", 0), ("g1", 1), ("wq", 2), ("wo", 1), ("wo", 2),
                            ("wdown", 2), ("wgate", 0), ("aux_g", 1), ("aux_a", 0), ("aux_b", 1)):
            rows = synth.tensor_shape(cfg, name)[0]
            r0, n = min(5, rows - 1), min(37, rows - min(5, rows - 1))
            a = sm.gen_tensor_rows(cfg, 20251001, name, layer, r0, n)
            b = sm.gen_tensor_rows(cfg, 20251001, name, layer, r0, n, use_fast=False)
            assert a.dtype == b.dtype == np.float32 and a.shape == b.shape
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), (cfg.dtype, name, layer)
            wide = sm.gen_tensor_rows(cfg, 20251001, name, layer, r0, n, dtype=np.float64)
            assert wide.dtype == np.float64 and np.array_equal(wide, b.astype(np.float64))

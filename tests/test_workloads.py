"""Host-side checks of the seeded input generators."""

import numpy as np
import torch

from workloads import synth


def test_draw_ranks_constraints_and_determinism():
    for seed in range(5):
        for stream in (0, 1):
            r = synth.draw_ranks(seed, stream, 8)
            assert sum(r) == 2048 and len(r) == 8
            assert all(96 <= v <= 416 and v % 32 == 0 for v in r)
            assert r == synth.draw_ranks(seed, stream, 8)
    assert synth.draw_ranks(0, 0, 8) != synth.draw_ranks(0, 1, 8)


def test_round_to_matches_torch():
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 37.0
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-5]          # ties and small values
    t = torch.from_numpy(x)
    np.testing.assert_array_equal(synth.round_to(x, "bf16"), t.to(torch.bfloat16).float().numpy())
    np.testing.assert_array_equal(synth.round_to(x, "f16"), t.to(torch.float16).float().numpy())


def test_config_layers():
    l2 = synth.config_layer("2")
    assert l2.n_groups == 8 and l2.R_k == 2048 and l2.R_v == 2048 and l2.b_elems("k") == 8 * 256 * 512
    l3 = synth.config_layer("3")
    assert l3.R_k == 2048 and l3.R_v == 2048 and l3.n_groups == 8
    assert synth.config_layer("5a").n_groups == 32 and synth.config_layer("5b").n_groups == 1
    assert synth.config_layer("5b").b_elems("k") == 2048 * 4096


def test_cases_are_representable_and_seeded():
    layer = synth.uniform_layer(4, 2, 32, d_head=32)
    a = synth.make_case_svd(layer, 2, 40, seed=3, d_model=128)
    b = synth.make_case_svd(layer, 2, 40, seed=3, d_model=128)
    for name in ("q", "Hk", "Hv", "Bk", "Bv", "Ak", "Av"):
        va, vb = getattr(a, name), getattr(b, name)
        np.testing.assert_array_equal(va, vb)
        np.testing.assert_array_equal(va, va.astype(np.float16).astype(np.float32))
    c = synth.make_case_orthonormal(layer, 1, 16, seed=0, dtype="bf16")
    np.testing.assert_array_equal(c.Hk, synth.round_to(c.Hk, "bf16"))
    # orthonormal rows scaled by sqrt(width / r)
    B0 = synth.make_orthonormal_B(layer, 0, "k")[: 32 * 64].reshape(32, 64)
    np.testing.assert_allclose(B0 @ B0.T, np.eye(32) * 2.0, atol=1e-12)

"""The seeded input generator: deterministic, correctly rounded, and shaped like the stated workloads."""
import numpy as np
import torch

from paper_2603_22276_amd import inputs as I


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(100000) * np.exp(rng.uniform(-20, 20, 100000))).astype(np.float32)
    a[:4] = [0.0, -0.0, np.inf, -np.inf]
    ours = I.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    back = I.bf16_bits_to_f32(ours)
    assert np.array_equal(back, torch.from_numpy(a).to(torch.bfloat16).float().numpy())
    # ties to even: 1 + 2^-8 is exactly halfway between 1 and 1 + 2^-7
    assert I.f32_to_bf16_bits(np.array([1 + 2.0 ** -8], np.float32))[0] == 0x3F80
    assert I.f32_to_bf16_bits(np.array([1 + 3 * 2.0 ** -8], np.float32))[0] == 0x3F82


def test_c1_recipe_and_determinism():
    a = I.make_inputs(I.C1)
    b = I.make_inputs(I.C1)
    for k in ("W", "A", "B", "m", "x", "dy"):
        assert np.array_equal(a[k], b[k])
    assert a["W"].shape == (256, 512) and a["A"].shape == (16, 512) and a["B"].shape == (256, 16)
    assert a["x"].shape == (64, 512) and a["dy"].shape == (64, 256) and a["m"].dtype == np.float32
    assert float(a["s"]) == 4.0 and a["eps"] == 1e-12
    assert abs(a["W"].std() * np.sqrt(512) - 1) < 0.02
    assert abs(a["B"].std() / 1e-2 - 1) < 0.05
    ratio = a["m"] / np.linalg.norm(a["W"].astype(np.float64), axis=1)
    assert abs(ratio.mean() - 1) < 5e-4 and 5e-4 < ratio.std() < 2e-3


def test_bf16_config_storage_and_stress_variant():
    cfg = I.C2.scaled(d_out=128, d_in=256, tokens=32, r=32)
    a = I.make_inputs(cfg)
    assert a["W"].dtype == np.uint16 and a["x"].dtype == np.uint16 and a["eps"] == 1e-6
    assert np.isclose(float(a["s"]), 32 / np.sqrt(32))
    st = I.stress(cfg)
    assert np.isclose(float(st.s) ** 2 * st.r * st.sigma_B ** 2, 1.0)
    assert len({I.c5_module(i, r).seed_offset for i in range(7) for r in (64, 384, 768)}) == 21

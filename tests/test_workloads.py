"""Input generators: determinism, dtypes, rounding.  CPU only."""
import numpy as np
import torch

import workloads


def test_deterministic_and_shapes():
    a = workloads.make(workloads.CONFIGS["C1"])
    b = workloads.make(workloads.CONFIGS["C1"])
    for key in ("W", "X", "Ip01", "Iz01"):
        assert np.array_equal(a[key], b[key])
    assert a["W"].shape == (500, 800) and a["W"].dtype == np.float32
    assert a["X"].shape == (800, 1)
    assert a["Ip01"].shape == (40, 100, 4) and a["Iz01"].shape == (40, 4, 100)
    assert set(np.unique(a["Ip01"])) <= {0, 1}


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(20000) * 3).astype(np.float32)
    bits = workloads.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = workloads.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_storage_roundtrip_exact():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(1000).astype(np.float32)
    for dt in ("f32", "f16", "bf16"):
        s = workloads.to_storage(x, dt)
        w = workloads.to_float64(s, dt)
        assert np.array_equal(workloads.to_storage(w, dt), s)


def test_factor_density():
    cfg = workloads.CONFIGS["C2"]
    d = workloads.make_factors_only(cfg)
    assert abs(d["Ip01"].mean() - cfg.p) < 0.002 and abs(d["Iz01"].mean() - cfg.p) < 0.002

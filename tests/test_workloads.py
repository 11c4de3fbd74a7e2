"""The synthetic input recipe: shapes, dtypes, determinism and the stated value structure (CPU only)."""
import numpy as np
import torch

from paper_2410_06577_amd import workloads as wl


def test_tiny_config_shapes_and_structure():
    d = wl.make_scan_inputs(wl.TINY)
    assert d["q"].shape == (1, 64, 1, 16) and d["v"].shape == (1, 64, 1, 32)
    assert d["q"].dtype == torch.float32 and d["log_alpha"].dtype == torch.float32
    assert d["S0"] is None
    assert (d["log_alpha"] <= 0).all() and (d["beta"] > 0).all() and (d["beta"] < 1).all()
    np.testing.assert_allclose(d["k"].double().norm(dim=-1).numpy(), 1.0, rtol=1e-5)


def test_bf16_config_and_seed_determinism():
    w = wl.shrink(wl.LAYER_1P6B, B=1, T=128, H=2)
    a, b = wl.make_scan_inputs(w), wl.make_scan_inputs(w)
    assert a["q"].dtype == torch.bfloat16 and a["beta"].dtype == torch.float32
    assert a["S0"].shape == (1, 2, 64, 256) and abs(float(a["S0"].std()) - 0.1) < 0.01
    for key in ("q", "k", "v", "log_alpha", "beta", "S0"):
        assert torch.equal(a[key], b[key])
    c = wl.make_scan_inputs(wl.shrink(w, seed=99))
    assert not torch.equal(a["q"], c["q"])


def test_long_context_gates_are_near_zero():
    d = wl.make_scan_inputs(wl.shrink(wl.LONG_CONTEXT, T=256, H=2))
    la = d["log_alpha"]
    assert -0.05 < float(la.mean()) < -0.01          # -softplus(N(-4,1)), tau == 1


def test_decode_inputs():
    w = wl.DecodeWorkload("d", N=3, H=2, dk=64, dv=256, steps=5, ring=2)
    d = wl.make_decode_inputs(w)
    assert d["S"].shape == (3, 2, 64, 256) and d["S"].dtype == torch.float32
    assert len(d["ring"]) == 2 and d["ring"][0]["v"].shape == (3, 2, 256)
    assert d["ring"][0]["q"].dtype == torch.bfloat16

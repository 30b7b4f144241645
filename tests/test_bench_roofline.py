"""Host-side checks of the benchmark's roofline arithmetic (no GPU): the figures of the gemm_xw launch
follow from the workload's shape and the event times alone, and the headline roof is the one that binds."""
import types

import pytest

import bench
from synth import workloads as W


def _args(**kw):
    a = types.SimpleNamespace(recompute=False, wgrad="pool", workload="C5")
    a.__dict__.update(kw)
    return a


def _agg(w, steps, xw_ms, wg_ms):
    # one bracket per expert_ffn_fwd / expert_ffn_bwd call, each holding two gemm_xw launches
    n = w.L * steps
    return {"expert_ffn_fwd": [2 * xw_ms] * n, "expert_ffn_bwd": [2 * xw_ms] * n, "expert_wgrad": [wg_ms] * steps,
            "route": [0.05] * n, "permute": [0.06] * n, "combine": [0.05] * (2 * n), "combine_bwd": [0.1] * n,
            "route_bwd": [0.15] * n}


def test_gemm_xw_launch_figures_follow_from_the_shape():
    w = W.WORKLOADS["C5"]
    steps, xw_ms = 3, 1.3
    xw, others = bench.roofline_of(w, _args(), None, _agg(w, steps, xw_ms, 53.0), steps)
    S = w.T * w.k
    assert xw["launches"] == 4 * w.L * steps
    assert xw["avg_launch_ms"] == pytest.approx(xw_ms)
    assert xw["flops_per_launch"] == pytest.approx(3.0 * S * w.d * w.f)            # (fwd + dgrad) / 4 launches
    assert xw["algorithmic_bytes_per_launch"] == pytest.approx((12.0 * w.E * w.d * w.f + 8.0 * S * w.d + 20.0 * S * w.f) / 4)
    assert xw["achieved"] == pytest.approx(xw["flops_per_launch"] / (xw_ms * 1e-3) / 1e12)
    assert xw["frac"] == pytest.approx(xw["achieved"] / 2500.0)
    # 341 rows per expert: below the ridge point, the HBM time is the longer one
    fl = xw["floor"]
    assert fl["longer"] == "hbm" and fl["t_hbm_ms"] > fl["t_mfma_ms"]
    assert fl["frac_of_longer"] == pytest.approx(fl["t_hbm_ms"] / xw_ms)
    # pooled weight gradient: a third of the GEMM work of the step
    assert others["wgrad_pool"]["TFLOP/s"] == pytest.approx(6.0 * S * w.d * w.f * w.L / (53.0e-3) / 1e12)
    assert others["route"]["algorithmic_bytes"] == 2 * w.T * w.d + 4 * w.T * w.E + 8 * w.T * w.k


def test_headline_roofline_is_the_binding_roof():
    w = W.WORKLOADS["C5"]
    xw, _ = bench.roofline_of(w, _args(), None, _agg(w, 2, 1.3, 53.0), 2)
    r = bench.xw_roofline(xw, "C5")
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert r["frac"] == pytest.approx(r["achieved"] / r["peak"]) == pytest.approx(xw["floor"]["frac_of_longer"])
    assert r["mfma"]["frac"] == pytest.approx(xw["frac"]) and r["mfma"]["peak"] == 2500.0
    assert r["traffic"] is not None and "profiles/" in r["traffic_source"]
    # a launch above the ridge point is reported against the MFMA roof
    dense = dict(xw)
    dense["floor"] = dict(xw["floor"], longer="mfma")
    r2 = bench.xw_roofline(dense, "none")
    assert r2["bound"] == "mfma" and r2["unit"] == "TFLOP/s" and r2["traffic"] is None

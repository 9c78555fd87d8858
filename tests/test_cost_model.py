"""The flop/byte accounting reproduces the numbers the paper prints (tests/golden/cost_model.txt)."""
import os

from paper_2602_10378_amd import cost_model as cm


def _golden():
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "cost_model.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) == 3:
                out[line[0]] = (float(line[1]), float(line[2]))
    return out


def test_paper_cost_model_values():
    g = _golden()
    got = {
        "flops_coeff_d16": cm.paper_flops_coeff(16),
        "bytes_per_tile": cm.paper_bytes_per_tile(64, 1024, 16),
        "bytes_coeff_d16": cm.paper_bytes_coeff(64, 1024, 16),
        "intensity_d16": cm.paper_flops_coeff(16) / cm.paper_bytes_coeff(64, 1024, 16),
        "flops_coeff_1d": cm.paper_flops_1d(8) / 64.0,
        "intensity_coeff_1d": cm.paper_intensity_1d(1000) / 1000.0,
    }
    for key, val in got.items():
        want, tol = g[key]
        assert abs(val - want) <= tol, (key, val, want)
    want, rel = g["flops_32k_d16"]
    assert abs(cm.paper_flops(32768, 16) - want) <= rel * want


def test_pair_count_matches_metric_definition():
    assert cm.pair_interactions(1048576, 131072) == 1048576.0**2 + 131072.0 * 1048576.0
    s, e = cm.mfma_flops(32768, 4096, 16)
    assert s == 64.0 * 32768**2 and e == 32.0 * 4096 * 32768


def test_mi355x_roofline_accounting():
    """The roofline bench.py reports: the bound is the resource that needs the longest at its published peak, frac is
    its work over the measured time over that peak.  Spot values: the figures of the first measured runs, recomputed
    by hand (4 d n^2 flops in 580.49 ms = 121.2 TFLOP/s = 0.771 of 157.3; eval 2 d m n in 43.43 ms = 0.644; the 1-D
    score, 8 vector slots per pair, 150.8 us = 0.72 of 78.6 T lane-slots/s)."""
    n, m = 1048576.0, 131072.0
    r = cm.roofline("score", 16, n * n, 580.49e-3)
    assert r["bound"] == "mfma" and r["resource"] == "mfma_f32" and r["peak"] == 157.3
    assert abs(r["achieved"] - 121.2) < 0.05 and abs(r["frac"] - 0.771) < 5e-4
    assert abs(r["frac_by_resource"]["mfma_f32"] - r["frac"]) < 1e-12 and r["frac_by_resource"]["alu"] < r["frac"]
    r = cm.roofline("eval", 16, m * n, 43.43e-3)
    assert abs(r["achieved"] - 101.3) < 0.05 and abs(r["frac"] - 0.644) < 5e-4
    r = cm.roofline("score", 1, 32768.0**2, 150.8e-6, thin=True)
    assert r["bound"] == "alu" and abs(r["frac"] - 0.724) < 2e-3 and abs(r["peak"] - 78.6432) < 1e-9
    # the lower-precision modes price each contraction at the peak of the units it runs on
    w = cm.pair_work("score", 16, "fp16x2")
    assert (w["mfma_f32"], w["mfma_f16"]) == (32.0, 128.0)          # Phi X stays fp32; (hi + lo)(hi + lo) = 4 products
    assert cm.pair_work("score", 16, "fp16x2_all")["mfma_f16"] == 256.0 and cm.pair_work("score", 16, "fp16x2_phi16")["mfma_f16"] == 192.0
    assert cm.pair_work("score", 16, "symmetric")["mfma_f32"] == 48.0 and cm.pair_work("score", 16, "symmetric")["exp"] == 0.5
    assert cm.roofline("score", 16, n * n, 0.375, "fp16x2")["resource"] == "mfma_f32"
    assert cm.roofline("score", 16, n * n, 0.26, "fp16x2_all")["resource"] == "mfma_f16"

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

"""Runtime and utilisation sweeps in the shapes of the paper's figures, through the GPU library.

  Results, 16-D runtime and utilisation sweep:   n_train in {2k, 4k, 8k, 16k, 32k}, n_test = n_train / 8, d = 16
  Appendix on low dimensions (1-D sweep):        n_train = powers of two from 1024 to 64k, n_test = n_train / 8, three seeds
  Results, runtime of the Laplace-corrected KDE: the fused Laplace-corrected evaluation beside the plain KDE and the whole
                                                 SD-KDE pass on the same shapes

Per shape: the whole SD-KDE pass (score at the samples, shift, KDE of the shifted samples; one sdkde_fit_eval call), the
plain KDE and the Laplace-corrected KDE of the raw samples at the same queries;
utilisation as the paper computes it (its flop model over the measured time, as a share of the matrix peak; for d = 1 its
1-D model over the vector peak) and as the share of the time the bound resource needs at MI355X's published peaks.
Inputs are the synthetic mixtures of the benchmark configs (sdkde_inputs), three seeds, median over seeds.

  python -m paper_2602_10378_amd.sweep        prints the two tables as markdown
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from . import cost_model as cm


def _ms(fn, reps: int) -> float:
    """ms per call: best of three runs of `reps` back-to-back calls by the host clock between synchronisations (an event
    after every call would add ~15 us to each, more than a third of the smallest shapes)."""
    import time
    for _ in range(5):
        fn()
    best = float("inf")
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        best = min(best, (time.perf_counter() - t0) / reps * 1e3)
    return best


def bound_seconds(n: int, m: int, d: int) -> float:
    """Time the score and eval main kernels need at the published peaks (the bound resource of each stage)."""
    total = 0.0
    for stage, rows in (("score", n), ("eval", m)):
        plan = B.sdkde_describe_plan(n, rows, d, 0 if stage == "score" else 2)
        r = cm.roofline(stage, d, float(rows) * n, 1.0, "fp32", bool(plan["thin"]))
        total += max(r["seconds_at_peak"].values())
    return total


def measure(name: str, n: int, m: int, seed: int, reps: int):
    import sdkde_inputs
    x, q, h = sdkde_inputs.make(name, seed=seed, n=n, m=m)
    d = x.shape[1]
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    ws = B.make_workspace(n, m, d, device=xd.device)
    s, x_sd = torch.empty_like(xd), torch.empty_like(xd)
    dens, logd = torch.empty(m, device="cuda"), torch.empty(m, device="cuda")

    def sd_kde():
        B.sdkde_fit_eval(xd, qd, h, score_out=s, samples_sd_out=x_sd, density_out=dens, log_density_out=logd, workspace=ws)

    def kde():
        B.sdkde_eval(xd, qd, h, density_out=dens, workspace=ws)

    def laplace():
        B.sdkde_eval_laplace(xd, qd, h, density_out=dens, workspace=ws)

    return {"d": d, "sd_kde_ms": _ms(sd_kde, reps), "kde_ms": _ms(kde, reps), "laplace_ms": _ms(laplace, reps)}


def sweep(name: str, sizes, seeds=(0, 1, 2), reps: int = 100):
    """[{n, m, d, <median over seeds of every timing>, utilisation figures}] for config `name`'s mixture."""
    rows = []
    for n in sizes:
        m = n // 8
        runs = [measure(name, n, m, seed, reps) for seed in seeds]
        row = {"n": n, "m": m, "d": runs[0]["d"]}
        for key in ("sd_kde_ms", "kde_ms", "laplace_ms"):
            row[key] = float(np.median([r[key] for r in runs]))
        d, sec = row["d"], row["sd_kde_ms"] * 1e-3
        row["pairs_per_s"] = cm.pair_interactions(n, m) / sec
        flops = cm.paper_flops_1d(n) if d == 1 else cm.paper_flops(n, d, m)
        row["paper_model_utilisation"] = flops / sec / cm.PEAK_MFMA_F32          # the vector peak is the same figure
        row["share_of_bound"] = bound_seconds(n, m, d) / sec
        rows.append(row)
    return rows


def markdown(rows, title):
    lines = [f"**{title}**", "",
             "| n_train | n_test | SD-KDE pass | pairs/s | paper's flop model / peak | time of the bound resource at peak / time | "
             "plain KDE | Laplace-corrected KDE (fused) | SD-KDE / Laplace |", "|---|---|---|---|---|---|---|---|---|"]
    for r in rows:
        lines.append(f"| {r['n']} | {r['m']} | {r['sd_kde_ms']:.4g} ms | {r['pairs_per_s']:.3g} | "
                     f"{r['paper_model_utilisation']:.3f} | {r['share_of_bound']:.3f} | {r['kde_ms']:.4g} ms | {r['laplace_ms']:.4g} ms | "
                     f"{r['sd_kde_ms'] / r['laplace_ms']:.1f}× |")
    return "\n".join(lines)


def main():
    B.load()
    print(markdown(sweep("C1", (2048, 4096, 8192, 16384, 32768)), "16-D mixture, n_test = n_train / 8 (the paper's 16-D runtime and utilisation sweep)"))
    print()
    print(markdown(sweep("C3", tuple(2 ** p for p in range(10, 17))), "1-D mixture, n_test = n_train / 8 (the paper's 1-D sweep)"))


if __name__ == "__main__":
    main()

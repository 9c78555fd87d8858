"""Benchmark of the SD-KDE hot path on one MI355X.

A step is one pass of the whole path (score at all samples -> debias -> KDE at the queries)
over one synthetic batch that is already resident in HBM.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C5] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
# HBM bytes per launch of the score main kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch,
# read counter x2 and write counter x1 after calibration on the debias kernel): profiles/pipeline_<config>_*.txt
SCORE_KERNEL_TRAFFIC_BYTES = {"C5": (4586089.0 * 2 + 557056.0) * 1024, "C4": (2387123.2 * 2 + 532480.0) * 1024}
# The paper's two timed shapes (one RTX A6000, TF32 dots), keyed by (config, n, m): seconds end to end.
PAPER_SECONDS = {("C5", 1048576, 131072): 2.3,        # abstract / conclusion
                 ("C2", 32768, 4096): 2.11e-3}        # runtime table of the Results section (run with --config C2 --m 4096)


def cpu_baseline(x, q, h, budget_s=15.0):
    """Times the double-precision oracle (as is) on a bounded sample of the same workload:
    the first r score rows against all n samples plus the first r*m/n queries against all n
    shifted samples, r sized from a short calibration so the whole leg takes ~budget_s."""
    import numpy as np
    import oracle
    n, d = x.shape
    m = q.shape[0]
    cal_rows, rate = 16, 0.0
    while True:                      # calibrate on a run long enough to amortise thread start-up
        cal_rows = min(n, cal_rows * 4)
        t0 = time.perf_counter()
        oracle.score(x, h, points=x[:cal_rows])
        cal = time.perf_counter() - t0
        rate = cal_rows * n / max(cal, 1e-9)
        if cal >= 0.5 or cal_rows == n:
            break
    rows = int(min(n, max(cal_rows, budget_s * rate / (n * (1.0 + m / n)))))
    qrows = int(min(m, max(1, round(rows * m / n))))
    t0 = time.perf_counter()
    s_rows = oracle.score(x, h, points=x[:rows])
    # eval leg: the shifted samples are an input here; any point set of the same shape costs
    # the same, so the unshifted samples stand in for them in the timing
    oracle.eval_log_density(x, q[:qrows], h)
    dt = time.perf_counter() - t0
    pairs = float(rows) * n + float(qrows) * n
    return {
        "value": pairs / dt, "unit": "pairs/s", "cores": oracle.threads(), "kind": "oracle",
        "sample": f"first {rows} of {n} score rows + first {qrows} of {m} queries, each against all {n} samples "
                  f"({pairs:.3g} pairs in {dt:.1f} s, fp64)",
    }, s_rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="C5")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--n", type=int, default=None, help="override the config's sample count (same distribution)")
    ap.add_argument("--m", type=int, default=None, help="override the config's query count")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-modes", action="store_true", help="skip the separately reported fp16x2-input mode")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build is single-GPU; run with --gpus 1 (no multi-GPU path exists)")

    import numpy as np
    import torch
    import paper_2602_10378_amd as P
    import sdkde_inputs

    cfg = sdkde_inputs.CONFIGS[args.config]
    x, q, h = sdkde_inputs.make(args.config, seed=args.seed, n=args.n, m=args.m)
    n, d = x.shape
    m = q.shape[0]
    P.load()
    dev = torch.device("cuda:0")
    xd, qd = torch.from_numpy(x).to(dev), torch.from_numpy(q).to(dev)
    ws = P.make_workspace(n, m, d, device=dev, flags=P.SDKDE_FLAG_SYMMETRIC)     # the largest footprint: serves every mode
    s = torch.empty_like(xd)
    x_sd = torch.empty_like(xd)
    dens = torch.empty(m, dtype=torch.float32, device=dev)
    logd = torch.empty(m, dtype=torch.float32, device=dev)

    def step(flags=P.SDKDE_PREC_FP32):
        P.sdkde_score(xd, h, out=s, workspace=ws, flags=flags)
        P.sdkde_debias(xd, s, h, out=x_sd)
        P.sdkde_eval(x_sd, qd, h, density_out=dens, log_density_out=logd, workspace=ws, flags=flags)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    P.sdkde_profile_enable(True)      # HIP events around the main kernels, on the stream they run on
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # per-step spread (same stream)
    t0 = time.perf_counter()
    marks[0].record()
    for k in range(args.steps):
        step()
        marks[k + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step_ms = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps))
    score_launches, score_ms = P.sdkde_profile_summary(0)
    eval_launches, eval_ms = P.sdkde_profile_summary(1)
    P.sdkde_profile_enable(False)

    s_fp32 = s.clone()
    logd_fp32 = logd.clone()
    other = None
    fused = None
    if not args.no_other_modes:
        # The same three steps through the one-call entry point (shift written by the score epilogue, one column
        # mean for both passes: two launches fewer); fp32 path, same outputs.
        def fused_step():
            P.sdkde_fit_eval(xd, qd, h, score_out=s, samples_sd_out=x_sd, density_out=dens, log_density_out=logd, workspace=ws)
        fused_step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            fused_step()
        torch.cuda.synchronize()
        dtf = time.perf_counter() - t1
        fused = {"value": (float(n) * n + float(m) * n) / (dtf / args.steps), "unit": "pairs/s",
                 "ms_per_step": dtf / args.steps * 1e3,
                 "max_abs_log_density_diff_vs_three_calls": float((logd - logd_fp32).abs().max()),
                 "note": "sdkde_fit_eval: score, shift and eval in one call (fp32 path)"}
    if not args.no_other_modes and d > 3:
        # Lower-precision-input modes, reported separately: same steps, same timing protocol.
        other = {}
        notes = {"fp16x2_inputs": "cross-term inputs split into fp16 hi+lo on the fp16 matrix units, fp32 accumulate",
                 "fp16x2_all": "both contractions on the fp16 matrix units (inputs and Phi split into fp16 hi+lo), "
                               "fp32 accumulate, exp and row sums fp32",
                 "symmetric_score": "fp32 path; the score computes each unordered pair of samples once (phi_ij = phi_ji) "
                                    "and is still counted as n^2 pairs, as the paper counts them"}
        modes = [("fp16x2_inputs", P.SDKDE_PREC_FP16X2)]
        if P.sdkde_describe_plan(n, n, d, 0, P.SDKDE_PREC_FP16X2_ALL)["xt_scale"] == 2:      # else it runs as fp16x2 (d > 16)
            modes.append(("fp16x2_all", P.SDKDE_PREC_FP16X2_ALL))
        if P.sdkde_describe_plan(n, n, d, 0, P.SDKDE_FLAG_SYMMETRIC)["symmetric"]:
            modes.append(("symmetric_score", P.SDKDE_FLAG_SYMMETRIC))
        for key, flags in modes:
            step(flags)
            torch.cuda.synchronize()
            P.sdkde_profile_enable(True)
            t1 = time.perf_counter()
            for _ in range(args.steps):
                step(flags)
            torch.cuda.synchronize()
            dt16 = time.perf_counter() - t1
            l16, ms16 = P.sdkde_profile_summary(0)
            P.sdkde_profile_enable(False)
            other[key] = {
                "value": (float(n) * n + float(m) * n) / (dt16 / args.steps), "unit": "pairs/s",
                "ms_per_step": dt16 / args.steps * 1e3, "score_pair_kernels_ms": ms16 / max(l16, 1),
                "score_rel_frobenius_vs_fp32_path": float((s - s_fp32).norm() / s_fp32.norm()),
                "max_abs_log_density_diff_vs_fp32_path": float((logd - logd_fp32).abs().max()),
                "note": notes[key] + "; error vs the oracle is measured in tests/test_gpu_full_size.py"}
    if not args.no_other_modes:
        s.copy_(s_fp32)       # the sample check below is of the fp32 three-call path

    pairs = float(n) * n + float(m) * n
    paper_s = PAPER_SECONDS.get((args.config, n, m))
    ms_per_step = dt / args.steps * 1e3
    value = pairs / (dt / args.steps)
    score_avg_ms = score_ms / max(score_launches, 1)
    eval_avg_ms = eval_ms / max(eval_launches, 1)
    # algorithmic MFMA flops of the score kernel: 4d per pair (cross term 2d + Phi X 2d), n^2 pairs per launch
    score_flops = 4.0 * d * float(n) * n
    achieved = score_flops / (score_avg_ms * 1e-3) / 1e12
    out = {
        "metric": "pair-interactions/sec (score n^2 + eval m*n)", "value": value, "unit": "pairs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": (paper_s / (dt / args.steps)) if paper_s else None,
        "baseline_note": (f"paper: {paper_s:g} s end-to-end at this shape on one RTX A6000 with TF32 dots "
                          "(context, other hardware)") if paper_s else None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: n={n} samples, m={m} queries, d={d}, Gaussian mixture, "
                               f"Silverman h={h:.4f}, score+debias+eval", "n": n, "m": m, "d": d, "seed": args.seed},
        "end_to_end_s": dt / args.steps,
        "ms_per_step_min": per_step_ms[0] if per_step_ms else None,
        "ms_per_step_median": per_step_ms[len(per_step_ms) // 2] if per_step_ms else None,
        "stages_ms": {"score_main_kernel": score_avg_ms, "eval_main_kernel": eval_avg_ms,
                      "everything_else": ms_per_step - score_avg_ms - eval_avg_ms},
    }
    if not P.sdkde_describe_plan(n, n, d, 0)["thin"]:
        out["roofline"] = {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                           "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                           "traffic": SCORE_KERNEL_TRAFFIC_BYTES.get(args.config) if (args.n is None and args.m is None) else None,
                           "kernel": "pair_mfma_kernel (score)", "launch_ms": score_avg_ms,
                           "flops_per_launch": score_flops,
                           # per 16 x 16 tile of pairs: 8 d/16 MFMAs of 32 clocks, and 4 v_exp_f32 + 8 v_add_f32 that
                           # cannot overlap them (fp32 MFMA and VALU do not co-issue on gfx950; measured by sdkde_peaks:
                           # profiles/peaks_mfma_valu_coissue.txt, which times this mix at 333 clocks for d = 16:
                           # 256 + 64 + 13 of switching between the two): the share of the time the MFMA pipe can have
                           "frac_ceiling_of_instruction_mix": (256.0 * d / 16) / (256.0 * d / 16 + 4 * 8 + 8 * 4 + 13),
                           "valu": {"exp_per_s": float(n) * n / (score_avg_ms * 1e-3),
                                    "peak_exp_per_s": 256 * 4 * 16 * 2.4e9 / 2.0,
                                    "note": "v_exp_f32: 8 clocks per wave instruction; sdkde_peaks measures 19.4e12/s back to back"}}
    else:
        # thin-d path (Appendix A): VALU bound.  Per score pair: d subs + d FMAs (r^2) + 1 add (D) + d FMAs
        # (numerator) = 3d + 1 plain instructions, and one v_exp_f32 at a quarter of their rate (4 slots).  Peak:
        # the chip's fp32 vector rate, 157.3 TFLOP/s = 78.6 T lane-instructions/s (256 CUs x 4 SIMDs x 32 lanes x
        # 2.4 GHz: a wave instruction per 2 clocks per SIMD).  sdkde_peaks measures 62 (v_fma_f32) to 72 (v_add_f32)
        # T lane-instructions/s for independent plain instructions from two or more waves, 19.4 for v_exp_f32, and
        # 20.3 clocks for one exp and four FMAs issued in groups (16 at the published rates): the mix ceiling below.
        slots = (3 * d + 1 + 4) * float(n) * n
        peak = 256 * 4 * 32 * 2.4e9 / 1e12
        ach = slots / (score_avg_ms * 1e-3) / 1e12
        out["roofline"] = {"bound": "alu", "achieved": ach, "peak": peak, "unit": "T lane-slots/s", "frac": ach / peak,
                           "traffic": None, "kernel": "pair_thin_kernel (score)", "launch_ms": score_avg_ms,
                           "slots_per_pair": 3 * d + 5,
                           "frac_ceiling_of_instruction_mix": (8.0 + 2.0 * (3 * d + 1)) / (8.1 + 3.05 * (3 * d + 1))}
    if not P.sdkde_describe_plan(n, m, d, 2)["thin"]:
        # the second kernel of the step, for completeness: 2d flops per pair (the cross term only); per tile 4 d/16
        # MFMAs against the same VALU work as the score kernel
        eval_tflops = 2.0 * d * float(m) * n / (eval_avg_ms * 1e-3) / 1e12
        out["roofline_eval_kernel"] = {"bound": "mfma", "achieved": eval_tflops, "peak": PEAK_FP32_MFMA_TFLOPS,
                                       "unit": "TFLOP/s", "frac": eval_tflops / PEAK_FP32_MFMA_TFLOPS,
                                       "launch_ms": eval_avg_ms,
                                       "frac_ceiling_of_instruction_mix": (128.0 * d / 16) / (128.0 * d / 16 + 4 * 8 + 8 * 4 + 6)}
    if fused:
        other = dict(other or {}, fused_call=fused)
    if other:
        out["other_modes"] = other
    if not args.no_cpu_baseline:
        base, s_rows = cpu_baseline(x, q, h)
        out["cpu_baseline"] = base
        got = s[: s_rows.shape[0]].cpu().numpy().astype(np.float64)
        out["parity_on_sample"] = {"score_rel_frobenius": float(np.linalg.norm(got - s_rows) / np.linalg.norm(s_rows)),
                                   "rows": int(s_rows.shape[0])}
    print(json.dumps(out))


if __name__ == "__main__":
    main()

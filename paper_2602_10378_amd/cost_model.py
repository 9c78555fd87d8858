"""The paper's FLOP/byte accounting ("Arithmetic intensity in d dimensions"; Appendix A) and the
MI355X accounting used by bench.py.  Pure arithmetic on sizes; no device code."""
from __future__ import annotations

EXP_FLOPS_PAPER = 8          # the paper prices one exp at 8 flops (its GPU's 128:16 ALU:SFU ratio)


def paper_flops(k: int, d: int, m: int | None = None) -> float:
    """FLOPs_d(k): 2dk^2 (score Gram) + 2dk^2 + 4k^2 + 8k^2 (Phi X, norms, exp) + (2d + 4 + 8) k m (eval);
    the paper fixes m = k/8."""
    m = k / 8 if m is None else m
    return (4 * d + 4 + EXP_FLOPS_PAPER) * k * k + (2 * d + 4 + EXP_FLOPS_PAPER) * k * m


def paper_flops_coeff(d: int) -> float:
    """Coefficient of k^2 at m = k/8: 4d + 12 + d/4 + 3/2."""
    return paper_flops(8, d) / 64.0


def paper_bytes_per_tile(block_m: int, block_n: int, d: int) -> int:
    """4 (BM d + BN d + BM + BM d): load BM query rows, stream BN train rows, write partial pdf + weighted sums."""
    return 4 * (2 * block_m * d + block_n * d + block_m)


def paper_bytes_coeff(block_m: int, block_n: int, d: int) -> float:
    return paper_bytes_per_tile(block_m, block_n, d) / (block_m * block_n)


def paper_flops_1d(k: int) -> float:
    """Appendix A: c1 = 16 flops per train-train pair, c2 = 14 per train-test pair, m = k/8."""
    return 16.0 * k * k + 14.0 * k * (k / 8)


def paper_intensity_1d(k: int) -> float:
    return paper_flops_1d(k) / (5.0 * k)


def pair_interactions(n: int, m: int) -> float:
    """The benchmark's unit of work: n^2 score pairs + m n eval pairs."""
    return float(n) * n + float(m) * n


def mfma_flops(n: int, m: int, d: int):
    """Algorithmic matrix flops on this build's path: score 4d per pair (cross term + Phi X), eval 2d."""
    return 4.0 * d * n * n, 2.0 * d * m * n


# ------------------------------------------------------------------------------------------------------
# MI355X roofline accounting of the pair kernels (what bench.py reports next to every measured time).
# Published dense peaks: fp32 matrix 157.3 TFLOP/s, fp16 matrix 2.5 PFLOP/s, fp32 vector 157.3 TFLOP/s
# (= 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz = 78.6 T lane-instructions/s); v_exp_f32 runs at a quarter of
# the plain vector rate, so one exp takes four issue slots.
# ------------------------------------------------------------------------------------------------------
PEAK_MFMA_F32 = 157.3e12
PEAK_MFMA_F16 = 2.5e15
PEAK_VALU_SLOTS = 256 * 4 * 32 * 2.4e9
EXP_SLOTS = 4

# stage: "score" | "eval"; mode: "fp32" | "fp16x2" | "fp16x2_all" | "fp16x2_phi16" | "symmetric"


def pair_work(stage: str, d: int, mode: str = "fp32", thin: bool = False) -> dict:
    """Work per ordered pair as the kernels of `mode` issue it: matrix flops by input type, exps, and plain
    vector instructions (one lane-slot each).  The fp32 matrix path spends 2d flops per pair on the cross term
    and 2d on Phi X (score only); the fp16x2 modes multiply (hi + lo)(hi + lo) = four products per term; the
    symmetric score forms the Gram tile and the exp once per unordered pair."""
    score = stage == "score"
    if thin:
        # direct differences: d subs + d FMAs (r^2), 1 add (D); the score adds d FMAs (numerator)
        return {"mfma_f32": 0.0, "mfma_f16": 0.0, "exp": 1.0, "valu": (3.0 * d + 1.0) if score else (2.0 * d + 1.0)}
    if mode == "symmetric" and score:
        # per unordered pair: Gram 2d, T_I and T_J 2d each, one exp, init + row sum + column sum adds
        return {"mfma_f32": 3.0 * d, "mfma_f16": 0.0, "exp": 0.5, "valu": 1.5}
    if mode == "fp16x2" or (mode in ("fp16x2_all", "fp16x2_phi16") and not score):
        return {"mfma_f32": 2.0 * d if score else 0.0, "mfma_f16": 8.0 * d, "exp": 1.0, "valu": 2.0}
    if mode == "fp16x2_all":
        # both contractions on the fp16 units; six more vector instructions per four values split Phi
        return {"mfma_f32": 0.0, "mfma_f16": 16.0 * d, "exp": 1.0, "valu": 3.5}
    if mode == "fp16x2_phi16":
        # cross term as fp16x2 (8d), Phi X as one K = 32 MFMA per block: fp16(phi) (x_hi + x_lo) = 4d; per four values
        # four init adds, two packed conversions, two dot products (the row sum) and two register copies
        return {"mfma_f32": 0.0, "mfma_f16": 12.0 * d, "exp": 1.0, "valu": 2.5}
    return {"mfma_f32": (4.0 if score else 2.0) * d, "mfma_f16": 0.0, "exp": 1.0, "valu": 2.0}


def roofline(stage: str, d: int, pairs: float, seconds: float, mode: str = "fp32", thin: bool = False) -> dict:
    """Roofline of one launch over `pairs` ordered pairs that took `seconds`: the time each resource needs at
    its published peak, the binding one (perfect overlap of the others assumed), and achieved / peak on it."""
    w = pair_work(stage, d, mode, thin)
    t = {"mfma_f32": w["mfma_f32"] * pairs / PEAK_MFMA_F32, "mfma_f16": w["mfma_f16"] * pairs / PEAK_MFMA_F16,
         "alu": (w["valu"] + EXP_SLOTS * w["exp"]) * pairs / PEAK_VALU_SLOTS}
    bound = max(t, key=t.get)
    if bound == "alu":
        work, peak, unit = (w["valu"] + EXP_SLOTS * w["exp"]) * pairs, PEAK_VALU_SLOTS, "T lane-slots/s"
    else:
        work, peak, unit = w[bound] * pairs, (PEAK_MFMA_F32 if bound == "mfma_f32" else PEAK_MFMA_F16), "TFLOP/s"
    return {"bound": "alu" if bound == "alu" else "mfma", "resource": bound, "achieved": work / seconds / 1e12,
            "peak": peak / 1e12, "unit": unit, "frac": work / seconds / peak, "work_per_pair": w,
            "seconds_at_peak": {k: v for k, v in t.items() if v > 0.0},
            # the same as fractions of each roof: time the resource needs at its peak over the measured time
            "frac_by_resource": {k: v / seconds for k, v in t.items() if v > 0.0},
            # all three resources at their peaks one after the other (no overlap at all): the other end of the range
            "frac_of_sum_of_resources": sum(t.values()) / seconds}

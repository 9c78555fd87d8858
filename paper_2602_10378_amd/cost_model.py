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

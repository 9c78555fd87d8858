// Pair kernel of the thin path (d <= 3; the score kinds up to d = 6): direct differences on the VALU.
#pragma once
#include "common.h"

namespace {

// ------------------------------------------------------------------------------------------
// Main pair kernel, thin-d path (Appendix A: per pair one exp and a handful of ALU ops, no
// matrix unit).  Each thread owns R evaluation rows; the streamed sample is wave-uniform, so
// its coordinates come through scalar loads.  Accumulates D_i and, for SCORE, the direct-form
// numerator N_i = sum_j phi_ij (x~_j - p~_i).  Same grid decomposition as the MFMA kernel with
// row blocks of kBlock*R rows and "tiles" of 16 samples.
// ------------------------------------------------------------------------------------------
template <int D, int R, int KIND>
__global__ __launch_bounds__(kBlock) void pair_thin_kernel(
    const float* __restrict__ ps, const float* __restrict__ xs, float* __restrict__ part_t,
    float* __restrict__ part_d, int ntiles, int tiles_per_split, int nsplit, int64_t m_pad, float laplace_c0,
    const float* __restrict__ shift)
{
    constexpr bool SCORE = KIND == kScoreSelf || KIND == kScorePoints;
    constexpr bool LAPLACE = KIND == kEvalLaplace;
    constexpr bool ROWMAX = KIND == kRowMax;
    // samples per stage: sixteen exponentials in a group for d <= 2, eight above (measured at n = 262144 with one
    // row per thread, 16 against 8: d = 1 8.5 / 9.4 ms, d = 2 12.5 / 12.6, d = 3 15.8 / 15.7, d = 6 27.3 / 26.9)
    constexpr int G = (D <= 2 ? 16 : 8) / R;
    const int split = blockIdx.x % nsplit;
    const int64_t row_block = blockIdx.x / nsplit;
    const int64_t row0 = row_block * (kBlock * R) + threadIdx.x;

    // sh[q]: the row's shift (max_j of -r^2, <= 0) in the max-shifted mode, else 0; the squared distance is
    // accumulated on top of it so that exp2(-(r^2 + sh)) = phi / 2^sh costs no extra instruction.
    // Two-level accumulation as in the matrix path: the running sums are folded into (dsum, nsum) every
    // kFlushTiles sample tiles, so that no fp32 accumulator sees a long chain of additions at its own magnitude.
    float p[R][D], dacc[R], nacc[R][SCORE ? D : 1], dsum[R], nsum[R][SCORE ? D : 1], sh[R];
#pragma unroll
    for (int q = 0; q < R; ++q) {
#pragma unroll
        for (int k = 0; k < D; ++k) p[q][k] = ps[(row0 + (int64_t)q * kBlock) * D + k];
        sh[q] = (!ROWMAX && shift) ? shift[row0 + (int64_t)q * kBlock] : 0.0f;
        dacc[q] = dsum[q] = ROWMAX ? kNegHuge : 0.0f;
#pragma unroll
        for (int k = 0; k < (SCORE ? D : 1); ++k) nacc[q][k] = nsum[q][k] = 0.0f;
    }
    auto fold = [&]() {
#pragma unroll
        for (int q = 0; q < R; ++q) {
            if (ROWMAX) {
                dsum[q] = fmaxf(dsum[q], dacc[q]);
            } else {
                dsum[q] += dacc[q];
                dacc[q] = 0.0f;
            }
#pragma unroll
            for (int k = 0; k < (SCORE ? D : 1); ++k) {
                nsum[q][k] += nacc[q][k];
                nacc[q][k] = 0.0f;
            }
        }
    };

    const int t_begin = split * tiles_per_split;
    const int t_end = min(ntiles, t_begin + tiles_per_split);
    for (int jt = t_begin; jt < t_end; ++jt) {
        if (((jt - t_begin) & (kFlushTiles - 1)) == kFlushTiles - 1) fold();
        const float* xj = xs + (int64_t)jt * kTile * D;    // wave-uniform address
        // G samples at a time, in three stages pinned by scheduling barriers: squared distances, then the
        // exponentials back to back, then the sums.  v_exp_f32 issued between other VALU work slows both down
        // (measured on this chip: an exp plus four FMAs take 22.7 clocks interleaved, 20.6 in groups).
#pragma unroll
        for (int j0 = 0; j0 < kTile; j0 += G) {
            float diff[G][R][SCORE ? D : 1], r2[G][R], phi[G][R];
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                float xv[D];
#pragma unroll
                for (int k = 0; k < D; ++k) xv[k] = xj[(j0 + jj) * D + k];
#pragma unroll
                for (int q = 0; q < R; ++q) {
                    float acc = sh[q];
#pragma unroll
                    for (int k = 0; k < D; ++k) {
                        const float df = xv[k] - p[q][k];
                        if (SCORE) diff[jj][q][k] = df;
                        acc = fmaf(df, df, acc);
                    }
                    r2[jj][q] = acc;
                }
            }
            if (ROWMAX) {
#pragma unroll
                for (int jj = 0; jj < G; ++jj)
#pragma unroll
                    for (int q = 0; q < R; ++q) dacc[q] = fmaxf(dacc[q], -r2[jj][q]);
                continue;
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int jj = 0; jj < G; ++jj)
#pragma unroll
                for (int q = 0; q < R; ++q) phi[jj][q] = __builtin_amdgcn_exp2f(-r2[jj][q]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
#pragma unroll
                for (int q = 0; q < R; ++q) {
                    // Laplace factor 1 + d/2 - r^2/2h^2, with the true r^2 = r2 - sh
                    if (LAPLACE) dacc[q] = fmaf(phi[jj][q], fmaf(sh[q] - r2[jj][q], kLn2, laplace_c0), dacc[q]);
                    else dacc[q] += phi[jj][q];
                    if (SCORE) {
#pragma unroll
                        for (int k = 0; k < D; ++k) nacc[q][k] = fmaf(phi[jj][q], diff[jj][q][k], nacc[q][k]);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    fold();
#pragma unroll
    for (int q = 0; q < R; ++q) {
        const int64_t row = row0 + (int64_t)q * kBlock;
        part_d[(int64_t)split * m_pad + row] = dsum[q];
        if (SCORE) {
#pragma unroll
            for (int k = 0; k < D; ++k) part_t[((int64_t)split * m_pad + row) * D + k] = nsum[q][k];
        }
    }
}

}  // namespace

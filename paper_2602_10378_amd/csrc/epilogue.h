// Reductions of the partial sums and the elementwise kernels: score / eval epilogues, debias, max-shift.
#pragma once
#include "common.h"

namespace {

// ------------------------------------------------------------------------------------------
// Split reduction + epilogues (fixed summation order over splits: deterministic).
// ------------------------------------------------------------------------------------------

// ps_split_half: p~ is stored as fp16 hi/lo pairs (fp16x2 input mode) and is rebuilt as hi + lo.
// mode 0 (MFMA path, separate points): score = (T/D - p~) * inv_ah2            (T = Phi X regrouping)
// mode 1 (thin path):                   score = (N/D) * inv_ah2                (direct-form numerator)
// mode 2 (MFMA path, at the samples):   score = (T' - p~ D') / (D' + 1) * inv_ah2
//        where T', D' exclude the pair (i, i), whose weight is exactly 1.
// inv_ah2 = 1 / (a h^2) undoes the coordinate scaling.  D == 0 gives 0.
// score and x_sd are both optional outputs; x_sd = x + half_h2 * score (x: the original points, same indexing).
__global__ __launch_bounds__(kBlock) void score_epilogue_kernel(
    const float* __restrict__ part_t, const float* __restrict__ part_d, const float* __restrict__ ps,
    int nsplit, int64_t m, int64_t m_pad, int d, int dp, int mode, int ps_split_half, float inv_ah2,
    float* __restrict__ score, const float* __restrict__ x, float half_h2, float* __restrict__ x_sd)
{
    int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= m * d) return;
    const int64_t i = idx / d;
    const int c = (int)(idx % d);
    float tsum = 0.0f, dsum = 0.0f;
    for (int s = 0; s < nsplit; ++s) {
        tsum += part_t[((int64_t)s * m_pad + i) * dp + c];
        dsum += part_d[(int64_t)s * m_pad + i];
    }
    float pc = 0.0f;                       // p~_i[c]
    if (mode != 1) {
        if (ps_split_half) {
            const _Float16* ph = reinterpret_cast<const _Float16*>(ps) + i * 2 * dp + (c / 16) * 32 + (c % 16);
            pc = (float)ph[0] + (float)ph[16];
        } else {
            pc = ps[i * dp + ((c & ~15) | ((c & 3) << 2) | ((c >> 2) & 3))];      // fp32 layout of the prepared rows
        }
    }
    float out = 0.0f;
    if (mode == 2) {
        out = fmaf(-pc, dsum, tsum) / (dsum + 1.0f) * inv_ah2;
    } else if (dsum > 0.0f) {
        float ratio = tsum / dsum;
        out = (mode == 1 ? ratio : ratio - pc) * inv_ah2;
    }
    if (score) score[idx] = out;
    if (x_sd) x_sd[idx] = fmaf(half_h2, out, x[idx]);      // fused debiasing shift (sdkde_fit_eval)
}

// log p = log D + lognorm, lognorm = -log n - d log h - (d/2) log 2 pi (formed on the host in double).
// signed != 0 (Laplace-corrected sum, which may be negative): density = sum * exp(lognorm) only.
// shift (may be null): per-query base-2 exponent shift of the max-shifted mode.
__global__ __launch_bounds__(kBlock) void eval_epilogue_kernel(const float* __restrict__ part_d, int nsplit,
                                                               int64_t m, int64_t m_pad, double lognorm, int is_signed,
                                                               const float* __restrict__ shift,
                                                               float* __restrict__ density,
                                                               float* __restrict__ log_density)
{
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= m) return;
    float dsum = 0.0f;
    for (int s = 0; s < nsplit; ++s) dsum += part_d[(int64_t)s * m_pad + i];
    // max-shifted mode: the sums were taken of phi / 2^shift
    const double shift_ln = shift ? (double)shift[i] * 0.69314718055994530942 : 0.0;
    if (is_signed) {
        if (density) density[i] = (float)((double)dsum * exp(lognorm + shift_ln));
        return;
    }
    double lp = log((double)dsum) + lognorm + shift_ln;      // -inf when dsum == 0
    if (log_density) log_density[i] = (float)lp;
    if (density) density[i] = (float)exp(lp);
}

__global__ __launch_bounds__(kBlock) void debias_kernel(const float* __restrict__ x, const float* __restrict__ s,
                                                        int64_t total, float half_h2, float* __restrict__ out)
{
    int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (idx < total) out[idx] = fmaf(half_h2, s[idx], x[idx]);
}


// shift[i] = max over splits of the row maxima left in part_d by a kRowMax pass; on the MFMA path the
// shift is also folded into the row constant pn (-|p~|^2 - shift), so the main pass needs no extra work.
__global__ __launch_bounds__(kBlock) void shift_kernel(const float* __restrict__ part_d, int nsplit, int64_t m_pad,
                                                       float* __restrict__ shift, float* __restrict__ pn)
{
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= m_pad) return;
    float mx = kNegHuge;
    for (int s = 0; s < nsplit; ++s) mx = fmaxf(mx, part_d[(int64_t)s * m_pad + i]);
    shift[i] = mx;
    if (pn) pn[i] -= mx;
}

}  // namespace

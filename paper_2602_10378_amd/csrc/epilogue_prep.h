// One launch for two stages of the one-call pass (sdkde_fit_eval): the score epilogue at the samples themselves with
// the debiasing shift, and the preparation of the eval pass's operands (the shifted samples, which this kernel has
// just formed, and the queries).  A small problem is a chain of dependent launches and little else; this removes one.
#pragma once
#include "epilogue.h"
#include "prep.h"

namespace {

// Workgroups [0, blocks_sd): rows r0 .. r0 + kPrepRows of the samples.  The (row, four columns) items of those rows
// are reduced over the split slots exactly as score_epilogue_quad_kernel does it (64 items per pass, slots shared by
// four parts and combined in part order: the same bits), score and shifted samples are written, and the shifted
// values stay in LDS, from where prep_rows writes the eval pass's prepared copy and norms.  `ps` (the score pass's
// prepared samples, read for p~) and sd_job.dst may be the same memory: a workgroup reads its own rows before it
// overwrites them and no other workgroup touches them.
// Workgroups [blocks_sd, ...): the queries, as prep_mfma_kernel prepares them (centre read from the workspace).
__global__ __launch_bounds__(kBlock) void score_epilogue_prep_kernel(
    const float* __restrict__ part_t, const float* __restrict__ part_d, const float* ps, int nsplit, int64_t m,
    int64_t m_pad, int d, int dp, int ps_split_half, float inv_ah2, float* __restrict__ score, const float* __restrict__ x,
    float half_h2, float* __restrict__ x_sd, int quad_io, PrepJob sd_job, PrepJob q_job, int blocks_sd,
    PrepCommon common, float a, int prec, Stamp stamp)
{
    constexpr int PARTS = kEpiPartsFew, LANES = kBlock / PARTS;
    __shared__ double red[kBlock];
    __shared__ float smean[SDKDE_MAX_D];
    __shared__ float raw[kPrepRows][SDKDE_MAX_D + 1];
    __shared__ float used[kPrepRows][SDKDE_MAX_D + 1];
    __shared__ f32x4 red_t[PARTS][LANES];
    __shared__ float red_d[PARTS][LANES];
    __shared__ int stamp_flag;
    const bool poisoned = stamp_poisons(stamp, &stamp_flag);
    prep_common(common, d, red, smean);
    if ((int)blockIdx.x >= blocks_sd) {
        prep_rows<false>(q_job, (int64_t)(blockIdx.x - blocks_sd) * kPrepRows, d, dp, a, prec, poisoned, smean, raw, used);
        return;
    }

    const int64_t r0 = (int64_t)blockIdx.x * kPrepRows;
    const int lane = threadIdx.x % LANES, part = threadIdx.x / LANES;
    const int quads = dp / 4;
    for (int first = 0; first < kPrepRows * quads; first += LANES) {        // kPrepRows * quads is a multiple of 64
        const int item = first + lane;
        const int64_t i = r0 + item / quads;
        const int c0 = (item % quads) * 4;
        const bool active = i < m;
        f32x4 tacc = {0.0f, 0.0f, 0.0f, 0.0f};
        float dacc = 0.0f;
        if (active) {
            for (int s = part; s < nsplit; s += PARTS) {
                tacc += *reinterpret_cast<const f32x4*>(part_t + ((int64_t)s * m_pad + i) * dp + c0);
                dacc += part_d[(int64_t)s * m_pad + i];
            }
        }
        red_t[part][lane] = tacc;
        red_d[part][lane] = dacc;
        __syncthreads();
        if (active && part == 0 && c0 < d) {
            f32x4 tsum = red_t[0][lane];
            float dsum = red_d[0][lane];
#pragma unroll
            for (int k = 1; k < PARTS; ++k) {
                tsum += red_t[k][lane];
                dsum += red_d[k][lane];
            }
            f32x4 out, shifted;
            const int64_t at = i * d + c0;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int c = c0 + v;       // may run past d in the last quad: computed from padding, not stored
                float pc;
                if (ps_split_half) {
                    const _Float16* ph = reinterpret_cast<const _Float16*>(ps) + i * 2 * dp + (c / 16) * 32 + (c % 16);
                    pc = (float)ph[0] + (float)ph[16];
                } else {
                    pc = ps[i * dp + ((c & ~15) | ((c & 3) << 2) | ((c >> 2) & 3))];
                }
                out[v] = fmaf(-pc, dsum, tsum[v]) / (dsum + 1.0f) * inv_ah2;      // the samples' own pair is not in the sums
            }
            if (quad_io) {                  // d is a multiple of four and the caller's arrays are 16-byte aligned
                const f32x4 xv = *reinterpret_cast<const f32x4*>(x + at);
#pragma unroll
                for (int v = 0; v < 4; ++v) shifted[v] = fmaf(half_h2, out[v], xv[v]);
                if (score) *reinterpret_cast<f32x4*>(score + at) = out;
                *reinterpret_cast<f32x4*>(x_sd + at) = shifted;
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if (c0 + v >= d) break;
                    shifted[v] = fmaf(half_h2, out[v], x[at + v]);
                    if (score) score[at + v] = out[v];
                    x_sd[at + v] = shifted[v];
                }
            }
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (c0 + v < d) raw[item / quads][c0 + v] = shifted[v];
        }
        __syncthreads();            // red_t / red_d are reused by the next pass; raw is read below
    }
    prep_rows<true>(sd_job, r0, d, dp, a, prec, poisoned, smean, raw, used);
}

}  // namespace

// Reductions of the partial sums and the elementwise kernels: score / eval epilogues, debias, max-shift.
#pragma once
#include "common.h"

namespace {

// ------------------------------------------------------------------------------------------
// Split reduction + epilogues (fixed summation order over splits: deterministic).
// ------------------------------------------------------------------------------------------

// The partial slots of one output are shared by PARTS threads (slots part, part + PARTS, ...), which keeps many
// loads in flight instead of one long dependent chain on a few compute units (a call with few points has up to
// thousands of slots and few outputs), and are combined through LDS in the fixed order part 0, 1, ..., PARTS - 1.
// The host picks PARTS from the slot and output counts alone (epilogue_parts), so a plan always sums in the same
// order: the many-thread form only where the outputs are too few to fill the chip otherwise, since its loads are
// narrow (kBlock / PARTS consecutive floats per slot).
constexpr int kEpiPartsFew = 4, kEpiPartsMany = 32;
constexpr int kEpiManySlots = 64;                   // least slot count and
constexpr int64_t kEpiFewOutputs = 65536;           // most outputs for kEpiPartsMany
inline int epilogue_parts(int nslots, int64_t outputs)
{
    return nslots >= kEpiManySlots && outputs <= kEpiFewOutputs ? kEpiPartsMany : kEpiPartsFew;
}

template <int PARTS, bool MAX>
__device__ __forceinline__ float reduce_slots(const float* __restrict__ first, int64_t stride, int nslots, bool active,
                                              float (*red)[kBlock / PARTS])
{
    constexpr int OUTPUTS = kBlock / PARTS;
    const int lane = threadIdx.x % OUTPUTS, part = threadIdx.x / OUTPUTS;
    float acc = MAX ? kNegHuge : 0.0f;
    if (active) {
        for (int s = part; s < nslots; s += PARTS) {
            const float v = first[(int64_t)s * stride];
            acc = MAX ? fmaxf(acc, v) : acc + v;
        }
    }
    red[part][lane] = acc;
    __syncthreads();
    float r = red[0][lane];
#pragma unroll
    for (int q = 1; q < PARTS; ++q) r = MAX ? fmaxf(r, red[q][lane]) : r + red[q][lane];
    __syncthreads();            // red is reused by the next reduction
    return r;
}

// ps_split_half: p~ is stored as fp16 hi/lo pairs (fp16x2 input mode) and is rebuilt as hi + lo.
// mode 0 (MFMA path, separate points): score = (T/D - p~) * inv_ah2            (T = Phi X regrouping)
// mode 1 (thin path):                   score = (N/D) * inv_ah2                (direct-form numerator)
// mode 2 (MFMA path, at the samples):   score = (T' - p~ D') / (D' + 1) * inv_ah2
//        where T', D' exclude the pair (i, i), whose weight is exactly 1.
// inv_ah2 = 1 / (a h^2) undoes the coordinate scaling.  D < min_sum (least_trusted_sum of the sample count) gives 0.
// score and x_sd are both optional outputs; x_sd = x + half_h2 * score (x: the original points, same indexing).
// Grid: one workgroup per kBlock / PARTS elements of the [m, d] output.
template <int PARTS>
__global__ __launch_bounds__(kBlock) void score_epilogue_kernel(
    const float* __restrict__ part_t, const float* __restrict__ part_d, const float* __restrict__ ps,
    int nsplit, int64_t m, int64_t m_pad, int d, int dp, int mode, int ps_split_half, float inv_ah2,
    float* __restrict__ score, const float* __restrict__ x, float half_h2, float* __restrict__ x_sd, float min_sum)
{
    constexpr int kEpiOutputs = kBlock / PARTS;
    __shared__ float red[PARTS][kEpiOutputs];
    const int64_t idx = (int64_t)blockIdx.x * kEpiOutputs + threadIdx.x % kEpiOutputs;
    const bool active = idx < m * d;
    const int64_t i = active ? idx / d : 0;
    const int c = active ? (int)(idx % d) : 0;
    const float tsum = reduce_slots<PARTS, false>(part_t + i * dp + c, m_pad * dp, nsplit, active, red);
    const float dsum = reduce_slots<PARTS, false>(part_d + i, m_pad, nsplit, active, red);
    if (!active || threadIdx.x >= kEpiOutputs) return;
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
    } else if (dsum >= min_sum) {
        float ratio = tsum / dsum;
        out = (mode == 1 ? ratio : ratio - pc) * inv_ah2;
    }
    if (score) score[idx] = out;
    if (x_sd) x_sd[idx] = fmaf(half_h2, out, x[idx]);      // fused debiasing shift (sdkde_fit_eval)
}

// Matrix-path form of score_epilogue_kernel<kEpiPartsFew> (modes 0 and 2): a thread takes four consecutive
// coordinates of one row, so the partial T is read with 16-byte loads (1 KiB per wave and slot instead of 256
// bytes) by a quarter of the workgroups.  Same summation order, hence the same bits.  quad_io: the outputs (and x)
// may be accessed 16 bytes at a time.
// Grid: one workgroup per kBlock / kEpiPartsFew (row, four columns) pairs of the [m, dp] partials.
__global__ __launch_bounds__(kBlock) void score_epilogue_quad_kernel(
    const float* __restrict__ part_t, const float* __restrict__ part_d, const float* __restrict__ ps,
    int nsplit, int64_t m, int64_t m_pad, int d, int dp, int mode, int ps_split_half, float inv_ah2,
    float* __restrict__ score, const float* __restrict__ x, float half_h2, float* __restrict__ x_sd, int quad_io,
    float min_sum)
{
    constexpr int PARTS = kEpiPartsFew, LANES = kBlock / PARTS;
    __shared__ f32x4 red_t[PARTS][LANES];
    __shared__ float red_d[PARTS][LANES];
    const int lane = threadIdx.x % LANES, part = threadIdx.x / LANES;
    const int quads = dp / 4;
    const int64_t q = (int64_t)blockIdx.x * LANES + lane;
    const bool active = q < m * quads;
    const int64_t i = active ? q / quads : 0;
    const int c0 = active ? (int)(q % quads) * 4 : 0;
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
    if (!active || part != 0 || c0 >= d) return;
    f32x4 tsum = red_t[0][lane];
    float dsum = red_d[0][lane];
#pragma unroll
    for (int k = 1; k < PARTS; ++k) {
        tsum += red_t[k][lane];
        dsum += red_d[k][lane];
    }
    f32x4 out;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int c = c0 + v;       // may run past d in the last quad: computed from padding, not stored
        float pc;
        if (ps_split_half) {
            const _Float16* ph = reinterpret_cast<const _Float16*>(ps) + i * 2 * dp + (c / 16) * 32 + (c % 16);
            pc = (float)ph[0] + (float)ph[16];
        } else {
            pc = ps[i * dp + ((c & ~15) | ((c & 3) << 2) | ((c >> 2) & 3))];      // fp32 layout of the prepared rows
        }
        float o = 0.0f;
        if (mode == 2) o = fmaf(-pc, dsum, tsum[v]) / (dsum + 1.0f) * inv_ah2;
        else if (dsum >= min_sum) o = (tsum[v] / dsum - pc) * inv_ah2;
        out[v] = o;
    }
    const int64_t at = i * d + c0;
    if (quad_io) {                  // d is a multiple of four and the caller's arrays are 16-byte aligned
        if (score) *reinterpret_cast<f32x4*>(score + at) = out;
        if (x_sd) {
            const f32x4 xv = *reinterpret_cast<const f32x4*>(x + at);
            f32x4 r;
#pragma unroll
            for (int v = 0; v < 4; ++v) r[v] = fmaf(half_h2, out[v], xv[v]);
            *reinterpret_cast<f32x4*>(x_sd + at) = r;
        }
    } else {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (c0 + v >= d) break;
            if (score) score[at + v] = out[v];
            if (x_sd) x_sd[at + v] = fmaf(half_h2, out[v], x[at + v]);
        }
    }
}

// log p = log D + lognorm, lognorm = -log n - d log h - (d/2) log 2 pi (formed on the host in double).
// signed != 0 (Laplace-corrected sum, which may be negative): density = sum * exp(lognorm) only.
// shift (may be null): per-query base-2 exponent shift of the max-shifted mode.  min_sum: least_trusted_sum(n).
// Grid: one workgroup per kBlock / PARTS queries.
template <int PARTS>
__global__ __launch_bounds__(kBlock) void eval_epilogue_kernel(const float* __restrict__ part_d, int nsplit,
                                                               int64_t m, int64_t m_pad, double lognorm, int is_signed,
                                                               const float* __restrict__ shift, float min_sum,
                                                               float* __restrict__ density,
                                                               float* __restrict__ log_density)
{
    constexpr int kEpiOutputs = kBlock / PARTS;
    __shared__ float red[PARTS][kEpiOutputs];
    const int64_t i = (int64_t)blockIdx.x * kEpiOutputs + threadIdx.x % kEpiOutputs;
    const bool active = i < m;
    float dsum = reduce_slots<PARTS, false>(part_d + (active ? i : 0), m_pad, nsplit, active, red);
    if (!active || threadIdx.x >= kEpiOutputs) return;
    // too close to the flush threshold of the weights: the all-underflow case (the signed sum of the Laplace-corrected
    // estimate may be small because its terms cancel, and is left as it is)
    if (!is_signed && dsum < min_sum) dsum = 0.0f;
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

// out may alias x or s (each thread reads its one element before it writes it): no __restrict__ here.
__global__ __launch_bounds__(kBlock) void debias_kernel(const float* x, const float* s, int64_t total, float half_h2,
                                                        float* out)
{
    int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (idx < total) out[idx] = fmaf(half_h2, s[idx], x[idx]);
}


// shift[i] = max over splits of the row maxima left in part_d by a kRowMax pass; on the MFMA path the
// shift is also folded into the row constant pn (-|p~|^2 - shift), so the main pass needs no extra work.
// Grid: one workgroup per kBlock / PARTS rows.
template <int PARTS>
__global__ __launch_bounds__(kBlock) void shift_kernel(const float* __restrict__ part_d, int nsplit, int64_t m_pad,
                                                       float* __restrict__ shift, float* __restrict__ pn)
{
    constexpr int kEpiOutputs = kBlock / PARTS;
    __shared__ float red[PARTS][kEpiOutputs];
    const int64_t i = (int64_t)blockIdx.x * kEpiOutputs + threadIdx.x % kEpiOutputs;
    const bool active = i < m_pad;
    const float mx = reduce_slots<PARTS, true>(part_d + (active ? i : 0), m_pad, nsplit, active, red);
    if (!active || threadIdx.x >= kEpiOutputs) return;
    shift[i] = mx;
    if (pn) pn[i] -= mx;
}

}  // namespace

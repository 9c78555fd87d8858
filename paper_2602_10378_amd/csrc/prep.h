// Prep kernels: centre + scale + pad (+ fp16 hi/lo split) into the layouts the pair kernels read.
#pragma once
#include "common.h"

namespace {

// ------------------------------------------------------------------------------------------
// Prep: the centre (mean of a strided subsample, formed by every workgroup for itself), then centre + scale + pad.
// ------------------------------------------------------------------------------------------

// The centre all coordinates are taken relative to: the column means of an evenly strided subsample of the
// samples (about kCentreElems input values, at least 32 rows), summed in double in a fixed order, so every
// workgroup that computes it gets the same bits.  Any point near the data serves (the exponent
// -|p - x|^2 / 2h^2 does not depend on it; it only keeps the norms of the Gram expansion small), so a few hundred
// rows spread over the whole array are as good as all of them and need no pass of their own.
// Result in smean[0 .. d); ends with a barrier.
__device__ __forceinline__ int64_t centre_rows(int64_t n, int d)
{
    const int64_t want = kCentreElems / d > 32 ? kCentreElems / d : 32;
    return n < want ? n : want;
}

__device__ __forceinline__ void block_centre(const float* __restrict__ src, int64_t n, int d, double* red, float* smean)
{
    const int rows_per_iter = kBlock / d;                 // d <= 128 < kBlock
    const int rr = threadIdx.x / d, c = threadIdx.x % d;
    const int64_t rows = centre_rows(n, d);
    const int64_t stride = n / rows;                      // >= 1
    double acc = 0.0;
    if (rr < rows_per_iter) {
#pragma unroll 16
        for (int64_t k = rr; k < rows; k += rows_per_iter) acc += (double)src[k * stride * d + c];
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if ((int)threadIdx.x < d) {
        double t = 0.0;
        for (int q = 0; q < rows_per_iter; ++q) t += red[q * d + threadIdx.x];
        smean[threadIdx.x] = (float)(t / (double)rows);
    }
    __syncthreads();
}

// Where a prep launch gets the centre from.
struct PrepCommon {
    const float* centre_src;   // samples to take the centre of (centre_rows of them, strided); null: read `centre`
    int64_t centre_n;          // rows of centre_src
    float* centre;             // in the workspace: written by workgroup 0 when computed, read otherwise
};

// Centre into smean (computed or read back).  Ends with a barrier.
__device__ __forceinline__ void prep_common(const PrepCommon& pc, int d, double* red, float* smean)
{
    if (pc.centre_src) {
        block_centre(pc.centre_src, pc.centre_n, d, red, smean);
        if (blockIdx.x == 0 && (int)threadIdx.x < d) pc.centre[threadIdx.x] = smean[threadIdx.x];
    } else {
        if ((int)threadIdx.x < d) smean[threadIdx.x] = pc.centre[threadIdx.x];
        __syncthreads();
    }
}

// One array to prepare: src[rows][d] -> dst (rows_pad rows), optional blocked transpose dst_t, norms dst_n.
struct PrepJob {
    const float* src;
    int64_t rows, rows_pad;
    float* dst;
    float* dst_t;
    float* dst_n;
    float pad_value;      // thin path only: coordinate value of padding rows
};

// Record of what a prep launch left in the workspace (sample arrays and column sums), kept in the workspace itself:
// a launch that prepares samples writes it, a launch that relies on earlier samples (SDKDE_FLAG_SAMPLES_PREPARED)
// compares it with what it expects and, on a mismatch, poisons its own outputs with NaN so that every result of the
// call is NaN instead of a plausible number from someone else's samples.
constexpr int kStampWords = 6;
struct Stamp {
    uint64_t* where;                // in the workspace; null: no record kept or checked
    int check;                      // 0: write `value` (workgroup 0), 1: compare with `value`
    uint64_t value[kStampWords];    // kind of call, samples pointer, n, d, precision mode, bits of the scale a
};

// Thread 0 of every workgroup reads or (workgroup 0) writes the record; returns whether this launch is poisoned.
// Ends with a barrier.
__device__ __forceinline__ bool stamp_poisons(const Stamp& stamp, int* flag)
{
    if (threadIdx.x == 0) {
        int bad = 0;
        if (stamp.where && stamp.check) {
            for (int k = 0; k < kStampWords; ++k) bad |= stamp.where[k] != stamp.value[k];
        } else if (stamp.where && blockIdx.x == 0) {
            for (int k = 0; k < kStampWords; ++k) stamp.where[k] = stamp.value[k];
        }
        *flag = bad;
    }
    __syncthreads();
    return *flag != 0;
}

constexpr int kPrepRows = 32;      // rows per workgroup of prep_mfma_kernel (two 16-sample tiles; 2 x 16.5 KiB of LDS)

// Centre, scale and pad for the MFMA path.  A workgroup stages kPrepRows rows in LDS and writes
//   dst[row][dp]   = a (x - mean), 0 in padding columns and rows (coalesced row writes); fp32: within each
//                    16-column block coordinate c sits at position 4 (c % 4) + c / 4,
//   dst_t[row/16][col][row%16] = the same values with each 16-sample tile transposed (if dst_t),
//   dst_n[row]     = -|dst[row]|^2 in double, rounded once; kPadNorm for padding rows.
// prec >= SDKDE_PREC_FP16X2 (fp16x2 input modes): dst holds, per 16-column block, 16 fp16 "hi" values
// followed by 16 fp16 "lo" values with hi + lo = the fp32 coordinate to ~22 mantissa bits (same bytes
// per row as fp32); the norm is then taken of hi + lo so that it matches what the MFMA multiplies.
// prec == SDKDE_PREC_FP16X2_ALL: dst_t holds fp16 pairs too, laid out as the A operand of the K = 32
// second contraction: for tile, column c and lane group g, eight halves [hi(4g..4g+3) | the same again]
// followed by eight halves [lo(4g..4g+3) | the same again] (twice the bytes of the fp32 layout).
// prec == SDKDE_PREC_FP16X2_PHI16: dst_t holds, for tile, column c and lane group g, eight halves
// [hi(4g..4g+3) | lo(4g..4g+3)].
// The body for one workgroup: rows r0 .. r0 + kPrepRows of `job`.  STAGED: the input values of those rows are
// already in raw[][] (a caller that has just computed them); otherwise they are read from job.src.
template <bool STAGED>
__device__ __forceinline__ void prep_rows(const PrepJob& job, int64_t r0, int d, int dp, float a, int prec, bool poisoned,
                                          const float* smean, float (*raw)[SDKDE_MAX_D + 1], float (*used)[SDKDE_MAX_D + 1])
{
    _Float16* dst_h = reinterpret_cast<_Float16*>(job.dst);
    for (int idx = threadIdx.x; idx < kPrepRows * dp; idx += kBlock) {
        const int rr = idx / dp, c = idx % dp;
        const int64_t row = r0 + rr;
        float v = 0.0f;
        if (row < job.rows && c < d) v = a * ((STAGED ? raw[rr][c] : job.src[row * d + c]) - smean[c]);
        raw[rr][c] = v;
        if (prec != SDKDE_PREC_FP32) {
            const _Float16 hi = (_Float16)v;
            const _Float16 lo = (_Float16)(v - (float)hi);
            _Float16* out = dst_h + row * 2 * dp + (c / 16) * 32 + (c % 16);
            out[0] = hi;
            out[16] = lo;
            v = (float)hi + (float)lo;
        } else {
            // fp32 layout: coordinate c of a 16-column block at position 4 (c % 4) + c / 4 (RowTiles, KLAST)
            job.dst[row * dp + ((c & ~15) | ((c & 3) << 2) | ((c >> 2) & 3))] = v;
        }
        used[rr][c] = v;
    }
    __syncthreads();
    if (job.dst_t && prec == SDKDE_PREC_FP16X2_PHI16) {
        // A operand of the K = 32 second contraction with single-fp16 weights: for tile, column c and lane group g,
        // eight halves [hi(4g..4g+3) | lo(4g..4g+3)] (the bytes of the fp32 layout)
        _Float16* base = reinterpret_cast<_Float16*>(job.dst_t) + (r0 / kTile) * (int64_t)dp * 32;
        for (int idx = threadIdx.x; idx < kPrepRows * dp * 2; idx += kBlock) {
            // idx = ((tile*dp + c)*4 + g)*8 + e
            const int e = idx % 8, g = (idx / 8) % 4, c = (idx / 32) % dp, tile = idx / (32 * dp);
            const float v = raw[tile * kTile + 4 * g + (e & 3)][c];
            const _Float16 hi = (_Float16)v;
            base[idx] = e < 4 ? hi : (_Float16)(v - (float)hi);
        }
    } else if (job.dst_t && prec != SDKDE_PREC_FP16X2_ALL) {
        float* base = job.dst_t + (r0 / kTile) * (int64_t)dp * kTile;
        for (int idx = threadIdx.x; idx < kPrepRows * dp; idx += kBlock) {
            const int tile = idx / (dp * kTile), c = (idx / kTile) % dp, rr = idx % kTile;
            base[idx] = raw[tile * kTile + rr][c];        // idx = (tile*dp + c)*16 + rr
        }
    } else if (job.dst_t) {
        _Float16* base = reinterpret_cast<_Float16*>(job.dst_t) + (r0 / kTile) * (int64_t)dp * 64;
        for (int idx = threadIdx.x; idx < kPrepRows * dp * 4; idx += kBlock) {
            // idx = ((tile*dp + c)*4 + g)*16 + e
            const int e = idx % 16, g = (idx / 16) % 4, c = (idx / 64) % dp, tile = idx / (64 * dp);
            const float v = raw[tile * kTile + 4 * g + (e & 3)][c];
            const _Float16 hi = (_Float16)v;
            base[idx] = e < 8 ? hi : (_Float16)(v - (float)hi);
        }
    }
    if (threadIdx.x < kPrepRows) {
        double acc = 0.0;
        for (int c = 0; c < dp; ++c) acc += (double)used[threadIdx.x][c] * (double)used[threadIdx.x][c];
        const int64_t row = r0 + threadIdx.x;
        job.dst_n[row] = poisoned ? __builtin_nanf("") : row < job.rows ? -(float)acc : kPadNorm;
    }
}

// Grid: job0's blocks first (blocks0 of them), then job1's.
__global__ __launch_bounds__(kBlock) void prep_mfma_kernel(PrepJob job0, PrepJob job1, int blocks0, int d, int dp,
                                                           PrepCommon common, float a, int prec, Stamp stamp)
{
    __shared__ double red[kBlock];
    __shared__ float smean[SDKDE_MAX_D];
    __shared__ float raw[kPrepRows][SDKDE_MAX_D + 1];     // a (x - mean)
    __shared__ float used[kPrepRows][SDKDE_MAX_D + 1];    // the value the first contraction multiplies (hi + lo, or raw)
    __shared__ int stamp_flag;
    const bool poisoned = stamp_poisons(stamp, &stamp_flag);
    prep_common(common, d, red, smean);

    const bool second = (int)blockIdx.x >= blocks0;
    const PrepJob& job = second ? job1 : job0;
    const int64_t r0 = (int64_t)(blockIdx.x - (second ? blocks0 : 0)) * kPrepRows;
    prep_rows<false>(job, r0, d, dp, a, prec, poisoned, smean, raw, used);
}

// Thin-d variant: dst[row][d] = a (x - mean), padding rows get pad_value in every coordinate.
// One thread per padded row; same two-job grid.
__global__ __launch_bounds__(kBlock) void prep_thin_kernel(PrepJob job0, PrepJob job1, int blocks0, int d,
                                                           PrepCommon common, float a, Stamp stamp)
{
    __shared__ double red[kBlock];
    __shared__ float smean[SDKDE_MAX_D];
    __shared__ int stamp_flag;
    const bool poisoned = stamp_poisons(stamp, &stamp_flag);
    prep_common(common, d, red, smean);
    const bool second = (int)blockIdx.x >= blocks0;
    const PrepJob& job = second ? job1 : job0;
    const int64_t row = (int64_t)(blockIdx.x - (second ? blocks0 : 0)) * kBlock + threadIdx.x;
    if (row >= job.rows_pad) return;
    for (int c = 0; c < d; ++c)
        job.dst[row * d + c] = poisoned ? __builtin_nanf("") : row < job.rows ? a * (job.src[row * d + c] - smean[c]) : job.pad_value;
}

}  // namespace

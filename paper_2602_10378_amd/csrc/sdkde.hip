// SD-KDE hot path for MI355X (gfx950 / CDNA4): prep, pair-interaction kernels (fp32 MFMA for
// d >= 4, direct differences for thin d), split reduction + epilogues, and the C ABI.
//
// Notation follows the paper: c = 1/(2h^2), phi_ij = exp(-c |p_i - x_j|^2),
// D_i = sum_j phi_ij, T_i = sum_j phi_ij x_j  (Method section: T = Phi X).
//
// All coordinates are centred on the sample mean and scaled by a = sqrt(c log2 e), so that
// the squared distance in scaled units is directly the (negated) argument of exp2:
//     phi_ij = exp2( 2 p~_i . x~_j - |p~_i|^2 - |x~_j|^2 ).
// The cross term is the Gram-matrix tile of the Method section, computed with fp32 MFMA;
// the score numerator uses Phi X with the Phi tile still in the registers the first MFMA
// left it in.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <math.h>
#include <type_traits>
#include "sdkde.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr int kWave = 64;
constexpr int kBlock = 256;            // 4 waves per workgroup
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kTile = 16;              // MFMA 16x16x4 tile edge
constexpr int kRowPad = 1024;          // row padding of every prepared array (>= rows per workgroup)
constexpr float kPadNorm = -1.0e30f;   // "-|x|^2" of a padding sample: exp2 of it is exactly 0
constexpr float kPadCoord = 1.0e18f;   // thin-d padding coordinate: squared distance ~1e36, exp2(-that) = 0
constexpr int kMeanBlocks = 128;
constexpr int kFlushTiles = 64;         // sample tiles between folds of the running sums (power of two)
constexpr int kThinMaxD = 3;           // direct-difference path for d <= 3, MFMA path above

// What a pair kernel accumulates.
enum PairKind {
    kScoreSelf = 0,     // D and T at the samples themselves (own sample tiles skipped)
    kScorePoints = 1,   // D and T at separate points
    kEval = 2,          // D only (Gaussian KDE)
    kEvalLaplace = 3,   // sum of phi * (1 + d/2 - r^2/2h^2) (Laplace-corrected KDE; signed)
    kRowMax = 4,        // max_j of the exponent (first pass of the max-shifted mode); kept in the D slot
    kScoreBand = 5      // as kScoreSelf, but only the samples of the rows' own block (symmetric mode)
};
constexpr float kNegHuge = -3.0e38f;
constexpr float kLn2 = 0.693147180559945309f;

inline int64_t round_up(int64_t v, int64_t q) { return (v + q - 1) / q * q; }

// ------------------------------------------------------------------------------------------
// Prep: column means (deterministic two-stage reduction), then centre + scale + pad.
// ------------------------------------------------------------------------------------------

// partial[b][c] = sum over this block's rows of x[row][c], double accumulation.
__global__ __launch_bounds__(kBlock) void mean_partial_kernel(const float* __restrict__ x, int64_t n,
                                                              int d, double* __restrict__ partial)
{
    __shared__ double red[kBlock];
    const int rows_per_iter = kBlock / d;              // d <= 128 < kBlock
    const int rr = threadIdx.x / d, c = threadIdx.x % d;
    double acc = 0.0;
    if (rr < rows_per_iter) {
        for (int64_t row = (int64_t)blockIdx.x * rows_per_iter + rr; row < n;
             row += (int64_t)gridDim.x * rows_per_iter)
            acc += (double)x[row * d + c];
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < d) {
        double s = 0.0;
        for (int r = 0; r < rows_per_iter; ++r) s += red[r * d + threadIdx.x];
        partial[(int64_t)blockIdx.x * d + threadIdx.x] = s;
    }
}

// Second stage of the column mean, done by every prep workgroup for itself (saves a launch):
// sums the kMeanBlocks partials of each column in a fixed order, so all workgroups get the same
// bits.  Result in smean[0 .. d); ends with a barrier.
__device__ __forceinline__ void block_mean(const double* __restrict__ partial, int d, int64_t n, double* red,
                                           float* smean)
{
    const int slices = kBlock / d;                        // d <= 128, so >= 2
    const int sl = threadIdx.x / d, c = threadIdx.x % d;
    double acc = 0.0;
    if (sl < slices)
        for (int b = sl; b < kMeanBlocks; b += slices) acc += partial[(int64_t)b * d + c];
    red[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < d) {
        double t = 0.0;
        for (int q = 0; q < slices; ++q) t += red[q * d + threadIdx.x];
        smean[threadIdx.x] = (float)(t / (double)n);
    }
    __syncthreads();
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

constexpr int kPrepRows = 32;      // rows per workgroup of prep_mfma_kernel (two 16-sample tiles; 2 x 16.5 KiB of LDS)

// Centre, scale and pad for the MFMA path.  A workgroup stages kPrepRows rows in LDS and writes
//   dst[row][dp]   = a (x - mean), 0 in padding columns and rows (coalesced row writes),
//   dst_t[row/16][col][row%16] = the same values with each 16-sample tile transposed (if dst_t),
//   dst_n[row]     = -|dst[row]|^2 in double, rounded once; kPadNorm for padding rows.
// prec >= SDKDE_PREC_FP16X2 (fp16x2 input modes): dst holds, per 16-column block, 16 fp16 "hi" values
// followed by 16 fp16 "lo" values with hi + lo = the fp32 coordinate to ~22 mantissa bits (same bytes
// per row as fp32); the norm is then taken of hi + lo so that it matches what the MFMA multiplies.
// prec == SDKDE_PREC_FP16X2_ALL: dst_t holds fp16 pairs too, laid out as the A operand of the K = 32
// second contraction: for tile, column c and lane group g, eight halves [hi(4g..4g+3) | the same again]
// followed by eight halves [lo(4g..4g+3) | the same again] (twice the bytes of the fp32 layout).
// Grid: job0's blocks first (blocks0 of them), then job1's; sample mean from mean_partial.
__global__ __launch_bounds__(kBlock) void prep_mfma_kernel(PrepJob job0, PrepJob job1, int blocks0, int d, int dp,
                                                           const double* __restrict__ mean_partial, int64_t n_mean,
                                                           float a, int prec)
{
    __shared__ double red[kBlock];
    __shared__ float smean[SDKDE_MAX_D];
    __shared__ float raw[kPrepRows][SDKDE_MAX_D + 1];     // a (x - mean)
    __shared__ float used[kPrepRows][SDKDE_MAX_D + 1];    // the value the first contraction multiplies (hi + lo, or raw)
    block_mean(mean_partial, d, n_mean, red, smean);

    const bool second = (int)blockIdx.x >= blocks0;
    const PrepJob& job = second ? job1 : job0;
    const int64_t r0 = (int64_t)(blockIdx.x - (second ? blocks0 : 0)) * kPrepRows;
    _Float16* dst_h = reinterpret_cast<_Float16*>(job.dst);

    for (int idx = threadIdx.x; idx < kPrepRows * dp; idx += kBlock) {
        const int rr = idx / dp, c = idx % dp;
        const int64_t row = r0 + rr;
        float v = 0.0f;
        if (row < job.rows && c < d) v = a * (job.src[row * d + c] - smean[c]);
        raw[rr][c] = v;
        if (prec != SDKDE_PREC_FP32) {
            const _Float16 hi = (_Float16)v;
            const _Float16 lo = (_Float16)(v - (float)hi);
            _Float16* out = dst_h + row * 2 * dp + (c / 16) * 32 + (c % 16);
            out[0] = hi;
            out[16] = lo;
            v = (float)hi + (float)lo;
        } else {
            job.dst[row * dp + c] = v;
        }
        used[rr][c] = v;
    }
    __syncthreads();
    if (job.dst_t && prec != SDKDE_PREC_FP16X2_ALL) {
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
        job.dst_n[row] = row < job.rows ? -(float)acc : kPadNorm;
    }
}

// Thin-d variant: dst[row][d] = a (x - mean), padding rows get pad_value in every coordinate.
// One thread per padded row; same two-job grid.
__global__ __launch_bounds__(kBlock) void prep_thin_kernel(PrepJob job0, PrepJob job1, int blocks0, int d,
                                                           const double* __restrict__ mean_partial, int64_t n_mean,
                                                           float a)
{
    __shared__ double red[kBlock];
    __shared__ float smean[SDKDE_MAX_D];
    block_mean(mean_partial, d, n_mean, red, smean);
    const bool second = (int)blockIdx.x >= blocks0;
    const PrepJob& job = second ? job1 : job0;
    const int64_t row = (int64_t)(blockIdx.x - (second ? blocks0 : 0)) * kBlock + threadIdx.x;
    if (row >= job.rows_pad) return;
    for (int c = 0; c < d; ++c)
        job.dst[row * d + c] = row < job.rows ? a * (job.src[row * d + c] - smean[c]) : job.pad_value;
}

// ------------------------------------------------------------------------------------------
// Main pair kernel, MFMA path.
//
// One wave owns NI tiles of 16 evaluation rows (kept in registers as the B operand) and
// streams 16-sample tiles of the other set.  For every (row tile, sample tile) pair:
//   C[j][i]  = -|p_i|^2 - |x_j|^2                        (VALU, accumulator initialisation)
//   C       += X_J (16 x dp) * (2 P_I)^T (dp x 16)       (dp/4 MFMA 16x16x4, fp32)
//   Phi^T    = exp2(C)                                   (v_exp_f32)
//   D_i     += sum_j Phi^T[j][i]                         (VALU, per-lane partial)
//   T^T     += X_J^T (dp x 16) * Phi^T (16 x 16)         (dp/4 MFMA; SCORE only)
// The 16x16x4 accumulator layout (lane l, register v) = (row 4*(l/16)+v, column l%16) is exactly
// the B-operand layout (k = l/16, n = l%16) of the second MFMA for the four samples
// j = 4*(l/16)+v, so Phi never leaves its registers: register v is the B operand of the MFMA
// whose A operand holds samples {v, 4+v, 8+v, 12+v}; the blocked-transposed copy xt supplies
// that A operand with one float4 load per lane.  The contraction order over coordinates in the
// first MFMA is likewise permuted (MFMA kk contracts coordinates {kk, 4+kk, 8+kk, 12+kk} of each
// 16-column block) so that both operands are plain float4 row loads.
//
// SELF (score at the samples themselves): the pair (i, i) must stay out of D and T, because
// T_i/D_i - x_i would otherwise cancel against the large self term whenever a point has few
// neighbours; the epilogue restores it analytically (phi_ii = 1).  This kernel therefore skips
// the NI sample tiles that are the wave's own row tiles; pair_diag_kernel covers them.
//
// Grid: blockIdx.x = row_block * S + split; each workgroup handles RB = 64*NI rows and the
// sample tiles [split*tiles_per_split, min(ntiles, (split+1)*tiles_per_split)).  With S a
// multiple of 8 the round-robin placement of workgroups on the 8 XCDs makes each XCD stream
// only its own eighth of the samples through its L2.
// All arrays are padded so that every access below is in bounds:
//   ps, pn : m_pad rows (multiple of kRowPad >= RB);  xs, xt, xn : ntiles*16 rows.
// ------------------------------------------------------------------------------------------

// fp16x2-all mode: Phi is produced as 2^kPhiScaleLog2 * phi (the offset rides on the row constant, so it
// is free) so that values down to 2^-28 keep full fp16 precision; phi <= 1 keeps the product below 65504.
constexpr int kPhiScaleLog2 = 14;

// [hi(x) hi(y) hi(z) hi(w) | lo(x) lo(y) lo(z) lo(w)] with hi = fp16(phi) (toward zero) and
// lo = fp16(phi - hi).  The residual is formed by the mixed-precision FMA (fp32 phi * 1.0 - fp16 hi, result
// rounded to fp16 into one half of the destination): six VALU instructions for four values.
__device__ __forceinline__ f16x8 split_phi(const f32x4& phi)
{
    const uint32_t h01 = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(phi.x, phi.y));
    const uint32_t h23 = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(phi.z, phi.w));
    uint32_t l01, l23;      // mixlo leaves the upper half as it was; mixhi then writes it
    asm("v_fma_mixlo_f16 %0, %1, 1.0, -%2 op_sel_hi:[0,0,1]" : "=v"(l01) : "v"(phi.x), "v"(h01));
    asm("v_fma_mixhi_f16 %0, %1, 1.0, -%2 op_sel:[0,0,1] op_sel_hi:[0,0,1]" : "+v"(l01) : "v"(phi.y), "v"(h01));
    asm("v_fma_mixlo_f16 %0, %1, 1.0, -%2 op_sel_hi:[0,0,1]" : "=v"(l23) : "v"(phi.z), "v"(h23));
    asm("v_fma_mixhi_f16 %0, %1, 1.0, -%2 op_sel:[0,0,1] op_sel_hi:[0,0,1]" : "+v"(l23) : "v"(phi.w), "v"(h23));
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    return __builtin_bit_cast(f16x8, (u32x4){h01, h23, l01, l23});
}

// Row-tile operands of one wave for NI row tiles starting at row0: -|p~|^2 and the B operand 2 * p~.
// fp32 inputs: lane (r, g) holds coordinates 16kb + 4g .. +3 of row r (b[t][kb]).
// fp16x2 inputs: two K = 32 operands per 16-column block, bh[t][kb][0] = [hi | hi] and
// bh[t][kb][1] = [lo | lo]; lane (r, g) holds elements 8g .. 8g+7 of that K axis, i.e. halves
// 8(g&1) .. +7 of the hi (resp. lo) part.  Against the streamed A operand [hi | lo] the two MFMAs
// sum hi*hi + lo*hi + hi*lo + lo*lo = the full product.
template <int KB, int NI, int PREC>
struct RowTiles {
    f32x4 b[PREC == SDKDE_PREC_FP32 ? NI : 1][KB];
    f16x8 bh[PREC != SDKDE_PREC_FP32 ? NI : 1][KB][2];
    float ni[NI];

    __device__ __forceinline__ void load(const float* __restrict__ ps, const float* __restrict__ pn, int64_t row0,
                                         int r, int g)
    {
        constexpr int DP = KB * 16;
#pragma unroll
        for (int t = 0; t < NI; ++t) {
            const int64_t row = row0 + t * kTile + r;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                if (PREC == SDKDE_PREC_FP32) {
                    f32x4 v = *reinterpret_cast<const f32x4*>(ps + row * DP + kb * 16 + g * 4);
                    b[t][kb] = v * 2.0f;
                } else {
                    const _Float16* ph = reinterpret_cast<const _Float16*>(ps) + row * 2 * DP + kb * 32 + (g & 1) * 8;
                    bh[t][kb][0] = *reinterpret_cast<const f16x8*>(ph) * (_Float16)2;
                    bh[t][kb][1] = *reinterpret_cast<const f16x8*>(ph + 16) * (_Float16)2;
                }
            }
            ni[t] = pn[row];
        }
    }

    // c += (16 samples x 16-column block kb) * (row tile t)^T; a = the lane's 16 bytes of the streamed operand.
    __device__ __forceinline__ f32x4 cross(int t, int kb, const f32x4& a, f32x4 c) const
    {
        if (PREC == SDKDE_PREC_FP32) {
            c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b[t][kb].x, c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b[t][kb].y, c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b[t][kb].z, c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b[t][kb].w, c, 0, 0, 0);
        } else {
            const f16x8 ah = __builtin_bit_cast(f16x8, a);
            c = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, bh[t][kb][0], c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, bh[t][kb][1], c, 0, 0, 0);
        }
        return c;
    }
};

// Writes one wave's partial sums: T^T accumulator (lane (r, g), register v) = coordinate
// 16mb + 4g + v of row r; D needs the sum over the four lane groups g.
template <int KB, int NI, bool SCORE, bool ROWMAX = false>
__device__ __forceinline__ void store_partials(float* __restrict__ part_t, float* __restrict__ part_d, int64_t slot,
                                               int64_t m_pad, int64_t row0, int r, int g,
                                               const f32x4 (&tsum)[NI][SCORE ? KB : 1], const float (&dsum)[NI])
{
    constexpr int DP = KB * 16;
#pragma unroll
    for (int t = 0; t < NI; ++t) {
        const int64_t row = row0 + t * kTile + r;
        if (SCORE) {
            float* dst = part_t + (slot * m_pad + row) * DP + g * 4;
#pragma unroll
            for (int mb = 0; mb < KB; ++mb) *reinterpret_cast<f32x4*>(dst + mb * 16) = tsum[t][mb];
        }
        float dtot = dsum[t];
        if (ROWMAX) {
            dtot = fmaxf(dtot, __shfl_xor(dtot, 16));
            dtot = fmaxf(dtot, __shfl_xor(dtot, 32));
        } else {
            dtot += __shfl_xor(dtot, 16);
            dtot += __shfl_xor(dtot, 32);
        }
        if (g == 0) part_d[slot * m_pad + row] = dtot;
    }
}

template <int KB, int NI, int KIND, int PREC>
__global__ __launch_bounds__(kBlock) void pair_mfma_kernel(
    const float* __restrict__ ps, const float* __restrict__ pn, const float* __restrict__ xs,
    const float* __restrict__ xt, const float* __restrict__ xn, float* __restrict__ part_t,
    float* __restrict__ part_d, int ntiles, int tiles_per_split, int nsplit, int64_t m_pad, float laplace_c0,
    const float* __restrict__ shift)
{
    static_assert(NI >= 2 && NI % 2 == 0, "the software pipeline alternates two accumulator sets");
    constexpr bool BAND = KIND == kScoreBand;
    constexpr bool SCORE = KIND == kScoreSelf || KIND == kScorePoints || BAND;
    constexpr bool SELF = KIND == kScoreSelf || BAND;
    constexpr bool LAPLACE = KIND == kEvalLaplace;
    constexpr bool ROWMAX = KIND == kRowMax;
    constexpr int DP = KB * 16;
    constexpr int NM = 4 * KB;                 // MFMAs per contraction and tile
    constexpr int KT = SCORE ? KB : 1;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);    // wave-uniform by construction
    const int r = lane & 15, g = lane >> 4;
    const int split = blockIdx.x % nsplit;
    const int64_t row_block = blockIdx.x / nsplit;
    const int64_t row0 = (row_block * kWavesPerBlock + wave) * (NI * kTile);

    RowTiles<KB, NI, PREC> rows;
    rows.load(ps, pn, row0, r, g);
    if (SCORE && PREC == SDKDE_PREC_FP16X2_ALL) {
        // every Phi of this kernel carries the factor 2^kPhiScaleLog2 (exact; removed from the sums at the end)
#pragma unroll
        for (int t = 0; t < NI; ++t) rows.ni[t] += (float)kPhiScaleLog2;
    }
    const float (&ni)[NI] = rows.ni;

    // Two-level accumulation: the running sums (tacc, dacc) are folded into (tsum, dsum) every
    // kFlushTiles sample tiles, so no fp32 accumulator sees more than a short chain of additions
    // at its own magnitude (keeps the rounding of T and D well below the cancellation in T/D - x).
    f32x4 tacc[NI][KT], tsum[NI][KT];
    float dacc[NI], dsum[NI];
    float lc0[LAPLACE ? NI : 1];          // Laplace factor constant per row tile: 1 + d/2 + shift_i ln 2
#pragma unroll
    for (int t = 0; t < NI; ++t) {
        dacc[t] = dsum[t] = ROWMAX ? kNegHuge : 0.0f;
#pragma unroll
        for (int mb = 0; mb < KT; ++mb) tacc[t][mb] = tsum[t][mb] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (LAPLACE) lc0[t] = fmaf(shift ? shift[row0 + t * kTile + r] : 0.0f, kLn2, laplace_c0);
    }

    // ntiles, tiles_per_split and NI are even (host side), so every span of sample tiles below
    // has even length and the loop can alternate two operand register sets without copies.
    const int dt0 = (int)(row0 / kTile);          // the wave's own row tiles are sample tiles dt0 .. dt0+NI-1
    int t_begin = split * tiles_per_split;
    int t_end = min(ntiles, t_begin + tiles_per_split);
    if (BAND) {
        // symmetric mode: only the samples of the rows' own block, tiles_per_split tiles long (the pairs
        // across blocks belong to pair_sym_kernel); nsplit is 1
        t_begin = dt0 / tiles_per_split * tiles_per_split;
        t_end = min(ntiles, t_begin + tiles_per_split);
    }

    // Operands of one sample tile, as each lane holds them.
    constexpr bool HALF2 = PREC == SDKDE_PREC_FP16X2_ALL;      // second contraction on the fp16 units too
    struct Operands {
        f32x4 a1[KB];     // first contraction, A: the lane's 16 bytes of sample r's row, block kb (fp32: coordinates
                          // 16kb + 4g .. +3; fp16x2: elements 8g .. 8g+7 of [hi | lo])
        f32x4 a2[KT];     // second contraction, A: lane (r, g) = coordinate 16mb + r of samples 4g .. 4g+3
                          // (fp32), or the eight halves [hi(4g..4g+3) | again] when HALF2
        f32x4 a2lo[HALF2 ? KT : 1];   // HALF2 only: [lo(4g..4g+3) | again]
        f32x4 nj;         // -|x|^2 of samples 4g .. 4g+3
    };
    Operands set_a, set_b;
    f32x4 creg[2], ph[2];

    // SELF: two spans, before and after the wave's own tiles; otherwise the whole range.
    for (int span = 0; span < (SELF ? 2 : 1); ++span) {
        int s_begin = t_begin, s_end = t_end;
        if (SELF) {
            if (span == 0) s_end = min(t_end, dt0);
            else s_begin = max(t_begin, dt0 + NI);
        }
        if (s_begin >= s_end) continue;

        const int t_last = s_end - 1;     // prefetches past the span re-read its last tile (in bounds)
        auto load_a1 = [&](int jt, Operands& o) {
            const float* xrow = xs + ((int64_t)min(jt, t_last) * kTile + r) * DP + g * 4;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) o.a1[kb] = *reinterpret_cast<const f32x4*>(xrow + kb * 16);
        };
        auto load_a2 = [&](int jt, Operands& o) {
            if (SCORE && !HALF2) {
                const float* trow = xt + ((int64_t)min(jt, t_last) * DP + r) * kTile + g * 4;
#pragma unroll
                for (int mb = 0; mb < KB; ++mb)
                    o.a2[mb] = *reinterpret_cast<const f32x4*>(trow + mb * 16 * kTile);
            } else if (SCORE) {
                // 32 bytes per (column, lane group): [hi | hi] then [lo | lo]
                const float* trow = xt + (((int64_t)min(jt, t_last) * DP + r) * 4 + g) * 8;
#pragma unroll
                for (int mb = 0; mb < KB; ++mb) {
                    o.a2[mb] = *reinterpret_cast<const f32x4*>(trow + mb * 16 * 32);
                    o.a2lo[mb] = *reinterpret_cast<const f32x4*>(trow + mb * 16 * 32 + 4);
                }
            }
        };
        auto load_nj = [&](int jt, Operands& o) {
            o.nj = *reinterpret_cast<const f32x4*>(xn + (int64_t)min(jt, t_last) * kTile + g * 4);
        };

        // Software pipeline over the flattened sequence of (sample tile, row tile) pairs u:
        //   [first contraction of pair u+1]  (4*KB MFMAs, back to back)
        //   [VALU clump: exp2 + row sum of pair u, accumulator init of pair u+2]
        //   [second contraction of pair u]   (4*KB MFMAs, back to back)
        // On gfx950 the fp32 MFMA does not overlap with VALU work of the same SIMD (measured:
        // every VALU instruction adds its full issue time, plus ~8 clocks each time the stream
        // switches between MFMA and VALU), so VALU work is gathered into one clump per pair
        // instead of being interleaved, and each clump only touches results that are at least
        // one MFMA group old, so it never waits.  creg[u & 1] holds the exponent tile of pair u,
        // ph[u & 1] its Phi^T tile.  Scheduling barriers pin the groups.
        //
        // Operand prefetch: two register sets alternate between "current" and "next" sample tile.
        // Each part of a set is reloaded for the tile after next as soon as its last reader has
        // issued, which puts every load about one full iteration (NI pairs) ahead of its use.
        load_a1(s_begin, set_a);
        load_a2(s_begin, set_a);
        load_nj(s_begin, set_a);
        creg[0] = set_a.nj + ni[0];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) creg[0] = rows.cross(0, kb, set_a.a1[kb], creg[0]);
        creg[1] = set_a.nj + ni[1];
        load_a1(s_begin + 1, set_b);
        load_nj(s_begin + 1, set_b);

        // Sample tile jt (operands in cur; those of jt+1 arriving in nxt) against all NI row tiles.
        auto iteration = [&](int jt, Operands& cur, Operands& nxt) {
            load_a2(jt + 1, nxt);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < NI; ++t) {
                const int slot = t & 1;
                const bool wrap1 = t + 1 >= NI, wrap2 = t + 2 >= NI;     // compile-time after unrolling
                f32x4& c = creg[slot];
                f32x4& phi = ph[slot];
                const float nin = ni[(t + 2) % NI];

                if (t == NI - 2) {              // cur.nj was last read by the clump of t = NI - 3
                    load_nj(jt + 2, cur);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
                    creg[slot ^ 1] = rows.cross((t + 1) % NI, kb, wrap1 ? nxt.a1[kb] : cur.a1[kb], creg[slot ^ 1]);
                __builtin_amdgcn_sched_barrier(0);
                if (t == NI - 2) load_a1(jt + 2, cur);    // cur.a1 was last read by the MFMAs above

                if (ROWMAX) {
                    dacc[t] = fmaxf(dacc[t], fmaxf(fmaxf(c.x, c.y), fmaxf(c.z, c.w)));
                } else {
                    phi.x = __builtin_amdgcn_exp2f(c.x);
                    phi.y = __builtin_amdgcn_exp2f(c.y);
                    phi.z = __builtin_amdgcn_exp2f(c.z);
                    phi.w = __builtin_amdgcn_exp2f(c.w);
                    if (LAPLACE) {
                        // c is the base-2 exponent -r^2/(2h^2) log2(e) (less the row's shift), so the Laplace
                        // factor 1 + d/2 - r^2/(2h^2) is lc0 + c ln 2 (Laplace-corrected KDE section).
                        float acc = dacc[t];
                        acc = fmaf(phi.x, fmaf(c.x, kLn2, lc0[t]), acc);
                        acc = fmaf(phi.y, fmaf(c.y, kLn2, lc0[t]), acc);
                        acc = fmaf(phi.z, fmaf(c.z, kLn2, lc0[t]), acc);
                        acc = fmaf(phi.w, fmaf(c.w, kLn2, lc0[t]), acc);
                        dacc[t] = acc;
                    } else {
                        dacc[t] += (phi.x + phi.y) + (phi.z + phi.w);
                    }
                }
                c = (wrap2 ? nxt.nj : cur.nj) + nin;             // accumulator init of pair u+2
                f16x8 bphi;
                if (SCORE && HALF2) bphi = split_phi(phi);       // part of the same VALU clump
                __builtin_amdgcn_sched_barrier(0);

                if (SCORE && !HALF2) {
#pragma unroll
                    for (int i = 0; i < NM; ++i) {
                        const int v = i / KB, mb = i % KB;     // the KB accumulator chains interleave
                        tacc[t][mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(cur.a2[mb][v], phi[v], tacc[t][mb], 0, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                } else if (SCORE) {
                    // Phi^T split as hi + lo (fp16 each; Phi carries a factor 2^14 so that its small values
                    // stay normal in fp16): K = 32 is [hi(4 samples) | lo(4 samples)] per lane group, against
                    // [x_hi | x_hi] and [x_lo | x_lo]: two MFMAs give (phi_hi + phi_lo)(x_hi + x_lo).
#pragma unroll
                    for (int mb = 0; mb < KB; ++mb) {
                        tacc[t][mb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, cur.a2[mb]), bphi,
                                                                             tacc[t][mb], 0, 0, 0);
                        tacc[t][mb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, cur.a2lo[mb]), bphi,
                                                                             tacc[t][mb], 0, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };

        for (int jt = s_begin; jt < s_end; jt += 2) {
            iteration(jt, set_a, set_b);
            iteration(jt + 1, set_b, set_a);
            if (((jt + 1 - s_begin) & (kFlushTiles - 1)) == kFlushTiles - 1) {    // wave-uniform
#pragma unroll
                for (int t = 0; t < NI; ++t) {
                    if (!ROWMAX) {
                        dsum[t] += dacc[t];
                        dacc[t] = 0.0f;
                    }
#pragma unroll
                    for (int mb = 0; mb < KT; ++mb) {
                        tsum[t][mb] += tacc[t][mb];
                        tacc[t][mb] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
                }
            }
        }
        // The pipeline has started pair (s_end, 0) on a re-read of the last tile; it is dropped.
    }
#pragma unroll
    for (int t = 0; t < NI; ++t) {
        dsum[t] = ROWMAX ? fmaxf(dsum[t], dacc[t]) : dsum[t] + dacc[t];
#pragma unroll
        for (int mb = 0; mb < KT; ++mb) tsum[t][mb] += tacc[t][mb];
        if (SCORE && PREC == SDKDE_PREC_FP16X2_ALL) {
            constexpr float unscale = 1.0f / (float)(1 << kPhiScaleLog2);
            dsum[t] *= unscale;
#pragma unroll
            for (int mb = 0; mb < KT; ++mb) tsum[t][mb] *= unscale;
        }
    }
    store_partials<KB, NI, SCORE, ROWMAX>(part_t, part_d, split, m_pad, row0, r, g, tsum, dsum);
}

// Diagonal blocks of the score at the samples themselves: every wave pairs its NI row tiles with
// the same NI tiles taken as samples, leaving out the pair of each point with itself, and writes
// the sums into partial slot `slot` (one past the splits of pair_mfma_kernel).  Same operand
// layouts as above; a plain loop, since this is NI*16 pairs per row out of n.
// Grid: one workgroup per row block, as in the main kernel.
template <int KB, int NI, int PREC>
__global__ __launch_bounds__(kBlock) void pair_diag_kernel(
    const float* __restrict__ xs, const float* __restrict__ xt, const float* __restrict__ xn,
    float* __restrict__ part_t, float* __restrict__ part_d, int ntiles, int slot, int64_t m_pad)
{
    constexpr int DP = KB * 16;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);    // wave-uniform by construction
    const int r = lane & 15, g = lane >> 4;
    const int64_t row0 = ((int64_t)blockIdx.x * kWavesPerBlock + wave) * (NI * kTile);
    const int dt0 = (int)(row0 / kTile);

    RowTiles<KB, NI, PREC> rows;
    rows.load(xs, xn, row0, r, g);
    if (PREC == SDKDE_PREC_FP16X2_ALL) {      // Phi carries 2^kPhiScaleLog2, as in pair_mfma_kernel
#pragma unroll
        for (int t = 0; t < NI; ++t) rows.ni[t] += (float)kPhiScaleLog2;
    }
    f32x4 tsum[NI][KB];
    float dsum[NI];
#pragma unroll
    for (int t = 0; t < NI; ++t) {
        dsum[t] = 0.0f;
#pragma unroll
        for (int mb = 0; mb < KB; ++mb) tsum[t][mb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (int dt = 0; dt < NI; ++dt) {
        const int jt = dt0 + dt;
        if (jt >= ntiles) break;               // rows past the last sample tile are padding
        constexpr bool HALF2 = PREC == SDKDE_PREC_FP16X2_ALL;
        f32x4 a1[KB], a2[KB], a2lo[HALF2 ? KB : 1];
        const float* xrow = xs + ((int64_t)jt * kTile + r) * DP + g * 4;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) a1[kb] = *reinterpret_cast<const f32x4*>(xrow + kb * 16);
        if (!HALF2) {
            const float* trow = xt + ((int64_t)jt * DP + r) * kTile + g * 4;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) a2[kb] = *reinterpret_cast<const f32x4*>(trow + kb * 16 * kTile);
        } else {
            const float* trow = xt + (((int64_t)jt * DP + r) * 4 + g) * 8;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                a2[kb] = *reinterpret_cast<const f32x4*>(trow + kb * 16 * 32);
                a2lo[kb] = *reinterpret_cast<const f32x4*>(trow + kb * 16 * 32 + 4);
            }
        }
        const f32x4 nj = *reinterpret_cast<const f32x4*>(xn + (int64_t)jt * kTile + g * 4);
#pragma unroll
        for (int t = 0; t < NI; ++t) {
            f32x4 c = nj + rows.ni[t];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) c = rows.cross(t, kb, a1[kb], c);
            f32x4 phi;
            // register v of lane (r, g) is the pair (sample 4g + v, row r) of this tile
            const bool own = t == dt;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float e = __builtin_amdgcn_exp2f(c[v]);
                phi[v] = (own && g * 4 + v == r) ? 0.0f : e;
            }
            dsum[t] += (phi.x + phi.y) + (phi.z + phi.w);
            if (!HALF2) {
#pragma unroll
                for (int mb = 0; mb < KB; ++mb)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        tsum[t][mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a2[mb][v], phi[v], tsum[t][mb], 0, 0, 0);
            } else {
                const f16x8 bphi = split_phi(phi);
#pragma unroll
                for (int mb = 0; mb < KB; ++mb) {
                    tsum[t][mb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a2[mb]), bphi, tsum[t][mb], 0, 0, 0);
                    tsum[t][mb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a2lo[mb]), bphi, tsum[t][mb], 0, 0, 0);
                }
            }
        }
    }
    if (PREC == SDKDE_PREC_FP16X2_ALL) {
        constexpr float unscale = 1.0f / (float)(1 << kPhiScaleLog2);
#pragma unroll
        for (int t = 0; t < NI; ++t) {
            dsum[t] *= unscale;
#pragma unroll
            for (int mb = 0; mb < KB; ++mb) tsum[t][mb] *= unscale;
        }
    }
    store_partials<KB, NI, true>(part_t, part_d, slot, m_pad, row0, r, g, tsum, dsum);
}

// ------------------------------------------------------------------------------------------
// Symmetric score at the samples themselves (separate mode, SDKDE_FLAG_SYMMETRIC).
//
// phi_ij = phi_ji, so each unordered pair of samples needs one Gram-matrix entry and one exp.  A
// wave that holds row tile I and streams sample tile J computes the tile Phi once and uses it twice:
//   T_I^T += X_J^T (dp x 16) * Phi^T (16 x 16)      as in pair_mfma_kernel, Phi^T from its registers,
//   T_J^T += X_I^T (dp x 16) * Phi   (16 x 16)      with the tile transposed through 1.25 KiB of LDS
// (three groups of MFMAs for two ordered pairs instead of four, and half the exps).
//
// The samples are cut into blocks of `rb` rows; only pairs (i in an earlier block, j in a later block)
// are handled here, pairs inside one block go through pair_mfma_kernel restricted to that block.
// A workgroup (8 waves) takes one item = (chunk c of `per_group` blocks, group gam >= c of `per_group`
// blocks) and, for every block b of the group:
//   - keeps the accumulators [T_J | D_J] of the block's rb rows in LDS ([KB][rb][16] + [rb] floats),
//   - walks over the rows of the chunk that lie before block b, 8 * NI * 16 at a time; each wave holds
//     NI row tiles (operands and T_I, D_I in registers) and streams one eighth of the block per phase,
//     wave w taking eighth (w + phase) mod 8, so that within a phase every LDS accumulator row has one
//     owner and the order of all additions is fixed (no atomics; barriers between phases),
//   - adds the wave's T_I, D_I into partial slot gam + 1 of its rows (the same lanes add the blocks of a
//     group one after the other: first a store, then read-add-write),
//   - writes the block's LDS accumulators into partial slot c.
// A row of chunk/group rho thus receives slots 0..rho (as streamed sample, one per chunk) and
// rho+1..ngroups (as row, one per group): ngroups + 1 slots, every one written exactly once (rows that meet
// no later block in their own group get zeros).
//
// Pipeline per (sample tile, row tile) pair u, on top of the schedule of pair_mfma_kernel:
//   [T_I MFMAs of u] [T_J MFMAs of u-1] [Gram MFMAs of u+2] | VALU clump of u+1: exp2, row sum, column sum of
//   the transposed tile of u, accumulator init; LDS: write Phi(u+1), read it back transposed | ...
// The T_J MFMAs run one pair behind so that the transposed tile has a whole stage to come back from LDS.
// The T_J accumulator of a sample tile is added into LDS during the next tile (rows read in the clump of
// its row tile 0, add and write in that of row tile 1), when its MFMAs have long finished.
// ------------------------------------------------------------------------------------------
constexpr int kSymWaves = 8;
constexpr int kSymBlock = kSymWaves * kWave;

// x summed over the four lanes that share lane % 16 (the four 16-lane rows of the wave), in every lane, as
// (row 0 + row 1) + (row 2 + row 3).  The row-swap instructions of gfx950 keep this on the VALU; a shuffle
// would go through the LDS crossbar and make the wave wait for its round trip.
__device__ __forceinline__ float sum_over_lane_rows(float x)
{
    float a = x, b = x;
    // lanes 16-31 of a <-> lanes 0-15 of b, lanes 48-63 of a <-> lanes 32-47 of b
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    a += b;
    b = a;
    // lanes 32-63 of a <-> lanes 0-31 of b
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return a + b;
}
constexpr int kTrStride = 20;      // floats per row of the 16 x 16 transpose tile: 16-byte aligned rows, no bank conflicts

inline size_t sym_lds_bytes(int kb, int rb)
{
    return sizeof(float) * ((size_t)kb * rb * 16 + rb + kSymWaves * 16 * kTrStride);
}

template <int KB, int NI, int PREC>
__global__ __launch_bounds__(kSymBlock) void pair_sym_kernel(
    const float* __restrict__ xs, const float* __restrict__ xt, const float* __restrict__ xn,
    float* __restrict__ part_t, float* __restrict__ part_d, int64_t n_pad, int rb, int nblocks, int per_group,
    int ngroups)
{
    static_assert(NI >= 2 && NI % 2 == 0, "the software pipeline alternates two accumulator sets");
    static_assert(PREC != SDKDE_PREC_FP16X2_ALL, "the transposed tile is consumed in fp32");
    extern __shared__ __align__(16) float sym_lds[];
    constexpr int DP = KB * 16;
    constexpr int SB = kSymWaves * NI * kTile;          // rows a workgroup holds at a time
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int r = lane & 15, g = lane >> 4;

    float* const lds_t = sym_lds;                            // [KB][rb][16]
    float* const lds_d = lds_t + (size_t)KB * rb * 16;       // [rb]
    float* const tr = lds_d + rb + wave * (16 * kTrStride);  // this wave's transpose tile
    f32x4* const tr_wr = reinterpret_cast<f32x4*>(tr + r * kTrStride + g * 4);    // row r, columns 4g .. 4g+3
    const float* const tr_rd = tr + g * 4 * kTrStride + r;                         // rows 4g .. 4g+3, column r

    // item -> (c, gam): the ngroups (ngroups - 1) / 2 full rectangles first, the triangular items c == gam last
    const int id = blockIdx.x;
    const int noff = ngroups * (ngroups - 1) / 2;
    int c, gam;
    if (id < noff) {
        gam = (int)((1.0f + sqrtf(1.0f + 8.0f * (float)id)) * 0.5f);
        while (gam * (gam - 1) / 2 > id) --gam;
        while ((gam + 1) * gam / 2 <= id) ++gam;
        c = id - gam * (gam - 1) / 2;
    } else {
        c = gam = id - noff;
    }
    const int b_lo = gam * per_group, b_hi = min(nblocks, b_lo + per_group);
    const int64_t a_lo = (int64_t)c * per_group * rb;
    const int64_t a_hi = min(n_pad, a_lo + (int64_t)per_group * rb);
    const int64_t slot_a = gam + 1, slot_b = c;
    const int tiles_per_phase = rb / (kSymWaves * kTile);    // an even power of two (host side)
    const int tp_shift = __ffs(tiles_per_phase) - 1;

    struct Operands {
        f32x4 a1[KB];     // Gram contraction, A: the lane's 16 bytes of sample r's row, block kb
        f32x4 a2[KB];     // T_I contraction, A: coordinate 16mb + r of samples 4g .. 4g+3
        f32x4 nj;         // -|x|^2 of samples 4g .. 4g+3
    };

    for (int b = b_lo; b < b_hi; ++b) {
        for (int idx = threadIdx.x; idx < KB * rb * 16 + rb; idx += kSymBlock) sym_lds[idx] = 0.0f;
        __syncthreads();
        const int bt0 = b * (rb / kTile);                     // first sample tile of the block
        const int64_t a_end = min(a_hi, (int64_t)b * rb);     // rows strictly before the block

        for (int64_t a0 = a_lo; a0 < a_end; a0 += SB) {
            const int64_t row0 = a0 + (int64_t)wave * (NI * kTile);
            RowTiles<KB, NI, PREC> rows;
            rows.load(xs, xn, row0, r, g);
            const float (&ni)[NI] = rows.ni;
            f32x4 xti[NI][KB];      // T_J contraction, A: coordinate 16mb + r of rows 4g .. 4g+3 of row tile t
#pragma unroll
            for (int t = 0; t < NI; ++t) {
                const float* trow = xt + ((row0 / kTile + t) * DP + r) * kTile + g * 4;
#pragma unroll
                for (int mb = 0; mb < KB; ++mb) xti[t][mb] = *reinterpret_cast<const f32x4*>(trow + mb * 16 * kTile);
            }
            f32x4 tacc[NI][KB];
            float dacc[NI];
#pragma unroll
            for (int t = 0; t < NI; ++t) {
                dacc[t] = 0.0f;
#pragma unroll
                for (int mb = 0; mb < KB; ++mb) tacc[t][mb] = f32x4{0.f, 0.f, 0.f, 0.f};
            }

            {
                // The wave's stream of sample tiles through the block: position q is tile q % TP of eighth
                // (wave + q / TP) mod 8 (TP = tiles_per_phase, a power of two).  The software pipeline runs through
                // the whole stream; at every multiple of TP the wave finishes its T_J sums and all waves meet.
                const int q_last = kSymWaves * tiles_per_phase - 1;     // prefetches past the stream re-read its last tile
                auto tile_of = [&](int q) {
                    q = min(q, q_last);
                    return bt0 + (((wave + (q >> tp_shift)) & (kSymWaves - 1)) << tp_shift) + (q & (tiles_per_phase - 1));
                };
                Operands set_a, set_b;
                f32x4 creg[2], ph[2], pht[2];
                f32x4 acc3[KB];          // T_J^T of the current sample tile: (lane (r, g), v) = coordinate 16mb + 4g + v
                                         // of sample r
                float cacc, cprev;       // sum over rows 4g .. 4g+3 of all row tiles of Phi[.][sample r]; the part of it
                                         // that arrives one clump late (last pair of the tile)
                f32x4 fold[KB];          // the LDS accumulator rows the next fold adds to, read one stage ahead
                float dfold;

                auto load_a1 = [&](int q, Operands& o) {
                    const float* xrow = xs + ((int64_t)tile_of(q) * kTile + r) * DP + g * 4;
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb) o.a1[kb] = *reinterpret_cast<const f32x4*>(xrow + kb * 16);
                };
                auto load_a2 = [&](int q, Operands& o) {
                    const float* trow = xt + ((int64_t)tile_of(q) * DP + r) * kTile + g * 4;
#pragma unroll
                    for (int mb = 0; mb < KB; ++mb) o.a2[mb] = *reinterpret_cast<const f32x4*>(trow + mb * 16 * kTile);
                };
                auto load_nj = [&](int q, Operands& o) {
                    o.nj = *reinterpret_cast<const f32x4*>(xn + (int64_t)tile_of(q) * kTile + g * 4);
                };
                // LDS accumulator rows of sample tile jt (block-local), this lane's 16 bytes of block mb
                auto lds_row = [&](int jt, int mb) {
                    return lds_t + ((size_t)mb * rb + (size_t)(jt - bt0) * kTile + r) * 16 + g * 4;
                };
                auto load_fold = [&](int jt) {
#pragma unroll
                    for (int mb = 0; mb < KB; ++mb) fold[mb] = *reinterpret_cast<const f32x4*>(lds_row(jt, mb));
                    dfold = lds_d[(jt - bt0) * kTile + r];
                };
                // adds the finished tile's T_J^T and column sums to the rows read by load_fold(jt)
                auto store_fold = [&](int jt) {
#pragma unroll
                    for (int mb = 0; mb < KB; ++mb) *reinterpret_cast<f32x4*>(lds_row(jt, mb)) = fold[mb] + acc3[mb];
                    // all four lanes of a column hold the same sum and write the same value
                    lds_d[(jt - bt0) * kTile + r] = dfold + sum_over_lane_rows(cacc + cprev);
                    cacc = 0.0f;
                };

                load_a1(0, set_a);
                load_a2(0, set_a);
                load_nj(0, set_a);
                creg[0] = set_a.nj + ni[0];
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) creg[0] = rows.cross(0, kb, set_a.a1[kb], creg[0]);
                creg[1] = set_a.nj + ni[1];
                load_a1(1, set_b);
                load_nj(1, set_b);
                pht[0] = pht[1] = f32x4{0.f, 0.f, 0.f, 0.f};
                cacc = cprev = 0.0f;
#pragma unroll
                for (int mb = 0; mb < KB; ++mb) acc3[mb] = f32x4{0.f, 0.f, 0.f, 0.f};

                // Stream position q (operands in cur) against all NI row tiles.  The T_J MFMAs run one pair behind
                // (their transposed tile was read from LDS a whole stage earlier), so the previous tile's T_J^T
                // is complete after the MFMAs of row tile 0 and is folded into LDS in the clump of row tile 1
                // (first tile of a phase: nothing is pending, zeros are added to the tile's own rows).
                auto iteration = [&](int q, Operands& cur, Operands& nxt) {
                    const int jt = tile_of(q);
                    const int jprev = (q & (tiles_per_phase - 1)) ? jt - 1 : jt;
                    load_a2(q + 1, nxt);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int t = 0; t < NI; ++t) {
                        const int slot = t & 1;
                        const bool wrap1 = t + 1 >= NI, wrap2 = t + 2 >= NI;
                        f32x4& cc = creg[slot];
                        f32x4& phi = ph[slot];
                        const float nin = ni[(t + 2) % NI];

                        if (t == NI - 2) {
                            load_nj(q + 2, cur);
                            __builtin_amdgcn_sched_barrier(0);
                        }
#pragma unroll
                        for (int kb = 0; kb < KB; ++kb)
                            creg[slot ^ 1] = rows.cross((t + 1) % NI, kb, wrap1 ? nxt.a1[kb] : cur.a1[kb], creg[slot ^ 1]);
                        __builtin_amdgcn_sched_barrier(0);
                        if (t == NI - 2) load_a1(q + 2, cur);

                        // VALU clump
                        phi.x = __builtin_amdgcn_exp2f(cc.x);
                        phi.y = __builtin_amdgcn_exp2f(cc.y);
                        phi.z = __builtin_amdgcn_exp2f(cc.z);
                        phi.w = __builtin_amdgcn_exp2f(cc.w);
                        dacc[t] += (phi.x + phi.y) + (phi.z + phi.w);
                        asm volatile("" : "+v"(dacc[t]));      // keeps the sum here (the compiler would otherwise sink it
                                                               // to the end of the loop body and hold every Phi tile live)
                        cc = (wrap2 ? nxt.nj : cur.nj) + nin;
                        if (t == 0) load_fold(jprev);
                        if (t == 1) store_fold(jprev);
                        {   // column sums of the pair before this one (its transposed tile is in pht[slot ^ 1])
                            const f32x4& q = pht[slot ^ 1];
                            const float cs = (q.x + q.y) + (q.z + q.w);
                            if (t == 0) cprev = cs;      // belongs to the previous tile, folded in the next clump
                            else cacc += cs;
                        }
                        // transpose Phi through LDS: lane (r, g) holds Phi[i = r][j = 4g + v]; it needs Phi[4g + v][r]
                        *tr_wr = phi;
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        pht[slot].x = tr_rd[0];
                        pht[slot].y = tr_rd[kTrStride];
                        pht[slot].z = tr_rd[2 * kTrStride];
                        pht[slot].w = tr_rd[3 * kTrStride];
                        __builtin_amdgcn_sched_barrier(0);

#pragma unroll
                        for (int i = 0; i < 4 * KB; ++i) {
                            const int v = i / KB, mb = i % KB;
                            tacc[t][mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(cur.a2[mb][v], phi[v], tacc[t][mb], 0, 0, 0);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        // T_J of the previous pair: row tile t - 1 of this sample tile, or the last row tile of the
                        // previous one (first pair of a phase: pht is zero)
#pragma unroll
                        for (int i = 0; i < 4 * KB; ++i) {
                            const int v = i / KB, mb = i % KB;
                            // row tile 1 runs the first T_J MFMAs of this sample tile (pair (jt, 0)): start from zero,
                            // the previous tile's sums have just been folded
                            const f32x4 c0 = (t == 1 && v == 0) ? f32x4{0.f, 0.f, 0.f, 0.f} : acc3[mb];
                            acc3[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(xti[(t + NI - 1) % NI][mb][v], pht[slot ^ 1][v],
                                                                           c0, 0, 0, 0);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                };

                for (int q = 0; q <= q_last; q += 2) {
                    iteration(q, set_a, set_b);
                    iteration(q + 1, set_b, set_a);
                    if (((q + 2) & (tiles_per_phase - 1)) == 0) {
                        // end of a phase: T_J and column sums of the last pair, the last sample tile, and the
                        // meeting point (operand loads and the Gram MFMAs of the next phase's first pair are in flight)
                        f32x4& last = pht[(NI - 1) & 1];
#pragma unroll
                        for (int i = 0; i < 4 * KB; ++i) {
                            const int v = i / KB, mb = i % KB;
                            acc3[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(xti[NI - 1][mb][v], last[v], acc3[mb], 0, 0, 0);
                        }
                        cprev = 0.0f;
                        cacc += (last.x + last.y) + (last.z + last.w);
                        const int jt = tile_of(q + 1);
                        load_fold(jt);
                        store_fold(jt);
#pragma unroll
                        for (int mb = 0; mb < KB; ++mb) acc3[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
                        last = f32x4{0.f, 0.f, 0.f, 0.f};     // the next stage's trailing T_J MFMAs add nothing
                        __syncthreads();
                    }
                }
            }

            // this wave's rows: add into partial slot gam + 1 (the first block that meets these rows stores)
            const bool first = b == max(b_lo, (int)(a0 / rb) + 1);
#pragma unroll
            for (int t = 0; t < NI; ++t) {
                const int64_t row = row0 + t * kTile + r;
                float* dst = part_t + (slot_a * n_pad + row) * DP + g * 4;
#pragma unroll
                for (int mb = 0; mb < KB; ++mb) {
                    f32x4 v = tacc[t][mb];
                    if (!first) v += *reinterpret_cast<const f32x4*>(dst + mb * 16);
                    *reinterpret_cast<f32x4*>(dst + mb * 16) = v;
                }
                const float dt = sum_over_lane_rows(dacc[t]);
                if (g == 0) {
                    float* dd = part_d + slot_a * n_pad + row;
                    *dd = first ? dt : *dd + dt;
                }
            }
        }

        // the block's accumulators -> partial slot c (every phase ended with a barrier; an empty walk leaves zeros)
        const int64_t brow = (int64_t)b * rb;
        for (int idx = threadIdx.x; idx < rb * DP; idx += kSymBlock) {
            const int j = idx / DP, col = idx % DP;
            part_t[(slot_b * n_pad + brow + j) * DP + col] = lds_t[((size_t)(col / 16) * rb + j) * 16 + (col % 16)];
        }
        for (int j = threadIdx.x; j < rb; j += kSymBlock) part_d[slot_b * n_pad + brow + j] = lds_d[j];
        __syncthreads();
    }

    // triangular item: the rows of the group's last block met no later block here; their slot gets zeros
    if (c == gam) {
        const int64_t z0 = (int64_t)(b_hi - 1) * rb;
        for (int idx = threadIdx.x; idx < rb * DP; idx += kSymBlock) part_t[(slot_a * n_pad + z0) * DP + idx] = 0.0f;
        for (int j = threadIdx.x; j < rb; j += kSymBlock) part_d[slot_a * n_pad + z0 + j] = 0.0f;
    }
}

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
    const int split = blockIdx.x % nsplit;
    const int64_t row_block = blockIdx.x / nsplit;
    const int64_t row0 = row_block * (kBlock * R) + threadIdx.x;

    // sh[q]: the row's shift (max_j of -r^2, <= 0) in the max-shifted mode, else 0; the squared distance is
    // accumulated on top of it so that exp2(-(r^2 + sh)) = phi / 2^sh costs no extra instruction.
    float p[R][D], dacc[R], nacc[R][SCORE ? D : 1], sh[R];
#pragma unroll
    for (int q = 0; q < R; ++q) {
#pragma unroll
        for (int k = 0; k < D; ++k) p[q][k] = ps[(row0 + (int64_t)q * kBlock) * D + k];
        sh[q] = (!ROWMAX && shift) ? shift[row0 + (int64_t)q * kBlock] : 0.0f;
        dacc[q] = ROWMAX ? kNegHuge : 0.0f;
#pragma unroll
        for (int k = 0; k < (SCORE ? D : 1); ++k) nacc[q][k] = 0.0f;
    }

    const int t_begin = split * tiles_per_split;
    const int t_end = min(ntiles, t_begin + tiles_per_split);
    for (int jt = t_begin; jt < t_end; ++jt) {
        const float* xj = xs + (int64_t)jt * kTile * D;    // wave-uniform address
#pragma unroll
        for (int jj = 0; jj < kTile; ++jj) {
            float xv[D];
#pragma unroll
            for (int k = 0; k < D; ++k) xv[k] = xj[jj * D + k];
#pragma unroll
            for (int q = 0; q < R; ++q) {
                float diff[D];
                float r2 = sh[q];
#pragma unroll
                for (int k = 0; k < D; ++k) {
                    diff[k] = xv[k] - p[q][k];
                    r2 = fmaf(diff[k], diff[k], r2);
                }
                if (ROWMAX) {
                    dacc[q] = fmaxf(dacc[q], -r2);
                    continue;
                }
                float phi = __builtin_amdgcn_exp2f(-r2);
                // Laplace factor 1 + d/2 - r^2/2h^2, with the true r^2 = r2 - sh
                if (LAPLACE) dacc[q] = fmaf(phi, fmaf(sh[q] - r2, kLn2, laplace_c0), dacc[q]);
                else dacc[q] += phi;
                if (SCORE) {
#pragma unroll
                    for (int k = 0; k < D; ++k) nacc[q][k] = fmaf(phi, diff[k], nacc[q][k]);
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < R; ++q) {
        const int64_t row = row0 + (int64_t)q * kBlock;
        part_d[(int64_t)split * m_pad + row] = dacc[q];
        if (SCORE) {
#pragma unroll
            for (int k = 0; k < D; ++k) part_t[((int64_t)split * m_pad + row) * D + k] = nacc[q][k];
        }
    }
}

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
            pc = ps[i * dp + c];
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

// ------------------------------------------------------------------------------------------
// Host side: plan, workspace layout, dispatch.
// ------------------------------------------------------------------------------------------

// Most row tiles per wave for which pair_mfma_kernel is instantiated (larger ones would spill registers).
constexpr int max_row_tiles(int kb, int kind, int prec = SDKDE_PREC_FP32)
{
    const bool second = kind == kScoreSelf || kind == kScorePoints || kind == kScoreBand;   // has the Phi X contraction
    if (prec == SDKDE_PREC_FP16X2_ALL && kb > 6) return 0;              // see effective_prec()
    if (kind == kScoreBand && (kb > 2 || prec != SDKDE_PREC_FP32)) return 0;          // see sym_row_tiles()
    return second ? (kb == 1 ? 8 : kb <= 4 ? 4 : 2) : (kb == 1 ? 16 : kb == 2 ? 8 : kb <= 4 ? 4 : 2);
}

// Precision mode a call actually runs in: the thin path is fp32 VALU code; the fp16 second contraction is
// built for dp <= 96 (beyond that its operands no longer fit the register file) and falls back to fp16x2.
inline uint32_t effective_prec(uint32_t flags, bool thin, int dp)
{
    const uint32_t prec = flags & 15u;
    if (thin) return SDKDE_PREC_FP32;
    if (prec == SDKDE_PREC_FP16X2_ALL && dp > 96) return SDKDE_PREC_FP16X2;
    return prec;
}

// The fp16 split of 2^14 phi resolves weights with ABSOLUTE precision 2^-39 (the fp16 subnormal step over the
// scale), which is harmless next to a weight of one: the sample's own term at the samples themselves, the
// largest term after a max shift.  A score at separate points without that shift has no such anchor (a point
// whose weights are all below ~1e-7 would lose them in T but not in D), so it runs the fp16x2 mode instead.
inline uint32_t anchored_flags(uint32_t flags, bool self)
{
    if ((flags & 15u) == SDKDE_PREC_FP16X2_ALL && !self && !(flags & SDKDE_FLAG_MAX_SHIFT))
        return (flags & ~15u) | SDKDE_PREC_FP16X2;
    return flags;
}

struct Plan {
    bool thin;
    int d, dp;            // true and padded dimension (thin: dp == d)
    int ni;               // MFMA: row tiles per wave; thin: rows per thread
    int rows_per_block;
    int64_t n_pad, m_pad; // padded sample / point row counts
    int ntiles;           // 16-sample tiles
    int nsplit, tiles_per_split;
    int64_t row_blocks;
    // symmetric mode of the score at the samples themselves (pair_sym_kernel), off unless sym_on
    bool sym_on;
    int sym_ni, sym_rb, sym_per_group, sym_nblocks, sym_ngroups;
};

int env_int(const char* name, int fallback)
{
    const char* v = getenv(name);
    if (!v || !*v) return fallback;
    return atoi(v);
}

// Workgroups needed to keep 256 CUs busy with a few waves per SIMD.
constexpr int64_t kTargetBlocks = 2048;

Plan make_plan(int64_t n, int64_t m, int d, bool score)
{
    Plan p{};
    p.d = d;
    p.thin = d <= kThinMaxD;
    p.dp = p.thin ? d : (int)round_up(d, 16);
    p.n_pad = round_up(n, kRowPad);
    p.m_pad = round_up(m > 0 ? m : 1, kRowPad);
    p.ntiles = (int)((n + 2 * kTile - 1) / (2 * kTile)) * 2;   // even: the pair kernel alternates two operand sets
    const int max_split = p.ntiles >= 32 ? p.ntiles / 16 : 1;   // at least 16 tiles per split

    // Candidate row-tile counts, largest (most operand reuse) first; a smaller one is taken
    // only when the grid would otherwise leave most of the chip idle.
    int cand[5];
    int nc = 0;
    if (p.thin) {
        cand[nc++] = 4; cand[nc++] = 2; cand[nc++] = 1;
    } else {
        const int kb = p.dp / 16;
        // measured: more row tiles per wave (operand reuse) beats a second wave per SIMD once dp >= 48
        const int top = max_row_tiles(kb, score ? kScoreSelf : kEval);
        for (int v = top; v >= 2; v /= 2) cand[nc++] = v;
    }
    const int forced_ni = env_int(score ? "SDKDE_SCORE_NI" : "SDKDE_EVAL_NI", 0);
    const int forced_split = env_int(score ? "SDKDE_SCORE_SPLIT" : "SDKDE_EVAL_SPLIT", 0);
    {
        // a forced value must be one the dispatch tables below instantiate
        const int kb = p.thin ? 0 : p.dp / 16;
        const int widest = p.thin ? 4 : max_row_tiles(kb, score ? kScoreSelf : kEval);
        const int narrowest = p.thin ? 1 : 2;
        if (forced_ni >= narrowest && forced_ni <= widest && (forced_ni & (forced_ni - 1)) == 0) {
            cand[0] = forced_ni;
            nc = 1;
        }
    }

    for (int k = 0; k < nc; ++k) {
        p.ni = cand[k];
        p.rows_per_block = p.thin ? kBlock * p.ni : kWavesPerBlock * kTile * p.ni;
        p.row_blocks = (m + p.rows_per_block - 1) / p.rows_per_block;
        if (p.row_blocks < 1) p.row_blocks = 1;
        int64_t want = (kTargetBlocks + p.row_blocks - 1) / p.row_blocks;
        if (max_split >= 8) {                       // one group of splits per XCD
            want = round_up(want < 8 ? 8 : want, 8);
            if (want > max_split) want = max_split / 8 * 8;
        } else if (want > max_split) {
            want = max_split;
        }
        p.nsplit = (int)want;
        if (forced_split > 0) p.nsplit = forced_split > p.ntiles ? p.ntiles : forced_split;
        if (p.row_blocks * p.nsplit >= kTargetBlocks / 2) break;
    }
    p.tiles_per_split = (p.ntiles + p.nsplit - 1) / p.nsplit;
    p.tiles_per_split += p.tiles_per_split & 1;
    return p;
}

// Row tiles per wave of the pair_sym_kernel instantiation for kb 16-column blocks; 0: not built, the flag is
// ignored.  Built where it pays (measured at n = 262144 against the ordinary kernels): fp32 inputs with
// dp = 16 (1.25x) and dp = 32 (1.17x).  With dp >= 48 only two row tiles per wave fit the 256 registers a wave
// has at two waves per SIMD and the gain was nil; with fp16x2 inputs the Gram MFMAs it saves are already cheap
// and the mode was slower than the ordinary kernel.
constexpr int sym_row_tiles(int kb, int prec)
{
    if (prec == SDKDE_PREC_FP32) return kb == 1 ? 8 : kb == 2 ? 4 : 0;
    return 0;
}

// Most groups of sample blocks in the symmetric mode (a row gets one partial slot per group, plus three).
constexpr int kSymMaxGroups = 64;

// Decomposition of the symmetric mode, if this call takes it: the score at the samples themselves on the
// matrix path, for the dimensions and input modes pair_sym_kernel is built for (sym_row_tiles).  Block size: as many rows as the LDS accumulators
// hold ((dp + 1) floats per row within ~136 KiB), halved while there would be too few items to fill the chip.
void apply_symmetric(Plan& p, int64_t n, uint32_t flags, bool self)
{
    if (!(flags & SDKDE_FLAG_SYMMETRIC) || !self || p.thin) return;
    const int kb = p.dp / 16;
    const int ni = sym_row_tiles(kb, (int)(flags & 15u));
    if (ni == 0) return;
    p.sym_ni = ni;
    const int sb = kSymWaves * p.sym_ni * kTile;           // rows a workgroup holds at a time: 512 or 256
    int rb = kb == 1 ? 2048 : kb == 2 ? 1024 : 512;
    auto items = [&](int rb_) {
        int64_t nb = (n + rb_ - 1) / rb_;
        if (nb > kSymMaxGroups) nb = kSymMaxGroups;
        return nb * (nb + 1) / 2;
    };
    while (rb > sb && items(rb) < 1024) rb /= 2;
    const int forced_rb = env_int("SDKDE_SYM_RB", 0);
    if (forced_rb >= sb && forced_rb <= rb * 8 && forced_rb % sb == 0 && (forced_rb & (forced_rb - 1)) == 0 &&
        sym_lds_bytes(kb, forced_rb) <= 160 * 1024)
        rb = forced_rb;
    int max_groups = env_int("SDKDE_SYM_GROUPS", kSymMaxGroups);
    if (max_groups < 1 || max_groups > kSymMaxGroups) max_groups = kSymMaxGroups;
    const int64_t n_pad = round_up(n, rb > kRowPad ? rb : kRowPad);
    const int64_t nblocks = n_pad / rb;
    if (nblocks > (1 << 20)) return;
    p.sym_on = true;
    p.sym_rb = rb;
    p.sym_nblocks = (int)nblocks;
    p.sym_per_group = (int)((nblocks + max_groups - 1) / max_groups);
    p.sym_ngroups = (int)((nblocks + p.sym_per_group - 1) / p.sym_per_group);
    p.n_pad = p.m_pad = n_pad;          // whole blocks; the points are the samples
}

struct Workspace {
    double* mean_partial;
    float* xs;  float* xt;  float* xn;     // samples: scaled rows, blocked transpose, -|x|^2
    float* ps;  float* pn;                 // evaluation points (alias xs/xn when they are the samples)
    float* shift;                          // per-point exponent shift of the max-shifted mode (separate points only)
    float* part_t;  float* part_d;
    size_t bytes;
};

// Lays out the workspace for `plan`; base may be null (size query).  separate_points: the
// evaluation points are an array of their own (eval, or score at points != samples).
Workspace layout(const Plan& p, bool score, bool separate_points, void* base, uint32_t flags = 0)
{
    Workspace w{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off += (bytes + 255) / 256 * 256;
        return base ? (char*)base + at : (char*)nullptr;
    };
    w.mean_partial = (double*)take(sizeof(double) * kMeanBlocks * SDKDE_MAX_D);
    w.xs = (float*)take(sizeof(float) * p.n_pad * p.dp);
    // blocked transpose for the second contraction: fp32, or hi/lo fp16 pairs stored twice (2x the bytes)
    const size_t xt_scale = effective_prec(flags, p.thin, p.dp) == SDKDE_PREC_FP16X2_ALL ? 2 : 1;
    w.xt = (score && !p.thin) ? (float*)take(sizeof(float) * xt_scale * p.n_pad * p.dp) : nullptr;
    w.xn = (float*)take(sizeof(float) * p.n_pad);
    if (separate_points) {
        w.ps = (float*)take(sizeof(float) * p.m_pad * p.dp);
        w.pn = (float*)take(sizeof(float) * p.m_pad);
        w.shift = (float*)take(sizeof(float) * p.m_pad);
    } else {
        w.ps = w.xs;
        w.pn = w.xn;
    }
    // one slot per split, plus the diagonal-block slot of the score at the samples themselves
    size_t slots = (size_t)p.nsplit + ((score && !separate_points && !p.thin) ? 1 : 0);
    if (p.sym_on) slots = (size_t)p.sym_ngroups + 3;     // pair_sym_kernel's, then the in-block pass and its diagonal
    w.part_t = score ? (float*)take(sizeof(float) * slots * p.m_pad * p.dp) : nullptr;
    w.part_d = (float*)take(sizeof(float) * slots * p.m_pad);
    w.bytes = off;
    return w;
}

bool bad_bandwidth(double h) { return !(h > 0.0) || !isfinite(h); }

// Optional instrumentation: event pairs around the main pair kernel of each call.
constexpr int kProfileSlots = 256;
struct Profile {
    bool enabled = false;
    hipEvent_t ev[2][kProfileSlots][2] = {};   // [score|eval][launch][begin|end], created lazily
    int count[2] = {0, 0};
} g_profile;

#define SDKDE_HIP(call)                                   \
    do {                                                  \
        if ((call) != hipSuccess) return SDKDE_EDEVICE;   \
    } while (0)

template <int KIND, int PREC>
int launch_pair(const Plan& p, const Workspace& w, const float* shift, hipStream_t st)
{
    const dim3 grid((unsigned)(p.row_blocks * p.nsplit)), block(kBlock);
    if ((int64_t)p.row_blocks * p.nsplit > 0x7fffffffLL) return SDKDE_EUNSUPPORTED;
    const float laplace_c0 = 1.0f + 0.5f * (float)p.d;
    // Host-side shape check: every row the grid touches exists in the padded arrays.
    if (p.row_blocks * p.rows_per_block > p.m_pad || (int64_t)p.ntiles * kTile > p.n_pad) return SDKDE_EINVAL;

#define SDKDE_LAUNCH_MFMA(KB_, NI_)                                                                               \
    do {                                                                                                          \
        hipLaunchKernelGGL((pair_mfma_kernel<KB_, NI_, KIND, PREC>), grid, block, 0, st, w.ps, w.pn, w.xs, w.xt,  \
                           w.xn, w.part_t, w.part_d, p.ntiles, p.tiles_per_split, p.nsplit, p.m_pad, laplace_c0,  \
                           shift);                                                                                \
        if constexpr (KIND == kScoreSelf || KIND == kScoreBand)                                                   \
            hipLaunchKernelGGL((pair_diag_kernel<KB_, NI_, PREC>), dim3((unsigned)p.row_blocks), block, 0, st,   \
                               w.xs, w.xt, w.xn, w.part_t, w.part_d, p.ntiles, p.nsplit, p.m_pad);                \
    } while (0)
#define SDKDE_LAUNCH_THIN(D_, R_)                                                                      \
    do {                                                                                               \
        if constexpr (KIND != kScoreBand)                                                              \
            hipLaunchKernelGGL((pair_thin_kernel<D_, R_, KIND>), grid, block, 0, st, w.ps, w.xs,       \
                               w.part_t, w.part_d, p.ntiles, p.tiles_per_split, p.nsplit, p.m_pad,     \
                               laplace_c0, shift);                                                     \
    } while (0)
#define SDKDE_CASE_NI(KB_, NI_)                                            \
    case NI_:                                                              \
        if constexpr (NI_ <= max_row_tiles(KB_, KIND, PREC)) SDKDE_LAUNCH_MFMA(KB_, NI_); \
        else return SDKDE_EUNSUPPORTED;                                    \
        break;

    if (p.thin) {
        if constexpr (KIND == kScoreBand) return SDKDE_EUNSUPPORTED;     // the symmetric mode is matrix-path only
        const int key = p.d * 10 + p.ni;
        switch (key) {
            case 14: SDKDE_LAUNCH_THIN(1, 4); break;
            case 12: SDKDE_LAUNCH_THIN(1, 2); break;
            case 11: SDKDE_LAUNCH_THIN(1, 1); break;
            case 24: SDKDE_LAUNCH_THIN(2, 4); break;
            case 22: SDKDE_LAUNCH_THIN(2, 2); break;
            case 21: SDKDE_LAUNCH_THIN(2, 1); break;
            case 34: SDKDE_LAUNCH_THIN(3, 4); break;
            case 32: SDKDE_LAUNCH_THIN(3, 2); break;
            case 31: SDKDE_LAUNCH_THIN(3, 1); break;
            default: return SDKDE_EUNSUPPORTED;
        }
    } else {
        const int kb = p.dp / 16;
        switch (kb) {
            case 1:
                switch (p.ni) { SDKDE_CASE_NI(1, 16) SDKDE_CASE_NI(1, 8) SDKDE_CASE_NI(1, 4) SDKDE_CASE_NI(1, 2) default: return SDKDE_EUNSUPPORTED; }
                break;
            case 2:
                switch (p.ni) { SDKDE_CASE_NI(2, 8) SDKDE_CASE_NI(2, 4) SDKDE_CASE_NI(2, 2) default: return SDKDE_EUNSUPPORTED; }
                break;
            case 3:
                switch (p.ni) { SDKDE_CASE_NI(3, 4) SDKDE_CASE_NI(3, 2) default: return SDKDE_EUNSUPPORTED; }
                break;
            case 4:
                switch (p.ni) { SDKDE_CASE_NI(4, 4) SDKDE_CASE_NI(4, 2) default: return SDKDE_EUNSUPPORTED; }
                break;
            case 5:
                switch (p.ni) { SDKDE_CASE_NI(5, 2) default: return SDKDE_EUNSUPPORTED; }
                break;
            case 6:
                switch (p.ni) { SDKDE_CASE_NI(6, 2) default: return SDKDE_EUNSUPPORTED; }
                break;
            case 7:
                switch (p.ni) { SDKDE_CASE_NI(7, 2) default: return SDKDE_EUNSUPPORTED; }
                break;
            case 8:
                switch (p.ni) { SDKDE_CASE_NI(8, 2) default: return SDKDE_EUNSUPPORTED; }
                break;
            default: return SDKDE_EUNSUPPORTED;
        }
    }
#undef SDKDE_CASE_NI
#undef SDKDE_LAUNCH_THIN
#undef SDKDE_LAUNCH_MFMA
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

template <int KIND>
int launch_pair_prec(const Plan& p, const Workspace& w, uint32_t flags, const float* shift, hipStream_t st)
{
    // the thin-d path has no matrix inputs: it runs the same fp32 VALU code for every mode
    const uint32_t prec = effective_prec(flags, p.thin, p.dp);
    constexpr bool has_second = KIND == kScoreSelf || KIND == kScorePoints || KIND == kScoreBand;
    if constexpr (has_second) {
        if (prec == SDKDE_PREC_FP16X2_ALL) return launch_pair<KIND, SDKDE_PREC_FP16X2_ALL>(p, w, shift, st);
    }
    // kinds without a second contraction: the two fp16 modes are the same kernel
    if (prec != SDKDE_PREC_FP32) return launch_pair<KIND, SDKDE_PREC_FP16X2>(p, w, shift, st);
    return launch_pair<KIND, SDKDE_PREC_FP32>(p, w, shift, st);
}

// Symmetric mode: pairs across blocks (pair_sym_kernel), then the pairs inside each block with the ordinary
// kernels restricted to the block (slots ngroups + 1 and ngroups + 2).
template <int KB, int NI, int PREC>
int launch_sym_kernel(const Plan& p, const Workspace& w, hipStream_t st)
{
    const size_t lds = sym_lds_bytes(KB, p.sym_rb);
    static size_t lds_allowed = 0;           // largest dynamic LDS size this instantiation has been enabled for
    if (lds > lds_allowed) {
        SDKDE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&pair_sym_kernel<KB, NI, PREC>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        lds_allowed = lds;
    }
    const int64_t items = (int64_t)p.sym_ngroups * (p.sym_ngroups + 1) / 2;
    hipLaunchKernelGGL((pair_sym_kernel<KB, NI, PREC>), dim3((unsigned)items), dim3(kSymBlock), lds, st, w.xs, w.xt,
                       w.xn, w.part_t, w.part_d, p.n_pad, p.sym_rb, p.sym_nblocks, p.sym_per_group, p.sym_ngroups);
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

template <int KB, int PREC>
int launch_sym_kb(const Plan& p, const Workspace& w, hipStream_t st)
{
    constexpr int NI = sym_row_tiles(KB, PREC);
    if constexpr (NI > 0) {
        if (p.sym_ni != NI) return SDKDE_EINVAL;
        return launch_sym_kernel<KB, NI, PREC>(p, w, st);
    } else {
        return SDKDE_EUNSUPPORTED;
    }
}

template <int PREC>
int launch_sym_prec(const Plan& p, const Workspace& w, hipStream_t st)
{
    // Host-side shape check: whole blocks, whole workgroup row sets, an even power of two of tiles per phase.
    const int sb = kSymWaves * p.sym_ni * kTile;
    if (p.sym_ni < 2 || p.sym_rb % sb || p.sym_rb % (2 * kSymWaves * kTile) || (p.sym_rb & (p.sym_rb - 1)) ||
        (int64_t)p.sym_nblocks * p.sym_rb != p.n_pad || sym_lds_bytes(p.dp / 16, p.sym_rb) > 160 * 1024)
        return SDKDE_EINVAL;
    switch (p.dp / 16) {
        case 1: return launch_sym_kb<1, PREC>(p, w, st);
        case 2: return launch_sym_kb<2, PREC>(p, w, st);
        default: return SDKDE_EUNSUPPORTED;
    }
}

int launch_symmetric(const Plan& p, const Workspace& w, uint32_t flags, hipStream_t st)
{
    if (effective_prec(flags, p.thin, p.dp) != SDKDE_PREC_FP32) return SDKDE_EUNSUPPORTED;   // see sym_row_tiles()
    int rc = launch_sym_prec<SDKDE_PREC_FP32>(p, w, st);
    if (rc != SDKDE_OK) return rc;
    Plan band = p;
    band.nsplit = 1;
    band.tiles_per_split = p.sym_rb / kTile;        // kScoreBand: the length of a block in tiles
    Workspace wb = w;                               // its slots follow pair_sym_kernel's
    wb.part_t = w.part_t + (size_t)(p.sym_ngroups + 1) * p.m_pad * p.dp;
    wb.part_d = w.part_d + (size_t)(p.sym_ngroups + 1) * p.m_pad;
    return launch_pair_prec<kScoreBand>(band, wb, flags, nullptr, st);
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

// First pass of the max-shifted mode for separate points: row maxima of the exponent, then shift_kernel.
int launch_max_shift(const Plan& p, const Workspace& w, uint32_t flags, hipStream_t st)
{
    int rc = launch_pair_prec<kRowMax>(p, w, flags, nullptr, st);
    if (rc != SDKDE_OK) return rc;
    hipLaunchKernelGGL(shift_kernel, dim3((unsigned)((p.m_pad + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, w.part_d,
                       p.nsplit, p.m_pad, w.shift, p.thin ? nullptr : w.pn);
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

// First stage of the column means of src[rows][d] (the prep kernels finish them).
int launch_mean(const float* src, int64_t rows, int d, const Workspace& w, hipStream_t st)
{
    hipLaunchKernelGGL(mean_partial_kernel, dim3(kMeanBlocks), dim3(kBlock), 0, st, src, rows, d, w.mean_partial);
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

// Centre/scale/pad one or two arrays in a single launch (second.src == nullptr: only the first).
// n_mean: number of rows the column means in w.mean_partial were taken over.
int launch_prep(const Plan& p, const PrepJob& first, const PrepJob& second, int64_t n_mean, float a,
                const Workspace& w, uint32_t flags, hipStream_t st)
{
    const int64_t per_block = p.thin ? kBlock : kPrepRows;
    if (first.rows_pad % per_block || (second.src && second.rows_pad % per_block)) return SDKDE_EINVAL;
    const int64_t blocks0 = first.rows_pad / per_block;
    const int64_t blocks1 = second.src ? second.rows_pad / per_block : 0;
    if (blocks0 + blocks1 > 0x7fffffffLL) return SDKDE_EUNSUPPORTED;
    const dim3 grid((unsigned)(blocks0 + blocks1)), block(kBlock);
    if (p.thin)
        hipLaunchKernelGGL(prep_thin_kernel, grid, block, 0, st, first, second, (int)blocks0, p.d, w.mean_partial,
                           n_mean, a);
    else
        hipLaunchKernelGGL(prep_mfma_kernel, grid, block, 0, st, first, second, (int)blocks0, p.d, p.dp,
                           w.mean_partial, n_mean, a, (int)effective_prec(flags, p.thin, p.dp));
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

int check_common(const void* samples, int64_t n, int64_t m, int32_t d, double h, uint32_t flags)
{
    if (!samples || n < 1 || m < 0 || d < 1 || bad_bandwidth(h)) return SDKDE_EINVAL;
    if (d > SDKDE_MAX_D || (flags & ~(15u | SDKDE_FLAG_MAX_SHIFT | SDKDE_FLAG_SYMMETRIC)) != 0 || (flags & 15u) > SDKDE_PREC_FP16X2_ALL)
        return SDKDE_EUNSUPPORTED;
    if (n > (int64_t)1 << 34 || m > (int64_t)1 << 34) return SDKDE_EUNSUPPORTED;
    return SDKDE_OK;
}

// edge 0: before the main kernel of a call of kind `which`; edge 1: after it.
int profile_mark(int which, int edge, hipStream_t st)
{
    if (!g_profile.enabled || g_profile.count[which] >= kProfileSlots) return SDKDE_OK;
    hipEvent_t& e = g_profile.ev[which][g_profile.count[which]][edge];
    if (!e) SDKDE_HIP(hipEventCreate(&e));
    SDKDE_HIP(hipEventRecord(e, st));
    if (edge == 1) ++g_profile.count[which];
    return SDKDE_OK;
}

// Shared body of sdkde_score and of the first half of sdkde_fit_eval.  samples_sd_out (optional, only at
// the samples themselves): also writes samples + (h^2/2) score from the same epilogue.
int score_impl(const float* samples, int64_t n, const float* points, int64_t m, int32_t d, double h,
               float* score_out, float* samples_sd_out, void* workspace, size_t workspace_bytes, uint32_t flags,
               void* stream)
{
    int rc = check_common(samples, n, m, d, h, flags);
    if (rc != SDKDE_OK) return rc;
    const bool self = points == nullptr || (points == samples && m == n);
    if (points == nullptr && m != n) return SDKDE_EINVAL;
    if (m == 0) return SDKDE_OK;
    if (!score_out && !samples_sd_out) return SDKDE_EINVAL;
    if (samples_sd_out && !self) return SDKDE_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255)) return SDKDE_EWORKSPACE;
    flags = anchored_flags(flags, self);

    Plan p = make_plan(n, m, d, true);
    apply_symmetric(p, n, flags, self);
    const Workspace w = layout(p, true, !self, workspace, flags);
    if (w.bytes > workspace_bytes) return SDKDE_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;

    const double a = sqrt(1.4426950408889634074 / (2.0 * h * h));   // sqrt(c log2 e)
    // When the points are the samples (m == n, so m_pad == n_pad), one prepared array serves
    // as both operands.
    if ((rc = launch_mean(samples, n, d, w, st)) != SDKDE_OK) return rc;
    const PrepJob sample_job{samples, n, p.n_pad, w.xs, w.xt, w.xn, kPadCoord};
    const PrepJob point_job{self ? nullptr : points, m, p.m_pad, w.ps, nullptr, w.pn, 0.0f};
    if ((rc = launch_prep(p, sample_job, point_job, n, (float)a, w, flags, st)) != SDKDE_OK) return rc;

    if ((rc = profile_mark(0, 0, st)) != SDKDE_OK) return rc;
    // at the samples themselves the largest weight is the self pair (exponent 0): nothing to shift
    const bool shifted = !self && (flags & SDKDE_FLAG_MAX_SHIFT) != 0;
    if (shifted && (rc = launch_max_shift(p, w, flags, st)) != SDKDE_OK) return rc;
    const float* shift = shifted ? w.shift : nullptr;
    rc = p.sym_on ? launch_symmetric(p, w, flags, st)
         : self   ? launch_pair_prec<kScoreSelf>(p, w, flags, nullptr, st)
                  : launch_pair_prec<kScorePoints>(p, w, flags, shift, st);
    if (rc != SDKDE_OK) return rc;
    if ((rc = profile_mark(0, 1, st)) != SDKDE_OK) return rc;

    const int64_t total = m * (int64_t)d;
    const float inv_ah2 = (float)(1.0 / (a * h * h));
    hipLaunchKernelGGL(score_epilogue_kernel, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, st,
                       w.part_t, w.part_d, w.ps, p.sym_on ? p.sym_ngroups + 3 : p.nsplit + ((self && !p.thin) ? 1 : 0), m,
                       p.m_pad, d, p.dp,
                       p.thin ? 1 : (self ? 2 : 0), effective_prec(flags, p.thin, p.dp) != SDKDE_PREC_FP32 ? 1 : 0, inv_ah2,
                       score_out, samples, (float)(0.5 * h * h), samples_sd_out);
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

// Shared body of sdkde_eval and sdkde_eval_laplace.
int eval_impl(const float* samples, int64_t n, const float* queries, int64_t m, int32_t d, double h,
              float* density_out, float* log_density_out, void* workspace, size_t workspace_bytes, uint32_t flags,
              void* stream, bool laplace, bool reuse_mean = false)
{
    int rc = check_common(samples, n, m, d, h, flags);
    if (rc != SDKDE_OK) return rc;
    if (m == 0) return SDKDE_OK;
    if (!queries || (!density_out && !log_density_out)) return SDKDE_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255)) return SDKDE_EWORKSPACE;

    const Plan p = make_plan(n, m, d, false);
    const Workspace w = layout(p, false, true, workspace, flags);
    if (w.bytes > workspace_bytes) return SDKDE_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;

    const double a = sqrt(1.4426950408889634074 / (2.0 * h * h));
    // reuse_mean: w.mean_partial still holds the column sums of an earlier pass over (nearly) the same points
    if (!reuse_mean && (rc = launch_mean(samples, n, d, w, st)) != SDKDE_OK) return rc;
    const PrepJob sample_job{samples, n, p.n_pad, w.xs, nullptr, w.xn, kPadCoord};
    const PrepJob query_job{queries, m, p.m_pad, w.ps, nullptr, w.pn, 0.0f};
    if ((rc = launch_prep(p, sample_job, query_job, n, (float)a, w, flags, st)) != SDKDE_OK) return rc;

    if ((rc = profile_mark(1, 0, st)) != SDKDE_OK) return rc;
    const bool shifted = (flags & SDKDE_FLAG_MAX_SHIFT) != 0;
    if (shifted && (rc = launch_max_shift(p, w, flags, st)) != SDKDE_OK) return rc;
    const float* shift = shifted ? w.shift : nullptr;
    rc = laplace ? launch_pair_prec<kEvalLaplace>(p, w, flags, shift, st) : launch_pair_prec<kEval>(p, w, flags, shift, st);
    if (rc != SDKDE_OK) return rc;
    if ((rc = profile_mark(1, 1, st)) != SDKDE_OK) return rc;

    const double lognorm = -log((double)n) - (double)d * log(h) - 0.5 * (double)d * log(6.283185307179586476925286766559);
    hipLaunchKernelGGL(eval_epilogue_kernel, dim3((unsigned)((m + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, w.part_d,
                       p.nsplit, m, p.m_pad, lognorm, laplace ? 1 : 0, shift, density_out, log_density_out);
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

}  // namespace

extern "C" {

int sdkde_workspace_bytes(int64_t n, int64_t m, int32_t d, uint32_t flags, size_t* bytes)
{
    if (!bytes) return SDKDE_EINVAL;
    int rc = check_common(bytes, n, m, d, 1.0, flags);
    if (rc != SDKDE_OK) return rc;
    // Largest of: score at the samples themselves, score at m separate points, eval at m queries.
    Plan self_plan = make_plan(n, n, d, true);
    apply_symmetric(self_plan, n, flags, true);
    size_t need = layout(self_plan, true, false, nullptr, flags).bytes;
    if (m > 0) {
        size_t b = layout(make_plan(n, m, d, true), true, true, nullptr, flags).bytes;
        need = b > need ? b : need;
        b = layout(make_plan(n, m, d, false), false, true, nullptr, flags).bytes;
        need = b > need ? b : need;
    }
    *bytes = need;
    return SDKDE_OK;
}

int sdkde_score(const float* samples, int64_t n, const float* points, int64_t m, int32_t d, double h,
                float* score_out, void* workspace, size_t workspace_bytes, uint32_t flags, void* stream)
{
    if (!score_out && m != 0) return SDKDE_EINVAL;
    return score_impl(samples, n, points, m, d, h, score_out, nullptr, workspace, workspace_bytes, flags, stream);
}

int sdkde_fit_eval(const float* samples, int64_t n, const float* queries, int64_t m, int32_t d, double h,
                   float* score_out, float* samples_sd_out, float* density_out, float* log_density_out,
                   void* workspace, size_t workspace_bytes, uint32_t flags, void* stream)
{
    if (!samples_sd_out) return SDKDE_EINVAL;
    int rc = check_common(samples, n, m, d, h, flags);
    if (rc != SDKDE_OK) return rc;
    if (m > 0 && (!queries || (!density_out && !log_density_out))) return SDKDE_EINVAL;
    rc = score_impl(samples, n, nullptr, n, d, h, score_out, samples_sd_out, workspace, workspace_bytes, flags, stream);
    if (rc != SDKDE_OK || m == 0) return rc;
    // The column means of the samples are still in the workspace; the shifted samples are centred on them
    // too (any centre is exact, it only has to be near the data), which saves the mean pass.
    return eval_impl(samples_sd_out, n, queries, m, d, h, density_out, log_density_out, workspace, workspace_bytes,
                     flags, stream, false, true);
}

int sdkde_debias(const float* samples, const float* score, int64_t n, int32_t d, double h, float* samples_sd_out,
                 void* stream)
{
    if (!samples || !score || !samples_sd_out || n < 0 || d < 1 || bad_bandwidth(h)) return SDKDE_EINVAL;
    const int64_t total = n * (int64_t)d;
    if (total == 0) return SDKDE_OK;
    hipLaunchKernelGGL(debias_kernel, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                       (hipStream_t)stream, samples, score, total, (float)(0.5 * h * h), samples_sd_out);
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

int sdkde_eval(const float* samples_sd, int64_t n, const float* queries, int64_t m, int32_t d, double h,
               float* density_out, float* log_density_out, void* workspace, size_t workspace_bytes, uint32_t flags,
               void* stream)
{
    return eval_impl(samples_sd, n, queries, m, d, h, density_out, log_density_out, workspace, workspace_bytes, flags,
                     stream, false);
}

int sdkde_eval_laplace(const float* samples, int64_t n, const float* queries, int64_t m, int32_t d, double h,
                       float* density_out, void* workspace, size_t workspace_bytes, uint32_t flags, void* stream)
{
    return eval_impl(samples, n, queries, m, d, h, density_out, nullptr, workspace, workspace_bytes, flags, stream,
                     true);
}

int sdkde_describe_plan(int64_t n, int64_t m, int32_t d, int32_t call, uint32_t flags, int64_t* out, int32_t out_len)
{
    if (!out || out_len < 20 || call < 0 || call > 2) return SDKDE_EINVAL;
    int rc = check_common(out, n, m, d, 1.0, flags);
    if (rc != SDKDE_OK) return rc;
    const bool score = call != 2;
    const bool separate = call != 0;
    const int64_t rows = call == 0 ? n : m;
    if (score) flags = anchored_flags(flags, !separate);
    Plan p = make_plan(n, rows, d, score);
    if (score) apply_symmetric(p, n, flags, !separate);
    char* const base = reinterpret_cast<char*>(uintptr_t(1) << 20);      // any aligned non-null address: offsets only
    const Workspace w = layout(p, score, separate, base, flags);
    auto off = [&](const void* q) { return q ? (int64_t)((const char*)q - base) : (int64_t)-1; };
    const int64_t slots = p.sym_on ? p.sym_ngroups + 3 : p.nsplit + ((score && !separate && !p.thin) ? 1 : 0);
    const int64_t xt_scale = effective_prec(flags, p.thin, p.dp) == SDKDE_PREC_FP16X2_ALL ? 2 : 1;
    const int64_t v[20] = {
        p.thin ? 1 : 0, p.dp, p.ni, p.rows_per_block, p.row_blocks, p.nsplit, p.tiles_per_split, p.ntiles,
        p.n_pad, p.m_pad, (int64_t)w.bytes, off(w.xs), off(w.xt), off(w.xn), off(w.ps), off(w.pn),
        off(w.part_t), off(w.part_d), slots, xt_scale};
    for (int k = 0; k < 20; ++k) out[k] = v[k];
    if (out_len >= 24) {
        out[20] = p.sym_on ? 1 : 0;
        out[21] = p.sym_on ? p.sym_rb : 0;
        out[22] = p.sym_on ? p.sym_per_group : 0;
        out[23] = p.sym_on ? p.sym_ngroups : 0;
    }
    return SDKDE_OK;
}

const char* sdkde_status_string(int status)
{
    switch (status) {
        case SDKDE_OK: return "ok";
        case SDKDE_EINVAL: return "invalid argument";
        case SDKDE_EUNSUPPORTED: return "unsupported dimension, size or flag";
        case SDKDE_EWORKSPACE: return "workspace missing, misaligned or too small";
        case SDKDE_EDEVICE: return "HIP runtime error";
        default: return "unknown status";
    }
}

int sdkde_profile_enable(int on)
{
    g_profile.enabled = on != 0;
    g_profile.count[0] = g_profile.count[1] = 0;
    return SDKDE_OK;
}

int sdkde_profile_summary(int which, int* launches, float* total_ms)
{
    if (which < 0 || which > 1 || !launches || !total_ms) return SDKDE_EINVAL;
    float total = 0.0f;
    for (int k = 0; k < g_profile.count[which]; ++k) {
        float ms = 0.0f;
        SDKDE_HIP(hipEventSynchronize(g_profile.ev[which][k][1]));
        SDKDE_HIP(hipEventElapsedTime(&ms, g_profile.ev[which][k][0], g_profile.ev[which][k][1]));
        total += ms;
    }
    *launches = g_profile.count[which];
    *total_ms = total;
    return SDKDE_OK;
}

}  // extern "C"

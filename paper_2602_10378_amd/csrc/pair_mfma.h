// Pair kernel of the matrix path (d >= 4): pair_mfma_kernel and its operand helpers.
#pragma once
#include "common.h"

namespace {

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
// that A operand with one float4 load per lane.  In the first contraction MFMA kk takes component kk of
// every lane's float4, i.e. positions {kk, 4+kk, 8+kk, 12+kk} of each 16-column block, so that both
// operands are plain float4 row loads; the fp32 prepared arrays place coordinate 4kk + g at position
// 4g + kk, which makes those the coordinates 4kk .. 4kk+3 (see KLAST below).
//
// SELF (score at the samples themselves): the pair (i, i) must stay out of D and T, because
// T_i/D_i - x_i would otherwise cancel against the large self term whenever a point has few
// neighbours; the epilogue restores it analytically (phi_ii = 1).  The pipelined loop therefore skips
// the NI sample tiles that are the wave's own row tiles (no masking code in the hot loop); a plain loop after it
// pairs the row tiles with those own tiles that lie in this workgroup's split, the diagonal masked.
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

// Single-fp16 weights (SDKDE_PREC_FP16X2_PHI16): [h(x) h(y) h(z) h(w) | the same again] with h = fp16(phi) toward zero,
// the B operand of one K = 32 MFMA against [x_hi | x_lo]; *rowsum gets the sum of the four ROUNDED weights added
// (v_dot2c_f32_f16 against ones: exact products, fp32 sum), so that D and T carry the same weights.
__device__ __forceinline__ f16x8 round_phi(const f32x4& phi, float* rowsum)
{
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const f16x2 h01 = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(phi.x, phi.y));
    const f16x2 h23 = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(phi.z, phi.w));
    const f16x2 ones = {(_Float16)1, (_Float16)1};
    *rowsum = __builtin_amdgcn_fdot2(h23, ones, __builtin_amdgcn_fdot2(h01, ones, *rowsum, false), false);
    const uint32_t u01 = __builtin_bit_cast(uint32_t, h01), u23 = __builtin_bit_cast(uint32_t, h23);
    return __builtin_bit_cast(f16x8, (u32x4){u01, u23, u01, u23});
}

// Row-tile operands of one wave for NI row tiles starting at row0: -|p~|^2 and the B operand 2 * p~.
// fp32 inputs: lane (r, g) holds coordinates 16kb + 4g .. +3 of row r (b[t][kb]).
// fp16x2 inputs: two K = 32 operands per 16-column block, bh[t][kb][0] = [hi | hi] and
// bh[t][kb][1] = [lo | lo]; lane (r, g) holds elements 8g .. 8g+7 of that K axis, i.e. halves
// 8(g&1) .. +7 of the hi (resp. lo) part.  Against the streamed A operand [hi | lo] the two MFMAs
// sum hi*hi + lo*hi + hi*lo + lo*lo = the full product.
// KLAST (fp32 inputs only): MFMAs of the last 16-column block that contract real coordinates.  The prepared
// fp32 arrays store coordinate c of a block at position 4 (c % 4) + c / 4, so that MFMA kk contracts
// coordinates 4kk .. 4kk+3 and a block with d - 16 (KB - 1) <= 4 KLAST real coordinates needs only KLAST of
// its four MFMAs (the skipped ones would multiply the zero padding).
template <int KB, int NI, int PREC, int KLAST = 4>
struct RowTiles {
    static_assert(KLAST >= 1 && KLAST <= 4 && (KLAST == 4 || PREC == SDKDE_PREC_FP32), "partial last block: fp32 inputs only");
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
            const int steps = kb == KB - 1 ? KLAST : 4;      // compile-time after unrolling
            c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b[t][kb].x, c, 0, 0, 0);
            if (steps > 1) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b[t][kb].y, c, 0, 0, 0);
            if (steps > 2) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b[t][kb].z, c, 0, 0, 0);
            if (steps > 3) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b[t][kb].w, c, 0, 0, 0);
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

template <int KB, int NI, int KIND, int PREC, int KLAST = 4>
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

    RowTiles<KB, NI, PREC, KLAST> rows;
    rows.load(ps, pn, row0, r, g);
    constexpr bool SCALED = SCORE && (PREC == SDKDE_PREC_FP16X2_ALL || PREC == SDKDE_PREC_FP16X2_PHI16);
    if (SCALED) {
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
    constexpr bool PHI16 = PREC == SDKDE_PREC_FP16X2_PHI16;    // the same with single-fp16 weights
    struct Operands {
        f32x4 a1[KB];     // first contraction, A: the lane's 16 bytes of sample r's row, block kb (fp32: coordinates
                          // 16kb + 4g .. +3; fp16x2: elements 8g .. 8g+7 of [hi | lo])
        f32x4 a2[KT];     // second contraction, A: lane (r, g) = coordinate 16mb + r of samples 4g .. 4g+3
                          // (fp32), the eight halves [hi(4g..4g+3) | again] when HALF2, [hi(4g..4g+3) | lo(4g..4g+3)]
                          // when PHI16
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
                // fp32 values, or (PHI16) hi/lo halves: 16 bytes per (column, lane group) either way
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
                    } else if (!(SCORE && PHI16)) {
                        dacc[t] += (phi.x + phi.y) + (phi.z + phi.w);
                    }
                }
                c = (wrap2 ? nxt.nj : cur.nj) + nin;             // accumulator init of pair u+2
                f16x8 bphi;
                if (SCORE && HALF2) bphi = split_phi(phi);       // part of the same VALU clump
                if (SCORE && PHI16) bphi = round_phi(phi, &dacc[t]);
                __builtin_amdgcn_sched_barrier(0);

                if (SCORE && PHI16) {
                    // one K = 32 MFMA per 16-column block: [h(4 samples) | again] against [x_hi | x_lo]
#pragma unroll
                    for (int mb = 0; mb < KB; ++mb)
                        tacc[t][mb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, cur.a2[mb]), bphi,
                                                                             tacc[t][mb], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                } else if (SCORE && !HALF2) {
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
    }
    if constexpr (SELF) {
        // The wave's own row tiles taken as samples, as far as they lie in this split: every pair but that of a
        // point with itself.  A plain loop: NI * 16 of a row's n pairs.
        const int d_end = min(t_end, dt0 + NI);
        for (int jt = max(t_begin, dt0); jt < d_end; ++jt) {
            const int dt = jt - dt0;
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
                f32x4 c = nj + ni[t];
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
                if (!PHI16) dsum[t] += (phi.x + phi.y) + (phi.z + phi.w);
                if (PHI16) {
                    const f16x8 bphi = round_phi(phi, &dsum[t]);
#pragma unroll
                    for (int mb = 0; mb < KB; ++mb)
                        tsum[t][mb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a2[mb]), bphi, tsum[t][mb], 0, 0, 0);
                } else if (!HALF2) {
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
    }
    if (SCALED) {
        constexpr float unscale = 1.0f / (float)(1 << kPhiScaleLog2);
#pragma unroll
        for (int t = 0; t < NI; ++t) {
            dsum[t] *= unscale;
#pragma unroll
            for (int mb = 0; mb < KT; ++mb) tsum[t][mb] *= unscale;
        }
    }
    store_partials<KB, NI, SCORE, ROWMAX>(part_t, part_d, split, m_pad, row0, r, g, tsum, dsum);
}

}  // namespace

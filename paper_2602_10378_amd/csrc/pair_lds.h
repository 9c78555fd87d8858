// Pair kernel of the matrix path for the kinds without a second contraction (eval, Laplace eval, row maximum)
// at large padded dimension: the streamed sample tile is staged in LDS once per workgroup.
#pragma once
#include "common.h"
#include "pair_mfma.h"

namespace {

// ------------------------------------------------------------------------------------------
// pair_mfma_kernel keeps two register sets of the streamed operand per wave (KB float4 each), next to the
// wave's row tiles (NI * KB float4).  From dp = 48 on that leaves room for few row tiles (two from dp = 80),
// so every wave re-reads the whole sample tile from the vector cache / L2 for little work: at d = 128 the
// eval kernel reached 0.64 of the fp32 MFMA peak and ran faster with one workgroup per compute unit than
// with two.  Here the four waves of a workgroup share one copy of the tile in LDS (double-buffered, filled
// by all 256 threads, one barrier per tile) and read their A operands from it one 16-column block at a
// time, which frees the registers for twice the row tiles and cuts the traffic from L2 fourfold.
//
// Same grid, operand layouts, padding rules and partial-sum slots as pair_mfma_kernel; fp32 inputs only.
// LDS row stride DP + 4 floats: the eight lanes a ds_read_b128 serves per clock (rows r .. r+7 of one lane
// group) fall in eight different groups of four banks, since (DP + 4) / 4 is odd.
// ------------------------------------------------------------------------------------------
template <int KB>
constexpr int lds_tile_floats() { return kTile * (KB * 16 + 4); }

template <int KB, int NI, int KIND>
__global__ __launch_bounds__(kBlock) void pair_lds_kernel(
    const float* __restrict__ ps, const float* __restrict__ pn, const float* __restrict__ xs,
    const float* __restrict__ xn, float* __restrict__ part_d, int ntiles, int tiles_per_split, int nsplit,
    int64_t m_pad, float laplace_c0, const float* __restrict__ shift)
{
    static_assert(KIND == kEval || KIND == kEvalLaplace || KIND == kRowMax, "kinds without a second contraction");
    constexpr bool LAPLACE = KIND == kEvalLaplace;
    constexpr bool ROWMAX = KIND == kRowMax;
    constexpr int DP = KB * 16;
    constexpr int STRIDE = DP + 4;
    constexpr int QUADS = kTile * DP / 4;                       // float4s of one sample tile
    constexpr int STAGE = (QUADS + kBlock - 1) / kBlock;        // float4s a thread moves per tile
    __shared__ float tile[2][lds_tile_floats<KB>()];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);    // wave-uniform by construction
    const int r = lane & 15, g = lane >> 4;
    const int split = blockIdx.x % nsplit;
    const int64_t row_block = blockIdx.x / nsplit;
    const int64_t row0 = (row_block * kWavesPerBlock + wave) * (NI * kTile);

    RowTiles<KB, NI, SDKDE_PREC_FP32> rows;
    rows.load(ps, pn, row0, r, g);

    float dacc[NI], dsum[NI];
    float lc0[LAPLACE ? NI : 1];          // Laplace factor constant per row tile: 1 + d/2 + shift_i ln 2
#pragma unroll
    for (int t = 0; t < NI; ++t) {
        dacc[t] = dsum[t] = ROWMAX ? kNegHuge : 0.0f;
        if (LAPLACE) lc0[t] = fmaf(shift ? shift[row0 + t * kTile + r] : 0.0f, kLn2, laplace_c0);
    }

    const int t_begin = split * tiles_per_split;
    const int t_end = min(ntiles, t_begin + tiles_per_split);       // the same for all waves of the workgroup
    if (t_begin < t_end) {
        const int t_last = t_end - 1;       // the prefetch past the end re-reads the last tile (in bounds)
        f32x4 stage[STAGE];
        // a sample tile is kTile consecutive rows of xs: QUADS consecutive float4s
        auto fetch = [&](int jt) {
            const f32x4* src = reinterpret_cast<const f32x4*>(xs + (int64_t)min(jt, t_last) * kTile * DP);
#pragma unroll
            for (int q = 0; q < STAGE; ++q) {
                const int idx = q * kBlock + threadIdx.x;
                if (QUADS % kBlock == 0 || idx < QUADS) stage[q] = src[idx];
            }
        };
        auto deposit = [&](float* buf) {
#pragma unroll
            for (int q = 0; q < STAGE; ++q) {
                const int idx = q * kBlock + threadIdx.x;
                if (QUADS % kBlock == 0 || idx < QUADS)
                    *reinterpret_cast<f32x4*>(buf + (idx / (DP / 4)) * STRIDE + (idx % (DP / 4)) * 4) = stage[q];
            }
        };
        fetch(t_begin);
        f32x4 nj = *reinterpret_cast<const f32x4*>(xn + (int64_t)t_begin * kTile + g * 4);
        deposit(tile[0]);
        __syncthreads();

        for (int jt = t_begin; jt < t_end; ++jt) {
            const float* cur = tile[(jt - t_begin) & 1] + r * STRIDE + g * 4;
            fetch(jt + 1);                  // lands in registers while this tile is worked on
            const f32x4 nj_next = *reinterpret_cast<const f32x4*>(xn + (int64_t)min(jt + 1, t_last) * kTile + g * 4);

            f32x4 c[NI];
#pragma unroll
            for (int t = 0; t < NI; ++t) c[t] = nj + rows.ni[t];
            f32x4 a = *reinterpret_cast<const f32x4*>(cur);
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                f32x4 a_next = a;
                if (kb + 1 < KB) a_next = *reinterpret_cast<const f32x4*>(cur + (kb + 1) * 16);
                __builtin_amdgcn_sched_barrier(0);      // the read stays a whole MFMA group ahead of its use
                // the NI accumulator chains interleave: consecutive MFMAs are independent
#pragma unroll
                for (int v = 0; v < 4; ++v) {
#pragma unroll
                    for (int t = 0; t < NI; ++t)
                        c[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[v], rows.b[t][kb][v], c[t], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                a = a_next;
            }
#pragma unroll
            for (int t = 0; t < NI; ++t) {
                if (ROWMAX) {
                    dacc[t] = fmaxf(dacc[t], fmaxf(fmaxf(c[t].x, c[t].y), fmaxf(c[t].z, c[t].w)));
                } else {
                    f32x4 phi;
                    phi.x = __builtin_amdgcn_exp2f(c[t].x);
                    phi.y = __builtin_amdgcn_exp2f(c[t].y);
                    phi.z = __builtin_amdgcn_exp2f(c[t].z);
                    phi.w = __builtin_amdgcn_exp2f(c[t].w);
                    if (LAPLACE) {
                        // factor 1 + d/2 - r^2/(2h^2) = lc0 + c ln 2, as in pair_mfma_kernel
                        float acc = dacc[t];
                        acc = fmaf(phi.x, fmaf(c[t].x, kLn2, lc0[t]), acc);
                        acc = fmaf(phi.y, fmaf(c[t].y, kLn2, lc0[t]), acc);
                        acc = fmaf(phi.z, fmaf(c[t].z, kLn2, lc0[t]), acc);
                        acc = fmaf(phi.w, fmaf(c[t].w, kLn2, lc0[t]), acc);
                        dacc[t] = acc;
                    } else {
                        dacc[t] += (phi.x + phi.y) + (phi.z + phi.w);
                    }
                }
            }
            if (!ROWMAX && ((jt + 1 - t_begin) & (kFlushTiles - 1)) == 0) {      // two-level accumulation
#pragma unroll
                for (int t = 0; t < NI; ++t) {
                    dsum[t] += dacc[t];
                    dacc[t] = 0.0f;
                }
            }
            // The other buffer was last read before the previous barrier; this barrier publishes the new tile
            // and ends the reads of the current one.
            deposit(tile[(jt + 1 - t_begin) & 1]);
            nj = nj_next;
            __syncthreads();
        }
    }
#pragma unroll
    for (int t = 0; t < NI; ++t) dsum[t] = ROWMAX ? fmaxf(dsum[t], dacc[t]) : dsum[t] + dacc[t];
    const f32x4 none[NI][1] = {};
    store_partials<KB, NI, false, ROWMAX>(nullptr, part_d, split, m_pad, row0, r, g, none, dsum);
}

}  // namespace

// Symmetric score kernel (SDKDE_FLAG_SYMMETRIC): every unordered pair of samples across sample blocks once.
#pragma once
#include "common.h"
#include "pair_mfma.h"

namespace {

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

template <int KB, int NI, int PREC, int KLAST = 4>
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
            RowTiles<KB, NI, PREC, KLAST> rows;      // KLAST: Gram MFMAs of a partly filled last block (pair_mfma.h)
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

}  // namespace

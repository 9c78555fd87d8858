// SD-KDE hot path for MI355X (gfx950 / CDNA4): prep, pair-interaction kernels (fp32 MFMA for
// d >= 4, direct differences for thin d), split reduction + epilogues, and the C ABI.
//
// Notation follows the paper: c = 1/(2h^2), phi_ij = exp(-c |p_i - x_j|^2),
// D_i = sum_j phi_ij, T_i = sum_j phi_ij x_j  (Method section: T = Phi X).
//
// All coordinates are taken relative to a centre of the samples and scaled by a = sqrt(c log2 e), so that
// the squared distance in scaled units is directly the (negated) argument of exp2:
//     phi_ij = exp2( 2 p~_i . x~_j - |p~_i|^2 - |x~_j|^2 ).
// The cross term is the Gram-matrix tile of the Method section, computed with fp32 MFMA;
// the score numerator uses Phi X with the Phi tile still in the registers the first MFMA
// left it in.
#include <string.h>
#include <atomic>
#include <mutex>
#include "common.h"
#include "prep.h"
#include "pair_mfma.h"
#include "pair_lds.h"
#include "pair_sym.h"
#include "pair_thin.h"
#include "epilogue.h"
#include "epilogue_prep.h"

namespace {

// ------------------------------------------------------------------------------------------
// Host side: plan, workspace layout, dispatch.
// ------------------------------------------------------------------------------------------

// Whether the kinds without a second contraction run pair_lds_kernel (sample tile staged in LDS) instead of
// pair_mfma_kernel: fp32 inputs from dp = 64 on.  Measured (eval, n = 262144, m = 65536, best plan of each):
// d = 32 9.42 against 9.10 ms (slower), d = 48 13.03 / 13.16, d = 64 16.37 / 17.57, d = 128 32.0 / 43.5 ms.
constexpr bool lds_staged(int kb, int prec) { return prec == SDKDE_PREC_FP32 && kb >= 4; }

// Most row tiles per wave for which the pair kernels are instantiated (larger ones would spill registers).
constexpr int max_row_tiles(int kb, int kind, int prec = SDKDE_PREC_FP32)
{
    const bool second = kind == kScoreSelf || kind == kScorePoints || kind == kScoreBand;   // has the Phi X contraction
    if ((prec == SDKDE_PREC_FP16X2_ALL || prec == SDKDE_PREC_FP16X2_PHI16) && kb > 1) return 0;      // see effective_prec()
    if (kind == kScoreBand && (kb > 2 || prec != SDKDE_PREC_FP32)) return 0;          // see sym_row_tiles()
    if (!second && lds_staged(kb, prec)) return 4;
    return second ? (kb == 1 ? 8 : (kb <= 4 || (kb == 5 && prec == SDKDE_PREC_FP32)) ? 4 : 2)
                  : (kb == 1 ? 16 : kb == 2 ? 8 : kb <= 4 ? 4 : 2);
}

// Whether pair_mfma_kernel is also built with fewer MFMAs for a partly filled last 16-column block (KLAST < 4):
// fp32 inputs and d <= 32, where the saving is largest (d = 5..8 needs 6 instead of 8 MFMAs per tile in the score,
// 2 instead of 4 in eval); every kind but the symmetric mode's in-block pass, which is a sliver of its work.
constexpr bool partial_last_block_built(int kb, int kind, int prec)
{
    return prec == SDKDE_PREC_FP32 && kb <= 2 && kind != kScoreBand;
}

// Precision mode a call actually runs in: the thin path is fp32 VALU code; the fp16 second contraction is
// used at dp = 16 only and falls back to fp16x2 above.  (Its split of Phi is VALU work that eight row tiles per
// wave amortise best, and from dp = 32 on only four fit: measured at n = 131072, fp16x2 against fp16x2-all,
// d = 32 10.7 / 11.3 ms and d = 64 21.7 / 22.3 ms, where d = 16 gives 6.0 / 4.4 ms.)
inline uint32_t effective_prec(uint32_t flags, bool thin, int dp)
{
    const uint32_t prec = flags & 15u;
    if (thin) return SDKDE_PREC_FP32;
    if ((prec == SDKDE_PREC_FP16X2_ALL || prec == SDKDE_PREC_FP16X2_PHI16) && dp > 16) return SDKDE_PREC_FP16X2;
    return prec;
}

// The fp16 split of 2^14 phi resolves weights with ABSOLUTE precision 2^-39 (the fp16 subnormal step over the
// scale), which is harmless next to a weight of one: the sample's own term at the samples themselves, the
// largest term after a max shift.  A score at separate points without that shift has no such anchor (a point
// whose weights are all below ~1e-7 would lose them in T but not in D), so it runs the fp16x2 mode instead.
inline uint32_t anchored_flags(uint32_t flags, bool self)
{
    const uint32_t prec = flags & 15u;
    if ((prec == SDKDE_PREC_FP16X2_ALL || prec == SDKDE_PREC_FP16X2_PHI16) && !self && !(flags & SDKDE_FLAG_MAX_SHIFT))
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
    int klast;            // MFMAs of the last 16-column block that contract real coordinates: ceil((d - (dp - 16)) / 4)
    // symmetric mode of the score at the samples themselves (pair_sym_kernel), off unless sym_on
    bool sym_on;
    int sym_ni, sym_rb, sym_per_group, sym_nblocks, sym_ngroups;
};

// Overrides of the plan's own choices, set through sdkde_set_tuning (tests and sweeps); 0: none.
std::atomic<int> g_tuning[SDKDE_TUNE_COUNT];

int tuning(int knob, int fallback)
{
    const int v = g_tuning[knob].load(std::memory_order_relaxed);
    return v > 0 ? v : fallback;
}

// Workgroups needed to keep 256 CUs busy with a few waves per SIMD (tiny problems).
constexpr int64_t kTargetBlocks = 2048;
constexpr int kComputeUnits = 256;

// Relative cost per unit of work of running the matrix-path kernels with `ni` row tiles per wave instead of the
// best count (operand reuse against register pressure), measured on MI355X at n = 65536 .. 262144 with fp32
// inputs: score d = 16: 2 / 4 / 8 row tiles 2.67 / 2.37 / 2.37 ms (n = 65536); d = 64: 2 / 4: 9.67 / 8.11 ms;
// eval d = 16 (n = 262144, m = 65536): 2 / 4 / 8 / 16: 5.70 / 5.55 / 5.51 / 5.57 ms; d = 32: 2 / 4 / 8:
// 9.57 / 9.21 / 9.10 ms; d = 48: 2 / 4: 14.3 / 13.1 ms; d = 64 and 128 (pair_lds_kernel): 2 / 4: 16.9 / 16.8 and
// 32.5 / 32.0 ms.
double row_tiles_penalty(bool score, int kb, int ni, uint32_t prec)
{
    if (prec != SDKDE_PREC_FP32) {
        // fp16 input modes (n = 131072 resp. n = 262144, m = 65536): the cheap MFMAs leave the operand loads and
        // the VALU work exposed, so few row tiles cost much more than with fp32 inputs.  Score, fp16x2: d = 16
        // 2 / 4 / 8 row tiles 6.51 / 6.02 / 6.13 ms, d = 32 2 / 4: 12.1 / 10.7, d = 64: 24.0 / 21.7; fp16x2-all
        // (d = 16 only): 9.88 / 5.25 / 4.36 ms.  Eval: d = 16 2 / 4 / 8 / 16: 3.01 / 2.41 / 2.27 / 2.95 ms,
        // d = 32 2 / 4 / 8: 8.15 / 4.30 / 3.39, d = 64 2 / 4: 15.3 / 7.9 ms.
        if (score && (prec == SDKDE_PREC_FP16X2_ALL || prec == SDKDE_PREC_FP16X2_PHI16)) return ni >= 8 ? 1.0 : ni == 4 ? 1.2 : 2.25;
        if (score) return kb >= 5 ? 1.0 : kb == 1 ? (ni >= 8 ? 1.018 : ni == 4 ? 1.0 : 1.08) : (ni >= 4 ? 1.0 : 1.12);
        if (kb == 1) return ni == 16 ? 1.32 : ni == 8 ? 1.0 : ni == 4 ? 1.065 : 1.33;
        if (kb == 2) return ni == 8 ? 1.0 : ni == 4 ? 1.27 : 2.4;
        return kb >= 5 ? 1.0 : ni == 4 ? 1.0 : 1.94;
    }
    if (score) {
        if (kb >= 6) return 1.0;                              // only ni = 2 is built
        // dp = 80: two row tiles leave room for two waves per SIMD, whose tile streams evict each other from the
        // vector cache (n = 262144: 201 ms against 162 ms with four row tiles and one wave per SIMD)
        if (kb == 5) return ni >= 4 ? 1.0 : 1.25;
        return ni >= 8 ? 1.0 : ni == 4 ? (kb == 1 ? 1.004 : 1.0) : (kb == 1 ? 1.12 : 1.15);
    }
    if (kb == 1) return ni == 16 ? 1.013 : ni == 8 ? 1.0 : ni == 4 ? 1.005 : 1.035;
    if (kb == 2) return ni == 8 ? 1.0 : ni == 4 ? 1.008 : 1.05;
    if (lds_staged(kb, (int)prec)) return ni == 4 ? 1.0 : 1.01;
    return ni == 4 ? 1.0 : 1.09;                              // kb = 3
}

// Estimated time of the pair kernel plus its share of the epilogue for `ni` row tiles per wave and `nsplit`
// splits, in units of one wave's time for one 16 x 16 tile.  A compute unit works through its
// ceil(workgroups / 256) workgroups at a rate that does not depend on how many are resident (the kernels are
// bound by instruction issue), so the time is rounds x (work of a workgroup), plus a tail that grows with the
// length of a workgroup, plus the traffic of one more partial slot per split (written once, read once, at about
// 3 TB/s).  Fitted to sweeps over (ni, nsplit) at d = 16 .. 128, n = 8192 .. 1048576, m = 1024 .. 200000: the
// pick is within 0.3 % of the best measured pair on average (2.3 % at worst), where "as many workgroups as
// fill the chip eight times" was 4.7 % off on average and up to 28 % at n = 8192 .. 24576.
double plan_cost(bool score, int kb, uint32_t prec, int64_t m, int64_t m_pad, int ntiles, int ni, int nsplit)
{
    const int64_t row_blocks = (m + kWavesPerBlock * kTile * ni - 1) / (kWavesPerBlock * kTile * ni);
    const int64_t groups = row_blocks * nsplit;
    const int64_t rounds = (groups + kComputeUnits - 1) / kComputeUnits;
    int tps = (ntiles + nsplit - 1) / nsplit;
    tps += tps & 1;
    const double work = (double)rounds * ni * (tps + 1.0) * row_tiles_penalty(score, kb, ni, prec);
    const double tail = 0.1 * ni * tps;
    // clocks per tile: the MFMAs at their measured issue time (33 clocks in fp32; the fp16 modes in proportion to
    // their measured kernel times), plus exp and sums
    double tile_clk = 33.0 * (score ? 8 : 4) * kb + 50.0;
    if (prec == SDKDE_PREC_FP16X2) tile_clk *= 0.62;
    if (prec == SDKDE_PREC_FP16X2_ALL) tile_clk *= score ? 0.41 : 0.62;
    if (prec == SDKDE_PREC_FP16X2_PHI16) tile_clk *= score ? 0.36 : 0.62;
    const double slot_bytes = (double)m_pad * (score ? 16 * kb + 1 : 1) * 8.0;
    const double slot = slot_bytes / 1250.0 / tile_clk;          // 1250 bytes per clock = 3 TB/s at 2.4 GHz
    return work + tail + nsplit * slot;
}

// The same estimate for the thin path (rows per thread `r`, 256 r rows per workgroup), in units of one thread's
// time for one row against one 16-sample tile.  One row per thread is the fastest form per pair (measured at
// n = 262144: d = 1 score 9.96 / 10.36 / 10.23 ms with 1 / 2 / 4 rows, d = 3 18.2 / 18.7 / 19.8 ms), and the
// tail weighs more than on the matrix path; fitted to sweeps at d = 1 and 3, n = 8192 .. 1048576: the pick is
// within 0.2 % of the best measured pair on average (1.3 % at worst), the earlier rule was 7 % off on average.
double plan_cost_thin(bool score, int d, int64_t m, int64_t m_pad, int ntiles, int r, int nsplit)
{
    const int64_t row_blocks = (m + (int64_t)kBlock * r - 1) / ((int64_t)kBlock * r);
    const int64_t groups = row_blocks * nsplit;
    const int64_t rounds = (groups + kComputeUnits - 1) / kComputeUnits;
    int tps = (ntiles + nsplit - 1) / nsplit;
    tps += tps & 1;
    const double penalty = r == 1 ? 1.0 : r == 2 ? 1.0 + 0.015 * (1 + d) : 1.0 + 0.03 * d;
    const double work = (double)rounds * r * (tps + 1.0) * penalty;
    const double tail = 0.6 * r * tps;
    // clocks per row and tile: 16 pairs of 3d + 3 (score) or 2d + 3 (eval) VALU issue slots of 4 clocks
    const double tile_clk = 64.0 * (score ? 3 * d + 3 : 2 * d + 3);
    const double slot = (double)m_pad * (score ? d + 1 : 1) * 8.0 / 1250.0 / tile_clk;
    return work + tail + nsplit * slot;
}

Plan make_plan(int64_t n, int64_t m, int d, bool score, uint32_t flags)
{
    Plan p{};
    p.d = d;
    // Direct differences on the VALU: up to d = 6 for the score kinds, up to d = 3 for eval.  Measured at
    // n = 262144, m = 65536, fp32, VALU form against matrix form (with the shortened last block): score d = 4
    // 19.8 / 26.2 ms, d = 5 22.9 / 29.9, d = 6 26.9 / 30.0, d = 7 30.6 / 30.0, d = 8 33.6 / 30.0; eval d = 4
    // 3.7 / 2.8 ms, d = 5 4.2 / 3.7, d = 6 4.7 / 3.7.
    p.thin = d <= (score ? kThinMaxDScore : kThinMaxDEval);
    p.dp = p.thin ? d : (int)round_up(d, 16);
    p.klast = p.thin ? 4 : (d - (p.dp - 16) + 3) / 4;
    p.n_pad = round_up(n, kRowPad);
    p.m_pad = round_up(m > 0 ? m : 1, kRowPad);
    p.ntiles = (int)((n + 2 * kTile - 1) / (2 * kTile)) * 2;   // even: the pair kernel alternates two operand sets
    const int max_split = p.ntiles >= 32 ? p.ntiles / 16 : 1;   // at least 16 tiles per split

    // Candidate row-tile counts, largest (most operand reuse) first.
    int cand[5];
    int nc = 0;
    if (p.thin && d > kThinMaxDEval) {
        cand[nc++] = 1;                 // built with one row per thread only
    } else if (p.thin) {
        cand[nc++] = 4; cand[nc++] = 2; cand[nc++] = 1;
    } else {
        const int kb = p.dp / 16;
        const int top = max_row_tiles(kb, score ? kScoreSelf : kEval, (int)effective_prec(flags, false, p.dp));
        for (int v = top; v >= 2; v /= 2) cand[nc++] = v;
    }
    const int forced_ni = tuning(score ? SDKDE_TUNE_SCORE_ROW_TILES : SDKDE_TUNE_EVAL_ROW_TILES, 0);
    int forced_split = tuning(score ? SDKDE_TUNE_SCORE_SPLITS : SDKDE_TUNE_EVAL_SPLITS, 0);
    if (forced_split > p.ntiles) forced_split = p.ntiles;
    {
        // a forced value must be one the dispatch tables below instantiate
        const int kb = p.thin ? 0 : p.dp / 16;
        const int widest = p.thin ? (d > kThinMaxDEval ? 1 : 4)
                                  : max_row_tiles(kb, score ? kScoreSelf : kEval, (int)effective_prec(flags, false, p.dp));
        const int narrowest = p.thin ? 1 : 2;
        if (forced_ni >= narrowest && forced_ni <= widest && (forced_ni & (forced_ni - 1)) == 0) {
            cand[0] = forced_ni;
            nc = 1;
        }
    }
    auto set_row_tiles = [&](int ni) {
        p.ni = ni;
        p.rows_per_block = p.thin ? kBlock * ni : kWavesPerBlock * kTile * ni;
        p.row_blocks = (m + p.rows_per_block - 1) / p.rows_per_block;
        if (p.row_blocks < 1) p.row_blocks = 1;
    };

    if (max_split >= 8) {
        // Enough samples for one group of splits per XCD: the (row tiles or rows per thread, splits) pair of least
        // estimated time; ties go to more rows per workgroup, then fewer splits.
        const uint32_t prec = effective_prec(flags, false, p.dp);
        const int most = max_split / 8 * 8 < 1024 ? max_split / 8 * 8 : 1024;
        double best = 0.0;
        int best_ni = 0, best_split = 0;
        for (int k = 0; k < nc; ++k) {
            for (int sp = forced_split > 0 ? forced_split : 8; sp <= (forced_split > 0 ? forced_split : most); sp += 8) {
                const double c = p.thin ? plan_cost_thin(score, d, m > 0 ? m : 1, p.m_pad, p.ntiles, cand[k], sp)
                                        : plan_cost(score, p.dp / 16, prec, m > 0 ? m : 1, p.m_pad, p.ntiles, cand[k], sp);
                if (best_ni == 0 || c < best) {
                    best = c;
                    best_ni = cand[k];
                    best_split = sp;
                }
            }
        }
        set_row_tiles(best_ni);
        p.nsplit = best_split;
    } else {
        // Tiny sample sets: the largest row count per workgroup that still gives the chip enough workgroups,
        // with as many splits as that takes.
        for (int k = 0; k < nc; ++k) {
            set_row_tiles(cand[k]);
            int64_t want = (kTargetBlocks + p.row_blocks - 1) / p.row_blocks;
            if (max_split >= 8) {                       // one group of splits per XCD
                want = round_up(want < 8 ? 8 : want, 8);
                if (want > max_split) want = max_split / 8 * 8;
            } else if (want > max_split) {
                want = max_split;
            }
            p.nsplit = (int)want;
            if (forced_split > 0) p.nsplit = forced_split;
            if (p.row_blocks * p.nsplit >= kTargetBlocks / 2) break;
        }
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
// matrix path, for the dimensions and input modes pair_sym_kernel is built for (sym_row_tiles).  Block size:
// as many rows as the LDS accumulators hold ((dp + 1) floats per row within ~136 KiB), halved while there
// would be too few items to fill the chip.
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
    const int forced_rb = tuning(SDKDE_TUNE_SYM_BLOCK_ROWS, 0);
    if (forced_rb >= sb && forced_rb <= rb * 8 && forced_rb % sb == 0 && (forced_rb & (forced_rb - 1)) == 0 &&
        sym_lds_bytes(kb, forced_rb) <= 160 * 1024)
        rb = forced_rb;
    int max_groups = tuning(SDKDE_TUNE_SYM_GROUPS, kSymMaxGroups);
    if (max_groups < 1 || max_groups > kSymMaxGroups) max_groups = kSymMaxGroups;
    const int64_t n_pad = round_up(n, rb > kRowPad ? rb : kRowPad);
    const int64_t nblocks = n_pad / rb;
    if (nblocks > (1 << 20)) return;
    const int per_group = (int)((nblocks + max_groups - 1) / max_groups);
    const int ngroups = (int)((nblocks + per_group - 1) / per_group);
    // Below ~512 work items (two rounds of one per CU) the ordinary kernels win: measured at d = 16 the mode pays
    // from n = 32768 (528 items) and loses 1.5x at n = 24576 (300 items), 4x at n = 8192; at d = 32 it pays from
    // n = 16384.  The flag is then ignored.  (SDKDE_TUNE_SYM_MIN_ITEMS: for tests of the mode at small sizes.)
    int min_items = tuning(SDKDE_TUNE_SYM_MIN_ITEMS, 512);
    if (min_items < 1) min_items = 1;
    if ((int64_t)ngroups * (ngroups + 1) / 2 < min_items) return;
    p.sym_on = true;
    p.sym_rb = rb;
    p.sym_nblocks = (int)nblocks;
    p.sym_per_group = per_group;
    p.sym_ngroups = ngroups;
    p.n_pad = p.m_pad = n_pad;          // whole blocks; the points are the samples
}

struct Workspace {
    float* centre;                         // the point all coordinates are taken relative to (prep.h)
    uint64_t* stamp;                       // record of the last sample preparation (prep.h)
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
    w.centre = (float*)take(sizeof(float) * SDKDE_MAX_D);
    w.stamp = (uint64_t*)take(sizeof(uint64_t) * kStampWords);
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
    // one slot per split
    size_t slots = (size_t)p.nsplit;
    if (p.sym_on) slots = (size_t)p.sym_ngroups + 2;     // pair_sym_kernel's, then the in-block pass
    w.part_t = score ? (float*)take(sizeof(float) * slots * p.m_pad * p.dp) : nullptr;
    w.part_d = (float*)take(sizeof(float) * slots * p.m_pad);
    w.bytes = off;
    return w;
}

bool bad_bandwidth(double h) { return !(h > 0.0) || !isfinite(h); }

// For a workspace smaller than the plan's own decomposition needs (a buffer sized for another m, say): halves the
// splits, down to one group per XCD (a single split for tiny sample sets).  False when already there.  Fewer
// splits mean fewer partial-sum slots; the call is then slower for few points but needs less memory.
bool fewer_splits(Plan& p)
{
    const int least = p.ntiles >= 128 ? 8 : 1;
    if (p.sym_on || p.nsplit <= least) return false;
    int s = p.nsplit / 2;
    if (least == 8) s = s / 8 * 8;
    p.nsplit = s < least ? least : s;
    p.tiles_per_split = (p.ntiles + p.nsplit - 1) / p.nsplit;
    p.tiles_per_split += p.tiles_per_split & 1;
    return true;
}

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

#define SDKDE_LAUNCH_MFMA_K(KB_, NI_, KLAST_)                                                                     \
    hipLaunchKernelGGL((pair_mfma_kernel<KB_, NI_, KIND, PREC, KLAST_>), grid, block, 0, st, w.ps, w.pn, w.xs,    \
                       w.xt, w.xn, w.part_t, w.part_d, p.ntiles, p.tiles_per_split, p.nsplit, p.m_pad,            \
                       laplace_c0, shift)
#define SDKDE_LAUNCH_MFMA(KB_, NI_)                                                                               \
    do {                                                                                                          \
        if constexpr (partial_last_block_built(KB_, KIND, PREC)) {                                                \
            switch (p.klast) {                                                                                    \
                case 1: SDKDE_LAUNCH_MFMA_K(KB_, NI_, 1); break;                                                  \
                case 2: SDKDE_LAUNCH_MFMA_K(KB_, NI_, 2); break;                                                  \
                case 3: SDKDE_LAUNCH_MFMA_K(KB_, NI_, 3); break;                                                  \
                default: SDKDE_LAUNCH_MFMA_K(KB_, NI_, 4); break;                                                 \
            }                                                                                                     \
        } else {                                                                                                  \
            SDKDE_LAUNCH_MFMA_K(KB_, NI_, 4);                                                                     \
        }                                                                                                         \
    } while (0)
#define SDKDE_LAUNCH_THIN(D_, R_)                                                                      \
    do {                                                                                               \
        if constexpr (KIND != kScoreBand)                                                              \
            hipLaunchKernelGGL((pair_thin_kernel<D_, R_, KIND>), grid, block, 0, st, w.ps, w.xs,       \
                               w.part_t, w.part_d, p.ntiles, p.tiles_per_split, p.nsplit, p.m_pad,     \
                               laplace_c0, shift);                                               \
    } while (0)
// d = 4 .. 6: the kinds a score call runs (one row per thread)
#define SDKDE_LAUNCH_THIN_SCORE(D_)                                                                    \
    do {                                                                                               \
        if constexpr (KIND == kScoreSelf || KIND == kScorePoints || KIND == kRowMax) SDKDE_LAUNCH_THIN(D_, 1); \
        else return SDKDE_EUNSUPPORTED;                                                                \
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
            case 41: SDKDE_LAUNCH_THIN_SCORE(4); break;
            case 51: SDKDE_LAUNCH_THIN_SCORE(5); break;
            case 61: SDKDE_LAUNCH_THIN_SCORE(6); break;
            default: return SDKDE_EUNSUPPORTED;
        }
    } else if (lds_staged(p.dp / 16, PREC) && (KIND == kEval || KIND == kEvalLaplace || KIND == kRowMax)) {
        if constexpr (PREC == SDKDE_PREC_FP32 && (KIND == kEval || KIND == kEvalLaplace || KIND == kRowMax)) {
#define SDKDE_LAUNCH_LDS(KB_, NI_)                                                                                \
    hipLaunchKernelGGL((pair_lds_kernel<KB_, NI_, KIND>), grid, block, 0, st, w.ps, w.pn, w.xs, w.xn, w.part_d,   \
                       p.ntiles, p.tiles_per_split, p.nsplit, p.m_pad, laplace_c0, shift)
#define SDKDE_CASE_LDS(KB_)                                                                   \
    case KB_:                                                                                 \
        switch (p.ni) {                                                                       \
            case 2: SDKDE_LAUNCH_LDS(KB_, 2); break;                                          \
            case 4: SDKDE_LAUNCH_LDS(KB_, 4); break;                                          \
            default: return SDKDE_EUNSUPPORTED;                                               \
        }                                                                                     \
        break;
            switch (p.dp / 16) {
                SDKDE_CASE_LDS(4) SDKDE_CASE_LDS(5) SDKDE_CASE_LDS(6) SDKDE_CASE_LDS(7) SDKDE_CASE_LDS(8)
                default: return SDKDE_EUNSUPPORTED;
            }
#undef SDKDE_CASE_LDS
#undef SDKDE_LAUNCH_LDS
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
                switch (p.ni) { SDKDE_CASE_NI(5, 4) SDKDE_CASE_NI(5, 2) default: return SDKDE_EUNSUPPORTED; }
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
#undef SDKDE_LAUNCH_THIN_SCORE
#undef SDKDE_LAUNCH_THIN
#undef SDKDE_LAUNCH_MFMA
#undef SDKDE_LAUNCH_MFMA_K
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
        if (prec == SDKDE_PREC_FP16X2_PHI16) return launch_pair<KIND, SDKDE_PREC_FP16X2_PHI16>(p, w, shift, st);
    }
    // kinds without a second contraction: the two fp16 modes are the same kernel
    if (prec != SDKDE_PREC_FP32) return launch_pair<KIND, SDKDE_PREC_FP16X2>(p, w, shift, st);
    return launch_pair<KIND, SDKDE_PREC_FP32>(p, w, shift, st);
}

// Symmetric mode: pairs across blocks (pair_sym_kernel), then the pairs inside each block with the ordinary
// kernel restricted to the block (slot ngroups + 1).
template <int KB, int NI, int PREC, int KLAST>
int launch_sym_kernel(const Plan& p, const Workspace& w, hipStream_t st)
{
    const size_t lds = sym_lds_bytes(KB, p.sym_rb);
    // more than 64 KiB of dynamic LDS has to be enabled per kernel and device; remembered, so that later calls
    // (also ones under stream capture) only launch
    constexpr int kMaxDevices = 64;
    static std::mutex guard;                          // host threads may call concurrently
    static size_t lds_allowed[kMaxDevices] = {};
    int dev = 0;
    SDKDE_HIP(hipGetDevice(&dev));
    {
        std::lock_guard<std::mutex> lock(guard);
        if (dev < 0 || dev >= kMaxDevices || lds > lds_allowed[dev]) {
            SDKDE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&pair_sym_kernel<KB, NI, PREC, KLAST>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            if (dev >= 0 && dev < kMaxDevices) lds_allowed[dev] = lds;
        }
    }
    const int64_t items = (int64_t)p.sym_ngroups * (p.sym_ngroups + 1) / 2;
    hipLaunchKernelGGL((pair_sym_kernel<KB, NI, PREC, KLAST>), dim3((unsigned)items), dim3(kSymBlock), lds, st, w.xs, w.xt,
                       w.xn, w.part_t, w.part_d, p.n_pad, p.sym_rb, p.sym_nblocks, p.sym_per_group, p.sym_ngroups);
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

template <int KB, int PREC>
int launch_sym_kb(const Plan& p, const Workspace& w, hipStream_t st)
{
    constexpr int NI = sym_row_tiles(KB, PREC);
    if constexpr (NI > 0) {
        if (p.sym_ni != NI) return SDKDE_EINVAL;
        switch (p.klast) {
            case 1: return launch_sym_kernel<KB, NI, PREC, 1>(p, w, st);
            case 2: return launch_sym_kernel<KB, NI, PREC, 2>(p, w, st);
            case 3: return launch_sym_kernel<KB, NI, PREC, 3>(p, w, st);
            default: return launch_sym_kernel<KB, NI, PREC, 4>(p, w, st);
        }
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

// Launches an epilogue kernel (template parameter: threads per output) over `outputs` outputs of `nslots` slots.
#define SDKDE_LAUNCH_EPILOGUE(KERNEL, nslots, outputs, st, ...)                                                    \
    do {                                                                                                           \
        if (epilogue_parts(nslots, outputs) == kEpiPartsMany) {                                                    \
            constexpr int per_wg = kBlock / kEpiPartsMany;                                                         \
            hipLaunchKernelGGL(KERNEL<kEpiPartsMany>, dim3((unsigned)(((outputs) + per_wg - 1) / per_wg)),         \
                               dim3(kBlock), 0, st, __VA_ARGS__);                                                  \
        } else {                                                                                                   \
            constexpr int per_wg = kBlock / kEpiPartsFew;                                                          \
            hipLaunchKernelGGL(KERNEL<kEpiPartsFew>, dim3((unsigned)(((outputs) + per_wg - 1) / per_wg)),          \
                               dim3(kBlock), 0, st, __VA_ARGS__);                                                  \
        }                                                                                                          \
    } while (0)

// First pass of the max-shifted mode for separate points: row maxima of the exponent, then shift_kernel.
int launch_max_shift(const Plan& p, const Workspace& w, uint32_t flags, hipStream_t st)
{
    int rc = launch_pair_prec<kRowMax>(p, w, flags, nullptr, st);
    if (rc != SDKDE_OK) return rc;
    SDKDE_LAUNCH_EPILOGUE(shift_kernel, p.nsplit, p.m_pad, st, w.part_d, p.nsplit, p.m_pad, w.shift,
                          p.thin ? nullptr : w.pn);
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

// Centre/scale/pad one or two arrays in a single launch (second.src == nullptr: only the first).
// centre_src: the samples whose strided subsample gives the centre (also left in w.centre); null: w.centre as an
// earlier launch on this workspace left it.
// What identifies prepared samples: the kind of call that prepared them (the score and eval layouts differ), the
// caller's array, its shape, the precision mode and the scale a = sqrt(log2 e / 2) / h as it reached the kernels.
Stamp make_stamp(const Workspace& w, bool check, bool score, const float* samples, int64_t n, int d, uint32_t prec, float a)
{
    Stamp s{};
    s.where = w.stamp;
    s.check = check ? 1 : 0;
    uint32_t abits;
    memcpy(&abits, &a, sizeof abits);
    const uint64_t v[kStampWords] = {score ? 1u : 2u, (uint64_t)(uintptr_t)samples, (uint64_t)n, (uint64_t)d, prec, abits};
    for (int k = 0; k < kStampWords; ++k) s.value[k] = v[k];
    return s;
}

int launch_prep(const Plan& p, const PrepJob& first, const PrepJob& second, const float* centre_src, int64_t centre_n,
                float a, const Workspace& w, uint32_t flags, const Stamp& stamp, hipStream_t st)
{
    const PrepCommon common{centre_src, centre_n, w.centre};
    const int64_t per_block = p.thin ? kBlock : kPrepRows;
    if (first.rows_pad % per_block || (second.src && second.rows_pad % per_block)) return SDKDE_EINVAL;
    const int64_t blocks0 = first.rows_pad / per_block;
    const int64_t blocks1 = second.src ? second.rows_pad / per_block : 0;
    if (blocks0 + blocks1 > 0x7fffffffLL) return SDKDE_EUNSUPPORTED;
    const dim3 grid((unsigned)(blocks0 + blocks1)), block(kBlock);
    if (p.thin)
        hipLaunchKernelGGL(prep_thin_kernel, grid, block, 0, st, first, second, (int)blocks0, p.d, common, a, stamp);
    else
        hipLaunchKernelGGL(prep_mfma_kernel, grid, block, 0, st, first, second, (int)blocks0, p.d, p.dp, common, a,
                           (int)effective_prec(flags, p.thin, p.dp), stamp);
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

int check_common(const void* samples, int64_t n, int64_t m, int32_t d, double h, uint32_t flags)
{
    if (!samples || n < 1 || m < 0 || d < 1 || bad_bandwidth(h)) return SDKDE_EINVAL;
    constexpr uint32_t known = 15u | SDKDE_FLAG_MAX_SHIFT | SDKDE_FLAG_SYMMETRIC | SDKDE_FLAG_SAMPLES_PREPARED;
    if (d > SDKDE_MAX_D || (flags & ~known) != 0 || (flags & 15u) > SDKDE_PREC_FP16X2_PHI16) return SDKDE_EUNSUPPORTED;
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

// What the score epilogue of sdkde_fit_eval needs in order to prepare the eval pass's operands in the same launch
// (score_epilogue_prep_kernel): where that pass expects its prepared samples and queries, and the record it leaves.
struct FusedPrep {
    PrepJob sd_job, q_job;
    Stamp stamp;
};

// Whether the one-call pass can fold the eval pass's preparation into the score epilogue, and with what.  Both passes
// must be on the matrix path with their own full decomposition fitting the workspace, the epilogue must be the
// four-part one, and everything the fused launch writes for the eval pass must lie where the score pass no longer
// reads: the prepared shifted samples over the prepared samples (a workgroup reads its rows before it overwrites
// them), their norms and the prepared queries inside the blocked transpose, which only the pair kernel reads.
bool plan_fused_prep(const float* samples_sd, int64_t n, const float* queries, int64_t m, int32_t d, double h, void* workspace,
                     size_t workspace_bytes, uint32_t flags, FusedPrep* out)
{
    if (m <= 0 || (flags & (SDKDE_FLAG_MAX_SHIFT | SDKDE_FLAG_SYMMETRIC | SDKDE_FLAG_SAMPLES_PREPARED))) return false;
    if (tuning(SDKDE_TUNE_SEPARATE_PREP, 0) == 1) return false;
    const uint32_t sflags = anchored_flags(flags, true);
    Plan ps = make_plan(n, n, d, true, sflags);
    apply_symmetric(ps, n, sflags, true);
    const Plan pe = make_plan(n, m, d, false, flags);
    if (ps.thin || pe.thin || ps.sym_on || ps.n_pad != pe.n_pad || ps.dp != pe.dp) return false;
    // One workgroup of the folded launch reduces 32 rows x dp/4 items in dp/8 passes, where the plain epilogue spreads
    // them over dp/8 workgroups: measured per pass of the whole call (folded / separate, same box), d = 16: n = 2048
    // 28.4 / 29.9 us, 4096 33.7 / 35.7, 8192 66.2 / 67.5, 32768 x 4096 662.3 / 665.0; d = 32: 4096 50.0 / 49.1;
    // d = 64: 4096 81.8 / 77.0; d = 128: 145.0 / 131.2.  It pays at dp = 16 only.
    if (ps.dp != 16) return false;
    if (effective_prec(sflags, false, ps.dp) != effective_prec(flags, false, pe.dp)) return false;
    const Workspace ws = layout(ps, true, false, workspace, sflags);
    const Workspace we = layout(pe, false, true, workspace, flags);
    if (ws.bytes > workspace_bytes || we.bytes > workspace_bytes) return false;
    if (epilogue_parts(ps.nsplit, n * (int64_t)d) != kEpiPartsFew) return false;
    if (ps.n_pad % kPrepRows || pe.m_pad % kPrepRows || (ps.n_pad + pe.m_pad) / kPrepRows > 0x7fffffffLL) return false;
    const char* dead_begin = (const char*)ws.xt;
    const char* dead_end = (const char*)ws.xn;                   // the blocked transpose ends where the norms begin
    const char* wr_begin = (const char*)we.xn;
    const char* wr_end = (const char*)(we.pn + pe.m_pad);
    if (we.xs != ws.xs || wr_begin < dead_begin || wr_end > dead_end) return false;
    if ((const char*)we.ps < (const char*)(we.xn + pe.n_pad)) return false;
    const double a = sqrt(1.4426950408889634074 / (2.0 * h * h));
    out->sd_job = PrepJob{samples_sd, n, pe.n_pad, we.xs, nullptr, we.xn, kPadCoord};
    out->q_job = PrepJob{queries, m, pe.m_pad, we.ps, nullptr, we.pn, 0.0f};
    out->stamp = make_stamp(we, false, false, samples_sd, n, d, effective_prec(flags, false, pe.dp), (float)a);
    return true;
}

// Shared body of sdkde_score and of the first half of sdkde_fit_eval.  samples_sd_out (optional, only at
// the samples themselves): also writes samples + (h^2/2) score from the same epilogue.
int score_impl(const float* samples, int64_t n, const float* points, int64_t m, int32_t d, double h,
               float* score_out, float* samples_sd_out, void* workspace, size_t workspace_bytes, uint32_t flags,
               void* stream, const FusedPrep* fused = nullptr)
{
    int rc = check_common(samples, n, m, d, h, flags);
    if (rc != SDKDE_OK) return rc;
    const bool self = points == nullptr || (points == samples && m == n);
    if (points == nullptr && m != n) return SDKDE_EINVAL;
    if (m == 0) return SDKDE_OK;
    if (!score_out && !samples_sd_out) return SDKDE_EINVAL;
    if (samples_sd_out && !self) return SDKDE_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255)) return SDKDE_EWORKSPACE;
    if (flags & SDKDE_FLAG_SAMPLES_PREPARED) return SDKDE_EUNSUPPORTED;      // sdkde_eval / sdkde_eval_laplace only
    flags = anchored_flags(flags, self);

    Plan p = make_plan(n, m, d, true, flags);
    apply_symmetric(p, n, flags, self);
    Workspace w = layout(p, true, !self, workspace, flags);
    while (w.bytes > workspace_bytes && fewer_splits(p)) w = layout(p, true, !self, workspace, flags);
    if (w.bytes > workspace_bytes) return SDKDE_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;

    const double a = sqrt(1.4426950408889634074 / (2.0 * h * h));   // sqrt(c log2 e)
    // at the samples themselves the largest weight is the self pair (exponent 0): nothing to shift
    const bool shifted = !self && (flags & SDKDE_FLAG_MAX_SHIFT) != 0;
    // When the points are the samples (m == n, so m_pad == n_pad), one prepared array serves
    // as both operands.
    const PrepJob sample_job{samples, n, p.n_pad, w.xs, w.xt, w.xn, kPadCoord};
    const PrepJob point_job{self ? nullptr : points, m, p.m_pad, w.ps, nullptr, w.pn, 0.0f};
    const Stamp stamp = make_stamp(w, false, true, samples, n, d, effective_prec(flags, p.thin, p.dp), (float)a);
    if ((rc = launch_prep(p, sample_job, point_job, samples, n, (float)a, w, flags, stamp, st)) != SDKDE_OK) return rc;

    if ((rc = profile_mark(0, 0, st)) != SDKDE_OK) return rc;
    if (shifted && (rc = launch_max_shift(p, w, flags, st)) != SDKDE_OK) return rc;
    const float* shift = shifted ? w.shift : nullptr;
    rc = p.sym_on ? launch_symmetric(p, w, flags, st)
         : self   ? launch_pair_prec<kScoreSelf>(p, w, flags, nullptr, st)
                  : launch_pair_prec<kScorePoints>(p, w, flags, shift, st);
    if (rc != SDKDE_OK) return rc;
    if ((rc = profile_mark(0, 1, st)) != SDKDE_OK) return rc;

    const int64_t total = m * (int64_t)d;
    const int nslots = p.sym_on ? p.sym_ngroups + 2 : p.nsplit;
    const int mode = p.thin ? 1 : (self ? 2 : 0);        // see score_epilogue_kernel
    const int ps_halves = effective_prec(flags, p.thin, p.dp) != SDKDE_PREC_FP32 ? 1 : 0;
    const float inv_ah2 = (float)(1.0 / (a * h * h)), half_h2 = (float)(0.5 * h * h);
    if (!p.thin && epilogue_parts(nslots, total) == kEpiPartsFew) {
        const int64_t quads = m * (p.dp / 4);
        constexpr int per_wg = kBlock / kEpiPartsFew;
        const uintptr_t io = (uintptr_t)score_out | (uintptr_t)samples_sd_out | (samples_sd_out ? (uintptr_t)samples : 0);
        const int quad_io = (d % 4 == 0 && (io & 15) == 0) ? 1 : 0;
        if (fused) {
            // plan_fused_prep has checked that this plan and layout are the ones it was made for
            if (!self || !samples_sd_out || p.sym_on || mode != 2) return SDKDE_EINVAL;
            const int blocks_sd = (int)(fused->sd_job.rows_pad / kPrepRows);
            const int blocks_q = (int)(fused->q_job.rows_pad / kPrepRows);
            hipLaunchKernelGGL(score_epilogue_prep_kernel, dim3((unsigned)(blocks_sd + blocks_q)), dim3(kBlock), 0, st, w.part_t,
                               w.part_d, w.ps, nslots, m, p.m_pad, d, p.dp, ps_halves, inv_ah2, score_out, samples, half_h2,
                               samples_sd_out, quad_io, fused->sd_job, fused->q_job, blocks_sd,
                               PrepCommon{nullptr, 0, w.centre}, (float)a, (int)effective_prec(flags, p.thin, p.dp), fused->stamp);
            return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
        }
        hipLaunchKernelGGL(score_epilogue_quad_kernel, dim3((unsigned)((quads + per_wg - 1) / per_wg)), dim3(kBlock), 0, st,
                           w.part_t, w.part_d, w.ps, nslots, m, p.m_pad, d, p.dp, mode, ps_halves, inv_ah2, score_out,
                           samples, half_h2, samples_sd_out, quad_io, least_trusted_sum(n));
    } else {
        SDKDE_LAUNCH_EPILOGUE(score_epilogue_kernel, nslots, total, st, w.part_t, w.part_d, w.ps, nslots, m, p.m_pad, d,
                              p.dp, mode, ps_halves, inv_ah2, score_out, samples, half_h2, samples_sd_out, least_trusted_sum(n));
    }
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

// Shared body of sdkde_eval and sdkde_eval_laplace.
int eval_impl(const float* samples, int64_t n, const float* queries, int64_t m, int32_t d, double h,
              float* density_out, float* log_density_out, void* workspace, size_t workspace_bytes, uint32_t flags,
              void* stream, bool laplace, bool reuse_centre = false, bool all_prepared = false)
{
    int rc = check_common(samples, n, m, d, h, flags);
    if (rc != SDKDE_OK) return rc;
    if (m == 0) return SDKDE_OK;
    if (!queries || (!density_out && !log_density_out)) return SDKDE_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255)) return SDKDE_EWORKSPACE;

    Plan p = make_plan(n, m, d, false, flags);
    Workspace w = layout(p, false, true, workspace, flags);
    while (w.bytes > workspace_bytes && fewer_splits(p)) w = layout(p, false, true, workspace, flags);
    if (w.bytes > workspace_bytes) return SDKDE_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;

    const double a = sqrt(1.4426950408889634074 / (2.0 * h * h));
    const bool shifted = (flags & SDKDE_FLAG_MAX_SHIFT) != 0;
    const PrepJob sample_job{samples, n, p.n_pad, w.xs, nullptr, w.xn, kPadCoord};
    const PrepJob query_job{queries, m, p.m_pad, w.ps, nullptr, w.pn, 0.0f};
    if (all_prepared) {
        // sdkde_fit_eval: the score epilogue has prepared samples and queries for this plan (plan_fused_prep)
    } else if (flags & SDKDE_FLAG_SAMPLES_PREPARED) {
        // the workspace still holds the centre and the prepared samples (their place in the workspace depends
        // on n, d and the precision mode only, not on m): only the queries are prepared
        // (a call whose record of the prepared samples does not match gets NaN for every output)
        const Stamp expect = make_stamp(w, true, false, samples, n, d, effective_prec(flags, p.thin, p.dp), (float)a);
        if ((rc = launch_prep(p, query_job, PrepJob{}, nullptr, 0, (float)a, w, flags, expect, st)) != SDKDE_OK) return rc;
    } else {
        // reuse_centre: w.centre still holds the centre of an earlier pass over (nearly) the same points
        const Stamp stamp = make_stamp(w, false, false, samples, n, d, effective_prec(flags, p.thin, p.dp), (float)a);
        if ((rc = launch_prep(p, sample_job, query_job, reuse_centre ? nullptr : samples, n, (float)a, w, flags, stamp, st)) != SDKDE_OK)
            return rc;
    }

    const double lognorm = -log((double)n) - (double)d * log(h) - 0.5 * (double)d * log(6.283185307179586476925286766559);
    if ((rc = profile_mark(1, 0, st)) != SDKDE_OK) return rc;
    if (shifted && (rc = launch_max_shift(p, w, flags, st)) != SDKDE_OK) return rc;
    const float* shift = shifted ? w.shift : nullptr;
    rc = laplace ? launch_pair_prec<kEvalLaplace>(p, w, flags, shift, st) : launch_pair_prec<kEval>(p, w, flags, shift, st);
    if (rc != SDKDE_OK) return rc;
    if ((rc = profile_mark(1, 1, st)) != SDKDE_OK) return rc;

    SDKDE_LAUNCH_EPILOGUE(eval_epilogue_kernel, p.nsplit, m, st, w.part_d, p.nsplit, m, p.m_pad, lognorm, laplace ? 1 : 0,
                          shift, least_trusted_sum(n), density_out, log_density_out);
    return hipGetLastError() == hipSuccess ? SDKDE_OK : SDKDE_EDEVICE;
}

}  // namespace

// Built-in scratch buffer of sdkde_fit_eval_static: one copy per GPU the library runs on, held until the
// process ends.  The name is a host-side stand-in; the device address is looked up once per device.
static __device__ __align__(256) unsigned char scratch[SDKDE_STATIC_SCRATCH_BYTES];

namespace {

// Address of `scratch` on the current device (resolved on the first call there; null on failure).
void* static_scratch_address()
{
    constexpr int kMaxDevices = 64;
    static std::mutex guard;
    static void* address[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(guard);
    if (!address[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        address[dev] = ptr;
    }
    return address[dev];
}

}  // namespace

extern "C" {

int sdkde_workspace_bytes(int64_t n, int64_t m, int32_t d, uint32_t flags, size_t* bytes)
{
    if (!bytes) return SDKDE_EINVAL;
    int rc = check_common(bytes, n, m, d, 1.0, flags);
    if (rc != SDKDE_OK) return rc;
    // Largest of: score at the samples themselves, score at m separate points, eval at m queries.
    Plan self_plan = make_plan(n, n, d, true, flags);
    apply_symmetric(self_plan, n, flags, true);
    size_t need = layout(self_plan, true, false, nullptr, flags).bytes;
    if (m > 0) {
        const uint32_t at_points = anchored_flags(flags, false);      // the mode a score at separate points runs in
        size_t b = layout(make_plan(n, m, d, true, at_points), true, true, nullptr, at_points).bytes;
        need = b > need ? b : need;
        b = layout(make_plan(n, m, d, false, flags), false, true, nullptr, flags).bytes;
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
    if (!workspace || ((uintptr_t)workspace & 255)) return SDKDE_EWORKSPACE;
    // The centre of the samples stays in the workspace; the shifted samples are centred on it too (any
    // centre is exact, it only has to be near the data).  Where the layouts allow it the score epilogue also
    // prepares the eval pass's operands: five launches instead of six.
    FusedPrep fused;
    const bool fuse = plan_fused_prep(samples_sd_out, n, queries, m, d, h, workspace, workspace_bytes, flags, &fused);
    rc = score_impl(samples, n, nullptr, n, d, h, score_out, samples_sd_out, workspace, workspace_bytes, flags, stream,
                    fuse ? &fused : nullptr);
    if (rc != SDKDE_OK || m == 0) return rc;
    return eval_impl(samples_sd_out, n, queries, m, d, h, density_out, log_density_out, workspace, workspace_bytes,
                     flags, stream, false, true, fuse);
}

int sdkde_fit_eval_static(const float* samples, int64_t n, const float* queries, int64_t m, int32_t d, double h,
                          float* score_out, float* samples_sd_out, float* density_out, float* log_density_out,
                          uint32_t flags, void* stream)
{
    if (!samples_sd_out) return SDKDE_EINVAL;
    int rc = check_common(samples, n, m, d, h, flags);
    if (rc != SDKDE_OK) return rc;
    // The whole pass must fit the built-in buffer with the decomposition the ordinary call would take, so that
    // both give the same bits; larger problems are refused, not run with fewer splits.
    size_t need = 0;
    if ((rc = sdkde_workspace_bytes(n, m, d, flags, &need)) != SDKDE_OK) return rc;
    if (need > (size_t)SDKDE_STATIC_SCRATCH_BYTES) return SDKDE_ETOOLARGE;
    void* ws = static_scratch_address();
    if (!ws) return SDKDE_EDEVICE;
    return sdkde_fit_eval(samples, n, queries, m, d, h, score_out, samples_sd_out, density_out, log_density_out, ws,
                          (size_t)SDKDE_STATIC_SCRATCH_BYTES, flags, stream);
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
    Plan p = make_plan(n, rows, d, score, flags);
    if (score) apply_symmetric(p, n, flags, !separate);
    char* const base = reinterpret_cast<char*>(uintptr_t(1) << 20);      // any aligned non-null address: offsets only
    const Workspace w = layout(p, score, separate, base, flags);
    auto off = [&](const void* q) { return q ? (int64_t)((const char*)q - base) : (int64_t)-1; };
    const int64_t slots = p.sym_on ? p.sym_ngroups + 2 : p.nsplit;
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
    if (out_len >= 25)
        out[24] = (!p.thin && partial_last_block_built(p.dp / 16, score ? kScoreSelf : kEval, (int)effective_prec(flags, p.thin, p.dp)))
                      ? p.klast : 4;
    if (out_len >= 26) {
        out[25] = 0;
        size_t need = 0;
        FusedPrep unused;
        if (call == 2 && sdkde_workspace_bytes(n, m, d, flags, &need) == SDKDE_OK)
            out[25] = plan_fused_prep(nullptr, n, nullptr, m, d, 1.0, base, need, flags, &unused) ? 1 : 0;
    }
    return SDKDE_OK;
}

int sdkde_set_tuning(int knob, int value)
{
    if (knob < 0 || knob >= SDKDE_TUNE_COUNT || value < 0) return SDKDE_EINVAL;
    g_tuning[knob].store(value, std::memory_order_relaxed);
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
        case SDKDE_ETOOLARGE: return "problem too large for the built-in scratch buffer";
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

// Types, constants and the kinds of pair kernel shared by every part of the SD-KDE library (gfx950).
#pragma once
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
constexpr int kCentreElems = 4096;      // the centre is the mean of about this many evenly strided input values
constexpr int kFlushTiles = 64;         // sample tiles between folds of the running sums (power of two)
constexpr int kThinMaxDScore = 6;      // direct-difference path for the score kinds up to this d, MFMA path above
constexpr int kThinMaxDEval = 3;       // the same for the kinds without a numerator (eval, Laplace eval)

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
// v_exp_f32 flushes results below the smallest normal fp32 number (2^-126) to zero, so a weight sum over n samples
// may have lost up to n * 2^-126.  A sum that this could change by more than one part in a thousand (the
// tolerance of the outputs) is treated as the all-underflow case (score 0, density 0, log density -inf) rather
// than returned as a plausible number: with three samples all ~13.1 bandwidths from a query the sum came out 44 %
// low.  least_trusted_sum(n) is that threshold.
constexpr double kMinNormal = 1.17549435e-38;
inline float least_trusted_sum(int64_t n) { return (float)((double)n * 1000.0 * kMinNormal); }
constexpr float kLn2 = 0.693147180559945309f;

inline int64_t round_up(int64_t v, int64_t q) { return (v + q - 1) / q * q; }

}  // namespace

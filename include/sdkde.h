/*
 * sdkde.h - C ABI of the MI355X (gfx950) SD-KDE library.
 *
 * The library computes the three steps of score-debiased kernel density estimation
 * exactly as the paper states the problem (Introduction; Method section): samples x_i in
 * R^d (n of them), a scalar bandwidth h, and query points y_j (m of them).
 *
 * Conventions for every call
 *  - All array arguments are DEVICE pointers to fp32, row-major, contiguous, owned by the
 *    caller.  The library never frees, retains or reallocates them.  `workspace` is device
 *    memory too (any 256-byte aligned block of at least sdkde_workspace_bytes() bytes); its
 *    contents are scratch and need no initialisation.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is only
 *    enqueued; no call synchronises with the host, and no call allocates device memory.
 *  - h is passed as double so that the derived constants are formed in double and rounded
 *    once; the pairwise arithmetic itself is fp32 (fp32 MFMA inputs, fp32 accumulation) unless
 *    `flags` selects another input mode.
 *  - Accuracy domain of the matrix path (d >= 7, and the eval calls at d >= 4): squared distances are formed as
 *    |p|^2 + |x|^2 - 2 p.x on coordinates taken relative to a centre of the samples (the mean of an evenly
 *    strided subsample of them).  With E = (|p - centre|^2 + max_j |x_j - centre|^2) / 2h^2 the size of the terms
 *    that cancel, each of the 2 + d/4 roundings can cost E 2^-24 in the exponent of phi, so the stated 1e-3
 *    tolerances are guaranteed while (2 + d/4) E 2^-24 <= 1e-3 (every point within about 50 h of the centre at
 *    d = 16, 30 h at d = 64, 20 h at d = 128) and typically hold to twice those distances.  The thin path (d <= 3,
 *    the score calls d <= 6) forms the differences directly, but of coordinates that were rounded to fp32 after
 *    centring and scaling: a difference is good to 2^-24 R (R = distance from the centre), not to the last bit
 *    of the inputs.  The score's numerator is formed the paper's way on the matrix path, p sum_j phi_j -
 *    sum_j phi_j x_j, two sums of size |p - centre| sum_j phi_j carried in fp32.  On either path, whatever the
 *    size of the result, about 1e-6 (1 + R/h) / h of the score is lost, which shows only where the true score is
 *    that small against 1/h (a sample whose only neighbours are its exact duplicates, a bandwidth so narrow that
 *    every neighbour's weight vanishes).  (Far outside that domain, R/h above ~1e18, the scaled
 *    coordinates overflow fp32 on either path and the outputs are NaN.)  Unless SDKDE_FLAG_MAX_SHIFT is set no running maximum
 *    is kept, and weights below the smallest normal fp32 number (2^-126) are flushed to zero: a point whose
 *    weights phi_j sum to less than 1000 n 2^-126 (so that the flushed ones could be more than one part in a
 *    thousand of the sum; the point is then farther than about 11.5 - 13 h from every sample, depending on n)
 *    gets the all-underflow results documented with each call instead of a number that may be wrong.
 *  - Results are deterministic: no atomics are used, so repeated calls with the same
 *    arguments (and a workspace of at least sdkde_workspace_bytes, or of the same size) give
 *    bit-identical outputs.
 *  - Stream capture: the calls only launch kernels (no allocation, no memset, no host
 *    synchronisation), so a sequence of them can be captured into a HIP graph.  One
 *    exception: the first SDKDE_FLAG_SYMMETRIC score on a device raises that kernel's dynamic
 *    LDS limit (a function attribute, set once per device and kernel), so make one such call
 *    outside capture first.  The optional instrumentation records events and must stay off
 *    during capture.
 *  - Return value: SDKDE_OK or an error code; nothing throws.  After an error the outputs
 *    are unspecified.  Two calls that share a workspace must be ordered on one stream.
 *  - Host threads: calls keep no state between them (the optional instrumentation and the test-only
 *    sdkde_set_tuning below aside), so
 *    several threads may call concurrently, each with its own workspace and stream, on the device that is
 *    current in that thread.
 */
#ifndef SDKDE_H
#define SDKDE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SDKDE_OK = 0,
    SDKDE_EINVAL = 1,       /* null pointer, n < 1, m < 0, d < 1, h not finite or <= 0 */
    SDKDE_EUNSUPPORTED = 2, /* d above SDKDE_MAX_D, unknown flag bits */
    SDKDE_EWORKSPACE = 3,   /* workspace missing, misaligned or too small */
    SDKDE_EDEVICE = 4,      /* a HIP launch or event call failed */
    SDKDE_ETOOLARGE = 5     /* sdkde_fit_eval_static: the sizes need more than SDKDE_STATIC_SCRATCH_BYTES */
};

enum {
    SDKDE_MAX_D = 128,
    /* flags: precision mode of the distance cross term (the Gram-matrix tile of the Method section) */
    SDKDE_PREC_FP32 = 0,    /* fp32 MFMA inputs, fp32 accumulate: the reference path */
    SDKDE_PREC_FP16X2 = 1,  /* each input split into two fp16 halves (hi + lo, ~22 mantissa bits) and
                               multiplied on the fp16 matrix units with fp32 accumulate; Phi X, exp and all
                               sums stay fp32.  A lower-precision-input mode: its error is reported
                               separately.  Ignored on the thin path (fp32 VALU: d <= 3, the score calls
                               d <= 6). */
    SDKDE_PREC_FP16X2_ALL = 2, /* as FP16X2, and Phi X on the fp16 matrix units too: Phi is split in registers
                               into fp16 hi + lo (scaled by 2^14 to stay normal), X into hi + lo in the
                               prepared copy; fp32 accumulate, exp and the row sums D stay fp32.  The split
                               resolves a weight to max(2^-22 phi, 2^-39) ABSOLUTE, i.e. relative to a
                               weight of one, so it is used where such a weight is present: the score at
                               the samples themselves (own term 1) and the score at separate points
                               together with SDKDE_FLAG_MAX_SHIFT (largest term 1).  The score error is
                               then at most n 2^-39 max_j |x_j - mean| / h^2 on top of the FP16X2 mode's;
                               only a data set in which nearly every sample is isolated (all neighbour
                               weights under ~1e-7) has scores that small.  A score at separate points
                               without the shift, calls without a Phi X contraction (eval), and d > 16
                               (where it is no faster than FP16X2) run as FP16X2. */
    SDKDE_PREC_FP16X2_PHI16 = 3, /* as FP16X2 for the cross term, and Phi X on the fp16 matrix units with every weight
                               rounded to ONE fp16 value (scaled by 2^14, X still hi + lo): the least precise input mode.
                               The row sums D are taken of the same rounded weights, so T - p D is exactly the direct-form
                               numerator sum_j fp16(phi_j) (x_j - p): the error is relative to the weights, not to the
                               size of the coordinates: 2^-11 per term, i.e. up to 5e-4 of sum_j phi_j |x_j - p| / (h^2 D),
                               a few 1e-4 of the score where the terms pull one way, and up to ~1.2e-3 of it (measured)
                               at a point with few neighbours whose pulls partly cancel;
                               fp32 accumulate, exp fp32.  Applies where FP16X2_ALL applies, and runs as FP16X2
                               elsewhere. */
    /* flags bit 4: two-pass, max-shifted sums for sdkde_eval, sdkde_eval_laplace and sdkde_score at
       separate points: a first pass finds max_j of the exponent for every point, the second sums
       phi_j / max phi, and the logarithm (or the signed density) gets the shift back.  Results then stay
       finite however far a point is from the samples (the log density never becomes -inf, the score at
       a far point is that of its nearest samples), at about 1.75x the time of the call. */
    SDKDE_FLAG_MAX_SHIFT = 16,
    /* flags bit 5: symmetric score.  phi_ij = phi_ji, so for the score at the samples themselves each
       unordered pair needs one Gram-matrix entry and one exp, used for both T_i and T_j (an algorithmic saving
       the paper does not take: "Arithmetic intensity in d dimensions" counts all n^2 pairs).  A separate
       mode, reported separately and against the same n^2 pair count.  Same results within the same tolerances,
       still without atomics and bit-reproducible, but more workspace (one partial [T | D] per row for each of
       up to 64 groups of sample blocks: about 4.6 GiB at n = 2^20, d = 16).  Takes effect where it pays: for
       sdkde_score at the samples themselves and sdkde_fit_eval with 7 <= d <= 32, SDKDE_PREC_FP32 and enough samples to fill the chip with its work
       items (n >= 32768 at d <= 16, n >= 16384 at d <= 32); ignored otherwise (sdkde_describe_plan tells). */
    SDKDE_FLAG_SYMMETRIC = 32,
    /* flags bit 6, sdkde_eval and sdkde_eval_laplace only (evaluating one fitted estimate at many batches of
       queries): the workspace still holds what the previous sdkde_eval / sdkde_eval_laplace call on it prepared
       from the same samples, n, d, h and precision mode, and nothing else has used the workspace since: the
       centre and the prepared samples are reused and only the queries are prepared (m may differ from
       call to call, the workspace being large enough for each m used; at n = 2^20 this saves about 0.3 ms per call).  The samples are not read.  The workspace
       keeps a record of what was prepared (kind of call, samples pointer, n, d, h, precision mode); a call whose
       arguments do not match that record returns SDKDE_OK like any other but writes NaN to every output, so a
       broken precondition cannot pass for a result.  (Samples changed in place behind the same pointer are not
       detected.)  Other calls return SDKDE_EUNSUPPORTED for the flag. */
    SDKDE_FLAG_SAMPLES_PREPARED = 64
};

/*
 * Bytes of workspace sufficient for each of: sdkde_score at the n samples themselves,
 * sdkde_score at m separate points, and sdkde_eval at m queries, all with n samples of
 * dimension d, called with these flags.  One block of this size serves the whole score ->
 * debias -> eval pipeline.  The size depends on n, m, d and flags together (the grid
 * decomposition, and with it the number of partial-sum slots, is chosen per shape and
 * precision mode).  A call given less than its own size (a buffer made for another m, say)
 * falls back to fewer splits of the samples - the same results to rounding, in a different but
 * equally fixed summation order, slower when there are few points - and returns
 * SDKDE_EWORKSPACE, doing nothing, only if its smallest decomposition does not fit either (a
 * buffer made for m points always serves fewer points with the same n, d and flags).  The
 * symmetric mode has one decomposition only and is refused without its full size.
 * bytes: host pointer, written on success.
 */
int sdkde_workspace_bytes(int64_t n, int64_t m, int32_t d, uint32_t flags, size_t *bytes);

/*
 * Empirical score of the Gaussian KDE of `samples` with bandwidth h (Introduction, formula
 * for s-hat; Method section, the identity that turns its numerator into T = Phi X):
 *     s(p) = sum_j -(p - x_j) phi_j / (h^2 sum_j phi_j),  phi_j = exp(-|p - x_j|^2 / 2h^2),
 * evaluated at each of the m `points`.  points == NULL means "at the samples themselves"
 * (then m must equal n); the sum always runs over all n samples, so a point that is a
 * sample includes its own term.  A point so far from every sample that sum_j phi_j is below
 * 1000 n 2^-126 (see above) gets score 0 (SDKDE_FLAG_MAX_SHIFT: a shifted sum instead).
 *   samples   [n, d] in      points [m, d] in (or NULL)      score_out [m, d] out
 * score_out must not overlap samples, points or workspace.
 */
int sdkde_score(const float *samples, int64_t n, const float *points, int64_t m, int32_t d,
                double h, float *score_out, void *workspace, size_t workspace_bytes,
                uint32_t flags, void *stream);

/*
 * Debiasing shift (Introduction; Method section): samples_sd = samples + (h^2 / 2) score,
 * elementwise over [n, d].  samples_sd_out may alias samples or score.  n = 0 is a no-op.
 */
int sdkde_debias(const float *samples, const float *score, int64_t n, int32_t d, double h,
                 float *samples_sd_out, void *stream);

/*
 * Gaussian KDE of `samples_sd` at the queries (Introduction, first display, with phi the
 * standard normal density so that the estimate integrates to one; Method section, the
 * train-query Gram matrix):
 *     p(q) = 1 / (n h^d (2 pi)^(d/2)) * sum_j exp(-|q - x_j|^2 / 2h^2).
 * density_out and log_density_out are [m] outputs; either may be NULL, not both.  The
 * density underflows to 0 where it is below the fp32 range (large d); the log density is
 * finite unless the sum of the weights is below 1000 n 2^-126 (see above; then -inf, density 0;
 * SDKDE_FLAG_MAX_SHIFT evaluates such queries with a shifted sum).  m = 0 is a no-op.
 *   samples_sd [n, d] in     queries [m, d] in
 */
int sdkde_eval(const float *samples_sd, int64_t n, const float *queries, int64_t m, int32_t d,
               double h, float *density_out, float *log_density_out, void *workspace,
               size_t workspace_bytes, uint32_t flags, void *stream);

/*
 * The whole SD-KDE pass in one call (Method section, opening paragraph: form the empirical SD-KDE,
 * score + shift, and evaluate the resulting density on the queries): sdkde_score at the samples,
 * the shift fused into its epilogue, then sdkde_eval of the shifted samples, with the shifted samples
 * centred on the centre already computed for the samples (one launch fewer than the three calls; at d <= 16,
 * where the queries' prepared copy fits beside the samples', the same epilogue also prepares the eval pass's
 * operands: two launches fewer, same bits).
 *   samples [n, d] in      queries [m, d] in
 *   score_out [n, d] out, may be NULL      samples_sd_out [n, d] out, required
 *   density_out / log_density_out [m] out, either may be NULL, not both (unless m = 0)
 * Results equal those of the three separate calls up to the rounding of the centring.
 */
int sdkde_fit_eval(const float *samples, int64_t n, const float *queries, int64_t m, int32_t d,
                   double h, float *score_out, float *samples_sd_out, float *density_out,
                   float *log_density_out, void *workspace, size_t workspace_bytes, uint32_t flags,
                   void *stream);

/*
 * sdkde_fit_eval without a workspace argument, for callers that cannot allocate device memory or keep a
 * workspace of their own (code under stream capture, tight serving loops, harnesses that forbid hipMalloc):
 * the partial sums and prepared operands live in a buffer of SDKDE_STATIC_SCRATCH_BYTES that is part of the
 * library's device image, one copy per GPU, held until the process ends.  No allocation of any kind happens
 * in the call; inputs and outputs are still the caller's device arrays, with the meaning they have in
 * sdkde_fit_eval, and the results are bit-identical to those of sdkde_fit_eval with a workspace of
 * sdkde_workspace_bytes(n, m, d, flags).  Sizes for which that figure exceeds SDKDE_STATIC_SCRATCH_BYTES are
 * refused with SDKDE_ETOOLARGE and nothing is launched (the buffer serves e.g. n = m = 32768 at d = 16,
 * n = 65536, m = 8192 at d = 16, n = m = 16384 at d = 64).  The buffer keeps the last call's contents; nothing
 * in it has to start at zero, every call rewrites what it reads.  All calls on one GPU share the one buffer:
 * two calls that overlap in time on the same GPU (different streams or host threads) race; order them on
 * one stream.  The first call on a device looks up the buffer's device address (no stream work); make it
 * outside stream capture.
 */
enum { SDKDE_STATIC_SCRATCH_BYTES = 64 * 1024 * 1024 };
int sdkde_fit_eval_static(const float *samples, int64_t n, const float *queries, int64_t m, int32_t d,
                          double h, float *score_out, float *samples_sd_out, float *density_out,
                          float *log_density_out, uint32_t flags, void *stream);

/*
 * Laplace-corrected KDE (Laplace-corrected KDE section: K_h^LC(x) = K_h(x) (1 + d/2 - |x|^2 / 2h^2),
 * p_LC(q) = (1/n) sum_j K_h^LC(q - x_j)), with the affine factor applied inside the same pass that
 * forms exp(-|q - x_j|^2 / 2h^2) (the fused "Flash-Laplace-KDE" of that section).  It takes the
 * UNSHIFTED samples and needs no score pass.  The estimate can be negative; density_out [m] is
 * signed and underflows to 0 where |p_LC| is below the fp32 range.  Arguments otherwise as in
 * sdkde_eval; sdkde_workspace_bytes(n, m, d) covers it.
 */
int sdkde_eval_laplace(const float *samples, int64_t n, const float *queries, int64_t m, int32_t d,
                       double h, float *density_out, void *workspace, size_t workspace_bytes,
                       uint32_t flags, void *stream);

/*
 * Introspection of the host-side plan (grid decomposition and workspace layout) that a call with these
 * sizes would use; touches no device.  call: 0 = sdkde_score at the samples, 1 = sdkde_score at m
 * separate points, 2 = sdkde_eval / sdkde_eval_laplace at m queries.  out (host, at least 20 entries):
 *   [0] thin path (0/1)      [1] padded dimension   [2] row tiles per wave (thin: rows per thread)
 *   [3] rows per workgroup   [4] row blocks         [5] splits of the sample axis
 *   [6] sample tiles per split   [7] sample tiles (of 16)   [8] padded sample rows   [9] padded point rows
 *   [10] workspace bytes     [11..17] byte offsets in the workspace of: prepared samples, their
 *   blocked transpose, their norms, prepared points, their norms, partial T, partial D (-1 = absent)
 *   [18] partial slots       [19] size factor of the transposed copy (2 in the FP16X2_ALL mode)
 * and, when out_len >= 24: [20] symmetric mode in effect   [21] rows per sample block   [22] blocks per group
 *   [23] groups (work items = groups (groups + 1) / 2)
 * and, when out_len >= 25: [24] matrix instructions of the first contraction spent on the last 16-column block
 *   (4 = all; fewer when the block holds at most 12 real coordinates: fp32 inputs, d <= 32)
 * and, when out_len >= 26: [25] call 2 only: 1 if sdkde_fit_eval at these sizes and flags, with a workspace of
 *   sdkde_workspace_bytes, prepares the eval pass's operands inside its score epilogue (five launches instead
 *   of six), else 0
 */
int sdkde_describe_plan(int64_t n, int64_t m, int32_t d, int32_t call, uint32_t flags, int64_t *out,
                        int32_t out_len);

/*
 * For tests and parameter sweeps only: overrides one of the choices the host-side plan otherwise makes from
 * the sizes alone (value 0 restores the library's own choice).  Values the kernels are not built for are
 * ignored.  The setting is process-global and changes the decomposition, hence the workspace size and the
 * (still fixed) summation order: set it before sdkde_workspace_bytes and leave it alone until the calls it
 * is meant for have been issued.  Normal use never calls this; the library reads no environment variables.
 */
enum {
    SDKDE_TUNE_SCORE_ROW_TILES = 0, /* row tiles per wave (thin path: rows per thread) of the score calls */
    SDKDE_TUNE_SCORE_SPLITS = 1,    /* splits of the sample axis of the score calls */
    SDKDE_TUNE_EVAL_ROW_TILES = 2,  /* the same two for sdkde_eval / sdkde_eval_laplace */
    SDKDE_TUNE_EVAL_SPLITS = 3,
    SDKDE_TUNE_SYM_BLOCK_ROWS = 4,  /* symmetric mode: rows per sample block (a power of two) */
    SDKDE_TUNE_SYM_GROUPS = 5,      /* symmetric mode: most groups of sample blocks (1 .. 64) */
    SDKDE_TUNE_SYM_MIN_ITEMS = 6,   /* symmetric mode: least number of work items for the flag to take effect
                                       (default 512) */
    SDKDE_TUNE_SEPARATE_PREP = 7,   /* 1: sdkde_fit_eval always prepares the eval pass's operands in a launch of
                                       its own (same results; for comparing the two forms) */
    SDKDE_TUNE_COUNT = 8
};
int sdkde_set_tuning(int knob, int value);

/* Static, human-readable name of a status code. */
const char *sdkde_status_string(int status);

/*
 * Optional instrumentation.  While enabled, sdkde_score and sdkde_eval bracket their main
 * pair-interaction kernel with HIP events on the caller's stream (up to 256 launches of each
 * kind are kept; enabling or disabling resets the record).  sdkde_profile_summary waits for
 * the recorded events of one kind (which: 0 = score, 1 = eval) and returns how many launches
 * were recorded and the sum of their durations in milliseconds (host pointers).  The state is
 * process-global and not thread-safe.
 */
int sdkde_profile_enable(int on);
int sdkde_profile_summary(int which, int *launches, float *total_ms);

#ifdef __cplusplus
}
#endif
#endif /* SDKDE_H */

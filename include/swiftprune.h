/*
 * swiftprune.h - C ABI of the SwiftPrune per-layer pruning path for AMD gfx950.
 *
 * Method: "SwiftPrune: Hessian-Free Weight Pruning for Large Language Models"
 * (arXiv 2501.16376).  One linear layer  y = W x  with  W[out, in]  is pruned
 * from calibration activations  X[tokens, in]  in four steps:
 *
 *   1. statistics   xsq[q] = sum_t X[t,q]^2,  S = sum_q xsq[q]      (Algorithm 1, first statement)
 *   2. score        L[r,q] = 1/2 * W[r,q]^2 / (1 - xsq[q]/S)         (Sec. 3.1, the score equation)
 *   3. selection    per row, an EWMA threshold walk (Sec. 3.2, Algorithm 1 loop),
 *                   or N:M group selection (Sec. 3.3)
 *   4. apply        pruned weights are set to zero in place           (Algorithm 1, "w_i = 0")
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller; the only
 *     host pointers are `params` and the out-arguments of the host helpers.
 *     The library allocates nothing, frees nothing and keeps no state.
 *   - Matrices are row-major; `ld*` is the row pitch in ELEMENTS (>= columns).
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and the call returns without synchronising.
 *   - Return value: SP_OK (0) or a negative sp_status.  Arguments are checked
 *     on the host before anything is launched; on error nothing was enqueued.
 *   - Keep mask format: uint32 words, `mask_words = (in + 31) / 32` per row,
 *     weight (r, q) is bit (q & 31) of word  r * mask_words + (q >> 5);
 *     1 = keep, 0 = prune; bits at q >= in are written as 0.
 */
#ifndef SWIFTPRUNE_H
#define SWIFTPRUNE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* storage type of X and W: IEEE binary32, bfloat16, IEEE binary16.  All arithmetic is fp32 (fp64 inside the
 * statistics sums) whatever the storage; a 16-bit element widens to fp32 exactly. */
typedef enum { SP_F32 = 0, SP_BF16 = 1, SP_F16 = 2 } sp_dtype;

typedef enum {
    SP_OK = 0,
    SP_EINVAL = -1, /* bad argument (null pointer, non-positive size, pitch < columns, unknown dtype or pattern, ...) */
    SP_ENOSPC = -2, /* workspace smaller than swiftprune_stats_workspace_bytes() */
    SP_EHIP = -3,   /* the HIP runtime refused a launch; hipGetLastError() has the code */
    SP_ERANGE = -4  /* swiftprune_calibrate_la: the target ratio is not reachable within the tolerance
                       (outputs hold the closest candidate found) */
} sp_status;

/* EWMA parameters of Algorithm 1.  alpha, beta in (0, 1];  la is the
 * threshold multiplier (the table of Sec. 3.1 maps pruning ratios of 50-90 %
 * to la).  The paper's only numeric alpha/beta is
 * 0.125 (Sec. 4.2).  If la is NaN it is looked up from `sparsity`. */
typedef struct {
    float alpha;
    float beta;
    float la;
} sp_ewma_params;

/* flags of the select entry points */
#define SP_SEQUENTIAL_ORDER 1u /* walk each row element by element in Algorithm 1's statement order, one
                                  rounding per operation, no fused multiply-add: reproduces a sequential
                                  fp32 evaluation bit for bit (slow; validation) */
#define SP_APPLY_INPLACE 2u    /* also zero the pruned weights of W in place (step 4 fused in) */

/*
 * Step 1 (Algorithm 1, first statement; Sec. 3.1 defines S as the sum of the squared activations).
 *
 *   X          [tokens, in], pitch ldx, dtype dt               (device, read)
 *   xsq        [in] fp32: accumulate == 0 -> overwritten with sum_t X[t,q]^2;
 *              accumulate != 0 -> that sum is ADDED to the values already there
 *              (so X may arrive in token chunks)              (device, read/write)
 *   S          [1] fp32, required: the total sum_q xsq[q]; overwritten when
 *              accumulate == 0, added to when accumulate != 0 (it must then hold
 *              what the previous chunk's call left)           (device, read/write)
 *   hr         [in] fp32, written only when finalize != 0 (may be NULL otherwise):
 *              hr[q] = 0.5 / (1 - xsq[q]/S), the per-channel factor of the score.
 *              S == 0 gives hr = 0.5; a denominator <= 0 is replaced by FLT_EPSILON.
 *   workspace  >= swiftprune_stats_workspace_bytes(tokens, in) bytes, 256-byte
 *              aligned, contents irrelevant on entry, clobbered (device)
 *
 * Per-lane sums run in fp32 over chains of at most 32 terms, are folded into
 * fp64 every 128 rows and combined in fp64 in a fixed order: xsq is within one
 * or two fp32 roundings of the exact sum and does not depend on scheduling.
 * S is the fp64 sum of the per-workgroup fp64 sums, rounded once.
 * Fast path: X 16-byte aligned, ldx and in multiples of 16 bytes worth of
 * elements; anything else takes an element-wise path with the same result.
 */
int swiftprune_layer_stats(const void *X, int64_t tokens, int64_t in, int64_t ldx, sp_dtype dt,
                           float *xsq, float *S, float *hr, int accumulate, int finalize,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * swiftprune_layer_stats for callers that cannot allocate device memory or have none to spare for a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, kernels and results as swiftprune_layer_stats, without `workspace`: the partial sums
 * live in a device array of SP_STATIC_WORKSPACE_BYTES that is part of the library's code object (every
 * GPU the library runs on holds its own copy until the process ends).  The call allocates and frees
 * nothing.  Shapes with swiftprune_stats_workspace_bytes(tokens, in) > SP_STATIC_WORKSPACE_BYTES are
 * refused with SP_ENOSPC (nothing is enqueued); all Llama / Pythia layer widths at 262144 tokens need
 * about 2 MB.  The device of `hip_stream` must be the current device.
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap (different streams
 * without an ordering between them, or host threads) race and give wrong sums; calls on one stream, or
 * otherwise ordered, are safe.  Nothing has to be cleared between calls.
 */
#define SP_STATIC_WORKSPACE_BYTES ((size_t)8 << 20)
int swiftprune_layer_stats_static(const void *X, int64_t tokens, int64_t in, int64_t ldx, sp_dtype dt,
                                  float *xsq, float *S, float *hr, int accumulate, int finalize,
                                  void *hip_stream);

/*
 * Step 1 from sums that the producer of X has formed itself (Algorithm 1, first statement: x_q^2 is a sum over
 * the calibration tokens, so it can be cut in pieces anywhere; Sec. 3.1: S and the score's denominator).  A kernel
 * that writes X (a GEMM or activation epilogue) adds up the squares of what it writes, per channel, over its own
 * piece of the tokens, and stores one fp32 row per piece; this call adds the pieces in fp64 and finishes the step.
 * Nothing of X is read, so the 2 bytes per activation that swiftprune_layer_stats streams are saved altogether.
 *   partials [parts, ld] fp32, row-major (device, read): partials[p*ld + q] = sum over the tokens of piece p of
 *            X[t,q]^2; parts >= 1 (at most 2^24), ld >= in; pieces may cover any numbers of tokens
 *   xsq      [in] fp32 (device): accumulate == 0: written; != 0: the pieces are added to what it holds
 *   S        [1]  fp32 (device, written): the sum over q of the xsq just written, formed in fp64 (with
 *            accumulate != 0 it is formed from the accumulated xsq; the old value is not read)
 *   hr       [in] fp32 (device): written when finalize != 0, as by swiftprune_layer_stats (same conventions for
 *            S == 0 and a non-positive denominator); may be NULL when finalize == 0
 * Two small launches on `hip_stream`; no workspace.  Errors: SP_EINVAL (null pointer, parts / in <= 0, ld < in,
 * misaligned pointer), SP_EHIP; nothing is enqueued on SP_EINVAL.
 */
int swiftprune_layer_stats_from_partials(const float *partials, int64_t parts, int64_t in, int64_t ld,
                                         float *xsq, float *S, float *hr, int accumulate, int finalize,
                                         void *hip_stream);

/*
 * The last part of step 1 on its own (denominator of the Sec. 3.1 score equation):
 *     hr[q] = 1/2 / (1 - xsq[q]/S),  with the conventions of swiftprune_layer_stats for S == 0 and a
 *     non-positive denominator.
 * For callers that add up xsq and S themselves - token shards reduced on several devices (each shard from
 * swiftprune_layer_stats with finalize == 0), or statistics kept from an earlier run.
 *   xsq [in], S [1], hr [in] fp32 (device; xsq and S read, hr written; hr may alias xsq)
 */
int swiftprune_channel_factor(const float *xsq, const float *S, int64_t in, float *hr, void *hip_stream);

/*
 * Steps 2+3, unstructured (Sec. 3.1 score equation; Sec. 3.2; Algorithm 1 loop body).
 * Per row, q ascending, state est = L_0, dev = 0:
 *     prune (r,q)  iff  L < est - la*dev      (state before q, strict)
 *     est <- (1-alpha) est + alpha L ;  dev <- (1-beta) dev + beta |est - L|   (updated est)
 * The sum S is held fixed during the walk (the paper's "S - w_i^2" update is
 * below fp32 resolution of S for calibration sums).
 *
 *   W           [out, in], pitch ldw, dtype dt  (device; read, and written when SP_APPLY_INPLACE)
 *   hr          [in] fp32 from swiftprune_layer_stats             (device, read)
 *   sparsity    target pruning ratio; only used to look up la when params->la is NaN
 *   params      host pointer; NULL = {0.125, 0.125, la from sparsity}
 *   keep_mask   [out, (in+31)/32] uint32, fully overwritten        (device, write)
 *   row_pruned  nullable [out] int32: number pruned in each row    (device, write)
 *   scores      nullable [out, in] fp32: L, for validation         (device, write)
 *   flags       SP_SEQUENTIAL_ORDER | SP_APPLY_INPLACE
 *
 * Default (scan) path: est/dev are evaluated as wavefront-wide linear-recurrence
 * scans; they differ from a sequential fp32 walk by a few ulp, so a decision
 * can differ only where L is within rounding of its threshold.
 * Scores are assumed finite and inside fp32's normal range: a NaN or infinite
 * score (a non-finite weight, or w*w overflowing) enters est and dev, after
 * which the decisions of the rest of that row are unspecified; other rows are
 * not affected.  No error is reported for it.
 */
int swiftprune_score_select(const void *W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                            const float *hr, float sparsity, const sp_ewma_params *params,
                            uint32_t *keep_mask, int32_t *row_pruned, float *scores,
                            uint32_t flags, void *hip_stream);

/*
 * Several weight matrices that multiply the SAME layer input (q / k / v of an attention block, gate / up
 * of an MLP) share the calibration statistics: Algorithm 1 forms S and the x_q^2 once from the input X,
 * so one swiftprune_layer_stats call serves all of them.  The two calls below prune such a group in one
 * launch: the rows of all matrices are spread over one grid, which also keeps a short matrix (1024
 * rows) from occupying the device alone.  Results are identical to calling swiftprune_score_select /
 * swiftprune_nm_select once per matrix with the same hr.
 *
 *   mats     host array of n_mats (1 .. SP_MAX_GROUP) descriptors; every matrix has `in` columns and
 *            dtype dt; W, keep_mask, row_pruned are device pointers as in the single-matrix calls
 *   others   as in swiftprune_score_select / swiftprune_nm_select (no scores output)
 * Matrices that miss the fast layout (16-byte alignment, in % 8) or flags / parameters that need the
 * general kernels (SP_SEQUENTIAL_ORDER, alpha == 1) are handled by one launch per matrix instead.
 * SP_EINVAL if any descriptor is invalid; nothing is enqueued then.
 */
typedef struct {
    void *W;              /* [out, in], pitch ldw */
    int64_t out;
    int64_t ldw;
    uint32_t *keep_mask;  /* [out, (in+31)/32], fully overwritten */
    int32_t *row_pruned;  /* nullable [out]; not used by the N:M call */
} sp_matrix;
#define SP_MAX_GROUP 8

int swiftprune_score_select_group(const sp_matrix *mats, int n_mats, int64_t in, sp_dtype dt,
                                  const float *hr, float sparsity, const sp_ewma_params *params,
                                  uint32_t flags, void *hip_stream);
int swiftprune_nm_select_group(const sp_matrix *mats, int n_mats, int64_t in, sp_dtype dt,
                               const float *hr, int n_keep, int m_group, uint32_t flags,
                               void *hip_stream);

/*
 * Threshold tuning (Sec. 3.1: the ratio -> la table covers 50..90 % only, and la is described as the
 * knob that sets the level of sparsity).  With S fixed, est and dev do not depend on la, so one pass over W
 * counts the pruned weights for several candidate la at once.
 *
 *   la       host array of n_la (1..16) finite candidates
 *   counts   [n_la] uint64, overwritten: counts[i] = number of weights of the whole matrix with
 *            L < est - la[i]*dev (scan evaluation, as in swiftprune_score_select)   (device, write)
 * Asynchronous on hip_stream like the other entry points.
 */
int swiftprune_count_pruned(const void *W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                            const float *hr, float alpha, float beta, const float *la, int n_la,
                            unsigned long long *counts, void *hip_stream);

/*
 * Searches la in [la_lo, la_hi] so that the pruned fraction of W is within `tolerance` of
 * `target_sparsity` (the fraction is non-increasing in la): up to 8 passes of 16 equally spaced
 * candidates, each pass one counting launch and one 128-byte copy to the host.
 * UNLIKE the other entry points this call SYNCHRONISES hip_stream before it returns.
 *
 *   counts_ws  device scratch, >= 16 uint64 (128 bytes), 8-byte aligned
 *   la, achieved   host out-arguments: the chosen la and the pruned fraction it gives
 * Returns SP_OK, or SP_ERANGE when no candidate came within the tolerance (outputs = the closest).
 */
int swiftprune_calibrate_la(const void *W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                            const float *hr, float alpha, float beta, float target_sparsity,
                            float tolerance, float la_lo, float la_hi, unsigned long long *counts_ws,
                            float *la, float *achieved, void *hip_stream);

/*
 * The same tuning without the host in the loop (Sec. 3.1 leaves la for ratios outside its table to tuning;
 * the appendix reports 10-40 % without their la).  With S fixed every weight has a critical multiplier
 *     lambda = (est_before - L) / dev_before     (+inf / -inf when dev_before == 0),
 * it is pruned exactly when la < lambda, so the la that prunes k weights is the (k+1)-th largest lambda:
 * a three-pass radix select over W, entirely on hip_stream, no synchronisation, no copy to the host.
 *
 *   target_sparsity  in (0, 1): k = round(target_sparsity * out * in)
 *   workspace        device scratch, >= swiftprune_la_workspace_bytes(), 256-byte aligned
 *   la_device        [1] fp32 (device, write): the multiplier; pass it to swiftprune_score_select_la
 *   pruned_device    nullable [1] uint64 (device, write): weights with lambda > la (= k unless lambdas tie)
 *   status_device    nullable [1] int32 (device, write): 0, or 1 when rank k falls among weights that are
 *                    pruned for every la or for none (la is then +-3e38)
 * est/dev are the scan evaluation of swiftprune_score_select's default path; the pruned count that call
 * then produces can differ from k by the few weights whose score lies within rounding of its threshold.
 */
size_t swiftprune_la_workspace_bytes(void);
int swiftprune_calibrate_la_device(const void *W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                                   const float *hr, float alpha, float beta, float target_sparsity,
                                   void *workspace, size_t workspace_bytes, float *la_device,
                                   unsigned long long *pruned_device, int *status_device, void *hip_stream);

/*
 * swiftprune_score_select (default path) with la taken from device memory when the kernel runs, so that a
 * multiplier calibrated on the same stream is used without a round trip to the host.
 * flags: SP_APPLY_INPLACE.  Other arguments as for swiftprune_score_select.
 */
int swiftprune_score_select_la(const void *W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                               const float *hr, float alpha, float beta, const float *la_device,
                               uint32_t *keep_mask, int32_t *row_pruned, uint32_t flags, void *hip_stream);

/*
 * Exact comparator (Sec. 3.1: order a row's scores and drop the lowest ones - the O(n log n) rule
 * the EWMA walk replaces).  In every row the k smallest scores are
 * pruned, equal scores in index order; k = k_per_row[r] when k_per_row != NULL (device, int32[out]),
 * else k_uniform; k is clamped to [0, in].  Implemented as a per-row radix select, no sort.
 * keep_mask as above; flags: SP_APPLY_INPLACE.  NaN scores rank above every number.
 */
int swiftprune_topk_select(const void *W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                           const float *hr, const int32_t *k_per_row, int64_t k_uniform,
                           uint32_t *keep_mask, uint32_t flags, void *hip_stream);

/*
 * Steps 2+3, structured N:M (Sec. 3.3): in every group of m_group consecutive
 * inputs of a row keep the n_keep entries of highest score and prune the rest;
 * among equal scores the lower index is pruned first.  Supported: m_group in
 * {4, 8, 16}, 0 < n_keep < m_group, in % m_group == 0 (else SP_EINVAL).
 * Arguments as for swiftprune_score_select; flags: SP_APPLY_INPLACE.
 * Deterministic and order-free: with equal hr the mask is unique.  Scores are
 * assumed not to be NaN: a group that holds one is not guaranteed to keep
 * exactly n_keep entries.
 */
int swiftprune_nm_select(const void *W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                         const float *hr, int n_keep, int m_group,
                         uint32_t *keep_mask, float *scores, uint32_t flags, void *hip_stream);

/*
 * Step 4 (Algorithm 1: pruned w_i = 0, output C = W): W[r,q] <- +0 where the keep
 * bit is 0; kept weights are left bit for bit.  W is modified in place.
 */
int swiftprune_apply(void *W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                     const uint32_t *keep_mask, void *hip_stream);

/*
 * Compact storage of an N:M-pruned matrix (Sec. 3.3 motivates N:M by formats that store only the kept
 * values and their positions).  Open layout, not a vendor format:
 *   values [out, in/m_group*n_keep] in W's dtype: values[r, g*N + j] = j-th kept entry (ascending
 *          column) of group g of row r                                            (device, write)
 *   meta   [out, swiftprune_nm_meta_words(in, n_keep, m_group)] uint32: the position 0..M-1 of that
 *          entry inside its group as a field of b bits (b = 2 for M = 4, else 4); field number
 *          g*N + j of the row, packed little-endian (field f = bits [f*b mod 32, +b) of word f*b/32)
 * keep_mask should keep exactly n_keep entries per group (as swiftprune_nm_select produces): extra kept
 * entries beyond the first n_keep of a group are dropped; a group with fewer is padded with +0 at
 * position 0.  Patterns as for swiftprune_nm_select.
 */
int swiftprune_compact_nm(const void *W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                          const uint32_t *keep_mask, int n_keep, int m_group, void *values,
                          uint32_t *meta, void *hip_stream);

/* Inverse of swiftprune_compact_nm: W_out[out, in] (pitch ldw_out) gets the stored values at their
 * positions and +0 everywhere else. */
int swiftprune_expand_nm(const void *values, const uint32_t *meta, int64_t out, int64_t in, sp_dtype dt,
                         int n_keep, int m_group, void *W_out, int64_t ldw_out, void *hip_stream);

/*
 * Diagnostic: the est and dev sequences of the EWMA walk (Sec. 3.2; state-update table of Sec. 3.1; the
 * tracking figure of Sec. 4.2 plots them against the mean and the mean deviation of the scores).
 *
 *   est, dev   [out, in] fp32, row-major with pitch in: the state AFTER the update with element q;
 *              either may be null, not both                                      (device, write)
 *   alpha, beta in (0, 1].  la takes no part: the two sequences do not depend on it.
 * Evaluated with the same wavefront scans as swiftprune_score_select's default path, so the values
 * differ from a sequential fp32 walk by a few ulp.  Asynchronous on hip_stream.
 */
int swiftprune_ewma_trace(const void *W, int64_t out, int64_t in, int64_t ldw, sp_dtype dt,
                          const float *hr, float alpha, float beta, float *est, float *dev,
                          void *hip_stream);

/*
 * Launch-shape overrides for measurements.  The kernels' launch shapes (rows in flight and workgroups of
 * the statistics kernel, wavefronts per row of the EWMA kernel, workgroups of the N:M / apply kernels) were
 * chosen from sweeps on MI355X.  Three environment variables, read at every call, replace them so that the
 * sweeps can be repeated; they change how the work is cut, never the results.  Malformed values are ignored.
 *   SWIFTPRUNE_STATS_PLAN  = "<rows in flight: 4|8|16>,<workgroups 1..4096>[,plain]"
 *                            (plain = ordinary instead of non-temporal loads, bf16 vector path only;
 *                            swiftprune_stats_workspace_bytes follows the override)
 *   SWIFTPRUNE_SELECT_TEAM = "<0|1|2|4>[,direct]"  (wavefronts per row, 0 = built-in choice; direct = every span
 *                            loads its weights and channel factors from global memory and waits for them,
 *                            instead of factors staged in LDS and weights requested one span ahead)
 *   SWIFTPRUNE_BAND_GROUPS = "<apply workgroups>,<N:M select workgroups>" (1..4096 each)
 */

/* ---- host helpers (no device work) ---- */

/* uint32 words of meta per row for swiftprune_compact_nm (0 on an unsupported pattern). */
size_t swiftprune_nm_meta_words(int64_t in, int n_keep, int m_group);


/* la for a pruning ratio from the paper's table (0.9 -> -1.5, 0.8 -> -0.9, 0.7 -> -0.2,
 * 0.6 -> 0.2, 0.5 -> 0.5), piecewise linear between entries.  SP_EINVAL outside [0.5, 0.9]. */
int swiftprune_la_for_sparsity(float sparsity, float *la);

/* Bytes of workspace swiftprune_layer_stats needs for this shape (0 on bad arguments). */
size_t swiftprune_stats_workspace_bytes(int64_t tokens, int64_t in);

/* Static description of a status code. */
const char *swiftprune_strerror(int code);

/* Library version, "major.minor.patch". */
const char *swiftprune_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SWIFTPRUNE_H */

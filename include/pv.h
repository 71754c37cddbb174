/*
 * pv.h -- C ABI of the MI355X (gfx950) library for the discrete-code update of
 * PV-Tuning (arXiv 2405.14852): the linearised subspace V step.
 *
 * One V step on one weight matrix is
 *     W  = pv_dequantize(codes)                       Alg. 3, line 1
 *     T  = pv_encode_targets(W, G, alpha)             Eq. 7; Alg. 3, V step
 *     S  = pv_select_topk_groups(T, W, k)             Alg. 2, line 5; Sec. 3.4
 *     codes[S] = pv_reencode_groups(T, S)             Eq. 7 argmin; Sec. 4.2; App. D, K
 * Further calls: pv_encode_targets_select (lines 2 and 3 in one sweep),
 * pv_encode_targets_adam[_select] (Sec. 3.4: an Adam update as the direction),
 * pv_reencode_trust_ratio (Sec. 4.3: the subspace size from the trust ratio),
 * pv_codebook_grads (Alg. 3 P step: gradients of codebooks and scales),
 * pv_dequantize_groups (dequantisation of the re-encoded groups only),
 * pv_select_topk_groups_noalloc (the selection for callers that cannot allocate),
 * pv_dequantize_scalar / pv_reencode_scalar (App. K's scalar uniform-grid representation).
 * Instrumentation: pv_set_search_mode, pv_timing_*, pv_reencode_stats, and the two ceiling
 * probes pv_probe_copy / pv_probe_mfma_f16.
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE pointers on the context's GPU, owned by the
 *     caller, 16-byte aligned, row-major, dense.  The library neither allocates
 *     nor frees caller-visible memory.  The context owns its scratch memory,
 *     grown on demand and released by pv_destroy.
 *   - A weight matrix is [out_features, in_features].  A group is group_size
 *     consecutive weights of one row (along the input dimension, App. K).  Groups
 *     are numbered row by row: n = o * (in_features / group_size) + j;
 *     N = number of groups must be < 2^31.
 *   - Calls enqueue work on the context's HIP stream and return without waiting;
 *     results are ordered by that stream.  One context per host thread.  The one
 *     exception: when a call needs more scratch memory than the context holds (the
 *     first call of a shape, or a larger k), it waits for the stream, frees the old
 *     block and allocates a larger one before it enqueues anything; calls of a shape
 *     the context has seen before never wait, allocate or free.
 *   - Graph capture: once a call of the same shape has sized the scratch, the calls of
 *     a step (dequantize, targets, selection, re-encode and their variants) only launch
 *     kernels on the context's stream, so a caller may capture them into a HIP graph and
 *     replay it; the inputs may change in place between replays (a codebook rewritten by
 *     the P step).  pv_reencode_stats, pv_timing_read and pv_destroy synchronise and do
 *     not belong into a capture.
 *   - Errors are reported by the return code only; on an error nothing has been
 *     enqueued or written.  pv_last_error gives a short text for the last error
 *     of a context.
 */
#ifndef PV_H
#define PV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pv_ctx pv_ctx; /* opaque */

typedef enum {
    PV_OK = 0,
    PV_ERR_INVALID_ARG = 1, /* NULL pointer, k out of range, beam_width < 1, ...     */
    PV_ERR_SHAPE = 2,       /* in_features % group_size != 0, N >= 2^31, B not in 1..16 */
    PV_ERR_UNSUPPORTED = 3, /* a legal shape this build has no kernel for           */
    PV_ERR_ALLOC = 4,       /* scratch allocation failed                            */
    PV_ERR_DEVICE = 5       /* a HIP call failed                                    */
} pv_status;

typedef struct {
    int64_t out_features;  /* rows of W                                        */
    int64_t in_features;   /* columns of W; multiple of group_size             */
    int32_t group_size;    /* g >= 1                                           */
    int32_t num_codebooks; /* M in 1..8 (additive codebooks)                   */
    int32_t nbits;         /* B in 1..16; each codebook holds 2^B codewords    */
} pv_layout;

/* Create a context bound to HIP device `device`; work is enqueued on
 * `hip_stream` (a hipStream_t; NULL = the device's default stream). */
pv_status pv_create(pv_ctx **out, int device, void *hip_stream);
void pv_destroy(pv_ctx *ctx);
const char *pv_last_error(const pv_ctx *ctx);

/* Eq. 7 / Alg. 3 V step: the target of the linearised subspace V step,
 * T = W - alpha * G elementwise (alpha plays 1/L_S; G is the gradient or the
 * Adam direction, the caller's choice), one fp32 rounding per element.
 * W, G, T: f32 [out_features, in_features].  T may alias W or G exactly
 * (same pointer) but must not partially overlap them. */
pv_status pv_encode_targets(pv_ctx *ctx, const pv_layout *layout, const float *W,
                            const float *G, float alpha, float *T);

/* Sec. 3.4: Eq. 7 with the gradient replaced by a single Adam update (Kingma & Ba's rule
 * with bias correction; App. K uses beta1 = 0.9, beta2 = 0.95):
 *     m <- beta1 m + (1 - beta1) G,   v <- beta2 v + (1 - beta2) G^2     (in place)
 *     T  = W - lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 * elementwise in fp32: m' = fma(beta1, m, (1-beta1)*G), v' = fma(beta2, v, (1-beta2)*(G*G)),
 * two divisions by the bias corrections (formed in double, rounded to fp32 once), a correctly
 * rounded square root and division, T = fma(-lr, update, W).  step >= 1 counts the updates.
 * W, G, T and the moments m, v: f32 [out_features, in_features]; T may alias W or G exactly;
 * T, m, v must be distinct.  Selecting on ||T - W|| afterwards ranks groups by the size of
 * their Adam update, as Sec. 3.4 prescribes. */
pv_status pv_encode_targets_adam(pv_ctx *ctx, const pv_layout *layout, const float *W,
                                 const float *G, float *m, float *v, int64_t step, float lr,
                                 float beta1, float beta2, float eps, float *T);

/* Alg. 2 line 5 ("arg top tau") with Sec. 3.4's rule (largest update norm, per
 * weight matrix), applied to weight groups: score_n = sum_i (T[n,i] - W[n,i])^2
 * accumulated in fp32 in index order with fused multiply-adds; the k groups with
 * the largest score are returned as ASCENDING flat group ids in out_idx[k]
 * (i32).  Equal scores: the lower id is preferred.  0 <= k <= N; k == 0 writes
 * nothing.  group_scores: optional f32 [N], receives every group's score. */
pv_status pv_select_topk_groups(pv_ctx *ctx, const pv_layout *layout, const float *T,
                                const float *W, int64_t k, int32_t *out_idx,
                                float *group_scores /* NULL ok */);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation): pv_select_topk_groups with the same
 * arguments and the same results, whose scratch (group scores when group_scores is NULL,
 * radix-select histograms, per-chunk counts) lives in one static device array of about
 * 16.1 MiB that every GPU the library runs on holds until the process ends.  It calls no
 * allocation or release routine of any kind, creates no events (timing brackets are off for
 * this call) and enqueues only kernels.  Limit: N <= 4 194 304 groups, else
 * PV_ERR_UNSUPPORTED.  All calls on one GPU share the array: calls that overlap on one GPU
 * (two streams, two contexts) race; calls ordered by one stream are safe. */
pv_status pv_select_topk_groups_noalloc(pv_ctx *ctx, const pv_layout *layout, const float *T,
                                        const float *W, int64_t k, int32_t *out_idx,
                                        float *group_scores /* NULL ok */);

/* pv_encode_targets followed by pv_select_topk_groups, as one sweep over memory
 * (Eq. 7 feeding Alg. 2 line 5): T is written and every group's score is taken
 * from the registers that hold T and W, so neither is read back.  Outputs (T,
 * out_idx, group_scores) are bit-identical to the two calls in sequence.
 * T may alias G exactly; it must not alias W.  k == 0 still writes T (and
 * group_scores when given). */
pv_status pv_encode_targets_select(pv_ctx *ctx, const pv_layout *layout, const float *W,
                                   const float *G, float alpha, float *T, int64_t k,
                                   int32_t *out_idx, float *group_scores);

/* pv_encode_targets_adam followed by pv_select_topk_groups as one sweep (Sec. 3.4: the
 * subspace is chosen by the size of the Adam update): m, v and T are written, the scores come
 * from the registers that hold T and W.  Outputs are bit-identical to the two calls in
 * sequence.  T may alias G exactly; T, W, m, v must be distinct. */
pv_status pv_encode_targets_adam_select(pv_ctx *ctx, const pv_layout *layout, const float *W,
                                        const float *G, float *m, float *v, int64_t step, float lr,
                                        float beta1, float beta2, float eps, float *T, int64_t k,
                                        int32_t *out_idx, float *group_scores /* NULL ok */);

/* Eq. 7 argmin restricted to the listed groups (Alg. 3 last line, "find_nearest"):
 * for each listed group with target t (g values of T), row scale s and current
 * code tuple p, minimise  obj(b) = || s * sum_m codebooks[m, b_m, :] - t ||^2
 * (double precision on the fp32 inputs).
 *   M == 1: exact nearest codeword over all 2^B codewords ("try every code",
 *           App. K).  Exact ties: p if p is a minimiser, else the lowest index.
 *           beam_width is ignored.
 *   M >= 2: beam search (Sec. 4.2, App. D, App. K): the beam starts as {p}; for
 *           m = 0..M-1 every beam entry spawns 2^B candidates (its m-th code
 *           replaced), candidates are ranked by (obj, tuple lexicographic) and
 *           the best beam_width kept; the final best replaces p only if it is
 *           strictly better.
 * codes: u16 [out_features, in_features/g, M], updated in place for the listed
 * groups only; all other codes are left untouched.  group_idx: i32 [k],
 * ascending, unique, each in [0, N) (ids outside the range are skipped).
 * scales: f32 [out_features]; a zero scale keeps the previous code.
 * num_changed: optional device int64, receives the number of groups whose code
 * tuple changed.
 * A stored code is read modulo 2^B (its low B bits): bits above B are ignored in the
 * search and in num_changed, and stay as they are in a group whose code is kept (a group
 * that changes is written with a clean B-bit code).
 * Limits (PV_ERR_UNSUPPORTED): group_size <= 64; for M >= 2 also beam_width <= 64 and
 * beam_width * 2^B <= 4096 (the candidate pool of one beam step lives in LDS). */
pv_status pv_reencode_groups(pv_ctx *ctx, const pv_layout *layout, const float *T,
                             const float *codebooks /* f32 [M, 2^B, g] */,
                             const float *scales /* f32 [out_features] */,
                             const int32_t *group_idx, int64_t k, int32_t beam_width,
                             uint16_t *codes, int64_t *num_changed /* NULL ok */);

/* Stochastic rounding of the listed groups (App. F: the K-nearest approximation for vector
 * quantisation, K = 2; App. K: temperature 0.2, i.e. power = 5), the baseline the paper
 * compares the V step with.  For each listed group n with target t and row scale s:
 *   - the two codewords with the smallest obj(c) = || s * codebook[c, :] - t ||^2 (double
 *     precision on the fp32 inputs, equal objectives in index order) are found: c_1 with
 *     d_1 = sqrt(obj(c_1)) and c_2 with d_2 >= d_1 - by the matrix-core filter of
 *     pv_reencode_groups with its certificate taken from the second nearest where that filter
 *     applies (g = 8 or 16, B >= 5, search mode 0), else by a scan of all 2^B codewords; both
 *     give the same pair;
 *   - p = 1 / (1 + (d_1 / d_2)^power), i.e. probabilities proportional to distance^-power
 *     (power = 1: the formula of App. F); d_1 = 0 gives p = 1;
 *   - u = (bits >> 11) * 2^-53 with bits the SplitMix64 output function applied to
 *     seed + (n + 1) * 0x9E3779B97F4A7C15 (a function of seed and group id only, so the result
 *     does not depend on the order or partition of the list);
 *   - the code becomes c_1 if u < p, else c_2.
 * One codebook only (PV_ERR_UNSUPPORTED for M >= 2; App. F speaks of one codebook or lattice);
 * group_size <= 64; 1 <= power <= 64.  Pointers, layouts, the treatment of ids outside [0, N),
 * of unlisted groups, of stored bits above B and of num_changed are those of
 * pv_reencode_groups.  The straight-through buffer of App. E needs no call of its own:
 * pv_encode_targets with T aliasing W keeps the buffer, pv_reencode_groups (all groups, or
 * those pv_select_topk_groups picks against the dequantised weights) projects it. */
pv_status pv_reencode_groups_stochastic(pv_ctx *ctx, const pv_layout *layout, const float *T,
                                        const float *codebooks /* f32 [1, 2^B, g] */,
                                        const float *scales /* f32 [out_features] */,
                                        const int32_t *group_idx, int64_t k, int32_t power,
                                        uint64_t seed, uint16_t *codes,
                                        int64_t *num_changed /* NULL ok */);

/* Subspace size from the trust ratio (Sec. 4.3; App. K, hyperparameter paragraph):
 * tau is not given but found, as the largest number of weights whose update keeps
 *     || x^{k+1} - x^k || / || x^k ||  <  ratio          (the paper uses 0.01)
 * where x is this matrix' dequantised weights.  Candidates are the k_max groups of
 * pv_select_topk_groups(T, W, k_max), ranked by that rule (largest update norm
 * first, lower id first).  The paper applies them `chunk` groups at a time and
 * undoes the tail of the chunk that broke the bound; the result is the longest
 * ranked prefix that satisfies it, and at least one group whose code moves is kept
 * (if it lies in the chunk at which the procedure stops).  The comparison is done
 * on squares in double: sum over kept groups of sum_i (w_new - w_old)^2 <
 * ratio^2 * sum x^2, with w the fp32 weights of pv_dequantize.
 * codes: in/out, re-encoded (as by pv_reencode_groups) for the kept groups only.
 * rank_idx: optional i32 [k_max], receives the candidates in rank order (the kept
 * ones are its first *num_applied entries).  num_applied: device int64.
 * stats: optional device f64 [2] = {squared change of the kept groups, ||x^k||^2}. */
pv_status pv_reencode_trust_ratio(pv_ctx *ctx, const pv_layout *layout, const float *T,
                                  const float *W, const float *codebooks, const float *scales,
                                  int64_t k_max, int64_t chunk, double ratio, int32_t beam_width,
                                  uint16_t *codes, int32_t *rank_idx /* NULL ok */,
                                  int64_t *num_applied, double *stats /* NULL ok */);

/* Alg. 3 line 1: W_out[o, j*g + i] = scales[o] * sum_m codebooks[m, codes[o,j,m], i]
 * with fp32 additions in codebook order and one fp32 multiply.  Codes are
 * masked to B bits. */
pv_status pv_dequantize(pv_ctx *ctx, const pv_layout *layout, const uint16_t *codes,
                        const float *codebooks, const float *scales, float *W_out);

/* pv_dequantize restricted to the listed groups (Alg. 3 line 1 after a V step that changed
 * only those): W_out[o, j*g .. j*g+g) is rewritten for each listed flat group id, every other
 * weight of W_out is left as it is.  If W_out held pv_dequantize of the codes before the V
 * step and group_idx is the list the step re-encoded, the result equals pv_dequantize of the
 * new codes.  group_idx: i32 [k], ids outside [0, N) are skipped. */
pv_status pv_dequantize_groups(pv_ctx *ctx, const pv_layout *layout, const uint16_t *codes,
                               const float *codebooks, const float *scales,
                               const int32_t *group_idx, int64_t k, float *W_out);

/* P step (Alg. 3, "grad_codebooks = backprop(grad_phi)"; App. K: codebooks and per-channel
 * scales are trained by backprop): the chain rule through pv_dequantize applied to
 * G = d phi / d W (f32 [out_features, in_features]):
 *   grad_codebooks[m, c, i] = sum over groups n = (o, j) with codes[o,j,m] == c of
 *                             scales[o] * G[o, j*g + i]                  f32 [M, 2^B, g]
 *   grad_scales[o]          = sum_j sum_i G[o, j*g + i] * (sum_m codebooks[m, codes[o,j,m], i])
 *                                                                        f32 [out_features], optional
 * Products are exact in double and every result is rounded to fp32 once.  Two routes, both a
 * function of the inputs only (a second call returns the same bits):
 *   - the table of M * 2^B * g sums does not fit one block's LDS as 8-byte entries (64 KiB), or
 *     fewer than 64 groups share a codeword on average: the groups are sorted by code and a
 *     codeword's sum runs over its groups in ascending order, in double - equal to a
 *     sequential loop - unless more than 128 groups share the codeword, in which case pieces
 *     of 128 are summed that way and added in order;
 *   - else (small codebooks): the terms are added in 64-bit fixed point scaled by a power of
 *     two taken from max|scales| * max|G|, exact up to 2^-39 of that product per term, in
 *     any order; if a gradient or a scale is not finite every entry of grad_codebooks is NaN.
 * A row's scale gradient is a tree sum in double.  Unused codewords get exactly 0.  Nothing
 * is accumulated into the outputs: they are overwritten.  G and codebooks must be 16-byte
 * aligned. */
pv_status pv_codebook_grads(pv_ctx *ctx, const pv_layout *layout, const float *G,
                            const uint16_t *codes, const float *codebooks, const float *scales,
                            float *grad_codebooks, float *grad_scales /* NULL ok */);

/* ---- the scalar representation of App. K ("GPTQ": uniform grid, block-wise scale and zero
 *      point): W[o, i] = scales[o, i/block] * (codes[o, i] - zeros[o, i/block]),
 *      codes u8 [out_features, in_features] with values in [0, 2^nbits), nbits <= 8,
 *      scales and zeros f32 [out_features, in_features / block_size].
 *      Targets and selection are the calls above with group_size = 1 (the unit is a weight). */

/* fp32: one subtraction, one multiplication per weight. */
pv_status pv_dequantize_scalar(pv_ctx *ctx, int64_t out_features, int64_t in_features,
                               int32_t block_size, int32_t nbits, const uint8_t *codes,
                               const float *scales, const float *zeros, float *W_out);

/* V step on that representation (App. K: rounding to the nearest scaled integer): for each
 * listed weight (flat ids, ascending, as pv_select_topk_groups returns them for group_size 1)
 * the grid value nearest to T, i.e. the q minimising (w_q - t)^2 in double with w_q the fp32
 * dequantised value; ties: the previous code if it is a minimiser, else the lowest q.
 * codes is updated in place for the listed weights only.  num_changed: optional device int64. */
pv_status pv_reencode_scalar(pv_ctx *ctx, int64_t out_features, int64_t in_features,
                             int32_t block_size, int32_t nbits, const float *T, const float *scales,
                             const float *zeros, const int32_t *weight_idx, int64_t k,
                             uint8_t *codes, int64_t *num_changed /* NULL ok */);

/* ---- instrumentation (does not change results) ------------------------- */

/* Search strategy: 0 = automatic (a matrix-core filter with exact certificates
 * where the shape allows: one codebook with g = 8 or 16, or two 8-bit codebooks
 * with g = 8 or 16 and beam <= 8; else the exact kernels), 1 = exact kernels only. */
pv_status pv_set_search_mode(pv_ctx *ctx, int mode);

typedef enum {
    PV_K_ENCODE_TARGETS = 0,
    PV_K_GROUP_SCORES = 1,
    PV_K_SELECT = 2,      /* all kernels of the radix select + compaction   */
    PV_K_PREP = 3,        /* codebook + target preparation for the filter   */
    PV_K_SCORE_MFMA = 4,  /* the distance contraction                       */
    PV_K_RERANK = 5,      /* exact re-rank + write-back                     */
    PV_K_EXACT_SCAN = 6,  /* exact scan (fallback list or whole call)       */
    PV_K_BEAM = 7,
    PV_K_DEQUANTIZE = 8,
    PV_K_TRUST_RATIO = 9, /* norms, ranking, prefix sums, roll-back of pv_reencode_trust_ratio */
    PV_K_PSTEP = 10,      /* all kernels of pv_codebook_grads                              */
    PV_K_PROBE_COPY = 11, /* pv_probe_copy                                                 */
    PV_K_PROBE_MFMA = 12, /* pv_probe_mfma_f16                                             */
    PV_K_STOCHASTIC = 13, /* pv_reencode_groups_stochastic                                 */
    PV_K_COUNT = 14
} pv_kernel_id;

/* With timing on, each kernel (group) above is bracketed by HIP events on the
 * context's stream; pv_timing_read waits for the stream and returns the sum of
 * durations in milliseconds and the number of launches since the last reset. */
pv_status pv_timing_enable(pv_ctx *ctx, int on);
pv_status pv_timing_reset(pv_ctx *ctx);
pv_status pv_timing_read(pv_ctx *ctx, int kernel_id, double *total_ms, int64_t *launches);

/* Machine ceilings measured with two kernels of this library, for callers that want to
 * relate a measured rate to what the same box reaches at that moment (bench.py reports
 * them beside the published peaks).  Both enqueue on the context's stream and are timed
 * like every other kernel (PV_K_PROBE_COPY, PV_K_PROBE_MFMA).
 * pv_probe_copy: dst[0 .. bytes) = src[0 .. bytes), device pointers, 16-byte aligned,
 * bytes a multiple of 16, non-overlapping: one streaming pass, 2 * bytes of HBM traffic.
 * pv_probe_mfma_f16: every wave of a grid that fills the chip (4 waves per SIMD) issues
 * `iters` independent v_mfma_f32_32x32x16_f16 (2 * 32 * 32 * 16 FLOP each) and nothing else;
 * sink: f32 [256 * 16 * 64] device buffer that receives the accumulators (so that the work
 * cannot be removed); *waves_out (host pointer, NULL ok) = number of waves launched. */
pv_status pv_probe_copy(pv_ctx *ctx, void *dst, const void *src, int64_t bytes);
pv_status pv_probe_mfma_f16(pv_ctx *ctx, int64_t iters, float *sink, int64_t *waves_out);

/* Counters of the last pv_reencode_groups call (waits for the stream):
 * stats[0] = groups decided by a matrix-core filter (one codebook: the fp16
 * contraction; two 8-bit codebooks: the fp64 beam filter), stats[1] = groups the
 * filter could not certify and that were re-done by the exact scan / exact beam
 * kernel, stats[2] = candidate codewords evaluated exactly in the re-rank (one
 * codebook), stats[3] = groups handled by exact scan / beam search from the start. */
pv_status pv_reencode_stats(pv_ctx *ctx, int64_t stats[4]);

#ifdef __cplusplus
}
#endif
#endif /* PV_H */

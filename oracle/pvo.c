/*
 * CPU oracle for the V-step re-encoding path of PV-Tuning (arXiv 2405.14852).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
 * statement of what the GPU path must compute.  It shares no code with the
 * HIP library and must never be called from the product path: only tests,
 * the smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * What follows the paper exactly, and what is a stated reading of it:
 *   pvo_encode_targets      Eq. 7 (linearised subspace V step): the target is
 *                           y - (1/L) * grad, with alpha = 1/L; Alg. 3 V step.
 *   pvo_encode_targets_adam Sec. 3.4: the same target with the gradient replaced by one
 *                           Adam update (pinned by exact rational arithmetic, a library
 *                           optimiser, the first-step closed form).
 *   pvo_select_topk_groups  Alg. 2 "arg top tau" + Sec. 3.4: largest update
 *                           norm, greedily per weight matrix.  Reading: the
 *                           unit is a weight group (one code covers it).
 *   pvo_reencode_groups     M = 1: the argmin of Eq. 7 restricted to one group,
 *                           i.e. "try every code, keep the minimiser" (App. K,
 *                           VQ) -- a plain definition (pinned by brute force,
 *                           the App. P worked example, nearest-neighbour
 *                           library routines, Lemma 3.1).
 *                           M >= 2: beam search over the codebooks (Sec. 4.2,
 *                           App. K "beam size 8", App. D local search extended
 *                           to beam search) -- a heuristic; the paper gives no
 *                           listing, so the reading is: seed the beam with the
 *                           current codes, visit codebooks in index order once,
 *                           score every replacement with the full objective,
 *                           keep the best `beam_width`.  Pinned only by: equals
 *                           brute force when the beam is wide enough, never
 *                           worse than the previous code (Lemma 3.2), reduces
 *                           to the M = 1 definition, beam 1 = one pass of greedy
 *                           single-index descent (App. D).  Beyond those bounds
 *                           the beam result is PARITY UNPINNED.
 *   pvo_reencode_stochastic App. F: the K = 2 nearest-codeword approximation of stochastic
 *                           rounding, probabilities proportional to distance^-power (App. K:
 *                           temperature 0.2, power 5); the variates come from a counter-based
 *                           generator defined here (pinned by the exact probabilities of a
 *                           two-point grid, the unbiasedness of the scalar case, App. F's
 *                           biased counter-example, brute force on the two nearest and the
 *                           reference output of the generator's published test vector).
 *   pvo_dequantize          Alg. 3 line 1: W = scale_row * sum_m codeword_m.
 *   pvo_dequantize_scalar / pvo_reencode_scalar  App. K's scalar representation (uniform grid,
 *                           block-wise scale and zero point): the V step is rounding to the
 *                           nearest grid value, written as a search over all values (pinned
 *                           by the closed-form rounding and a sorted-grid bisection).
 *   pvo_codebook_grads      Alg. 3 P step: chain rule through the dequantiser (pinned by
 *                           automatic differentiation of an independent dequantiser and by
 *                           finite differences of a quadratic loss).
 *   pvo_reencode_trust_ratio  Sec. 4.3 / App. K: subspace size from the trust ratio,
 *                           the chunked procedure of App. K step by step (pinned by
 *                           brute force over all prefix lengths, a closed-form case,
 *                           independence of the chunk size and the limits ratio = 0 / inf).
 *
 * Arithmetic: objectives in IEEE double on the fp32 inputs, evaluated in index
 * order without contraction (compile with -ffp-contract=off).  The selection
 * score and the dequantised weights are fixed fp32 chains so that they are
 * reproducible bit for bit.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define PVO_OK 0
#define PVO_ERR 1

#define PVO_NEAR_TIE_REL 1e-6

/* ------------------------------------------------------------------ targets */

/* T = W - alpha * G, one rounding per element (Eq. 7 with 1/L_S = alpha). */
int pvo_encode_targets(int64_t out_features, int64_t in_features, const float *W,
                       const float *G, float alpha, float *T)
{
    if (!W || !G || !T || out_features < 0 || in_features < 0) return PVO_ERR;
    int64_t n = out_features * in_features;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) T[i] = fmaf(-alpha, G[i], W[i]);
    return PVO_OK;
}

/* beta^t in double by repeated squaring (a fixed sequence of IEEE multiplications) */
static double powi(double b, int64_t t)
{
    double r = 1.0;
    while (t > 0) {
        if (t & 1) r = r * b;
        b = b * b;
        t >>= 1;
    }
    return r;
}

/* Sec. 3.4: the gradient of Eq. 7 is replaced by a single Adam update (Kingma & Ba's rule
 * with bias correction; App. K uses beta1 = 0.9, beta2 = 0.95):
 *     m <- beta1 m + (1 - beta1) g          v <- beta2 v + (1 - beta2) g^2
 *     T  = W - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)
 * All in fp32, one rounding per written operation below, so that the result is
 * reproducible bit for bit; the two bias corrections are formed in double and rounded to
 * fp32 once.  m and v are updated in place; t >= 1 is the number of this update. */
int pvo_encode_targets_adam(int64_t out_features, int64_t in_features, const float *W,
                            const float *G, float *m, float *v, int64_t t, float lr, float beta1,
                            float beta2, float eps, float *T)
{
    if (!W || !G || !m || !v || !T || out_features < 0 || in_features < 0 || t < 1) return PVO_ERR;
    const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
    const float c1 = (float)(1.0 - powi((double)beta1, t));
    const float c2 = (float)(1.0 - powi((double)beta2, t));
    int64_t n = out_features * in_features;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float g = G[i];
        float mi = fmaf(beta1, m[i], omb1 * g);
        float vi = fmaf(beta2, v[i], omb2 * (g * g));
        float mhat = mi / c1;
        float vhat = vi / c2;
        float upd = mhat / (sqrtf(vhat) + eps);
        m[i] = mi;
        v[i] = vi;
        T[i] = fmaf(-lr, upd, W[i]);
    }
    return PVO_OK;
}

/* ---------------------------------------------------------------- selection */

/* Squared norm of one group's update, as an fp32 chain in index order. */
static float group_score(const float *t, const float *w, int g)
{
    float s = 0.0f;
    for (int i = 0; i < g; ++i) {
        float d = t[i] - w[i];
        s = fmaf(d, d, s);
    }
    return s;
}

typedef struct { float score; int32_t id; } scored_t;

/* larger score first; equal scores: lower id first */
static int cmp_scored(const void *a, const void *b)
{
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->id > y->id) - (x->id < y->id);
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* The k groups with the largest update norm (Alg. 2 line 5, per matrix as in
 * Sec. 3.4), returned as ascending flat group ids.  Full sort, no shortcuts. */
int pvo_select_topk_groups(int64_t out_features, int64_t in_features, int g,
                           const float *T, const float *W, int64_t k,
                           int32_t *out_idx, float *out_scores /* [N] or NULL */)
{
    if (!T || !W || g < 1 || in_features % g) return PVO_ERR;
    int64_t N = out_features * (in_features / g);
    if (k < 0 || k > N || N >= INT32_MAX) return PVO_ERR;
    if (k > 0 && !out_idx) return PVO_ERR;
    scored_t *all = (scored_t *)malloc(sizeof(scored_t) * (size_t)(N > 0 ? N : 1));
    if (!all) return PVO_ERR;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        all[n].score = group_score(T + n * g, W + n * g, g);
        all[n].id = (int32_t)n;
        if (out_scores) out_scores[n] = all[n].score;
    }
    qsort(all, (size_t)N, sizeof(scored_t), cmp_scored);
    for (int64_t i = 0; i < k; ++i) out_idx[i] = all[i].id;
    qsort(out_idx, (size_t)k, sizeof(int32_t), cmp_i32);
    free(all);
    return PVO_OK;
}

/* ---------------------------------------------------------------- re-encode */

/* || s * sum_m C_m[b_m] - t ||^2 in double; codewords summed over m ascending. */
static double tuple_objective(const float *codebooks, int M, int64_t csize, int g,
                              const uint16_t *b, float s, const float *t)
{
    double obj = 0.0;
    for (int i = 0; i < g; ++i) {
        double acc = (double)codebooks[((int64_t)0 * csize + b[0]) * g + i];
        for (int m = 1; m < M; ++m)
            acc = acc + (double)codebooks[((int64_t)m * csize + b[m]) * g + i];
        double r = (double)s * acc - (double)t[i];
        obj = obj + r * r;
    }
    return obj;
}

static int near_tie(double lo, double hi)
{
    /* lo <= hi are the two objectives being separated */
    return (hi - lo) < PVO_NEAR_TIE_REL * hi || hi == lo;
}

/* M = 1: exact nearest codeword (argmin of Eq. 7 over one group's code).
 * Ties: the previous code if it is a minimiser, else the lowest index. */
static void reencode_one_m1(const float *codebook, int64_t csize, int g, float s,
                            const float *t, uint16_t *code, int *flag_near,
                            double *obj_new, double *obj_prev)
{
    uint16_t prev = *code;
    double best = INFINITY, second = INFINITY;
    int64_t best_c = -1;
    for (int64_t c = 0; c < csize; ++c) {
        uint16_t cc = (uint16_t)c;
        double o = tuple_objective(codebook, 1, csize, g, &cc, s, t);
        if (o < best) { second = best; best = o; best_c = c; }
        else if (o < second) second = o;
    }
    double o_prev = tuple_objective(codebook, 1, csize, g, &prev, s, t);
    if (o_prev == best) best_c = prev;      /* previous code wins exact ties */
    if (!(best_c >= 0)) best_c = prev;      /* every objective is NaN: keep   */
    *code = (uint16_t)best_c;
    if (flag_near) *flag_near = (csize > 1) ? near_tie(best, second) : 0;
    if (obj_new) *obj_new = best;
    if (obj_prev) *obj_prev = o_prev;
}

#define PVO_MAX_M 8

typedef struct { double obj; uint16_t b[PVO_MAX_M]; } beam_t;

static int g_cmp_M; /* qsort has no context argument; set per thread below */
#pragma omp threadprivate(g_cmp_M)

/* objective ascending; equal objectives: tuples in lexicographic order */
static int cmp_beam(const void *a, const void *b)
{
    const beam_t *x = (const beam_t *)a, *y = (const beam_t *)b;
    if (x->obj < y->obj) return -1;
    if (x->obj > y->obj) return 1;
    for (int m = 0; m < g_cmp_M; ++m) {
        if (x->b[m] < y->b[m]) return -1;
        if (x->b[m] > y->b[m]) return 1;
    }
    return 0;
}

/* M >= 1: beam search seeded with the current tuple, one sweep over the
 * codebooks in index order.  At codebook m every beam entry spawns 2^B
 * candidates (its m-th code replaced by each codeword, the others held); all
 * candidates are ranked by the full objective and the best beam_width kept.
 * The winner replaces the previous tuple only if it is strictly better. */
static void reencode_one_beam(const float *codebooks, int M, int64_t csize, int g,
                              float s, const float *t, int beam_width,
                              uint16_t *code, beam_t *cand, int *flag_near,
                              double *obj_new, double *obj_prev)
{
    beam_t *cur = cand;                            /* first beam_width slots  */
    beam_t *pool = cand + beam_width;              /* beam_width * csize slots */
    int ncur = 1, near = 0;
    memset(&cur[0], 0, sizeof(beam_t));
    for (int m = 0; m < M; ++m) cur[0].b[m] = code[m];
    double o_prev = tuple_objective(codebooks, M, csize, g, cur[0].b, s, t);
    cur[0].obj = o_prev;
    g_cmp_M = M;
    for (int m = 0; m < M; ++m) {
        int64_t np = 0;
        for (int e = 0; e < ncur; ++e)
            for (int64_t c = 0; c < csize; ++c) {
                beam_t *q = &pool[np++];
                *q = cur[e];
                q->b[m] = (uint16_t)c;
                q->obj = tuple_objective(codebooks, M, csize, g, q->b, s, t);
            }
        qsort(pool, (size_t)np, sizeof(beam_t), cmp_beam);
        int keep = (int)(np < beam_width ? np : beam_width);
        if (np > keep && near_tie(pool[keep - 1].obj, pool[keep].obj)) near = 1;
        memcpy(cur, pool, sizeof(beam_t) * (size_t)keep);
        ncur = keep;
        if (m == M - 1 && np > 1 && near_tie(pool[0].obj, pool[1].obj)) near = 1;
    }
    /* the keep-or-replace decision against the previous tuple is a boundary too */
    {
        int same = 1;
        for (int m = 0; m < M; ++m) same &= (cur[0].b[m] == code[m]);
        if (!same && near_tie(cur[0].obj < o_prev ? cur[0].obj : o_prev,
                              cur[0].obj < o_prev ? o_prev : cur[0].obj)) near = 1;
    }
    if (cur[0].obj < o_prev)
        for (int m = 0; m < M; ++m) code[m] = cur[0].b[m];
    if (flag_near) *flag_near = near;
    if (obj_new) *obj_new = (cur[0].obj < o_prev) ? cur[0].obj : o_prev;
    if (obj_prev) *obj_prev = o_prev;
}

/* Re-assign the codes of the listed groups (ascending flat ids); every other
 * code is left untouched (Eq. 7: entries outside the subspace keep y's value).
 * use_beam = 0 forces the M = 1 definition; use_beam = 1 runs the beam routine
 * for any M (used to pin that it reduces to the definition at M = 1).
 * Optional per-selected-group outputs: near-tie flag, new / previous objective. */
int pvo_reencode_groups(int64_t out_features, int64_t in_features, int g, int M, int B,
                        const float *T, const float *codebooks, const float *scales,
                        const int32_t *group_idx, int64_t k, int beam_width, int use_beam,
                        uint16_t *codes, int64_t *num_changed, uint8_t *near_tie_flags,
                        double *obj_new, double *obj_prev)
{
    if (!T || !codebooks || !scales || !codes) return PVO_ERR;
    if (g < 1 || in_features % g || M < 1 || M > PVO_MAX_M || B < 1 || B > 16) return PVO_ERR;
    if (beam_width < 1 || k < 0) return PVO_ERR;
    if (k > 0 && !group_idx) return PVO_ERR;
    int64_t gpr = in_features / g, N = out_features * gpr, csize = (int64_t)1 << B;
    for (int64_t j = 0; j < k; ++j) {
        if (group_idx[j] < 0 || group_idx[j] >= N) return PVO_ERR;
        /* a stored code is an index into a codebook of 2^B codewords (Sec. 3.1: the partition
         * assigns each group one of the c values); anything else is not a code */
        for (int m = 0; m < M; ++m)
            if (codes[(int64_t)group_idx[j] * M + m] >= csize) return PVO_ERR;
    }
    int beam_path = use_beam || M > 1;
    int64_t changed = 0;
    int failed = 0;
#pragma omp parallel reduction(+ : changed)
    {
        beam_t *cand = NULL;
        if (beam_path) {
            cand = (beam_t *)malloc(sizeof(beam_t) * (size_t)(beam_width + beam_width * csize));
            if (!cand) {
#pragma omp atomic write
                failed = 1;
            }
        }
#pragma omp for schedule(dynamic, 16)
        for (int64_t j = 0; j < k; ++j) {
            if (beam_path && !cand) continue;
            int64_t n = group_idx[j];
            int64_t o = n / gpr;
            const float *t = T + n * g;
            uint16_t *code = codes + n * M;
            uint16_t before[PVO_MAX_M];
            for (int m = 0; m < M; ++m) before[m] = code[m];
            int flag = 0;
            double on = 0.0, op = 0.0;
            if (beam_path)
                reencode_one_beam(codebooks, M, csize, g, scales[o], t, beam_width, code,
                                  cand, &flag, &on, &op);
            else
                reencode_one_m1(codebooks, csize, g, scales[o], t, code, &flag, &on, &op);
            int diff = 0;
            for (int m = 0; m < M; ++m) diff |= (before[m] != code[m]);
            changed += diff;
            if (near_tie_flags) near_tie_flags[j] = (uint8_t)flag;
            if (obj_new) obj_new[j] = on;
            if (obj_prev) obj_prev[j] = op;
        }
        free(cand);
    }
    if (failed) return PVO_ERR;
    if (num_changed) *num_changed = changed;
    return PVO_OK;
}

/* ------------------------------------------------------- stochastic rounding */

/* Random bits of (seed, counter): the output function of the SplitMix64 generator (Steele, Lea
 * and Flood, 2014) on the state seed + (counter + 1) * its odd increment.  Counter-based: one
 * variate per weight group, whatever order the groups are visited in. */
uint64_t pvo_random_bits(uint64_t seed, uint64_t counter)
{
    uint64_t z = seed + (counter + 1u) * UINT64_C(0x9E3779B97F4A7C15);
    z = (z ^ (z >> 30)) * UINT64_C(0xBF58476D1CE4E5B9);
    z = (z ^ (z >> 27)) * UINT64_C(0x94D049BB133111EB);
    return z ^ (z >> 31);
}

/* the top 53 bits as a double in [0, 1) */
double pvo_uniform(uint64_t seed, uint64_t counter)
{
    return (double)(pvo_random_bits(seed, counter) >> 11) * 0x1.0p-53;
}

/* Stochastic rounding for vector quantisation, the K = 2 approximation of App. F: find the two
 * codewords nearest to the target (objective of Eq. 7 restricted to the group; equal objectives
 * in index order) and round to one of them with probability proportional to
 * distance^(-power), distance = sqrt(objective).  power = 1 is the formula of App. F,
 * power = 5 the temperature 0.2 of App. K.  The variate of group n is pvo_uniform(seed, n); the
 * nearest codeword is taken when it is below p(nearest) = 1 / (1 + (d_1 / d_2)^power).
 * Reading: a target that coincides with a codeword is rounded to it with certainty, and a
 * codebook of one codeword leaves no choice.  One codebook only: App. F speaks of a codebook or
 * lattice, additive codes have no list of "nearest vectors" short of the full product.
 * Optional outputs per listed group: the two indices, both objectives, p(nearest), the variate
 * and a flag for decisions that rounding could turn (the second and third objectives, or the
 * first two, within the near-tie tolerance; the variate within 1e-9 of p). */
int pvo_reencode_stochastic(int64_t out_features, int64_t in_features, int g, int B,
                            const float *T, const float *codebook, const float *scales,
                            const int32_t *group_idx, int64_t k, int power, uint64_t seed,
                            uint16_t *codes, int64_t *num_changed, int32_t *nearest_two,
                            double *objective_two, double *p_nearest, double *variate,
                            uint8_t *near_flags)
{
    if (!T || !codebook || !scales || !codes) return PVO_ERR;
    if (g < 1 || in_features % g || B < 1 || B > 16 || power < 1 || power > 64 || k < 0)
        return PVO_ERR;
    if (k > 0 && !group_idx) return PVO_ERR;
    int64_t gpr = in_features / g, N = out_features * gpr, csize = (int64_t)1 << B;
    for (int64_t j = 0; j < k; ++j)
        if (group_idx[j] < 0 || group_idx[j] >= N) return PVO_ERR;
    int64_t changed = 0;
#pragma omp parallel for schedule(dynamic, 16) reduction(+ : changed)
    for (int64_t j = 0; j < k; ++j) {
        int64_t n = group_idx[j];
        const float *t = T + n * g;
        float s = scales[n / gpr];
        double o1 = INFINITY, o2 = INFINITY, o3 = INFINITY;
        int64_t c1 = -1, c2 = -1;
        for (int64_t c = 0; c < csize; ++c) {       /* ascending: '<' keeps the lower index */
            uint16_t cc = (uint16_t)c;
            double o = tuple_objective(codebook, 1, csize, g, &cc, s, t);
            if (o < o1) { o3 = o2; o2 = o1; c2 = c1; o1 = o; c1 = c; }
            else if (o < o2) { o3 = o2; o2 = o; c2 = c; }
            else if (o < o3) o3 = o;
        }
        double p = 1.0;
        if (c2 >= 0 && o1 > 0.0) {
            double r = sqrt(o1 / o2), rn = r;
            for (int e = 1; e < power; ++e) rn = rn * r;
            p = 1.0 / (1.0 + rn);
        }
        double u = pvo_uniform(seed, (uint64_t)n);
        int64_t pick = (c2 < 0 || u < p) ? c1 : c2;
        if (c1 < 0) pick = codes[n];                /* every objective is NaN: keep */
        changed += (codes[n] != (uint16_t)pick);
        codes[n] = (uint16_t)pick;
        if (nearest_two) { nearest_two[2 * j] = (int32_t)c1; nearest_two[2 * j + 1] = (int32_t)c2; }
        if (objective_two) { objective_two[2 * j] = o1; objective_two[2 * j + 1] = o2; }
        if (p_nearest) p_nearest[j] = p;
        if (variate) variate[j] = u;
        if (near_flags)
            near_flags[j] = (uint8_t)(c2 >= 0 && (near_tie(o1, o2) || (csize > 2 && near_tie(o2, o3)) ||
                                                   fabs(u - p) <= 1e-9));
    }
    if (num_changed) *num_changed = changed;
    return PVO_OK;
}

/* Objective of arbitrary code tuples for the listed groups, in the oracle's
 * arithmetic (used to judge a differing choice on a near-tie group). */
int pvo_group_objective(int64_t out_features, int64_t in_features, int g, int M, int B,
                        const float *T, const float *codebooks, const float *scales,
                        const int32_t *group_idx, int64_t k,
                        const uint16_t *tuples /* [k, M] */, double *obj /* [k] */)
{
    if (!T || !codebooks || !scales || !tuples || !obj || g < 1 || in_features % g) return PVO_ERR;
    if (M < 1 || M > PVO_MAX_M || B < 1 || B > 16) return PVO_ERR;
    int64_t gpr = in_features / g, csize = (int64_t)1 << B;
    (void)out_features;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < k; ++j) {
        int64_t n = group_idx[j];
        obj[j] = tuple_objective(codebooks, M, csize, g, tuples + j * M, scales[n / gpr],
                                 T + n * g);
    }
    return PVO_OK;
}

/* --------------------------------------------------------------- dequantize */

/* W[o, j*g + i] = scales[o] * (C_0[b_0, i] + C_1[b_1, i] + ...), fp32 adds in
 * codebook order then one fp32 multiply (Alg. 3 line 1). */
int pvo_dequantize(int64_t out_features, int64_t in_features, int g, int M, int B,
                   const uint16_t *codes, const float *codebooks, const float *scales,
                   float *W_out)
{
    if (!codes || !codebooks || !scales || !W_out || g < 1 || in_features % g) return PVO_ERR;
    if (M < 1 || B < 1 || B > 16) return PVO_ERR;
    int64_t gpr = in_features / g, N = out_features * gpr, csize = (int64_t)1 << B;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float s = scales[n / gpr];
        for (int m = 0; m < M; ++m)
            if (codes[n * M + m] >= csize) {
#pragma omp atomic write
                bad = 1;
            }
        if (bad) continue;
        for (int i = 0; i < g; ++i) {
            float acc = codebooks[((int64_t)0 * csize + codes[n * M]) * g + i];
            for (int m = 1; m < M; ++m)
                acc = acc + codebooks[((int64_t)m * csize + codes[n * M + m]) * g + i];
            W_out[n * g + i] = s * acc;
        }
    }
    return bad ? PVO_ERR : PVO_OK;
}

/* ------------------------------------------------- trust-ratio subspace size */

/* Squared change of one group's dequantised weights when its code tuple goes from
 * `before` to `after`: the fp32 weights of pvo_dequantize, difference and square in
 * double, index order. */
static double group_change(const float *codebooks, int M, int64_t csize, int g, float s,
                           const uint16_t *before, const uint16_t *after)
{
    double d = 0.0;
    for (int i = 0; i < g; ++i) {
        float a = codebooks[((int64_t)0 * csize + before[0]) * g + i];
        float b = codebooks[((int64_t)0 * csize + after[0]) * g + i];
        for (int m = 1; m < M; ++m) {
            a = a + codebooks[((int64_t)m * csize + before[m]) * g + i];
            b = b + codebooks[((int64_t)m * csize + after[m]) * g + i];
        }
        double diff = (double)(s * b) - (double)(s * a);
        d = d + diff * diff;
    }
    return d;
}

/* The subspace size of Sec. 4.3 / App. K (hyperparameter paragraph): tau is the largest
 * number of weights whose update keeps the trust ratio ||x^{k+1} - x^k|| / ||x^k|| below
 * `ratio`.  Followed step by step: candidates are taken in the order of the selection
 * rule (largest update norm first, lower id first), `chunk` groups at a time; each chunk
 * is re-encoded and its change added to the total; when the total no longer satisfies the
 * bound, groups of that last chunk are put back to their previous codes, from the end of
 * the chunk, until it does; at least one group whose code changed is always kept.
 * Reading: the unit is a weight group, x is this matrix' dequantised weights (the trust
 * ratio is taken per weight matrix like the selection of Sec. 3.4), the comparison is
 * strict and done on squares:  sum of changes < ratio^2 * ||x^k||^2, all in double.
 * At most k_max groups are tried.  Returns the number of groups kept in *num_applied
 * (the first *num_applied entries of rank_idx), stats[0] = their squared change,
 * stats[1] = ||x^k||^2. */
int pvo_reencode_trust_ratio(int64_t out_features, int64_t in_features, int g, int M, int B,
                             const float *T, const float *W, const float *codebooks,
                             const float *scales, int64_t k_max, int64_t chunk, double ratio,
                             int beam_width, uint16_t *codes, int32_t *rank_idx,
                             int64_t *num_applied, double *stats)
{
    if (!T || !W || !codebooks || !scales || !codes || !rank_idx || !num_applied) return PVO_ERR;
    if (g < 1 || in_features % g || M < 1 || M > PVO_MAX_M || B < 1 || B > 16) return PVO_ERR;
    int64_t gpr = in_features / g, N = out_features * gpr, csize = (int64_t)1 << B;
    if (k_max < 0 || k_max > N || chunk < 1 || beam_width < 1 || !(ratio >= 0.0)) return PVO_ERR;

    /* order of the selection rule */
    scored_t *all = (scored_t *)malloc(sizeof(scored_t) * (size_t)(N > 0 ? N : 1));
    uint16_t *saved = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)(k_max > 0 ? k_max * M : 1));
    double *prefix = (double *)malloc(sizeof(double) * (size_t)(k_max + 1));
    if (!all || !saved || !prefix) { free(all); free(saved); free(prefix); return PVO_ERR; }
    for (int64_t n = 0; n < N; ++n) {
        all[n].score = group_score(T + n * g, W + n * g, g);
        all[n].id = (int32_t)n;
    }
    qsort(all, (size_t)N, sizeof(scored_t), cmp_scored);
    for (int64_t r = 0; r < k_max; ++r) rank_idx[r] = all[r].id;
    free(all);

    /* ||x^k||^2 of the current dequantised matrix */
    double normsq = 0.0;
    for (int64_t n = 0; n < N; ++n) {
        float s = scales[n / gpr];
        for (int i = 0; i < g; ++i) {
            float acc = codebooks[((int64_t)0 * csize + codes[n * M]) * g + i];
            for (int m = 1; m < M; ++m)
                acc = acc + codebooks[((int64_t)m * csize + codes[n * M + m]) * g + i];
            double w = (double)(s * acc);
            normsq = normsq + w * w;
        }
    }
    const double bound = ratio * ratio * normsq;

    int64_t applied = 0, first_changed = -1;
    prefix[0] = 0.0;
    int rc = PVO_OK;
    for (int64_t start = 0; start < k_max && rc == PVO_OK; start += chunk) {
        int64_t end = start + chunk < k_max ? start + chunk : k_max;
        for (int64_t r = start; r < end; ++r)
            for (int m = 0; m < M; ++m) saved[r * M + m] = codes[(int64_t)rank_idx[r] * M + m];
        rc = pvo_reencode_groups(out_features, in_features, g, M, B, T, codebooks, scales,
                                 rank_idx + start, end - start, beam_width, 0, codes, NULL, NULL,
                                 NULL, NULL);
        if (rc != PVO_OK) break;
        for (int64_t r = start; r < end; ++r) {
            int64_t n = rank_idx[r];
            double d = group_change(codebooks, M, csize, g, scales[n / gpr], saved + r * M,
                                    codes + n * M);
            int diff = 0;
            for (int m = 0; m < M; ++m) diff |= (saved[r * M + m] != codes[n * M + m]);
            if (diff && first_changed < 0) first_changed = r;
            prefix[r + 1] = prefix[r] + d;
        }
        applied = end;
        if (!(prefix[applied] < bound)) {
            /* undo from the end of this chunk until the bound holds; keep one changed group */
            while (applied > start && !(prefix[applied] < bound)) {
                if (first_changed >= 0 && applied - 1 <= first_changed) break;
                int64_t n = rank_idx[applied - 1];
                for (int m = 0; m < M; ++m) codes[n * M + m] = saved[(applied - 1) * M + m];
                --applied;
            }
            break;
        }
    }
    *num_applied = applied;
    if (stats) {
        stats[0] = prefix[applied];
        stats[1] = normsq;
    }
    free(saved);
    free(prefix);
    return rc;
}

/* ------------------------------------------------- scalar uniform grids (App. K) */

/* The scalar representation of App. K ("GPTQ": uniform grid, block-wise scales and zero
 * points along the input dimension): W[o, i] = s[o, i/blk] * (q[o, i] - z[o, i/blk]) with
 * q in [0, 2^b).  fp32: one subtraction, one multiplication. */
int pvo_dequantize_scalar(int64_t out_features, int64_t in_features, int blk, int b,
                          const uint8_t *codes, const float *scales, const float *zeros,
                          float *W_out)
{
    if (!codes || !scales || !zeros || !W_out || blk < 1 || in_features % blk) return PVO_ERR;
    if (b < 1 || b > 8) return PVO_ERR;
    int64_t bpr = in_features / blk;
    for (int64_t o = 0; o < out_features; ++o)
        for (int64_t i = 0; i < in_features; ++i) {
            int q = codes[o * in_features + i];
            if (q >= (1 << b)) return PVO_ERR;
            float d = (float)q - zeros[o * bpr + i / blk];
            W_out[o * in_features + i] = scales[o * bpr + i / blk] * d;
        }
    return PVO_OK;
}

/* V step on that representation (App. K: "V step performs simple rounding to nearest
 * (scaled) integer"): for every listed weight the grid value nearest to the target, written
 * as the definition - every q is tried, objective (w_q - t)^2 in double with w_q the fp32
 * dequantised value; ties: the previous code if it is a minimiser, else the lowest q. */
int pvo_reencode_scalar(int64_t out_features, int64_t in_features, int blk, int b, const float *T,
                        const float *scales, const float *zeros, const int32_t *weight_idx,
                        int64_t k, uint8_t *codes, int64_t *num_changed)
{
    if (!T || !scales || !zeros || !codes || blk < 1 || in_features % blk) return PVO_ERR;
    if (b < 1 || b > 8 || k < 0 || (k > 0 && !weight_idx)) return PVO_ERR;
    int64_t bpr = in_features / blk, n = out_features * in_features, changed = 0;
    for (int64_t j = 0; j < k; ++j) {
        int64_t e = weight_idx[j];
        if (e < 0 || e >= n) return PVO_ERR;
        int64_t o = e / in_features, i = e % in_features;
        float s = scales[o * bpr + i / blk], z = zeros[o * bpr + i / blk];
        int prev = codes[e], best = -1;
        double best_obj = 0.0, prev_obj = 0.0;
        for (int q = 0; q < (1 << b); ++q) {
            float w = s * ((float)q - z);
            double r = (double)w - (double)T[e];
            double obj = r * r;
            if (q == prev) prev_obj = obj;
            if (best < 0 || obj < best_obj) { best = q; best_obj = obj; }
        }
        if (prev < (1 << b) && prev_obj == best_obj) best = prev;
        if (best != prev) { codes[e] = (uint8_t)best; ++changed; }
    }
    if (num_changed) *num_changed = changed;
    return PVO_OK;
}

/* ------------------------------------------------------------ P-step gradients */

/* The P step updates the continuous parameters "by backprop" (Alg. 3, P step; Sec. 3.1:
 * the c-dimensional gradient over the distinct values; App. K: codebooks and per-channel
 * scales).  With W[o, j*g + i] = s_o * sum_m C_m[b(o,j,m), i] and G = d phi / d W the chain
 * rule gives
 *     d phi / d C_m[c, i] = sum over groups n = (o, j) with b(o,j,m) = c of  s_o * G[o, j*g + i]
 *     d phi / d s_o       = sum_j sum_i G[o, j*g + i] * (C_0[b_0, i] + C_1[b_1, i] + ...)
 * Products are formed in double (exact for fp32 factors), sums run in double in ascending
 * group / index order, results are rounded to fp32 once.  The inner codeword sum of the
 * scale gradient is the fp32 chain of pvo_dequantize (without the scale). */
int pvo_codebook_grads(int64_t out_features, int64_t in_features, int g, int M, int B,
                       const float *G, const uint16_t *codes, const float *codebooks,
                       const float *scales, float *grad_codebooks /* [M, 2^B, g] */,
                       float *grad_scales /* [out] or NULL */)
{
    if (!G || !codes || !codebooks || !scales || !grad_codebooks) return PVO_ERR;
    if (g < 1 || in_features % g || M < 1 || B < 1 || B > 16) return PVO_ERR;
    int64_t gpr = in_features / g, N = out_features * gpr, csize = (int64_t)1 << B;
    double *acc = (double *)calloc((size_t)(M * csize * g), sizeof(double));
    if (!acc) return PVO_ERR;
    for (int64_t n = 0; n < N; ++n) {
        double s = (double)scales[n / gpr];
        for (int m = 0; m < M; ++m) {
            int64_t c = codes[n * M + m];
            if (c >= csize) { free(acc); return PVO_ERR; }
            double *row = acc + ((int64_t)m * csize + c) * g;
            for (int i = 0; i < g; ++i) row[i] = row[i] + s * (double)G[n * g + i];
        }
    }
    for (int64_t e = 0; e < (int64_t)M * csize * g; ++e) grad_codebooks[e] = (float)acc[e];
    free(acc);
    if (grad_scales)
        for (int64_t o = 0; o < out_features; ++o) {
            double a = 0.0;
            for (int64_t j = 0; j < gpr; ++j) {
                int64_t n = o * gpr + j;
                for (int i = 0; i < g; ++i) {
                    float q = codebooks[((int64_t)0 * csize + codes[n * M]) * g + i];
                    for (int m = 1; m < M; ++m)
                        q = q + codebooks[((int64_t)m * csize + codes[n * M + m]) * g + i];
                    a = a + (double)G[n * g + i] * (double)q;
                }
            }
            grad_scales[o] = (float)a;
        }
    return PVO_OK;
}

int pvo_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}

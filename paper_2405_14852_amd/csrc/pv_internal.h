// Internal declarations shared by the translation units of libpv (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "pv.h"

// native 16-byte vector (the nontemporal builtins do not take HIP's float4 struct)
typedef float pv_f4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------- context

struct pv_buffer {
    void *ptr = nullptr;
    size_t bytes = 0;
};

struct pv_timer {
    std::vector<hipEvent_t> pending;  // start/stop pairs not yet read back
    double total_ms = 0.0;
    int64_t launches = 0;
};

struct pv_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    char err[256] = {0};
    int search_mode = 0;
    int meta_phase = 0;        // which of the two statistics slots of cb_meta the next filter call uses
    int rr_blocks_last = 0;    // blocks of the last call's re-rank kernel (their counters are summed on request)
    bool timing = false;
    pv_timer timers[PV_K_COUNT];
    std::vector<hipEvent_t> event_pool;

    // scratch, grown on demand (never shrunk)
    pv_buffer sel_scores;   // f32 [N]            group scores when the caller passes none
    pv_buffer sel_hist;     // u32 [copies + 2][bins]  radix-select histograms (kept zero between calls)
    pv_buffer sel_blocks;   // u32 [nblocks][2]   per-block (greater, equal) counts
    pv_buffer sel_state;    // u32 [4]            threshold key, ties to take
    pv_buffer stats;        // i64 [8]            counters of the last re-encode
    pv_buffer cb_f16;       // prepared codebook operand for the matrix-core filter
    pv_buffer cb_meta;      // u32 [2][8]         two slots of codebook statistics (scale, norms, rounding bound)
    pv_buffer x_f16;        // prepared target operand [k_pad / 32][2][32][8] halves
    pv_buffer x_meta;       // f32 [k_pad][4]     per-group bounds and flags
    pv_buffer partials;     // i32 [P][k_pad][2]  best / runner-up keys per partition
    pv_buffer fb_list;      // counters (work-item hand-out) and, for the beam path, the groups left to the exact kernel
    pv_buffer rr_counts;    // u32 [blocks][4]    per-block counters of the re-rank kernel
    pv_buffer trust;        // scratch of the trust-ratio call (saved codes, keys, prefix sums, sort space)
    pv_buffer pstep;        // scratch of the P-step gradients (digit histograms, keys and group ids of the sorting passes, segment starts, piece sums)
};

// RAII bracket that records HIP events around a group of launches when timing is on.
struct pv_timed {
    pv_ctx *c;
    int id;
    hipEvent_t start = nullptr;
    pv_timed(pv_ctx *ctx, int kernel_id);
    ~pv_timed();
};

pv_status pv_fail(pv_ctx *ctx, pv_status st, const char *fmt, ...);
pv_status pv_ensure(pv_ctx *ctx, pv_buffer &buf, size_t bytes, bool zero_new = false);

#define PV_HIP(ctx, call)                                                              \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess)                                                          \
            return pv_fail(ctx, PV_ERR_DEVICE, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

static inline int64_t pv_num_groups(const pv_layout *l)
{
    return l->out_features * (l->in_features / l->group_size);
}

// ---------------------------------------------------------------- Adam direction (Sec. 3.4)
// The gradient of Eq. 7 replaced by one Adam update.  Per element, in fp32 with one rounding
// per operation written here (division and square root correctly rounded):
//   m' = fma(b1, m, (1 - b1) * g)     v' = fma(b2, v, (1 - b2) * (g * g))
//   T  = fma(-lr, (m' / c1) / (sqrt(v' / c2) + eps), W)
// c1, c2: the bias corrections 1 - b^t, formed on the host in double and rounded once.
struct pv_adam_t {
    float lr, b1, b2, omb1, omb2, c1, c2, eps;
};

pv_adam_t pv_make_adam(int64_t step, float lr, float beta1, float beta2, float eps);

#ifdef __HIPCC__
// floor(n / d) for n, d < 2^31 from inv = 1.0 / d (rounded once): (n + 0.5) / d lies at least
// 0.5 / d away from every integer, and the two roundings move the product by less than
// 2^-21 / d, so the truncation is the exact quotient.  Four instructions instead of the
// thirty of an integer division.
__device__ __forceinline__ unsigned pv_row_of(unsigned n, double inv)
{
    return (unsigned)(((double)n + 0.5) * inv);
}

__device__ __forceinline__ float pv_adam_one(float w, float g, float &m, float &v, const pv_adam_t &a)
{
    m = fmaf(a.b1, m, a.omb1 * g);
    v = fmaf(a.b2, v, a.omb2 * (g * g));
    // plain '/' and sqrtf compile to the correctly rounded sequences (the __fsqrt_rn
    // intrinsic of this toolchain does not: it differs from IEEE in 14 % of random inputs)
    const float mhat = m / a.c1;
    const float vhat = v / a.c2;
    const float upd = mhat / (sqrtf(vhat) + a.eps);
    return fmaf(-a.lr, upd, w);
}
#endif

// ---------------------------------------------------------------- launchers
// (each enqueues on ctx->stream; arguments were validated by the caller)

pv_status pv_launch_encode_targets(pv_ctx *ctx, const float *W, const float *G, float alpha,
                                   float *T, int64_t n);
pv_status pv_launch_encode_targets_adam(pv_ctx *ctx, const float *W, const float *G, float *m,
                                        float *v, int64_t step, float lr, float beta1, float beta2,
                                        float eps, float *T, int64_t n);
pv_status pv_launch_dequantize(pv_ctx *ctx, const pv_layout *l, const uint16_t *codes,
                               const float *codebooks, const float *scales, float *W_out);
pv_status pv_launch_dequantize_groups(pv_ctx *ctx, const pv_layout *l, const uint16_t *codes,
                                      const float *codebooks, const float *scales,
                                      const int32_t *group_idx, int64_t k, float *W_out);
// A request to the scoring sweep to take, on its way, the squared norm of the dequantised
// weights sum (scales[o] * codebooks[codes[n]][i])^2 (one codebook, g = 8 or 16): the gathers
// from the L2-resident codebook ride under the sweep's memory traffic.  partial: device f64,
// at least pv_select_norm_parts() entries; the sweep leaves `parts` partial sums there, to be
// added in index order.  pv_select_norm_supported says whether a layout is covered.
struct pv_norm_req {
    const uint16_t *codes;
    const float *codebooks;
    const float *scales;
    double *partial;
    int parts;          // out
};
bool pv_select_norm_supported(const pv_layout *l);
int pv_select_norm_parts();
// G != nullptr: T is an output, formed in the scoring sweep as W - alpha * G, or, with adam and
// the moments m, v given, as W minus one Adam update of G
pv_status pv_launch_select(pv_ctx *ctx, const pv_layout *l, const float *T, const float *W,
                           int64_t k, int32_t *out_idx, float *scores, const float *G = nullptr,
                           float alpha = 0.0f, const pv_adam_t *adam = nullptr, float *m = nullptr,
                           float *v = nullptr, pv_norm_req *norm = nullptr);
// selection with its scratch in the library's static device array (no allocation of any kind)
pv_status pv_static_scratch_init(pv_ctx *ctx, int device);   // `device` must be current
int64_t pv_static_max_groups();
pv_status pv_launch_select_static(pv_ctx *ctx, const pv_layout *l, const float *T, const float *W,
                                  int64_t k, int32_t *out_idx, float *scores);
pv_status pv_launch_exact_scan(pv_ctx *ctx, const pv_layout *l, const float *T,
                               const float *codebooks, const float *scales,
                               const int32_t *list, const uint32_t *d_count, int64_t max_count,
                               uint16_t *codes, int64_t *num_changed, int64_t *d_stat_counter);
pv_status pv_launch_beam(pv_ctx *ctx, const pv_layout *l, const float *T, const float *codebooks,
                         const float *scales, const int32_t *group_idx, int64_t k,
                         int32_t beam_width, uint16_t *codes, int64_t *num_changed);
// two 8-bit codebooks, g = 8, beam <= 8: fp32 / fp16 matrix-core filter; groups it cannot
// certify are appended to redo_list (count in *redo_count) for the exact kernel
pv_status pv_launch_beam_2x8_f16(pv_ctx *ctx, const float *T, const float *codebooks,
                                 const float *scales, const int32_t *group_idx, int64_t k,
                                 int32_t beam_width, uint16_t *codes, int64_t *num_changed,
                                 unsigned long long *stat_fast, int32_t *redo_list,
                                 unsigned long long *redo_count, int gpr, int N);
bool pv_mfma_supported(const pv_layout *l);
// power == 0: the nearest codeword (deterministic V step); power >= 1: stochastic rounding over
// the two nearest with that power and seed
pv_status pv_launch_mfma_search(pv_ctx *ctx, const pv_layout *l, const float *T,
                                const float *codebooks, const float *scales,
                                const int32_t *group_idx, int64_t k, uint16_t *codes,
                                int64_t *num_changed, int32_t power = 0, uint64_t seed = 0);
// Stochastic rounding over the two nearest codewords (App. F, K = 2; App. K: power 5): given the
// two smallest objectives of a group (o1 <= o2, index kNoCode = absent) the code to take.  The
// nearest one is taken when the group's variate u - the top 53 bits of the SplitMix64 output
// function at seed + (group + 1) * increment - lies below p = 1 / (1 + (d1 / d2)^power),
// d = sqrt(objective).  Every step is a correctly rounded double operation, so every kernel
// that calls this (and the CPU reference, which writes the same chain) decides alike.
#ifdef __HIPCC__
constexpr int kPvNoCode = 0x7fffffff;
__device__ __forceinline__ int pv_round_pick(double o1, int i1, double o2, int i2, int power,
                                             unsigned long long seed, unsigned long long group)
{
    double p = 1.0;
    if (i2 != kPvNoCode && o1 > 0.0) {
        const double r = __dsqrt_rn(__ddiv_rn(o1, o2));
        double rn = r;
        for (int e = 1; e < power; ++e) rn = __dmul_rn(rn, r);
        p = __ddiv_rn(1.0, __dadd_rn(1.0, rn));
    }
    unsigned long long z = seed + (group + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z = z ^ (z >> 31);
    const double u = (double)(z >> 11) * 0x1.0p-53;
    return (i2 == kPvNoCode || u < p) ? i1 : i2;
}
#endif

pv_status pv_launch_round_two_nearest(pv_ctx *ctx, const pv_layout *l, const float *T,
                                      const float *codebook, const float *scales,
                                      const int32_t *group_idx, int64_t k, int32_t power,
                                      uint64_t seed, uint16_t *codes, int64_t *num_changed);
pv_status pv_launch_fill_f32(pv_ctx *ctx, float *p, int64_t n, float value);
pv_status pv_launch_fill_i64(pv_ctx *ctx, int64_t *p, int64_t n, int64_t value,
                             int64_t *also = nullptr);   // *also = value too, in the same launch
pv_status pv_launch_probe_copy(pv_ctx *ctx, void *dst, const void *src, int64_t bytes);
pv_status pv_launch_probe_mfma(pv_ctx *ctx, int64_t iters, float *sink, int64_t *waves_out);
// the search of pv_reencode_groups after argument validation (k may be 0)
pv_status pv_reencode_dispatch(pv_ctx *ctx, const pv_layout *l, const float *T,
                               const float *codebooks, const float *scales,
                               const int32_t *group_idx, int64_t k, int32_t beam_width,
                               uint16_t *codes, int64_t *num_changed);
pv_status pv_launch_dequantize_scalar(pv_ctx *ctx, int64_t out_features, int64_t in_features, int blk,
                                      const uint8_t *codes, const float *scales, const float *zeros,
                                      float *W_out);
pv_status pv_launch_reencode_scalar(pv_ctx *ctx, int64_t out_features, int64_t in_features, int blk,
                                    int nbits, const float *T, const float *scales,
                                    const float *zeros, const int32_t *weight_idx, int64_t k,
                                    uint8_t *codes, int64_t *num_changed);
pv_status pv_launch_codebook_grads(pv_ctx *ctx, const pv_layout *l, const float *G,
                                   const uint16_t *codes, const float *codebooks,
                                   const float *scales, float *grad_codebooks, float *grad_scales);
pv_status pv_launch_trust_ratio(pv_ctx *ctx, const pv_layout *l, const float *T, const float *W,
                                const float *codebooks, const float *scales, int64_t k_max,
                                int64_t chunk, double ratio, int32_t beam_width, uint16_t *codes,
                                int32_t *rank_idx, int64_t *num_applied, double *stats);

// C-ABI entry points of libpv: context handling, argument validation, dispatch.
// Every step of the path runs in the kernels of the other translation units.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>

#include "pv_internal.h"

// ---------------------------------------------------------------- helpers

pv_status pv_fail(pv_ctx *ctx, pv_status st, const char *fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return st;
}

pv_status pv_ensure(pv_ctx *ctx, pv_buffer &buf, size_t bytes, bool zero_new)
{
    if (buf.bytes >= bytes && buf.ptr) return PV_OK;
    size_t want = bytes < 256 ? 256 : bytes;
    if (buf.ptr) {
        // queued kernels may still read the old block
        PV_HIP(ctx, hipStreamSynchronize(ctx->stream));
        PV_HIP(ctx, hipFree(buf.ptr));
        buf.ptr = nullptr;
        buf.bytes = 0;
        want += want / 4;
    }
    void *p = nullptr;
    if (hipMalloc(&p, want) != hipSuccess) {
        (void)hipGetLastError();
        return pv_fail(ctx, PV_ERR_ALLOC, "scratch allocation of %zu bytes failed", want);
    }
    buf.ptr = p;
    buf.bytes = want;
    if (zero_new) PV_HIP(ctx, hipMemsetAsync(p, 0, want, ctx->stream));
    return PV_OK;
}

static hipEvent_t take_event(pv_ctx *c)
{
    if (!c->event_pool.empty()) {
        hipEvent_t e = c->event_pool.back();
        c->event_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

pv_timed::pv_timed(pv_ctx *ctx, int kernel_id) : c(ctx), id(kernel_id)
{
    if (!c->timing) return;
    start = take_event(c);
    if (start) (void)hipEventRecord(start, c->stream);
}

pv_timed::~pv_timed()
{
    if (!start) return;
    hipEvent_t stop = take_event(c);
    if (!stop) {
        c->event_pool.push_back(start);
        return;
    }
    (void)hipEventRecord(stop, c->stream);
    c->timers[id].pending.push_back(start);
    c->timers[id].pending.push_back(stop);
}

static pv_status check_layout(pv_ctx *ctx, const pv_layout *l)
{
    if (!l) return pv_fail(ctx, PV_ERR_INVALID_ARG, "layout is NULL");
    if (l->out_features < 0 || l->in_features < 0)
        return pv_fail(ctx, PV_ERR_SHAPE, "negative matrix shape");
    if (l->group_size < 1 || l->in_features % l->group_size != 0)
        return pv_fail(ctx, PV_ERR_SHAPE, "in_features %lld is not a multiple of group_size %d",
                       (long long)l->in_features, l->group_size);
    if (l->num_codebooks < 1 || l->num_codebooks > 8)
        return pv_fail(ctx, PV_ERR_SHAPE, "num_codebooks %d not in 1..8", l->num_codebooks);
    if (l->nbits < 1 || l->nbits > 16)
        return pv_fail(ctx, PV_ERR_SHAPE, "nbits %d not in 1..16", l->nbits);
    int64_t gpr = l->in_features / l->group_size;
    if (l->out_features > 0 && gpr > 0 && gpr > (INT64_C(0x7fffffff) - 1) / l->out_features)
        return pv_fail(ctx, PV_ERR_SHAPE, "number of groups must be below 2^31");
    return PV_OK;
}

static bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// ---------------------------------------------------------------- context

extern "C" pv_status pv_create(pv_ctx **out, int device, void *hip_stream)
{
    if (!out) return PV_ERR_INVALID_ARG;
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) {
        (void)hipGetLastError();
        return PV_ERR_DEVICE;
    }
    if (hipSetDevice(device) != hipSuccess) return PV_ERR_DEVICE;
    pv_ctx *c = new (std::nothrow) pv_ctx();
    if (!c) return PV_ERR_ALLOC;
    c->device = device;
    c->stream = static_cast<hipStream_t>(hip_stream);
    // address of the static scratch array on this device (for pv_select_topk_groups_noalloc)
    if (pv_static_scratch_init(c, device) != PV_OK) {
        delete c;
        return PV_ERR_DEVICE;
    }
    *out = c;
    return PV_OK;
}

extern "C" void pv_destroy(pv_ctx *c)
{
    if (!c) return;
    (void)hipSetDevice(c->device);
    (void)hipStreamSynchronize(c->stream);
    pv_buffer *bufs[] = {&c->sel_scores, &c->sel_hist, &c->sel_blocks, &c->sel_state, &c->stats,
                         &c->cb_f16,     &c->cb_meta,  &c->x_f16,      &c->x_meta,    &c->partials,
                         &c->fb_list, &c->rr_counts, &c->trust, &c->pstep};
    for (pv_buffer *b : bufs)
        if (b->ptr) (void)hipFree(b->ptr);
    for (auto &t : c->timers)
        for (hipEvent_t e : t.pending) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->event_pool) (void)hipEventDestroy(e);
    delete c;
}

extern "C" const char *pv_last_error(const pv_ctx *c) { return c ? c->err : "context is NULL"; }

// ---------------------------------------------------------------- the path

extern "C" pv_status pv_encode_targets(pv_ctx *ctx, const pv_layout *l, const float *W,
                                       const float *G, float alpha, float *T)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_layout(ctx, l);
    if (st != PV_OK) return st;
    if (!W || !G || !T) return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (misaligned(W) || misaligned(G) || misaligned(T))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    int64_t n = l->out_features * l->in_features;
    if (n == 0) return PV_OK;
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_launch_encode_targets(ctx, W, G, alpha, T, n);
}

extern "C" pv_status pv_encode_targets_adam(pv_ctx *ctx, const pv_layout *l, const float *W,
                                            const float *G, float *m, float *v, int64_t step,
                                            float lr, float beta1, float beta2, float eps, float *T)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_layout(ctx, l);
    if (st != PV_OK) return st;
    if (!W || !G || !m || !v || !T) return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (misaligned(W) || misaligned(G) || misaligned(m) || misaligned(v) || misaligned(T))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (step < 1) return pv_fail(ctx, PV_ERR_INVALID_ARG, "step must be >= 1");
    if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "beta1 and beta2 must lie in [0, 1)");
    if (T == (float *)m || T == (float *)v || m == v)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "T, m and v must be distinct buffers");
    int64_t n = l->out_features * l->in_features;
    if (n == 0) return PV_OK;
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_launch_encode_targets_adam(ctx, W, G, m, v, step, lr, beta1, beta2, eps, T, n);
}

extern "C" pv_status pv_encode_targets_adam_select(pv_ctx *ctx, const pv_layout *l, const float *W,
                                                   const float *G, float *m, float *v, int64_t step,
                                                   float lr, float beta1, float beta2, float eps,
                                                   float *T, int64_t k, int32_t *out_idx,
                                                   float *group_scores)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_layout(ctx, l);
    if (st != PV_OK) return st;
    int64_t N = pv_num_groups(l);
    if (k < 0 || k > N)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "k = %lld outside [0, %lld]", (long long)k,
                       (long long)N);
    if (!W || !G || !m || !v || !T) return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (k > 0 && !out_idx) return pv_fail(ctx, PV_ERR_INVALID_ARG, "out_idx is NULL");
    if (misaligned(W) || misaligned(G) || misaligned(m) || misaligned(v) || misaligned(T) ||
        misaligned(group_scores))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (step < 1) return pv_fail(ctx, PV_ERR_INVALID_ARG, "step must be >= 1");
    if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "beta1 and beta2 must lie in [0, 1)");
    if (T == W || T == m || T == v || m == v)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "T, W, m and v must be distinct buffers");
    if (N == 0) return PV_OK;
    PV_HIP(ctx, hipSetDevice(ctx->device));
    const int g = l->group_size;
    if (!(g == 4 || g == 8 || g == 16 || g == 32 || g == 64)) {
        // no fused kernel for this group size: the two calls in sequence
        st = pv_launch_encode_targets_adam(ctx, W, G, m, v, step, lr, beta1, beta2, eps, T,
                                           l->out_features * l->in_features);
        if (st != PV_OK) return st;
        if (k == 0 && !group_scores) return PV_OK;
        return pv_launch_select(ctx, l, T, W, k, out_idx, group_scores);
    }
    const pv_adam_t a = pv_make_adam(step, lr, beta1, beta2, eps);
    return pv_launch_select(ctx, l, T, W, k, out_idx, group_scores, G, 0.0f, &a, m, v);
}

extern "C" pv_status pv_select_topk_groups(pv_ctx *ctx, const pv_layout *l, const float *T,
                                           const float *W, int64_t k, int32_t *out_idx,
                                           float *group_scores)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_layout(ctx, l);
    if (st != PV_OK) return st;
    int64_t N = pv_num_groups(l);
    if (k < 0 || k > N)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "k = %lld outside [0, %lld]", (long long)k,
                       (long long)N);
    if (!T || !W) return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (k > 0 && !out_idx) return pv_fail(ctx, PV_ERR_INVALID_ARG, "out_idx is NULL");
    if (misaligned(T) || misaligned(W) || misaligned(group_scores))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (N == 0 || (k == 0 && !group_scores)) return PV_OK;
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_launch_select(ctx, l, T, W, k, out_idx, group_scores);
}

extern "C" pv_status pv_select_topk_groups_noalloc(pv_ctx *ctx, const pv_layout *l, const float *T,
                                                   const float *W, int64_t k, int32_t *out_idx,
                                                   float *group_scores)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_layout(ctx, l);
    if (st != PV_OK) return st;
    int64_t N = pv_num_groups(l);
    if (N > pv_static_max_groups())
        return pv_fail(ctx, PV_ERR_UNSUPPORTED,
                       "%lld groups exceed the %lld the static scratch array is sized for",
                       (long long)N, (long long)pv_static_max_groups());
    if (k < 0 || k > N)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "k = %lld outside [0, %lld]", (long long)k,
                       (long long)N);
    if (!T || !W) return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (k > 0 && !out_idx) return pv_fail(ctx, PV_ERR_INVALID_ARG, "out_idx is NULL");
    if (misaligned(T) || misaligned(W) || misaligned(group_scores))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (N == 0 || (k == 0 && !group_scores)) return PV_OK;
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_launch_select_static(ctx, l, T, W, k, out_idx, group_scores);
}

extern "C" pv_status pv_encode_targets_select(pv_ctx *ctx, const pv_layout *l, const float *W,
                                              const float *G, float alpha, float *T, int64_t k,
                                              int32_t *out_idx, float *group_scores)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_layout(ctx, l);
    if (st != PV_OK) return st;
    int64_t N = pv_num_groups(l);
    if (k < 0 || k > N)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "k = %lld outside [0, %lld]", (long long)k,
                       (long long)N);
    if (!W || !G || !T) return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (k > 0 && !out_idx) return pv_fail(ctx, PV_ERR_INVALID_ARG, "out_idx is NULL");
    if (misaligned(W) || misaligned(G) || misaligned(T) || misaligned(group_scores))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (T == W) return pv_fail(ctx, PV_ERR_INVALID_ARG, "T must not alias W (W is scored against T)");
    if (N == 0) return PV_OK;
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_launch_select(ctx, l, T, W, k, out_idx, group_scores, G, alpha);
}

static pv_status check_reencode_args(pv_ctx *ctx, const pv_layout *l, int64_t k,
                                     int32_t beam_width, const float *T, const float *codebooks,
                                     const float *scales, const uint16_t *codes)
{
    int64_t N = pv_num_groups(l);
    if (k < 0 || k > N)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "k = %lld outside [0, %lld]", (long long)k,
                       (long long)N);
    if (beam_width < 1) return pv_fail(ctx, PV_ERR_INVALID_ARG, "beam_width must be >= 1");
    if (!T || !codebooks || !scales || !codes)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (misaligned(T) || misaligned(codebooks))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (l->num_codebooks > 1) {
        int64_t pool = (int64_t)beam_width << l->nbits;
        if (beam_width > 64 || pool > 4096)
            return pv_fail(ctx, PV_ERR_UNSUPPORTED,
                           "beam search supports beam_width <= 64 and beam_width * 2^B <= 4096");
        if (l->group_size > 64)
            return pv_fail(ctx, PV_ERR_UNSUPPORTED, "beam search supports group_size <= 64");
    } else if (l->group_size > 64) {
        return pv_fail(ctx, PV_ERR_UNSUPPORTED, "nearest-codeword search supports group_size <= 64");
    }
    return PV_OK;
}

pv_status pv_reencode_dispatch(pv_ctx *ctx, const pv_layout *l, const float *T,
                               const float *codebooks, const float *scales,
                               const int32_t *group_idx, int64_t k, int32_t beam_width,
                               uint16_t *codes, int64_t *num_changed)
{
    const int M = l->num_codebooks;
    pv_status st = pv_ensure(ctx, ctx->stats, 8 * sizeof(int64_t));
    if (st != PV_OK) return st;
    int64_t *stats = static_cast<int64_t *>(ctx->stats.ptr);
    ctx->rr_blocks_last = 0;
    const bool filter = M == 1 && k > 0 && ctx->search_mode == 0 && pv_mfma_supported(l);
    if (filter)   // its first kernel clears the counters
        return pv_launch_mfma_search(ctx, l, T, codebooks, scales, group_idx, k, codes, num_changed);
    st = pv_launch_fill_i64(ctx, stats, 8, 0, num_changed);
    if (st != PV_OK) return st;
    if (k == 0) return PV_OK;
    if (M > 1) return pv_launch_beam(ctx, l, T, codebooks, scales, group_idx, k, beam_width, codes,
                                     num_changed);
    return pv_launch_exact_scan(ctx, l, T, codebooks, scales, group_idx, nullptr, k, codes,
                                num_changed, stats + 3);
}

extern "C" pv_status pv_reencode_groups(pv_ctx *ctx, const pv_layout *l, const float *T,
                                        const float *codebooks, const float *scales,
                                        const int32_t *group_idx, int64_t k, int32_t beam_width,
                                        uint16_t *codes, int64_t *num_changed)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_layout(ctx, l);
    if (st != PV_OK) return st;
    st = check_reencode_args(ctx, l, k, beam_width, T, codebooks, scales, codes);
    if (st != PV_OK) return st;
    if (k > 0 && !group_idx) return pv_fail(ctx, PV_ERR_INVALID_ARG, "group_idx is NULL");
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_reencode_dispatch(ctx, l, T, codebooks, scales, group_idx, k, beam_width, codes,
                                num_changed);
}

extern "C" pv_status pv_reencode_groups_stochastic(pv_ctx *ctx, const pv_layout *l, const float *T,
                                                   const float *codebooks, const float *scales,
                                                   const int32_t *group_idx, int64_t k,
                                                   int32_t power, uint64_t seed, uint16_t *codes,
                                                   int64_t *num_changed)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_layout(ctx, l);
    if (st != PV_OK) return st;
    st = check_reencode_args(ctx, l, k, 1, T, codebooks, scales, codes);
    if (st != PV_OK) return st;
    if (l->num_codebooks != 1)
        return pv_fail(ctx, PV_ERR_UNSUPPORTED, "stochastic rounding is defined for one codebook");
    if (power < 1 || power > 64)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "power = %d outside [1, 64]", (int)power);
    if (k > 0 && !group_idx) return pv_fail(ctx, PV_ERR_INVALID_ARG, "group_idx is NULL");
    PV_HIP(ctx, hipSetDevice(ctx->device));
    if (k > 0 && ctx->search_mode == 0 && pv_mfma_supported(l)) {
        // the matrix-core filter with the certificate taken from the second nearest; its first
        // kernel clears the counters
        st = pv_ensure(ctx, ctx->stats, 8 * sizeof(int64_t));
        if (st != PV_OK) return st;
        return pv_launch_mfma_search(ctx, l, T, codebooks, scales, group_idx, k, codes, num_changed,
                                     power, seed);
    }
    if (num_changed) {
        st = pv_launch_fill_i64(ctx, num_changed, 1, 0);
        if (st != PV_OK) return st;
    }
    if (k == 0) return PV_OK;
    return pv_launch_round_two_nearest(ctx, l, T, codebooks, scales, group_idx, k, power, seed,
                                       codes, num_changed);
}

extern "C" pv_status pv_reencode_trust_ratio(pv_ctx *ctx, const pv_layout *l, const float *T,
                                             const float *W, const float *codebooks,
                                             const float *scales, int64_t k_max, int64_t chunk,
                                             double ratio, int32_t beam_width, uint16_t *codes,
                                             int32_t *rank_idx, int64_t *num_applied,
                                             double *stats)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_layout(ctx, l);
    if (st != PV_OK) return st;
    st = check_reencode_args(ctx, l, k_max, beam_width, T, codebooks, scales, codes);
    if (st != PV_OK) return st;
    if (!W) return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (misaligned(W)) return pv_fail(ctx, PV_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (chunk < 1) return pv_fail(ctx, PV_ERR_INVALID_ARG, "chunk must be >= 1");
    if (!(ratio >= 0.0)) return pv_fail(ctx, PV_ERR_INVALID_ARG, "ratio must be >= 0");
    if (!num_applied) return pv_fail(ctx, PV_ERR_INVALID_ARG, "num_applied is NULL");
    if (pv_num_groups(l) == 0) return pv_launch_fill_i64(ctx, num_applied, 1, 0);
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_launch_trust_ratio(ctx, l, T, W, codebooks, scales, k_max, chunk, ratio, beam_width,
                                 codes, rank_idx, num_applied, stats);
}

extern "C" pv_status pv_codebook_grads(pv_ctx *ctx, const pv_layout *l, const float *G,
                                       const uint16_t *codes, const float *codebooks,
                                       const float *scales, float *grad_codebooks,
                                       float *grad_scales)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_layout(ctx, l);
    if (st != PV_OK) return st;
    if (!G || !codes || !codebooks || !scales || !grad_codebooks)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (misaligned(G) || misaligned(codebooks))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (l->group_size > 64)
        return pv_fail(ctx, PV_ERR_UNSUPPORTED, "codebook gradients support group_size <= 64");
    PV_HIP(ctx, hipSetDevice(ctx->device));
    if (pv_num_groups(l) == 0) {   // empty matrix: all sums are empty
        const size_t cb_bytes = sizeof(float) * (size_t)l->num_codebooks *
                                ((size_t)1 << l->nbits) * (size_t)l->group_size;
        pv_status fs = pv_launch_fill_f32(ctx, grad_codebooks, (int64_t)(cb_bytes / sizeof(float)), 0.0f);
        if (fs != PV_OK) return fs;
        if (grad_scales && l->out_features > 0) {
            fs = pv_launch_fill_f32(ctx, grad_scales, l->out_features, 0.0f);
            if (fs != PV_OK) return fs;
        }
        return PV_OK;
    }
    return pv_launch_codebook_grads(ctx, l, G, codes, codebooks, scales, grad_codebooks,
                                    grad_scales);
}

extern "C" pv_status pv_dequantize(pv_ctx *ctx, const pv_layout *l, const uint16_t *codes,
                                   const float *codebooks, const float *scales, float *W_out)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_layout(ctx, l);
    if (st != PV_OK) return st;
    if (!codes || !codebooks || !scales || !W_out)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (misaligned(codebooks) || misaligned(W_out))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (pv_num_groups(l) == 0) return PV_OK;
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_launch_dequantize(ctx, l, codes, codebooks, scales, W_out);
}

extern "C" pv_status pv_dequantize_groups(pv_ctx *ctx, const pv_layout *l, const uint16_t *codes,
                                          const float *codebooks, const float *scales,
                                          const int32_t *group_idx, int64_t k, float *W_out)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_layout(ctx, l);
    if (st != PV_OK) return st;
    if (k < 0 || k > pv_num_groups(l))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "k = %lld outside [0, %lld]", (long long)k,
                       (long long)pv_num_groups(l));
    if (!codes || !codebooks || !scales || !W_out)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (k > 0 && !group_idx) return pv_fail(ctx, PV_ERR_INVALID_ARG, "group_idx is NULL");
    if (misaligned(codebooks) || misaligned(W_out))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (k == 0) return PV_OK;
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_launch_dequantize_groups(ctx, l, codes, codebooks, scales, group_idx, k, W_out);
}

// ---------------------------------------------------------------- scalar grids

static pv_status check_scalar(pv_ctx *ctx, int64_t out_features, int64_t in_features,
                              int32_t block_size, int32_t nbits)
{
    if (out_features < 0 || in_features < 0) return pv_fail(ctx, PV_ERR_SHAPE, "negative matrix shape");
    if (block_size < 1 || in_features % block_size != 0)
        return pv_fail(ctx, PV_ERR_SHAPE, "in_features %lld is not a multiple of block_size %d",
                       (long long)in_features, block_size);
    if (nbits < 1 || nbits > 8) return pv_fail(ctx, PV_ERR_SHAPE, "nbits %d not in 1..8", nbits);
    if (out_features > 0 && in_features > (INT64_C(0x7fffffff) - 1) / out_features)
        return pv_fail(ctx, PV_ERR_SHAPE, "number of weights must be below 2^31");
    return PV_OK;
}

extern "C" pv_status pv_dequantize_scalar(pv_ctx *ctx, int64_t out_features, int64_t in_features,
                                          int32_t block_size, int32_t nbits, const uint8_t *codes,
                                          const float *scales, const float *zeros, float *W_out)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_scalar(ctx, out_features, in_features, block_size, nbits);
    if (st != PV_OK) return st;
    if (!codes || !scales || !zeros || !W_out)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (misaligned(W_out) || (reinterpret_cast<uintptr_t>(codes) & 3u))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "W_out must be 16-byte and codes 4-byte aligned");
    if (out_features * in_features == 0) return PV_OK;
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_launch_dequantize_scalar(ctx, out_features, in_features, block_size, codes, scales, zeros,
                                       W_out);
}

extern "C" pv_status pv_reencode_scalar(pv_ctx *ctx, int64_t out_features, int64_t in_features,
                                        int32_t block_size, int32_t nbits, const float *T,
                                        const float *scales, const float *zeros,
                                        const int32_t *weight_idx, int64_t k, uint8_t *codes,
                                        int64_t *num_changed)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = check_scalar(ctx, out_features, in_features, block_size, nbits);
    if (st != PV_OK) return st;
    if (k < 0 || k > out_features * in_features)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "k = %lld outside [0, %lld]", (long long)k,
                       (long long)(out_features * in_features));
    if (!T || !scales || !zeros || !codes) return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL tensor pointer");
    if (k > 0 && !weight_idx) return pv_fail(ctx, PV_ERR_INVALID_ARG, "weight_idx is NULL");
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_launch_reencode_scalar(ctx, out_features, in_features, block_size, nbits, T, scales, zeros,
                                     weight_idx, k, codes, num_changed);
}

// ---------------------------------------------------------------- instrumentation

extern "C" pv_status pv_set_search_mode(pv_ctx *ctx, int mode)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    if (mode != 0 && mode != 1) return pv_fail(ctx, PV_ERR_INVALID_ARG, "search mode must be 0 or 1");
    ctx->search_mode = mode;
    return PV_OK;
}

extern "C" pv_status pv_probe_copy(pv_ctx *ctx, void *dst, const void *src, int64_t bytes)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    if (!dst || !src) return pv_fail(ctx, PV_ERR_INVALID_ARG, "NULL pointer");
    if (bytes < 0 || (bytes & 15) || misaligned(dst) || misaligned(src))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "pointers and size must be multiples of 16 bytes");
    if (bytes / 16 / 256 >= (int64_t)1 << 31) return pv_fail(ctx, PV_ERR_INVALID_ARG, "size too large");
    if (bytes == 0) return PV_OK;
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_launch_probe_copy(ctx, dst, src, bytes);
}

extern "C" pv_status pv_probe_mfma_f16(pv_ctx *ctx, int64_t iters, float *sink, int64_t *waves_out)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    if (!sink) return pv_fail(ctx, PV_ERR_INVALID_ARG, "sink is NULL");
    if (iters < 4 || iters > ((int64_t)1 << 24) || (iters & 3))
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "iters must be a multiple of 4 in [4, 2^24]");
    PV_HIP(ctx, hipSetDevice(ctx->device));
    return pv_launch_probe_mfma(ctx, iters, sink, waves_out);
}

extern "C" pv_status pv_timing_enable(pv_ctx *ctx, int on)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    ctx->timing = on != 0;
    return PV_OK;
}

static pv_status drain_timers(pv_ctx *ctx)
{
    PV_HIP(ctx, hipSetDevice(ctx->device));
    PV_HIP(ctx, hipStreamSynchronize(ctx->stream));
    for (auto &t : ctx->timers) {
        for (size_t i = 0; i + 1 < t.pending.size(); i += 2) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, t.pending[i], t.pending[i + 1]) == hipSuccess) {
                t.total_ms += ms;
                t.launches += 1;
            } else {
                (void)hipGetLastError();
            }
            ctx->event_pool.push_back(t.pending[i]);
            ctx->event_pool.push_back(t.pending[i + 1]);
        }
        t.pending.clear();
    }
    return PV_OK;
}

extern "C" pv_status pv_timing_reset(pv_ctx *ctx)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    pv_status st = drain_timers(ctx);
    for (auto &t : ctx->timers) {
        t.total_ms = 0.0;
        t.launches = 0;
    }
    return st;
}

extern "C" pv_status pv_timing_read(pv_ctx *ctx, int kernel_id, double *total_ms, int64_t *launches)
{
    if (!ctx) return PV_ERR_INVALID_ARG;
    if (kernel_id < 0 || kernel_id >= PV_K_COUNT || !total_ms || !launches)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "bad timing query");
    pv_status st = drain_timers(ctx);
    if (st != PV_OK) return st;
    *total_ms = ctx->timers[kernel_id].total_ms;
    *launches = ctx->timers[kernel_id].launches;
    return PV_OK;
}

extern "C" pv_status pv_reencode_stats(pv_ctx *ctx, int64_t stats[4])
{
    if (!ctx || !stats) return PV_ERR_INVALID_ARG;
    for (int i = 0; i < 4; ++i) stats[i] = 0;
    if (!ctx->stats.ptr) return PV_OK;
    PV_HIP(ctx, hipSetDevice(ctx->device));
    PV_HIP(ctx, hipStreamSynchronize(ctx->stream));
    int64_t host[8];
    PV_HIP(ctx, hipMemcpy(host, ctx->stats.ptr, sizeof(host), hipMemcpyDeviceToHost));
    for (int i = 0; i < 4; ++i) stats[i] = host[i];
    if (ctx->rr_blocks_last > 0 && ctx->rr_counts.ptr) {
        // the one-codebook filter leaves its counters per block of the re-rank kernel:
        // {decided by the filter, codes changed, candidates evaluated, finished by a scan}
        std::vector<uint32_t> per_block((size_t)ctx->rr_blocks_last * 4);
        PV_HIP(ctx, hipMemcpy(per_block.data(), ctx->rr_counts.ptr, per_block.size() * sizeof(uint32_t),
                              hipMemcpyDeviceToHost));
        for (int b = 0; b < ctx->rr_blocks_last; ++b) {
            stats[0] += per_block[4 * (size_t)b + 0];
            stats[1] += per_block[4 * (size_t)b + 3];
            stats[2] += per_block[4 * (size_t)b + 2];
        }
    }
    return PV_OK;
}

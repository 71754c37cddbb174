// HBM-bound streaming kernels: target formation (Eq. 7) and dequantisation
// (Alg. 3 line 1).  One pass over memory each, 16-byte accesses per lane,
// consecutive lanes on consecutive addresses.
#include "pv_internal.h"

namespace {

constexpr int kBlock = 256;

// T = W - alpha * G with a single rounding per element.
// Each block covers kUnroll * kBlock consecutive pv_f4; the (< 4) tail floats
// are handled by the last thread that has no full vector.
constexpr int kUnroll = 4;

__global__ __launch_bounds__(kBlock) void k_encode_targets(const float *W,
                                                           const float *G,
                                                           float *T, int64_t n,
                                                           float alpha)
{
    const int64_t n4 = n >> 2;
    const pv_f4 *W4 = reinterpret_cast<const pv_f4 *>(W);
    const pv_f4 *G4 = reinterpret_cast<const pv_f4 *>(G);
    pv_f4 *T4 = reinterpret_cast<pv_f4 *>(T);
    const int64_t base = (int64_t)blockIdx.x * (kUnroll * kBlock) + threadIdx.x;
    pv_f4 w[kUnroll], g[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        int64_t i = base + (int64_t)u * kBlock;
        if (i < n4) {
            w[u] = __builtin_nontemporal_load(&W4[i]);
            g[u] = __builtin_nontemporal_load(&G4[i]);
        }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        int64_t i = base + (int64_t)u * kBlock;
        if (i < n4) {
            pv_f4 t;
            t.x = fmaf(-alpha, g[u].x, w[u].x);
            t.y = fmaf(-alpha, g[u].y, w[u].y);
            t.z = fmaf(-alpha, g[u].z, w[u].z);
            t.w = fmaf(-alpha, g[u].w, w[u].w);
            T4[i] = t;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0)
        for (int64_t i = n4 << 2; i < n; ++i) T[i] = fmaf(-alpha, G[i], W[i]);
}

// (the Adam arithmetic itself, pv_adam_t / pv_adam_one, is declared with the internal launchers)
constexpr int kAdamUnroll = 2;

__global__ __launch_bounds__(kBlock) void k_encode_targets_adam(const float *W, const float *G,
                                                                float *m, float *v, float *T,
                                                                int64_t n, pv_adam_t a)
{
    const int64_t n4 = n >> 2;
    const pv_f4 *W4 = reinterpret_cast<const pv_f4 *>(W);
    const pv_f4 *G4 = reinterpret_cast<const pv_f4 *>(G);
    pv_f4 *M4 = reinterpret_cast<pv_f4 *>(m);
    pv_f4 *V4 = reinterpret_cast<pv_f4 *>(v);
    pv_f4 *T4 = reinterpret_cast<pv_f4 *>(T);
    const int64_t base = (int64_t)blockIdx.x * (kAdamUnroll * kBlock) + threadIdx.x;
    pv_f4 w[kAdamUnroll], g[kAdamUnroll], mm[kAdamUnroll], vv[kAdamUnroll];
#pragma unroll
    for (int u = 0; u < kAdamUnroll; ++u) {
        int64_t i = base + (int64_t)u * kBlock;
        if (i < n4) {
            w[u] = __builtin_nontemporal_load(&W4[i]);
            g[u] = __builtin_nontemporal_load(&G4[i]);
            mm[u] = __builtin_nontemporal_load(&M4[i]);
            vv[u] = __builtin_nontemporal_load(&V4[i]);
        }
    }
#pragma unroll
    for (int u = 0; u < kAdamUnroll; ++u) {
        int64_t i = base + (int64_t)u * kBlock;
        if (i < n4) {
            pv_f4 t;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float mi = mm[u][e], vi = vv[u][e];
                t[e] = pv_adam_one(w[u][e], g[u][e], mi, vi, a);
                mm[u][e] = mi;
                vv[u][e] = vi;
            }
            M4[i] = mm[u];
            V4[i] = vv[u];
            T4[i] = t;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0)
        for (int64_t i = n4 << 2; i < n; ++i) {
            float mi = m[i], vi = v[i];
            T[i] = pv_adam_one(W[i], G[i], mi, vi, a);
            m[i] = mi;
            v[i] = vi;
        }
}

// One thread per VEC consecutive weights of a group: reads the group's code(s),
// gathers VEC floats of each codeword (the codebook stays in L2), adds them in
// codebook order, multiplies by the row scale, writes VEC floats.
// VEC == 4: a thread takes kDeqAhead vectors a block-width apart and has all their codes, then
// all their codewords, in flight together (two round trips per thread whatever the count:
// with one vector a thread the kernel is bound by those trips, not by the 4 bytes a weight
// it writes).
#ifndef PV_DEQ_AHEAD
#define PV_DEQ_AHEAD 2   // measured: 1 leaves two-codebook layouts bound by round trips, 4 and 8 lose to register pressure
#endif
constexpr int kDeqAhead = PV_DEQ_AHEAD;
// PARTS: 16-byte vectors per group when known at compile time (1, 2 or 4), else 0
template <int VEC, int PARTS>
__global__ __launch_bounds__(kBlock) void k_dequantize(const uint16_t *__restrict__ codes,
                                                       const float *__restrict__ codebooks,
                                                       const float *__restrict__ scales,
                                                       float *__restrict__ W_out, int64_t total,
                                                       int g, int M, int nbits, int gpr,
                                                       double inv_gpr)
{
    const unsigned mask = (1u << nbits) - 1u;
    const int64_t csize = (int64_t)1 << nbits;
    if constexpr (VEC == 4) {
        const int parts = PARTS > 0 ? PARTS : g / 4;
        const pv_f4 *cb4 = reinterpret_cast<const pv_f4 *>(codebooks);
        const int64_t first = (int64_t)blockIdx.x * (kBlock * kDeqAhead) + threadIdx.x;
        int64_t at[kDeqAhead];
        int q[kDeqAhead];
        unsigned code[kDeqAhead];
        float s[kDeqAhead];
        const uint16_t *cp[kDeqAhead];
#pragma unroll
        for (int u = 0; u < kDeqAhead; ++u) {
            const int64_t idx = first + (int64_t)u * kBlock;
            at[u] = idx < total ? idx : total - 1;
            const int n = (int)(at[u] / parts);
            q[u] = (int)(at[u] - (int64_t)n * parts);
            cp[u] = codes + (int64_t)n * M;
            code[u] = cp[u][0] & mask;
            s[u] = scales[pv_row_of((unsigned)n, inv_gpr)];
        }
        pv_f4 acc[kDeqAhead];
#pragma unroll
        for (int u = 0; u < kDeqAhead; ++u) acc[u] = cb4[((int64_t)code[u] * g) / 4 + q[u]];
        for (int m = 1; m < M; ++m) {
            pv_f4 c[kDeqAhead];
#pragma unroll
            for (int u = 0; u < kDeqAhead; ++u)
                c[u] = cb4[((m * csize + (cp[u][m] & mask)) * g) / 4 + q[u]];
#pragma unroll
            for (int u = 0; u < kDeqAhead; ++u) {
                acc[u].x = acc[u].x + c[u].x;
                acc[u].y = acc[u].y + c[u].y;
                acc[u].z = acc[u].z + c[u].z;
                acc[u].w = acc[u].w + c[u].w;
            }
        }
#pragma unroll
        for (int u = 0; u < kDeqAhead; ++u) {
            pv_f4 out;
            out.x = s[u] * acc[u].x;
            out.y = s[u] * acc[u].y;
            out.z = s[u] * acc[u].z;
            out.w = s[u] * acc[u].w;
            if (first + (int64_t)u * kBlock < total)
                __builtin_nontemporal_store(out, &reinterpret_cast<pv_f4 *>(W_out)[at[u]]);
        }
    } else {
        const int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
        if (idx >= total) return;
        const int n = (int)(idx / g);
        const int q = (int)(idx - (int64_t)n * g);
        const float s = scales[n / gpr];
        const uint16_t *cp = codes + (int64_t)n * M;
        float acc = codebooks[(int64_t)(cp[0] & mask) * g + q];
        for (int m = 1; m < M; ++m) acc = acc + codebooks[(m * csize + (cp[m] & mask)) * g + q];
        W_out[idx] = s * acc;
    }
}

// One codebook, g = 8, whole chunks of 256 groups per wave: a lane loads four codes with one
// 8-byte load (a wave's codes are 512 contiguous bytes instead of eight rounds of 2-byte
// loads), the codes reach the lanes that need them through wave shuffles, and the eight
// codeword gathers of a lane are in flight together.  Lane pairs share a group as above, so
// every store instruction still writes 1 KiB of contiguous weights.
constexpr int kWideRounds = 8;   // rounds of 64 vectors a wave: four codes a lane
__global__ __launch_bounds__(kBlock) void k_dequantize_g8_wide(const uint16_t *__restrict__ codes,
                                                              const float *__restrict__ codebooks,
                                                              const float *__restrict__ scales,
                                                              float *__restrict__ W_out, int nbits,
                                                              double inv_gpr)
{
    constexpr int kRounds = kWideRounds;                // 64 vectors (32 groups) of the wave each
    constexpr int kGroups = 32 * kRounds;               // groups per wave
    static_assert(kRounds == 8, "four codes a lane");
    const unsigned mask = (1u << nbits) - 1u;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t g0 = ((int64_t)blockIdx.x * (kBlock / 64) + wave) * kGroups;   // first group of the wave
    const uint2 four = *reinterpret_cast<const uint2 *>(codes + g0 + 4 * lane);
    const pv_f4 *cb4 = reinterpret_cast<const pv_f4 *>(codebooks);
    pv_f4 *out4 = reinterpret_cast<pv_f4 *>(W_out) + g0 * 2;
    const int half = lane & 1, gl = lane >> 1;          // vector of the group, group of the round
    pv_f4 acc[kRounds];
    float sc[kRounds];
#pragma unroll
    for (int k = 0; k < kRounds; ++k) {
        // group 32 k + gl of the wave: code number (gl & 3) of lane 8 k + gl / 4
        const int src = 8 * k + (gl >> 2);
        const unsigned lo = (unsigned)__shfl((int)four.x, src), hi = (unsigned)__shfl((int)four.y, src);
        const unsigned word = (gl & 2) ? hi : lo;
        const unsigned code = ((gl & 1) ? word >> 16 : word) & 0xFFFFu & mask;
        acc[k] = cb4[(int64_t)code * 2 + half];
        sc[k] = scales[pv_row_of((unsigned)(g0 + 32 * k + gl), inv_gpr)];
    }
#pragma unroll
    for (int k = 0; k < kRounds; ++k) {
        pv_f4 o;
        o.x = sc[k] * acc[k].x;
        o.y = sc[k] * acc[k].y;
        o.z = sc[k] * acc[k].z;
        o.w = sc[k] * acc[k].w;
        __builtin_nontemporal_store(o, &out4[64 * k + lane]);
    }
}

// The same for a list of groups only (the groups a V step re-encoded): every other weight of
// W_out keeps its value.  One thread per weight vector of a listed group.
template <int VEC>
__global__ __launch_bounds__(kBlock) void k_dequantize_groups(const uint16_t *__restrict__ codes,
                                                              const float *__restrict__ codebooks,
                                                              const float *__restrict__ scales,
                                                              const int32_t *__restrict__ group_idx,
                                                              int64_t total, float *__restrict__ W_out,
                                                              int g, int M, int nbits, int gpr, int N)
{
    const int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= total) return;
    const int parts = g / VEC;
    const int64_t j = idx / parts;
    const int q = (int)(idx - j * parts);
    const int n = group_idx[j];
    if (n < 0 || n >= N) return;
    const unsigned mask = (1u << nbits) - 1u;
    const int64_t csize = (int64_t)1 << nbits;
    const float s = scales[n / gpr];
    const uint16_t *cp = codes + (int64_t)n * M;
    if constexpr (VEC == 4) {
        const pv_f4 *cb4 = reinterpret_cast<const pv_f4 *>(codebooks);
        pv_f4 acc = cb4[((int64_t)(cp[0] & mask) * g) / 4 + q];
        for (int m = 1; m < M; ++m) {
            pv_f4 c = cb4[((m * csize + (cp[m] & mask)) * g) / 4 + q];
            acc.x = acc.x + c.x;
            acc.y = acc.y + c.y;
            acc.z = acc.z + c.z;
            acc.w = acc.w + c.w;
        }
        pv_f4 out;
        out.x = s * acc.x;
        out.y = s * acc.y;
        out.z = s * acc.z;
        out.w = s * acc.w;
        reinterpret_cast<pv_f4 *>(W_out)[((int64_t)n * g) / 4 + q] = out;
    } else {
        float acc = codebooks[(int64_t)(cp[0] & mask) * g + q];
        for (int m = 1; m < M; ++m) acc = acc + codebooks[(m * csize + (cp[m] & mask)) * g + q];
        W_out[(int64_t)n * g + q] = s * acc;
    }
}

// plain streaming copy, one 16-byte vector per thread (the ceiling the streaming kernels of
// this file are compared with)
__global__ __launch_bounds__(kBlock) void k_probe_copy(const pv_f4 *__restrict__ src,
                                                       pv_f4 *__restrict__ dst, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) __builtin_nontemporal_store(__builtin_nontemporal_load(&src[i]), &dst[i]);
}

// p[0 .. n) = v and, when q is given, *q = v (the counters of a call and the caller's
// num_changed in one launch)
__global__ void k_fill_i64(int64_t *p, int64_t n, int64_t v, int64_t *q)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
    if (q && i == 0) *q = v;
}

// p[0 .. n) = v (a kernel rather than a memset node: callers may capture the stream in a graph)
__global__ __launch_bounds__(kBlock) void k_fill_f32(float *p, int64_t n, float v)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) p[i] = v;
}

}  // namespace

pv_status pv_launch_encode_targets(pv_ctx *ctx, const float *W, const float *G, float alpha,
                                   float *T, int64_t n)
{
    pv_timed t(ctx, PV_K_ENCODE_TARGETS);
    int64_t n4 = n >> 2;
    int64_t blocks = (n4 + kUnroll * kBlock - 1) / (kUnroll * kBlock);
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_encode_targets, dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream, W, G,
                       T, n, alpha);
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

pv_adam_t pv_make_adam(int64_t step, float lr, float beta1, float beta2, float eps)
{
    auto powi = [](double b, int64_t t) {   // b^t by repeated squaring, IEEE double products
        double r = 1.0;
        while (t > 0) {
            if (t & 1) r = r * b;
            b = b * b;
            t >>= 1;
        }
        return r;
    };
    pv_adam_t a;
    a.lr = lr;
    a.b1 = beta1;
    a.b2 = beta2;
    a.omb1 = 1.0f - beta1;
    a.omb2 = 1.0f - beta2;
    a.c1 = (float)(1.0 - powi((double)beta1, step));
    a.c2 = (float)(1.0 - powi((double)beta2, step));
    a.eps = eps;
    return a;
}

pv_status pv_launch_encode_targets_adam(pv_ctx *ctx, const float *W, const float *G, float *m,
                                        float *v, int64_t step, float lr, float beta1, float beta2,
                                        float eps, float *T, int64_t n)
{
    pv_timed t(ctx, PV_K_ENCODE_TARGETS);
    const pv_adam_t a = pv_make_adam(step, lr, beta1, beta2, eps);
    int64_t n4 = n >> 2;
    int64_t blocks = (n4 + kAdamUnroll * kBlock - 1) / (kAdamUnroll * kBlock);
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_encode_targets_adam, dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream,
                       W, G, m, v, T, n, a);
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

pv_status pv_launch_dequantize(pv_ctx *ctx, const pv_layout *l, const uint16_t *codes,
                               const float *codebooks, const float *scales, float *W_out)
{
    pv_timed t(ctx, PV_K_DEQUANTIZE);
    const int g = l->group_size;
    const int64_t N = pv_num_groups(l);
    const int gpr = (int)(l->in_features / g);
    if (g % 4 == 0) {
        int64_t total = N * (g / 4);
        int64_t blocks = (total + kBlock * kDeqAhead - 1) / (kBlock * kDeqAhead);
#define PV_DEQ(P_)                                                                               \
    hipLaunchKernelGGL((k_dequantize<4, P_>), dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream, \
                       codes, codebooks, scales, W_out, total, g, l->num_codebooks, l->nbits,   \
                       gpr, 1.0 / (double)gpr)
        constexpr int kWideGroups = (kBlock / 64) * 32 * kWideRounds;      // groups per block of the wide kernel
        if (g == 8 && l->num_codebooks == 1 && N % kWideGroups == 0 && N < (INT64_C(1) << 31) &&
            (reinterpret_cast<uintptr_t>(codes) & 7u) == 0)
            hipLaunchKernelGGL(k_dequantize_g8_wide, dim3((unsigned)(N / kWideGroups)), dim3(kBlock), 0,
                               ctx->stream, codes, codebooks, scales, W_out, l->nbits, 1.0 / (double)gpr);
        else if (g == 8) PV_DEQ(2);
        else if (g == 16) PV_DEQ(4);
        else if (g == 4) PV_DEQ(1);
        else PV_DEQ(0);
#undef PV_DEQ
    } else {
        int64_t total = N * g;
        int64_t blocks = (total + kBlock - 1) / kBlock;
        hipLaunchKernelGGL((k_dequantize<1, 0>), dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream,
                           codes, codebooks, scales, W_out, total, g, l->num_codebooks, l->nbits,
                           gpr, 1.0 / (double)gpr);
    }
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

pv_status pv_launch_dequantize_groups(pv_ctx *ctx, const pv_layout *l, const uint16_t *codes,
                                      const float *codebooks, const float *scales,
                                      const int32_t *group_idx, int64_t k, float *W_out)
{
    pv_timed t(ctx, PV_K_DEQUANTIZE);
    const int g = l->group_size;
    const int gpr = (int)(l->in_features / g);
    const int N = (int)pv_num_groups(l);
    if (g % 4 == 0) {
        const int64_t total = k * (g / 4);
        hipLaunchKernelGGL(k_dequantize_groups<4>, dim3((unsigned)((total + kBlock - 1) / kBlock)),
                           dim3(kBlock), 0, ctx->stream, codes, codebooks, scales, group_idx, total,
                           W_out, g, l->num_codebooks, l->nbits, gpr, N);
    } else {
        const int64_t total = k * g;
        hipLaunchKernelGGL(k_dequantize_groups<1>, dim3((unsigned)((total + kBlock - 1) / kBlock)),
                           dim3(kBlock), 0, ctx->stream, codes, codebooks, scales, group_idx, total,
                           W_out, g, l->num_codebooks, l->nbits, gpr, N);
    }
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

pv_status pv_launch_probe_copy(pv_ctx *ctx, void *dst, const void *src, int64_t bytes)
{
    pv_timed t(ctx, PV_K_PROBE_COPY);
    const int64_t n = bytes / 16;
    const int64_t blocks = (n + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(k_probe_copy, dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream,
                       static_cast<const pv_f4 *>(src), static_cast<pv_f4 *>(dst), n);
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

pv_status pv_launch_fill_f32(pv_ctx *ctx, float *p, int64_t n, float value)
{
    if (n <= 0) return PV_OK;
    int64_t blocks = (n + kBlock - 1) / kBlock;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(k_fill_f32, dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream, p, n, value);
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

pv_status pv_launch_fill_i64(pv_ctx *ctx, int64_t *p, int64_t n, int64_t value, int64_t *also)
{
    hipLaunchKernelGGL(k_fill_i64, dim3((unsigned)((n + 63) / 64)), dim3(64), 0, ctx->stream, p, n,
                       value, also);
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

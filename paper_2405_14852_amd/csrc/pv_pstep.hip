// Gradients of the continuous parameters for the P step (Alg. 3, P step: "backprop";
// App. K: codebooks and per-channel scales): the chain rule through
//     W[o, j*g + i] = s_o * sum_m C_m[b(o,j,m), i]
// applied to G = d phi / d W:
//     d phi / d C_m[c, i] = sum over groups n = (o, j) with b(o,j,m) = c of  s_o * G[n, i]
//     d phi / d s_o       = sum_j sum_i G[o, j*g + i] * (C_0[b_0, i] + C_1[b_1, i] + ...)
//
// The codebook gradient is a scatter-add of N * g values into 2^B * g sums.  Atomics
// would serialise on popular codewords and give run-dependent roundings; instead the
// groups are SORTED by code (stable radix sort of 16-bit keys: equal codes stay in
// ascending group order) and every codeword's segment is summed by g lanes in that
// order, in double, with exact products - the same sum, in the same order, as a plain
// loop over the groups.  Segments longer than kLong groups are cut into pieces of kLong,
// summed by separate teams and added in piece order (a different association:
// reproducible, but no longer the sequential order).  Small codebooks take another route
// (k_pg_small below).  The scale gradient is one block-wide tree sum per row.
#include <hipcub/hipcub.hpp>

#include "pv_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kLong = 128;    // groups per piece: a segment up to this long is summed by one team alone

__global__ __launch_bounds__(kBlock) void k_pg_keys(const uint16_t *__restrict__ codes, int64_t N,
                                                    int M, int m, unsigned mask,
                                                    uint16_t *__restrict__ keys,
                                                    int32_t *__restrict__ vals)
{
    const int64_t n = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (n >= N) return;
    keys[n] = (uint16_t)(codes[n * M + m] & mask);
    vals[n] = (int32_t)n;
}

// start[c] = first position of code c in the sorted order (= position of the next present
// code when c is absent); start[csize] = N
__global__ __launch_bounds__(kBlock) void k_pg_starts(const uint16_t *__restrict__ sorted, int64_t N,
                                                      int csize, int32_t *__restrict__ start)
{
    const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (r >= N) return;
    const int cur = sorted[r];
    const int prev = r == 0 ? -1 : (int)sorted[r - 1];
    for (int c = prev + 1; c <= cur; ++c) start[c] = (int32_t)r;
    if (r == N - 1)
        for (int c = cur + 1; c <= csize; ++c) start[c] = (int32_t)N;
}

// Sum of s_o * G[n, i] over the sorted positions [lo, hi), in order, four groups in flight.
__device__ __forceinline__ double segment_sum(const int32_t *__restrict__ order,
                                              const float *__restrict__ G,
                                              const float *__restrict__ scales, int gpr, int g,
                                              int i, int lo, int hi)
{
    double acc = 0.0;
    int r = lo;
    for (; r + 4 <= hi; r += 4) {
        int n[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) n[u] = order[r + u];
        float gv[4], sv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            gv[u] = G[(int64_t)n[u] * g + i];
            sv[u] = scales[n[u] / gpr];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = acc + (double)sv[u] * (double)gv[u];
    }
    for (; r < hi; ++r) {
        const int n = order[r];
        acc = acc + (double)scales[n / gpr] * (double)G[(int64_t)n * g + i];
    }
    return acc;
}

// extra[c] = number of pieces of the codewords before c beyond their first ones (an exclusive
// prefix sum, extra[csize] = total), by the library's device scan over this functor.  A
// segment of len groups has ceil(len / kLong) pieces.
struct extra_pieces {
    const int32_t *start;
    int csize;
    __host__ __device__ int operator()(int c) const
    {
        if (c >= csize) return 0;
        const int len = start[c + 1] - start[c];
        return len > kLong ? (len + kLong - 1) / kLong - 1 : 0;
    }
};
typedef hipcub::TransformInputIterator<int, extra_pieces, hipcub::CountingInputIterator<int>> extra_iter;

// TEAM lanes per work item (the group size rounded up to a power of two); lane i sums
// dimension i.  Items [0, csize): the first piece of every codeword - written straight to
// the output when it is the only one.  Items csize + e: extra piece e (its codeword is found
// by bisection over the prefix `extra`); partial sums go to `partial` for k_pg_combine.
template <int TEAM>
__global__ __launch_bounds__(kBlock) void k_pg_accumulate(const int32_t *__restrict__ start,
                                                          const int32_t *__restrict__ extra,
                                                          const int32_t *__restrict__ order,
                                                          const float *__restrict__ G,
                                                          const float *__restrict__ scales,
                                                          int gpr, int g, int csize,
                                                          double *__restrict__ first_partial,
                                                          double *__restrict__ partial,
                                                          float *__restrict__ out)
{
    constexpr int kTeams = kBlock / TEAM;
    const int i = threadIdx.x % TEAM;
    const int64_t item = (int64_t)blockIdx.x * kTeams + threadIdx.x / TEAM;
    if (i >= g) return;
    if (item < csize) {
        const int c = (int)item;
        const int lo = start[c], hi = start[c + 1];
        const bool single = hi - lo <= kLong;
        const double acc = segment_sum(order, G, scales, gpr, g, i, lo, single ? hi : lo + kLong);
        if (single) out[(int64_t)c * g + i] = (float)acc;
        else first_partial[(int64_t)c * g + i] = acc;
        return;
    }
    const int e = (int)(item - csize);
    if (e >= extra[csize]) return;
    int lo_c = 0, hi_c = csize;               // largest c with extra[c] <= e
    while (hi_c - lo_c > 1) {
        const int mid = (lo_c + hi_c) >> 1;
        if (extra[mid] <= e) lo_c = mid;
        else hi_c = mid;
    }
    const int c = lo_c;
    const int piece = e - extra[c] + 1;
    const int lo = start[c] + piece * kLong;
    const int end = start[c + 1];
    const int hi = lo + kLong < end ? lo + kLong : end;
    partial[(int64_t)e * g + i] = segment_sum(order, G, scales, gpr, g, i, lo, hi);
}

// codewords with several pieces: the piece sums added in piece order
__global__ __launch_bounds__(kBlock) void k_pg_combine(const int32_t *__restrict__ extra, int g,
                                                       int csize,
                                                       const double *__restrict__ first_partial,
                                                       const double *__restrict__ partial,
                                                       float *__restrict__ out)
{
    const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (t >= (int64_t)csize * g) return;
    const int c = (int)(t / g), i = (int)(t % g);
    const int e0 = extra[c], e1 = extra[c + 1];
    if (e1 == e0) return;
    double acc = first_partial[t];
    int e = e0;
    for (; e + 4 <= e1; e += 4) {             // four loads in flight, added in piece order
        double p[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) p[u] = partial[(int64_t)(e + u) * g + i];
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = acc + p[u];
    }
    for (; e < e1; ++e) acc = acc + partial[(int64_t)e * g + i];
    out[t] = (float)acc;
}

// Small codebooks (all M * 2^B * g sums fit one block's LDS as doubles): every codeword is
// shared by thousands of groups, so sorting buys nothing.  Each block sweeps a contiguous
// range of groups once, 16 bytes of G per thread, and adds s_o * G into its own LDS table
// with LDS atomics; the tables are then added up over the blocks in block order.  The order
// of the atomic additions inside a block is not fixed, so the double sums may differ in
// their last bits from run to run (the fp32 results almost never do).
__global__ __launch_bounds__(kBlock) void k_pg_small(const float *__restrict__ G,
                                                     const uint16_t *__restrict__ codes,
                                                     const float *__restrict__ scales, int64_t N,
                                                     int64_t per_block, int g, int M, int nbits,
                                                     int gpr, double *__restrict__ partial)
{
    extern __shared__ double tab[];                     // [M][2^B][g]
    const int csize = 1 << nbits;
    const unsigned mask = (unsigned)csize - 1u;
    const int entries = M * csize * g;
    for (int e = threadIdx.x; e < entries; e += kBlock) tab[e] = 0.0;
    __syncthreads();
    const int vpg = g / 4;                              // 16-byte vectors per group
    const int64_t lo = (int64_t)blockIdx.x * per_block;
    const int64_t hi = lo + per_block < N ? lo + per_block : N;
    const pv_f4 *G4 = reinterpret_cast<const pv_f4 *>(G);
    for (int64_t v = lo * vpg + threadIdx.x; v < hi * vpg; v += kBlock) {
        const int64_t n = v / vpg;
        const int q4 = (int)(v - n * vpg);
        const pv_f4 gv = __builtin_nontemporal_load(&G4[v]);
        const double s = (double)scales[n / gpr];
        for (int m = 0; m < M; ++m) {
            const int c = codes[n * M + m] & mask;
            double *row = tab + ((int64_t)m * csize + c) * g + q4 * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) atomicAdd(&row[e], s * (double)gv[e]);
        }
    }
    __syncthreads();
    double *out = partial + (int64_t)blockIdx.x * entries;
    for (int e = threadIdx.x; e < entries; e += kBlock) out[e] = tab[e];
}

// sums the per-block tables in block order, rounds once
__global__ __launch_bounds__(kBlock) void k_pg_small_final(const double *__restrict__ partial,
                                                           int blocks, int entries,
                                                           float *__restrict__ out)
{
    const int e = blockIdx.x * kBlock + threadIdx.x;
    if (e >= entries) return;
    double acc = 0.0;
    int b = 0;
    for (; b + 4 <= blocks; b += 4) {
        double p[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) p[u] = partial[(int64_t)(b + u) * entries + e];
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = acc + p[u];
    }
    for (; b < blocks; ++b) acc = acc + partial[(int64_t)b * entries + e];
    out[e] = (float)acc;
}

// one block per output row; VEC: g % 4 == 0, a thread takes 16-byte vectors
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_pg_scales(const float *__restrict__ G,
                                                      const uint16_t *__restrict__ codes,
                                                      const float *__restrict__ codebooks, int g,
                                                      int M, int nbits, int gpr,
                                                      float *__restrict__ grad_scales)
{
    __shared__ double tmp[kBlock / 64];
    const int64_t o = blockIdx.x;
    const int64_t csize = (int64_t)1 << nbits;
    const unsigned mask = (unsigned)csize - 1u;
    const int64_t in_features = (int64_t)gpr * g;
    double acc = 0.0;
    if constexpr (VEC) {
        const int vpg = g / 4;                                  // vectors per group
        const int64_t nv = in_features / 4;
        const pv_f4 *G4 = reinterpret_cast<const pv_f4 *>(G + o * in_features);
        const pv_f4 *C4 = reinterpret_cast<const pv_f4 *>(codebooks);
        for (int64_t e = threadIdx.x; e < nv; e += kBlock) {
            const int64_t n = o * gpr + e / vpg;
            const int q4 = (int)(e % vpg);
            const pv_f4 gv = __builtin_nontemporal_load(&G4[e]);
            pv_f4 q = C4[((int64_t)(codes[n * M] & mask) * g) / 4 + q4];
            for (int m = 1; m < M; ++m) {
                const pv_f4 c = C4[((m * csize + (codes[n * M + m] & mask)) * g) / 4 + q4];
                q.x = q.x + c.x;
                q.y = q.y + c.y;
                q.z = q.z + c.z;
                q.w = q.w + c.w;
            }
            // per thread the terms are added in index order
            acc = acc + (double)gv.x * (double)q.x;
            acc = acc + (double)gv.y * (double)q.y;
            acc = acc + (double)gv.z * (double)q.z;
            acc = acc + (double)gv.w * (double)q.w;
        }
    } else {
        for (int64_t e = threadIdx.x; e < in_features; e += kBlock) {
            const int64_t n = o * gpr + e / g;
            const int i = (int)(e % g);
            float q = codebooks[(int64_t)(codes[n * M] & mask) * g + i];
            for (int m = 1; m < M; ++m)
                q = q + codebooks[(m * csize + (codes[n * M + m] & mask)) * g + i];
            acc = acc + (double)G[o * in_features + e] * (double)q;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc = acc + __shfl_down(acc, off);
    if ((threadIdx.x & 63) == 0) tmp[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < kBlock / 64; ++w) t = t + tmp[w];
        grad_scales[o] = (float)t;
    }
}

inline size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

pv_status pv_launch_codebook_grads(pv_ctx *ctx, const pv_layout *l, const float *G,
                                   const uint16_t *codes, const float *codebooks,
                                   const float *scales, float *grad_codebooks, float *grad_scales)
{
    const int64_t N = pv_num_groups(l);
    const int g = l->group_size, M = l->num_codebooks;
    const int gpr = (int)(l->in_features / g);
    const int csize = 1 << l->nbits;
    const unsigned mask = (unsigned)csize - 1u;
    hipStream_t sm = ctx->stream;

    // small codebooks: per-block LDS tables instead of a sort
    const int64_t entries = (int64_t)M * csize * g;
    if (g % 4 == 0 && entries * 8 <= 64 * 1024 && N / csize >= 64) {
        int blocks = (int)((N + 4095) / 4096);
        if (blocks > 512) blocks = 512;
        if (blocks < 1) blocks = 1;
        const int64_t per_block = (N + blocks - 1) / blocks;
        pv_status st2 = pv_ensure(ctx, ctx->pstep, (size_t)blocks * entries * 8);
        if (st2 != PV_OK) return st2;
        double *partial = static_cast<double *>(ctx->pstep.ptr);
        pv_timed t(ctx, PV_K_PSTEP);
        hipLaunchKernelGGL(k_pg_small, dim3(blocks), dim3(kBlock), (size_t)entries * 8, sm, G, codes,
                           scales, N, per_block, g, M, l->nbits, gpr, partial);
        hipLaunchKernelGGL(k_pg_small_final, dim3((unsigned)((entries + kBlock - 1) / kBlock)),
                           dim3(kBlock), 0, sm, partial, blocks, (int)entries, grad_codebooks);
        if (grad_scales) {
            hipLaunchKernelGGL(k_pg_scales<true>, dim3((unsigned)l->out_features), dim3(kBlock), 0, sm,
                               G, codes, codebooks, g, M, l->nbits, gpr, grad_scales);
        }
        PV_HIP(ctx, hipGetLastError());
        return PV_OK;
    }

    size_t sort_bytes = 0, scan_bytes = 0;
    PV_HIP(ctx, hipcub::DeviceRadixSort::SortPairs(nullptr, sort_bytes, (const uint16_t *)nullptr,
                                                   (uint16_t *)nullptr, (const int32_t *)nullptr,
                                                   (int32_t *)nullptr, (int)N, 0, l->nbits, sm));
    PV_HIP(ctx, hipcub::DeviceScan::ExclusiveSum(
                    nullptr, scan_bytes,
                    extra_iter(hipcub::CountingInputIterator<int>(0), extra_pieces{nullptr, csize}),
                    (int32_t *)nullptr, csize + 1, sm));
    if (scan_bytes > sort_bytes) sort_bytes = scan_bytes;   // one temporary area serves both
    const size_t nn = (size_t)N;
    const int64_t max_extra = N / kLong + 1;
    size_t o_keys = 0;
    size_t o_keys2 = o_keys + align_up(nn * 2);
    size_t o_vals = o_keys2 + align_up(nn * 2);
    size_t o_order = o_vals + align_up(nn * 4);
    size_t o_start = o_order + align_up(nn * 4);
    size_t o_extra = o_start + align_up((size_t)(csize + 1) * 4);
    size_t o_first = o_extra + align_up((size_t)(csize + 1) * 4);
    size_t o_part = o_first + align_up((size_t)csize * g * 8);
    size_t o_sort = o_part + align_up((size_t)max_extra * g * 8);
    size_t total = o_sort + align_up(sort_bytes);
    pv_status st = pv_ensure(ctx, ctx->pstep, total);
    if (st != PV_OK) return st;
    char *base = static_cast<char *>(ctx->pstep.ptr);
    uint16_t *keys = reinterpret_cast<uint16_t *>(base + o_keys);
    uint16_t *keys2 = reinterpret_cast<uint16_t *>(base + o_keys2);
    int32_t *vals = reinterpret_cast<int32_t *>(base + o_vals);
    int32_t *order = reinterpret_cast<int32_t *>(base + o_order);
    int32_t *start = reinterpret_cast<int32_t *>(base + o_start);
    int32_t *extra = reinterpret_cast<int32_t *>(base + o_extra);
    double *first_partial = reinterpret_cast<double *>(base + o_first);
    double *partial = reinterpret_cast<double *>(base + o_part);
    void *sort_tmp = base + o_sort;

    pv_timed t(ctx, PV_K_PSTEP);
    const unsigned nblocks = (unsigned)((N + kBlock - 1) / kBlock);
    int team = 1;
    while (team < g) team <<= 1;      // lanes per work item (g <= 64 checked by the caller)
    const int teams_per_block = kBlock / team;
    const unsigned ablocks = (unsigned)((csize + max_extra + teams_per_block - 1) / teams_per_block);
    const unsigned cblocks = (unsigned)(((int64_t)csize * g + kBlock - 1) / kBlock);
    for (int m = 0; m < M; ++m) {
        hipLaunchKernelGGL(k_pg_keys, dim3(nblocks), dim3(kBlock), 0, sm, codes, N, M, m, mask, keys,
                           vals);
        PV_HIP(ctx, hipcub::DeviceRadixSort::SortPairs(sort_tmp, sort_bytes, keys, keys2, vals, order,
                                                       (int)N, 0, l->nbits, sm));
        hipLaunchKernelGGL(k_pg_starts, dim3(nblocks), dim3(kBlock), 0, sm, keys2, N, csize, start);
        PV_HIP(ctx, hipcub::DeviceScan::ExclusiveSum(
                        sort_tmp, sort_bytes,
                        extra_iter(hipcub::CountingInputIterator<int>(0), extra_pieces{start, csize}),
                        extra, csize + 1, sm));
        float *out = grad_codebooks + (int64_t)m * csize * g;
#define PV_ACC(TEAM_)                                                                            \
    hipLaunchKernelGGL(k_pg_accumulate<TEAM_>, dim3(ablocks), dim3(kBlock), 0, sm, start, extra,    \
                       order, G, scales, gpr, g, csize, first_partial, partial, out)
        switch (team) {
        case 1: PV_ACC(1); break;
        case 2: PV_ACC(2); break;
        case 4: PV_ACC(4); break;
        case 8: PV_ACC(8); break;
        case 16: PV_ACC(16); break;
        case 32: PV_ACC(32); break;
        default: PV_ACC(64); break;
        }
#undef PV_ACC
        hipLaunchKernelGGL(k_pg_combine, dim3(cblocks), dim3(kBlock), 0, sm, extra, g, csize,
                           first_partial, partial, out);
    }
    if (grad_scales) {
        if (g % 4 == 0)
            hipLaunchKernelGGL(k_pg_scales<true>, dim3((unsigned)l->out_features), dim3(kBlock), 0, sm,
                               G, codes, codebooks, g, M, l->nbits, gpr, grad_scales);
        else
            hipLaunchKernelGGL(k_pg_scales<false>, dim3((unsigned)l->out_features), dim3(kBlock), 0, sm,
                               G, codes, codebooks, g, M, l->nbits, gpr, grad_scales);
    }
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

// Subspace size from the trust ratio (Sec. 4.3; App. K, hyperparameter paragraph):
// keep the largest number of groups, taken in the order of the selection rule
// (largest update norm first, lower id first), whose re-encoding keeps
//     || x^{k+1} - x^k ||^2  <  ratio^2 * || x^k ||^2
// for this matrix' dequantised weights x; always keep one group whose code moved.
//
// The paper grows the subspace chunk by chunk and undoes the tail of the last
// chunk.  Since the change only grows with the number of groups, the result is
// the longest prefix of the ranked candidates that satisfies the bound, so the
// work is done once for all candidates:
//   ranked candidates (radix select, then a stable sort of the k_max selected
//   keys) -> all candidates re-encoded in place (previous codes saved) ->
//   squared change per candidate -> prefix sums in rank order -> first prefix
//   that breaks the bound -> codes of the candidates behind it restored.
// Everything stays on the device; the kept count is written to device memory.
//
// Arithmetic: a group's change is the sum over its weights of
// (double(w_new) - double(w_old))^2 with w the fp32 dequantised weights; the
// prefix sums and ||x^k||^2 are double sums in a fixed (launch-independent)
// association, so a run is reproducible; they differ from a sequential sum by
// rounding only.
#include <hipcub/hipcub.hpp>

#include "pv_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kPer = 8;                       // ranks per thread in the scan kernels
constexpr int kTile = kBlock * kPer;          // ranks per block there
constexpr unsigned kNone = 0xFFFFFFFFu;

struct tr_state {
    unsigned first_violation;   // lowest rank r whose prefix of r + 1 groups breaks the bound
    unsigned first_moved;       // lowest rank whose code tuple moved
    unsigned kept;              // result
    unsigned pad;
    double normsq;
};

// fixed-order sum over the block; result valid in thread 0
__device__ __forceinline__ double block_sum(double v, double *tmp)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = v + __shfl_down(v, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) tmp[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
    if (threadIdx.x == 0)
        for (int w = 0; w < kBlock / 64; ++w) t = t + tmp[w];
    return t;
}

// keys and previous codes of the candidates; block 0 also adds up the partial norms
__global__ __launch_bounds__(kBlock) void k_tr_gather(const int32_t *__restrict__ idx, int k,
                                                      const float *__restrict__ scores,
                                                      const uint16_t *__restrict__ codes, int M,
                                                      uint16_t *__restrict__ old_codes,
                                                      unsigned *__restrict__ keys,
                                                      int32_t *__restrict__ pos,
                                                      const double *__restrict__ norm_partial,
                                                      int norm_parts, tr_state *__restrict__ state)
{
    __shared__ double tmp[kBlock / 64];
    const int j = blockIdx.x * kBlock + threadIdx.x;
    if (j < k) {
        const int64_t n = idx[j];
        keys[j] = __float_as_uint(scores[n]);   // scores are >= +0: the bits order like the values
        pos[j] = j;
        for (int m = 0; m < M; ++m) old_codes[(int64_t)j * M + m] = codes[n * M + m];
    }
    if (blockIdx.x == 0) {
        double acc = 0.0;
        for (int i = threadIdx.x; i < norm_parts; i += kBlock) acc = acc + norm_partial[i];
        acc = block_sum(acc, tmp);
        if (threadIdx.x == 0) {
            state->normsq = acc;
            state->first_violation = kNone;
            state->first_moved = kNone;
            state->kept = 0;
        }
    }
}

// dequantised weight i of a group (fp32 additions in codebook order, one multiply)
__device__ __forceinline__ float deq_weight(const float *__restrict__ codebooks,
                                            const uint16_t *code, int M, int64_t csize, int g,
                                            unsigned mask, float s, int i)
{
    float acc = codebooks[((int64_t)(code[0] & mask)) * g + i];
    for (int m = 1; m < M; ++m) acc = acc + codebooks[(m * csize + (code[m] & mask)) * g + i];
    return s * acc;
}

// squared change of candidate j (its previous codes against the codes now in place)
__device__ __forceinline__ double candidate_change(int64_t n, int64_t j,
                                                   const uint16_t *__restrict__ old_codes,
                                                   const uint16_t *__restrict__ codes,
                                                   const float *__restrict__ codebooks,
                                                   const float *__restrict__ scales, int g, int M,
                                                   int nbits, int gpr, bool *moved)
{
    const int64_t csize = (int64_t)1 << nbits;
    const unsigned mask = (unsigned)csize - 1u;
    const float s = scales[n / gpr];
    const uint16_t *a = old_codes + j * M;
    const uint16_t *b = codes + n * M;
    bool mv = false;
    for (int m = 0; m < M; ++m) mv |= (a[m] & mask) != (b[m] & mask);
    double d = 0.0;
    if (mv)
        for (int i = 0; i < g; ++i) {
            double diff = (double)deq_weight(codebooks, b, M, csize, g, mask, s, i) -
                          (double)deq_weight(codebooks, a, M, csize, g, mask, s, i);
            d = d + diff * diff;
        }
    *moved = mv;
    return d;
}

// ||x^k||^2: block b sums the groups [b * per_block, (b + 1) * per_block), thread t of it the
// groups t, t + 256, ... of that range, in an order fixed by the code below.  kGroups groups
// are in flight per thread (codes first, then the codewords): the kernel is a gather from the
// L2-resident codebook and bound by round trips otherwise.
template <int M_, bool VEC>
__global__ __launch_bounds__(kBlock) void k_tr_normsq(const uint16_t *__restrict__ codes,
                                                      const float *__restrict__ codebooks,
                                                      const float *__restrict__ scales, int64_t N,
                                                      int64_t per_block, int g, int M_rt, int nbits,
                                                      int gpr, double *__restrict__ partial)
{
    __shared__ double tmp[kBlock / 64];
    constexpr int kGroups = 8;
    const int M = M_ > 0 ? M_ : M_rt;
    const int64_t csize = (int64_t)1 << nbits;
    const unsigned mask = (unsigned)csize - 1u;
    const int64_t lo = (int64_t)blockIdx.x * per_block;
    const int64_t hi = lo + per_block < N ? lo + per_block : N;
    double acc = 0.0;
    for (int64_t n0 = lo + threadIdx.x; n0 < hi; n0 += (int64_t)kBlock * kGroups) {
        if constexpr (VEC && M_ == 1) {
            unsigned code[kGroups];
            float s[kGroups];
#pragma unroll
            for (int u = 0; u < kGroups; ++u) {
                const int64_t n = n0 + (int64_t)u * kBlock;
                code[u] = n < hi ? (codes[n] & mask) : 0u;
                s[u] = n < hi ? scales[n / gpr] : 0.0f;
            }
            for (int v4 = 0; v4 < g / 4; ++v4) {
                pv_f4 c[kGroups];
#pragma unroll
                for (int u = 0; u < kGroups; ++u)
                    c[u] = reinterpret_cast<const pv_f4 *>(codebooks + (int64_t)code[u] * g)[v4];
#pragma unroll
                for (int u = 0; u < kGroups; ++u) {
                    if (n0 + (int64_t)u * kBlock < hi) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            double w = (double)(s[u] * c[u][e]);
                            acc = acc + w * w;
                        }
                    }
                }
            }
        } else {
            for (int u = 0; u < kGroups; ++u) {
                const int64_t n = n0 + (int64_t)u * kBlock;
                if (n >= hi) break;
                const float sc = scales[n / gpr];
                const uint16_t *c = codes + n * M;
                for (int i = 0; i < g; ++i) {
                    double w = (double)deq_weight(codebooks, c, M, csize, g, mask, sc, i);
                    acc = acc + w * w;
                }
            }
        }
    }
    acc = block_sum(acc, tmp);
    if (threadIdx.x == 0) partial[blockIdx.x] = acc;
}

// change of every candidate, stored in rank order (one thread per rank)
__global__ __launch_bounds__(kBlock) void k_tr_delta(
    const int32_t *__restrict__ idx, const int32_t *__restrict__ order, int k,
    const uint16_t *__restrict__ old_codes, const uint16_t *__restrict__ codes,
    const float *__restrict__ codebooks, const float *__restrict__ scales, int g, int M, int nbits,
    int gpr, double *__restrict__ delta, uint8_t *__restrict__ moved)
{
    const int r = blockIdx.x * kBlock + threadIdx.x;
    if (r >= k) return;
    const int j = order[r];
    bool mv;
    delta[r] = candidate_change(idx[j], j, old_codes, codes, codebooks, scales, g, M, nbits, gpr, &mv);
    moved[r] = mv ? 1 : 0;
}

// Position of a thread's kPer values inside its tile: wave-wide inclusive scan with a fixed
// association, wave totals added in wave order.  Returns the sum of everything before the
// thread; *total = sum of the tile.  s_wave: kBlock / 64 doubles of LDS.
__device__ __forceinline__ double tile_exclusive(double mine, double *s_wave, double *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    double inc = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        double u = __shfl_up(inc, off);
        if (lane >= off) inc = u + inc;
    }
    double excl = __shfl_up(inc, 1);
    if (lane == 0) excl = 0.0;
    __syncthreads();
    if (lane == 63) s_wave[wave] = inc;
    __syncthreads();
    double before = 0.0, tot = 0.0;
#pragma unroll
    for (int w = 0; w < kBlock / 64; ++w) {
        if (w < wave) before = before + s_wave[w];
        tot = tot + s_wave[w];
    }
    *total = tot;
    return before + excl;
}

// sum over the ranks [b * kTile, (b + 1) * kTile)
__global__ __launch_bounds__(kBlock) void k_tr_tile_sums(const double *__restrict__ delta, int k,
                                                         double *__restrict__ tile_sum)
{
    __shared__ double s_wave[kBlock / 64];
    const int64_t r0 = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kPer;
    double acc = 0.0;
#pragma unroll
    for (int e = 0; e < kPer; ++e)
        if (r0 + e < k) acc = acc + delta[r0 + e];
    double total;
    (void)tile_exclusive(acc, s_wave, &total);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
}

// one block: exclusive prefix of the tile sums, in place, tile order
__global__ __launch_bounds__(kBlock) void k_tr_tile_offsets(double *__restrict__ tile_sum, int tiles)
{
    __shared__ double s_in[kBlock];
    __shared__ double s_carry;
    if (threadIdx.x == 0) s_carry = 0.0;
    __syncthreads();
    for (int base = 0; base < tiles; base += kBlock) {
        const int i = base + threadIdx.x;
        s_in[threadIdx.x] = i < tiles ? tile_sum[i] : 0.0;
        __syncthreads();
        if (threadIdx.x == 0) {               // short and exactly ordered
            double run = s_carry;
            for (int t = 0; t < kBlock; ++t) {
                double v = s_in[t];
                s_in[t] = run;
                run = run + v;
            }
            s_carry = run;
        }
        __syncthreads();
        if (i < tiles) tile_sum[i] = s_in[threadIdx.x];
        __syncthreads();
    }
}

// prefix sums in rank order; the first prefix that breaks the bound and the first moved
// group are recorded with atomic minima
__global__ __launch_bounds__(kBlock) void k_tr_prefix(const double *__restrict__ delta,
                                                      const uint8_t *__restrict__ moved, int k,
                                                      const double *__restrict__ tile_off,
                                                      double ratio, double *__restrict__ prefix,
                                                      tr_state *__restrict__ state)
{
    __shared__ double s_wave[kBlock / 64];
    const int64_t r0 = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kPer;
    double d[kPer];
    unsigned mv = 0;
    double mine = 0.0;
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
        d[e] = 0.0;
        if (r0 + e < k) {
            d[e] = delta[r0 + e];
            mv |= (unsigned)(moved[r0 + e] != 0) << e;
        }
        mine = mine + d[e];
    }
    double total;
    const double off = tile_off[blockIdx.x] + tile_exclusive(mine, s_wave, &total);
    const double bound = ratio * ratio * state->normsq;
    unsigned viol = kNone, first_mv = kNone;
    double run = off;
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
        if (r0 + e < k) {
            run = run + d[e];
            prefix[r0 + e + 1] = run;
            if (!(run < bound) && viol == kNone) viol = (unsigned)(r0 + e);
            if (((mv >> e) & 1u) && first_mv == kNone) first_mv = (unsigned)(r0 + e);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) prefix[0] = 0.0;
    if (viol != kNone) atomicMin(&state->first_violation, viol);
    if (first_mv != kNone) atomicMin(&state->first_moved, first_mv);
}

// the kept count with the rule that one moved group always stays
__device__ __forceinline__ int64_t kept_count(const tr_state *state, int k, int64_t chunk)
{
    int64_t kept = state->first_violation == kNone ? k : (int64_t)state->first_violation;
    if (kept < k && state->first_moved != kNone) {
        // the chunk that was being applied when the bound broke ends here
        int64_t chunk_end = (kept / chunk + 1) * chunk;
        if (chunk_end > k) chunk_end = k;
        const int64_t fm = (int64_t)state->first_moved;
        if (fm >= kept && fm < chunk_end) kept = fm + 1;
    }
    return kept;
}

// previous codes back into the candidates behind the kept prefix; ranked ids and results out
__global__ __launch_bounds__(kBlock) void k_tr_rollback(
    const int32_t *__restrict__ idx, const int32_t *__restrict__ order, int k,
    const uint16_t *__restrict__ old_codes, uint16_t *__restrict__ codes, int M,
    const tr_state *__restrict__ state, const double *__restrict__ prefix, int64_t chunk,
    int32_t *__restrict__ rank_idx, int64_t *__restrict__ num_applied, double *__restrict__ stats)
{
    const int64_t kept = kept_count(state, k, chunk);   // the same in every thread
    const int r = blockIdx.x * kBlock + threadIdx.x;
    if (r == 0) {
        if (num_applied) *num_applied = kept;
        if (stats) {
            stats[0] = k > 0 ? prefix[kept] : 0.0;
            stats[1] = state->normsq;
        }
    }
    if (r >= k) return;
    const int j = order[r];
    const int64_t n = idx[j];
    if (rank_idx) rank_idx[r] = (int32_t)n;
    if (r >= kept)
        for (int m = 0; m < M; ++m) codes[n * M + m] = old_codes[(int64_t)j * M + m];
}

inline size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

pv_status pv_launch_trust_ratio(pv_ctx *ctx, const pv_layout *l, const float *T, const float *W,
                                const float *codebooks, const float *scales, int64_t k_max,
                                int64_t chunk, double ratio, int32_t beam_width, uint16_t *codes,
                                int32_t *rank_idx, int64_t *num_applied, double *stats)
{
    const int64_t N = pv_num_groups(l);
    const int g = l->group_size, M = l->num_codebooks;
    const int gpr = (int)(l->in_features / g);
    const int k = (int)k_max;
    const int tiles = (k + kTile - 1) / kTile;
    int norm_blocks = (int)((N + 4095) / 4096);
    if (norm_blocks > 1024) norm_blocks = 1024;
    if (norm_blocks < 1) norm_blocks = 1;
    const int64_t per_block = (N + norm_blocks - 1) / norm_blocks;

    size_t sort_bytes = 0;
    if (k > 0)
        PV_HIP(ctx, hipcub::DeviceRadixSort::SortPairsDescending(
                        nullptr, sort_bytes, (const unsigned *)nullptr, (unsigned *)nullptr,
                        (const int32_t *)nullptr, (int32_t *)nullptr, k, 0, 32, ctx->stream));
    // one scratch block, carved up
    const size_t kk = (size_t)(k > 0 ? k : 1);
    size_t o_state = 0;
    size_t o_idx = o_state + align_up(sizeof(tr_state));
    size_t o_keys = o_idx + align_up(kk * 4);
    size_t o_keys2 = o_keys + align_up(kk * 4);
    size_t o_pos = o_keys2 + align_up(kk * 4);
    size_t o_order = o_pos + align_up(kk * 4);
    size_t o_old = o_order + align_up(kk * 4);
    size_t o_delta = o_old + align_up(kk * M * 2);
    size_t o_prefix = o_delta + align_up(kk * 8);
    size_t o_moved = o_prefix + align_up((kk + 1) * 8);
    size_t o_tiles = o_moved + align_up(kk);
    size_t o_norm = o_tiles + align_up((size_t)(tiles > 0 ? tiles : 1) * 8);
    size_t o_sort = o_norm + align_up((size_t)norm_blocks * 8);
    size_t total = o_sort + align_up(sort_bytes);
    pv_status st = pv_ensure(ctx, ctx->trust, total);
    if (st != PV_OK) return st;
    st = pv_ensure(ctx, ctx->sel_scores, (size_t)N * sizeof(float) + 16);
    if (st != PV_OK) return st;
    char *base = static_cast<char *>(ctx->trust.ptr);
    tr_state *state = reinterpret_cast<tr_state *>(base + o_state);
    int32_t *idx = reinterpret_cast<int32_t *>(base + o_idx);
    unsigned *keys = reinterpret_cast<unsigned *>(base + o_keys);
    unsigned *keys2 = reinterpret_cast<unsigned *>(base + o_keys2);
    int32_t *pos = reinterpret_cast<int32_t *>(base + o_pos);
    int32_t *order = reinterpret_cast<int32_t *>(base + o_order);
    uint16_t *old_codes = reinterpret_cast<uint16_t *>(base + o_old);
    double *delta = reinterpret_cast<double *>(base + o_delta);
    double *prefix = reinterpret_cast<double *>(base + o_prefix);
    uint8_t *moved = reinterpret_cast<uint8_t *>(base + o_moved);
    double *tile_sum = reinterpret_cast<double *>(base + o_tiles);
    double *norm_partial = reinterpret_cast<double *>(base + o_norm);
    void *sort_tmp = base + o_sort;
    float *scores = static_cast<float *>(ctx->sel_scores.ptr);
    hipStream_t sm = ctx->stream;

    // ||x^k||^2 of the codes as they are now (partial sums; the gather kernel adds them up)
    {
        pv_timed t(ctx, PV_K_TRUST_RATIO);
        if (M == 1 && g % 4 == 0)
            hipLaunchKernelGGL((k_tr_normsq<1, true>), dim3(norm_blocks), dim3(kBlock), 0, sm, codes,
                               codebooks, scales, N, per_block, g, M, l->nbits, gpr, norm_partial);
        else
            hipLaunchKernelGGL((k_tr_normsq<0, false>), dim3(norm_blocks), dim3(kBlock), 0, sm, codes,
                               codebooks, scales, N, per_block, g, M, l->nbits, gpr, norm_partial);
    }
    // candidates: the k_max groups of the selection rule (ascending ids) and every score
    st = pv_launch_select(ctx, l, T, W, k, idx, scores);
    if (st != PV_OK) return st;
    const unsigned kblocks = (unsigned)((k + kBlock - 1) / kBlock);
    {
        pv_timed t(ctx, PV_K_TRUST_RATIO);
        hipLaunchKernelGGL(k_tr_gather, dim3(kblocks > 0 ? kblocks : 1), dim3(kBlock), 0, sm, idx, k,
                           scores, codes, M, old_codes, keys, pos, norm_partial, norm_blocks, state);
        // equal keys keep their order (ascending ids): the sort is stable
        if (k > 0)
            PV_HIP(ctx, hipcub::DeviceRadixSort::SortPairsDescending(sort_tmp, sort_bytes, keys, keys2,
                                                                     pos, order, k, 0, 32, sm));
    }
    if (k > 0) {
        st = pv_reencode_dispatch(ctx, l, T, codebooks, scales, idx, k, beam_width, codes, nullptr);
        if (st != PV_OK) return st;
    }
    {
        pv_timed t(ctx, PV_K_TRUST_RATIO);
        if (k > 0) {
            hipLaunchKernelGGL(k_tr_delta, dim3(kblocks), dim3(kBlock), 0, sm, idx, order, k, old_codes,
                               codes, codebooks, scales, g, M, l->nbits, gpr, delta, moved);
            hipLaunchKernelGGL(k_tr_tile_sums, dim3(tiles), dim3(kBlock), 0, sm, delta, k, tile_sum);
            hipLaunchKernelGGL(k_tr_tile_offsets, dim3(1), dim3(kBlock), 0, sm, tile_sum, tiles);
            hipLaunchKernelGGL(k_tr_prefix, dim3(tiles), dim3(kBlock), 0, sm, delta, moved, k,
                               tile_sum, ratio, prefix, state);
        }
        hipLaunchKernelGGL(k_tr_rollback, dim3(kblocks > 0 ? kblocks : 1), dim3(kBlock), 0, sm, idx,
                           order, k, old_codes, codes, M, state, prefix, chunk, rank_idx, num_applied,
                           stats);
    }
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

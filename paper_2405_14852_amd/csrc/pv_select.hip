// Group scores and top-k selection (Alg. 2 line 5, per matrix as in Sec. 3.4).
//
// score_n = sum_i (T[n,i] - W[n,i])^2 as an fp32 fused-multiply-add chain in
// index order, so that every implementation of this rule gives the same bits.
// Scores are non-negative floats, so their bit patterns order like unsigned
// integers.  The k-th largest key is found by a 3-digit radix select (11+11+10
// bits, most significant first); groups above the threshold are taken, groups
// equal to it are taken lowest id first, and the ids are written in ascending
// order through a two-level prefix sum.  Nothing returns to the host.
//
// Launches: [scores + digit-0 histogram] [digit-1 histogram] [digit-2 histogram]
// [per-block counts] [ordered write].  Every block re-derives the digits chosen
// so far from the (tiny) histograms instead of waiting for a separate kernel.
#include "pv_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kBins = 2048;
constexpr int kItems = 8;                      // groups per thread in the compaction kernels
constexpr int kChunk = kBlock * kItems;        // groups per block there

__device__ __forceinline__ int digit_of(unsigned key, int pass)
{
    return pass == 0 ? (int)(key >> 21) : pass == 1 ? (int)((key >> 10) & 2047u) : (int)(key & 1023u);
}

// Add one count per valid lane to an LDS histogram.  Lanes of a wave that hit
// the same bin are merged first (two rounds catch the dominant bins of a
// narrow score distribution); the rest fall back to one atomic each.
__device__ __forceinline__ void hist_add(unsigned *hist, int bin, bool valid)
{
    const int lane = threadIdx.x & 63;
    unsigned long long todo = __ballot(valid);
#pragma unroll 1
    for (int round = 0; round < 2 && todo; ++round) {
        int leader = __ffsll((long long)todo) - 1;
        int lb = __shfl(bin, leader);
        unsigned long long same = __ballot(valid && bin == lb);
        if (lane == leader) atomicAdd(&hist[lb], (unsigned)__popcll(same));
        if (valid && bin == lb) valid = false;
        todo &= ~same;
    }
    if (valid) atomicAdd(&hist[bin], 1u);
}

// Exclusive prefix sum of one value per thread over the block (thread order);
// *total receives the block sum.  `tmp` needs kBlock / 64 unsigneds of LDS.
__device__ __forceinline__ unsigned block_excl_scan(unsigned v, unsigned *tmp, unsigned *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        unsigned u = __shfl_up(inc, off);
        if (lane >= off) inc += u;
    }
    __syncthreads();
    if (lane == 63) tmp[wave] = inc;
    __syncthreads();
    unsigned before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kBlock / 64; ++w) {
        unsigned x = tmp[w];
        before += w < wave ? x : 0u;
        all += x;
    }
    __syncthreads();
    *total = all;
    return before + inc - v;
}

// Given a histogram of `bins` digits and the rank `kk` (1-based, counted from the
// largest digit), find the digit d with  count(> d) < kk <= count(>= d)  and
// return kk - count(> d).  All threads of the block call this; the result goes
// to all.  `tmp` is kBlock + 2 unsigneds of LDS.
__device__ void pick_digit(const unsigned *__restrict__ ghist, int bins, unsigned kk,
                           unsigned *tmp, int *digit, unsigned *kk_rem)
{
    constexpr int per = kBins / kBlock;  // 8 bins per thread; thread 0 owns the TOP bins
    const int tid = threadIdx.x;
    unsigned local[per];
    unsigned sum = 0;
#pragma unroll
    for (int j = 0; j < per; ++j) {
        int bin = bins - 1 - (tid * per + j);
        local[j] = bin >= 0 ? ghist[bin] : 0u;
        sum += local[j];
    }
    unsigned total;
    unsigned above = block_excl_scan(sum, tmp, &total);
#pragma unroll
    for (int j = 0; j < per; ++j) {
        int bin = bins - 1 - (tid * per + j);
        if (bin >= 0 && above < kk && kk <= above + local[j]) {
            tmp[kBlock] = (unsigned)bin;
            tmp[kBlock + 1] = kk - above;
        }
        above += local[j];
    }
    __syncthreads();
    *digit = (int)tmp[kBlock];
    *kk_rem = tmp[kBlock + 1];
    __syncthreads();
}

__device__ __forceinline__ float score_group(const float *__restrict__ t,
                                             const float *__restrict__ w, int g)
{
    float s = 0.0f;
    if ((g & 3) == 0) {
        const pv_f4 *t4 = reinterpret_cast<const pv_f4 *>(t);
        const pv_f4 *w4 = reinterpret_cast<const pv_f4 *>(w);
        for (int i = 0; i < g / 4; ++i) {
            pv_f4 a = __builtin_nontemporal_load(&t4[i]);
            pv_f4 b = __builtin_nontemporal_load(&w4[i]);
            float d;
            d = a.x - b.x; s = fmaf(d, d, s);
            d = a.y - b.y; s = fmaf(d, d, s);
            d = a.z - b.z; s = fmaf(d, d, s);
            d = a.w - b.w; s = fmaf(d, d, s);
        }
    } else {
        for (int i = 0; i < g; ++i) {
            float d = t[i] - w[i];
            s = fmaf(d, d, s);
        }
    }
    return s;
}

// Pass 0: one thread per group: score, store, histogram of the top 11 key bits.
__global__ __launch_bounds__(kBlock) void k_scores_hist0(const float *__restrict__ T,
                                                         const float *__restrict__ W,
                                                         float *__restrict__ scores,
                                                         unsigned *__restrict__ hist0, int N, int g)
{
    __shared__ unsigned lh[kBins];
    for (int b = threadIdx.x; b < kBins; b += kBlock) lh[b] = 0;
    __syncthreads();
    const int64_t n = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const bool valid = n < N;
    unsigned key = 0;
    if (valid) {
        float s = score_group(T + n * g, W + n * g, g);
        scores[n] = s;
        key = __float_as_uint(s);
    }
    hist_add(lh, digit_of(key, 0), valid);
    __syncthreads();
    for (int b = threadIdx.x; b < kBins; b += kBlock) {
        unsigned v = lh[b];
        if (v) atomicAdd(&hist0[b], v);
    }
}

// Passes 1 and 2: histogram of the next digit among keys that match the digits
// chosen so far.
__global__ __launch_bounds__(kBlock) void k_hist_next(const float *__restrict__ scores,
                                                      const unsigned *__restrict__ hist_all,
                                                      unsigned *__restrict__ hist_out, int N,
                                                      unsigned k, int pass)
{
    __shared__ unsigned lh[kBins];
    __shared__ unsigned tmp[kBlock + 2];
    for (int b = threadIdx.x; b < kBins; b += kBlock) lh[b] = 0;
    int d0, d1 = 0;
    unsigned kk;
    pick_digit(hist_all, kBins, k, tmp, &d0, &kk);
    if (pass == 2) pick_digit(hist_all + kBins, kBins, kk, tmp, &d1, &kk);
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kChunk;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        int64_t n = base + j * kBlock + threadIdx.x;
        bool valid = n < N;
        unsigned key = valid ? __float_as_uint(scores[n]) : 0u;
        valid = valid && digit_of(key, 0) == d0 && (pass == 1 || digit_of(key, 1) == d1);
        hist_add(lh, digit_of(key, pass), valid);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kBins; b += kBlock) {
        unsigned v = lh[b];
        if (v) atomicAdd(&hist_out[b], v);
    }
}

__device__ __forceinline__ unsigned block_sum(unsigned v, unsigned *tmp)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) tmp[threadIdx.x >> 6] = v;
    __syncthreads();
    unsigned total = 0;
    for (int w = 0; w < kBlock / 64; ++w) total += tmp[w];
    __syncthreads();
    return total;
}

// Threshold key and number of ties to take, then per-block (greater, equal) counts.
__global__ __launch_bounds__(kBlock) void k_block_counts(const float *__restrict__ scores,
                                                         const unsigned *__restrict__ hist_all,
                                                         unsigned *__restrict__ state,
                                                         unsigned *__restrict__ block_counts, int N,
                                                         unsigned k)
{
    __shared__ unsigned tmp[kBlock + 2];
    int d0, d1, d2;
    unsigned kk;
    pick_digit(hist_all, kBins, k, tmp, &d0, &kk);
    pick_digit(hist_all + kBins, kBins, kk, tmp, &d1, &kk);
    pick_digit(hist_all + 2 * kBins, 1024, kk, tmp, &d2, &kk);
    const unsigned thr = ((unsigned)d0 << 21) | ((unsigned)d1 << 10) | (unsigned)d2;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        state[0] = thr;
        state[1] = kk;  // how many keys equal to thr are selected (lowest ids first)
    }
    const int64_t base = (int64_t)blockIdx.x * kChunk + (int64_t)threadIdx.x * kItems;
    unsigned gt = 0, eq = 0;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        int64_t n = base + j;
        if (n < N) {
            unsigned key = __float_as_uint(scores[n]);
            gt += key > thr;
            eq += key == thr;
        }
    }
    gt = block_sum(gt, tmp);
    eq = block_sum(eq, tmp);
    if (threadIdx.x == 0) {
        block_counts[2 * blockIdx.x] = gt;
        block_counts[2 * blockIdx.x + 1] = eq;
    }
}

// Ordered write: position of a selected group = (#greater with a lower id) +
// min(#equal with a lower id, ties to take).  Also re-zeroes the histograms for
// the next call.
__global__ __launch_bounds__(kBlock) void k_compact_write(const float *__restrict__ scores,
                                                          const unsigned *__restrict__ state,
                                                          const unsigned *__restrict__ block_counts,
                                                          unsigned *__restrict__ hist_all,
                                                          int32_t *__restrict__ out_idx, int N)
{
    __shared__ unsigned tmp[kBlock + 2];
    const unsigned thr = state[0], need_eq = state[1];
    // counts of all earlier blocks
    unsigned pg = 0, pe = 0;
    for (int b = threadIdx.x; b < (int)blockIdx.x; b += kBlock) {
        pg += block_counts[2 * b];
        pe += block_counts[2 * b + 1];
    }
    pg = block_sum(pg, tmp);
    pe = block_sum(pe, tmp);
    const int64_t base = (int64_t)blockIdx.x * kChunk + (int64_t)threadIdx.x * kItems;
    unsigned keys[kItems];
    unsigned gt = 0, eq = 0;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        int64_t n = base + j;
        keys[j] = n < N ? __float_as_uint(scores[n]) : 0u;
        if (n < N) {
            gt += keys[j] > thr;
            eq += keys[j] == thr;
        }
    }
    unsigned tot;
    unsigned rg = pg + block_excl_scan(gt, tmp, &tot);  // greater keys before this thread's items
    unsigned re = pe + block_excl_scan(eq, tmp, &tot);  // equal keys before them
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        int64_t n = base + j;
        if (n < N) {
            if (keys[j] > thr) {
                out_idx[rg + (re < need_eq ? re : need_eq)] = (int32_t)n;
                ++rg;
            } else if (keys[j] == thr) {
                if (re < need_eq) out_idx[rg + re] = (int32_t)n;
                ++re;
            }
        }
    }
    // leave the histograms zero for the next call (all their readers ran in earlier launches)
    const int64_t z = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (z < 3 * kBins) hist_all[z] = 0;
    if (gridDim.x * kBlock < 3 * kBins && blockIdx.x == 0)
        for (int i = gridDim.x * kBlock + threadIdx.x; i < 3 * kBins; i += kBlock) hist_all[i] = 0;
}

// scores only (k == 0 with a score output requested)
__global__ __launch_bounds__(kBlock) void k_scores_only(const float *__restrict__ T,
                                                        const float *__restrict__ W,
                                                        float *__restrict__ scores, int N, int g)
{
    const int64_t n = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (n < N) scores[n] = score_group(T + n * g, W + n * g, g);
}

}  // namespace

pv_status pv_launch_select(pv_ctx *ctx, const pv_layout *l, const float *T, const float *W,
                           int64_t k, int32_t *out_idx, float *scores)
{
    const int N = (int)pv_num_groups(l);
    const int g = l->group_size;
    pv_status st;
    if (!scores) {
        st = pv_ensure(ctx, ctx->sel_scores, (size_t)N * sizeof(float));
        if (st != PV_OK) return st;
        scores = static_cast<float *>(ctx->sel_scores.ptr);
    }
    const unsigned blocks1 = (unsigned)((N + kBlock - 1) / kBlock);
    const unsigned blocksC = (unsigned)((N + kChunk - 1) / kChunk);
    if (k == 0) {
        pv_timed t(ctx, PV_K_GROUP_SCORES);
        hipLaunchKernelGGL(k_scores_only, dim3(blocks1), dim3(kBlock), 0, ctx->stream, T, W, scores,
                           N, g);
        PV_HIP(ctx, hipGetLastError());
        return PV_OK;
    }
    st = pv_ensure(ctx, ctx->sel_hist, 3 * kBins * sizeof(unsigned), /*zero_new=*/true);
    if (st != PV_OK) return st;
    st = pv_ensure(ctx, ctx->sel_blocks, (size_t)blocksC * 2 * sizeof(unsigned));
    if (st != PV_OK) return st;
    st = pv_ensure(ctx, ctx->sel_state, 4 * sizeof(unsigned));
    if (st != PV_OK) return st;
    unsigned *hist = static_cast<unsigned *>(ctx->sel_hist.ptr);
    unsigned *bc = static_cast<unsigned *>(ctx->sel_blocks.ptr);
    unsigned *state = static_cast<unsigned *>(ctx->sel_state.ptr);
    {
        pv_timed t(ctx, PV_K_GROUP_SCORES);
        hipLaunchKernelGGL(k_scores_hist0, dim3(blocks1), dim3(kBlock), 0, ctx->stream, T, W, scores,
                           hist, N, g);
    }
    {
        pv_timed t(ctx, PV_K_SELECT);
        hipLaunchKernelGGL(k_hist_next, dim3(blocksC), dim3(kBlock), 0, ctx->stream, scores, hist,
                           hist + kBins, N, (unsigned)k, 1);
        hipLaunchKernelGGL(k_hist_next, dim3(blocksC), dim3(kBlock), 0, ctx->stream, scores, hist,
                           hist + 2 * kBins, N, (unsigned)k, 2);
        hipLaunchKernelGGL(k_block_counts, dim3(blocksC), dim3(kBlock), 0, ctx->stream, scores, hist,
                           state, bc, N, (unsigned)k);
        hipLaunchKernelGGL(k_compact_write, dim3(blocksC), dim3(kBlock), 0, ctx->stream, scores,
                           state, bc, hist, out_idx, N);
    }
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

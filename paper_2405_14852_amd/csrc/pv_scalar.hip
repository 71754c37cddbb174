// The scalar representation of App. K ("GPTQ": uniform grid of 2^b values, scale and zero
// point per block of `blk` consecutive weights of a row):
//     W[o, i] = s[o, i/blk] * (q[o, i] - z[o, i/blk])
// Dequantisation is a stream; the V step on this representation is rounding to the nearest
// grid value (App. K), done as the definition states it - every value tried, objective in
// double on the fp32 dequantised value, previous code kept on a tie - so the result is the
// oracle's bit for bit.  At most 256 candidates per weight: no search structure is needed.
#include "pv_internal.h"

namespace {

constexpr int kBlock = 256;

// one thread per four consecutive weights (they share a block when blk % 4 == 0)
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_dequantize_scalar(const uint8_t *__restrict__ codes,
                                                              const float *__restrict__ scales,
                                                              const float *__restrict__ zeros,
                                                              float *__restrict__ W_out, int64_t n,
                                                              int64_t in_features, int blk)
{
    const int64_t bpr = in_features / blk;
    if constexpr (VEC) {
        const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
        if (v * 4 >= n) return;
        const int64_t e = v * 4;
        const int64_t o = e / in_features, i = e - o * in_features;
        const float s = scales[o * bpr + i / blk], z = zeros[o * bpr + i / blk];
        const uchar4 q = reinterpret_cast<const uchar4 *>(codes)[v];
        pv_f4 w;
        w.x = s * ((float)q.x - z);
        w.y = s * ((float)q.y - z);
        w.z = s * ((float)q.z - z);
        w.w = s * ((float)q.w - z);
        __builtin_nontemporal_store(w, &reinterpret_cast<pv_f4 *>(W_out)[v]);
    } else {
        const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
        if (e >= n) return;
        const int64_t o = e / in_features, i = e - o * in_features;
        W_out[e] = scales[o * bpr + i / blk] * ((float)codes[e] - zeros[o * bpr + i / blk]);
    }
}

__global__ __launch_bounds__(kBlock) void k_reencode_scalar(const float *__restrict__ T,
                                                            const float *__restrict__ scales,
                                                            const float *__restrict__ zeros,
                                                            const int32_t *__restrict__ weight_idx,
                                                            int64_t k, uint8_t *__restrict__ codes,
                                                            unsigned long long *__restrict__ num_changed,
                                                            int64_t n, int64_t in_features, int blk,
                                                            int nvals)
{
    __shared__ unsigned s_changed;
    if (threadIdx.x == 0) s_changed = 0;
    __syncthreads();
    const int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    bool moved = false;
    if (j < k) {
        const int64_t e = weight_idx[j];
        if (e >= 0 && e < n) {
            const int64_t bpr = in_features / blk;
            const int64_t o = e / in_features, i = e - o * in_features;
            const float s = scales[o * bpr + i / blk], z = zeros[o * bpr + i / blk];
            const double t = (double)T[e];
            const int prev = codes[e];
            int best = -1;
            double best_obj = 0.0, prev_obj = 0.0;
            for (int q = 0; q < nvals; ++q) {
                const float w = s * ((float)q - z);
                const double r = (double)w - t;
                const double obj = r * r;
                if (q == prev) prev_obj = obj;
                if (best < 0 || obj < best_obj) {
                    best = q;
                    best_obj = obj;
                }
            }
            if (prev < nvals && prev_obj == best_obj) best = prev;
            if (best != prev) {
                codes[e] = (uint8_t)best;
                moved = true;
            }
        }
    }
    const unsigned long long b = __ballot(moved);
    if ((threadIdx.x & 63) == 0 && b) atomicAdd(&s_changed, (unsigned)__popcll(b));
    __syncthreads();
    if (threadIdx.x == 0 && s_changed && num_changed) atomicAdd(num_changed, (unsigned long long)s_changed);
}

}  // namespace

pv_status pv_launch_dequantize_scalar(pv_ctx *ctx, int64_t out_features, int64_t in_features, int blk,
                                      const uint8_t *codes, const float *scales, const float *zeros,
                                      float *W_out)
{
    pv_timed t(ctx, PV_K_DEQUANTIZE);
    const int64_t n = out_features * in_features;
    if (blk % 4 == 0) {
        const int64_t blocks = (n / 4 + kBlock - 1) / kBlock;
        hipLaunchKernelGGL(k_dequantize_scalar<true>, dim3((unsigned)blocks), dim3(kBlock), 0,
                           ctx->stream, codes, scales, zeros, W_out, n, in_features, blk);
    } else {
        const int64_t blocks = (n + kBlock - 1) / kBlock;
        hipLaunchKernelGGL(k_dequantize_scalar<false>, dim3((unsigned)blocks), dim3(kBlock), 0,
                           ctx->stream, codes, scales, zeros, W_out, n, in_features, blk);
    }
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

pv_status pv_launch_reencode_scalar(pv_ctx *ctx, int64_t out_features, int64_t in_features, int blk,
                                    int nbits, const float *T, const float *scales,
                                    const float *zeros, const int32_t *weight_idx, int64_t k,
                                    uint8_t *codes, int64_t *num_changed)
{
    if (num_changed) {
        pv_status st = pv_launch_fill_i64(ctx, num_changed, 1, 0);
        if (st != PV_OK) return st;
    }
    if (k == 0) return PV_OK;
    pv_timed t(ctx, PV_K_EXACT_SCAN);
    const int64_t blocks = (k + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(k_reencode_scalar, dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream, T, scales,
                       zeros, weight_idx, k, codes, reinterpret_cast<unsigned long long *>(num_changed),
                       out_features * in_features, in_features, blk, 1 << nbits);
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

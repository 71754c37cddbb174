// Stochastic rounding over the two nearest codewords (App. F: the K-nearest
// approximation for vector quantisation with K = 2; App. K: temperature 0.2,
// i.e. probabilities proportional to distance^-5).
//
// For every listed group the kernel scans the whole codebook, keeps the two
// smallest objectives  obj(c) = || s * C[c] - t ||^2  (double, index order, no
// contraction; equal objectives in index order) and rounds to the nearest one
// when the group's variate u is below
//     p = 1 / (1 + (d_1 / d_2)^power),      d = sqrt(obj),
// else to the second.  u is a function of (seed, group id) only: the output
// function of SplitMix64 (Steele, Lea, Flood 2014) on seed + (id + 1) * increment,
// top 53 bits.  Every operation on the way from the objectives to the decision
// (division, square root, products in a fixed order) is correctly rounded, so
// the decision is a function of the inputs and not of the machine.
#include "pv_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kMaxG = 64;
constexpr int GPB = 4;                       // list entries per work item
constexpr double kInf = __builtin_huge_val();
constexpr int kNone = 0x7fffffff;

struct two_t {
    double o1, o2;
    int i1, i2;
};

__device__ __forceinline__ bool better(double o1, int i1, double o2, int i2)
{
    return o1 < o2 || (o1 == o2 && i1 < i2);
}

// the two smallest of the union of two sorted pairs, (objective, index) order
__device__ __forceinline__ two_t merge(const two_t &a, const two_t &b)
{
    two_t r;
    if (better(b.o1, b.i1, a.o1, a.i1)) {
        r.o1 = b.o1; r.i1 = b.i1;
        const bool a_next = better(a.o1, a.i1, b.o2, b.i2);
        r.o2 = a_next ? a.o1 : b.o2;
        r.i2 = a_next ? a.i1 : b.i2;
    } else {
        r.o1 = a.o1; r.i1 = a.i1;
        const bool b_next = better(b.o1, b.i1, a.o2, a.i2);
        r.o2 = b_next ? b.o1 : a.o2;
        r.i2 = b_next ? b.i1 : a.i2;
    }
    return r;
}

__device__ __forceinline__ void insert(two_t &b, double o, int c)
{
    // ascending scan inside a thread: strict '<' keeps the lower index among equals
    if (o < b.o1) {
        b.o2 = b.o1; b.i2 = b.i1;
        b.o1 = o; b.i1 = c;
    } else if (o < b.o2) {
        b.o2 = o; b.i2 = c;
    }
}

__device__ __forceinline__ two_t wave_two(two_t b)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        two_t o;
        o.o1 = __shfl_down(b.o1, off);
        o.o2 = __shfl_down(b.o2, off);
        o.i1 = __shfl_down(b.i1, off);
        o.i2 = __shfl_down(b.i2, off);
        b = merge(b, o);
    }
    return b;
}

// G > 0: group size known at compile time; G == 0: any group size up to kMaxG.
template <int G>
__global__ __launch_bounds__(kBlock) void k_round_two_nearest(
    const float *__restrict__ T, const float *__restrict__ codebook,
    const float *__restrict__ scales, const int32_t *__restrict__ list, int64_t count,
    uint16_t *__restrict__ codes, unsigned long long *__restrict__ num_changed, int power,
    unsigned long long seed, int g_rt, int nbits, int gpr, int N)
{
    constexpr int GS = G > 0 ? G : kMaxG;
    const int g = G > 0 ? G : g_rt;
    __shared__ float s_t[GPB][GS];
    __shared__ float s_scale[GPB];
    __shared__ int s_group[GPB];
    __shared__ two_t s_two[GPB][kBlock / 64];
    const int csize = 1 << nbits;
    const int64_t items = (count + GPB - 1) / GPB;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned blk_changed = 0u;    // per thread; added up once at the end (one atomic per block)
    for (int64_t item = blockIdx.x; item < items; item += gridDim.x) {
        const int64_t base = item * GPB;
        __syncthreads();
        if (threadIdx.x < GPB) {
            int64_t j = base + threadIdx.x;
            int n = j < count ? list[j] : -1;
            if (n < 0 || n >= N) n = -1;
            s_group[threadIdx.x] = n;
            s_scale[threadIdx.x] = n >= 0 ? scales[n / gpr] : 0.0f;
        }
        __syncthreads();
        for (int e = threadIdx.x; e < GPB * g; e += kBlock) {
            int q = e / g, i = e - q * g;
            int n = s_group[q];
            s_t[q][i] = n >= 0 ? T[(int64_t)n * g + i] : 0.0f;
        }
        __syncthreads();
        two_t best[GPB];
#pragma unroll
        for (int q = 0; q < GPB; ++q) {
            best[q].o1 = best[q].o2 = kInf;
            best[q].i1 = best[q].i2 = kNone;
        }
        if constexpr (G > 0) {
            double sc[GPB], tt[GPB][GS];
#pragma unroll
            for (int q = 0; q < GPB; ++q) {
                sc[q] = (double)s_scale[q];
#pragma unroll
                for (int i = 0; i < GS; ++i) tt[q][i] = (double)s_t[q][i];
            }
            constexpr int kBatch = GS <= 8 ? 4 : 2;    // codewords whose loads are in flight together
            for (int c0 = threadIdx.x; c0 < csize; c0 += kBlock * kBatch) {
                pv_f4 cv[kBatch][GS / 4];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int c = c0 + u * kBlock;
                    const pv_f4 *cw4 =
                        reinterpret_cast<const pv_f4 *>(codebook + (int64_t)(c < csize ? c : 0) * GS);
#pragma unroll
                    for (int v4 = 0; v4 < GS / 4; ++v4) cv[u][v4] = cw4[v4];
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int c = c0 + u * kBlock;
                    double obj[GPB];
#pragma unroll
                    for (int q = 0; q < GPB; ++q) obj[q] = 0.0;
#pragma unroll
                    for (int v4 = 0; v4 < GS / 4; ++v4) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            double acc = (double)cv[u][v4][e];
#pragma unroll
                            for (int q = 0; q < GPB; ++q) {
                                // s * c is exact in double (two 24-bit factors): the fused form
                                // rounds like the product followed by the subtraction
                                double r = fma(sc[q], acc, -tt[q][v4 * 4 + e]);
                                obj[q] = obj[q] + r * r;
                            }
                        }
                    }
                    if (c < csize) {
#pragma unroll
                        for (int q = 0; q < GPB; ++q) insert(best[q], obj[q], c);
                    }
                }
            }
        } else {
            for (int c = threadIdx.x; c < csize; c += kBlock) {
                const float *cw = codebook + (int64_t)c * g;
                double obj[GPB];
#pragma unroll
                for (int q = 0; q < GPB; ++q) obj[q] = 0.0;
                for (int i = 0; i < g; ++i) {
                    double acc = (double)cw[i];
#pragma unroll
                    for (int q = 0; q < GPB; ++q) {
                        double r = (double)s_scale[q] * acc - (double)s_t[q][i];
                        obj[q] = obj[q] + r * r;
                    }
                }
#pragma unroll
                for (int q = 0; q < GPB; ++q) insert(best[q], obj[q], c);
            }
        }
#pragma unroll
        for (int q = 0; q < GPB; ++q) {
            two_t w = wave_two(best[q]);
            if (lane == 0) s_two[q][wave] = w;
        }
        __syncthreads();
        if (threadIdx.x < GPB && s_group[threadIdx.x] >= 0) {
            const int q = threadIdx.x;
            const int n = s_group[q];
            two_t b = s_two[q][0];
            for (int w = 1; w < kBlock / 64; ++w) b = merge(b, s_two[q][w]);
            const int prev = (int)(codes[n] & (csize - 1));
            int pick = prev;                           // every objective NaN: keep
            if (b.i1 != kNone)
                pick = pv_round_pick(b.o1, b.i1, b.o2, b.i2, power, seed, (unsigned long long)n);
            if (pick != prev) {
                codes[n] = (uint16_t)pick;
                ++blk_changed;
            }
        }
    }
    // threads 0 .. GPB - 1 counted; they sit in the first wave
    if (threadIdx.x < 64) {
        for (int off = 32; off > 0; off >>= 1) blk_changed += __shfl_down(blk_changed, off);
        if (threadIdx.x == 0 && blk_changed && num_changed)
            atomicAdd(num_changed, (unsigned long long)blk_changed);
    }
}

}  // namespace

pv_status pv_launch_round_two_nearest(pv_ctx *ctx, const pv_layout *l, const float *T,
                                      const float *codebook, const float *scales,
                                      const int32_t *group_idx, int64_t k, int32_t power,
                                      uint64_t seed, uint16_t *codes, int64_t *num_changed)
{
    pv_timed t(ctx, PV_K_STOCHASTIC);
    const int g = l->group_size;
    const int gpr = (int)(l->in_features / g);
    const int N = (int)pv_num_groups(l);
    int64_t blocks = (k + GPB - 1) / GPB;
    if (blocks > 8192) blocks = 8192;
    if (blocks < 1) blocks = 1;
    auto nc = reinterpret_cast<unsigned long long *>(num_changed);
#define PV_ROUND(G_)                                                                             \
    hipLaunchKernelGGL(k_round_two_nearest<G_>, dim3((unsigned)blocks), dim3(kBlock), 0,         \
                       ctx->stream, T, codebook, scales, group_idx, k, codes, nc, (int)power,    \
                       (unsigned long long)seed, g, l->nbits, gpr, N)
    if (g == 8) PV_ROUND(8);
    else if (g == 16) PV_ROUND(16);
    else if (g == 4) PV_ROUND(4);
    else PV_ROUND(0);
#undef PV_ROUND
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

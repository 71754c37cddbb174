// Exact searches in double precision: the full nearest-codeword scan for one
// codebook ("try every code", App. K) and the beam search over several
// codebooks (Sec. 4.2, App. D, App. K).  Objectives are evaluated exactly as
//     acc = C_0[b_0,i] (+ C_1[b_1,i] + ...)        in double, codebook order
//     r   = s * acc - t_i ;  obj = obj + r * r      in double, index order
// with no contraction, so that the decision is taken in one fixed arithmetic.
//
// The scan serves two callers: whole calls for shapes the matrix-core filter
// does not cover, and the (short) list of groups that filter could not certify.
// The two-codebook beam search has the same pair: a filter on the fp64 matrix
// instruction (k_beam_2x8_mfma) whose results are accepted only under
// double-precision certificates, and the exact kernel behind it.
#include "pv_internal.h"

#include <type_traits>

namespace {

constexpr int kBlock = 256;
constexpr int kMaxG = 64;
constexpr double kInf = __builtin_huge_val();

struct best_t {
    double obj;
    int idx;
};

__device__ __forceinline__ unsigned umin3(unsigned a, unsigned b, unsigned c)
{
    return min(min(a, b), c);
}

__device__ __forceinline__ bool better(double o1, int i1, double o2, int i2)
{
    return o1 < o2 || (o1 == o2 && i1 < i2);
}

__device__ __forceinline__ best_t wave_min(best_t b)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        double o = __shfl_down(b.obj, off);
        int i = __shfl_down(b.idx, off);
        if (better(o, i, b.obj, b.idx)) {
            b.obj = o;
            b.idx = i;
        }
    }
    return b;
}

// Block-wide lexicographic minimum of (obj, idx); valid in thread 0.
__device__ __forceinline__ best_t block_min(best_t b, double *s_obj, int *s_idx)
{
    b = wave_min(b);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) {
        s_obj[wave] = b.obj;
        s_idx[wave] = b.idx;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / 64; ++w)
            if (better(s_obj[w], s_idx[w], b.obj, b.idx)) {
                b.obj = s_obj[w];
                b.idx = s_idx[w];
            }
    }
    return b;
}

// ------------------------------------------------------------------ M = 1 scan
//
// Work item = GPB consecutive list entries.  Thread t scores codewords t, t + 256, ...
// against the GPB targets (a codeword is read once for GPB groups).  Ascending scan +
// strict '<' keeps the lowest index among equal objectives; the block-wide lexicographic
// (obj, idx) minimum is then the lowest index, the previous code wins an exact tie with
// the minimum, and the code is written.
// G > 0: group size known at compile time (vector loads, targets in
// registers); G == 0: any group size up to kMaxG.
constexpr int GPB = 4;

template <int G>
__global__ __launch_bounds__(kBlock) void k_exact_scan(
    const float *__restrict__ T, const float *__restrict__ codebook,
    const float *__restrict__ scales, const int32_t *__restrict__ list,
    const uint32_t *__restrict__ d_count, int64_t max_count, uint16_t *__restrict__ codes,
    unsigned long long *__restrict__ num_changed, unsigned long long *__restrict__ stat_counter,
    int g_rt, int nbits, int gpr, int N)
{
    constexpr int GS = G > 0 ? G : kMaxG;
    const int g = G > 0 ? G : g_rt;
    __shared__ float s_t[GPB][GS];
    __shared__ float s_scale[GPB];
    __shared__ int s_group[GPB];
    __shared__ double s_obj[kBlock / 64];
    __shared__ int s_idx[kBlock / 64];
    __shared__ int s_prev[GPB];          // previous code of each group and its codeword,
    __shared__ float s_cprev[GPB][GS];   // fetched up front: the final tie rule needs them
    const int64_t count = d_count ? (int64_t)*d_count : max_count;
    const int csize = 1 << nbits;
    const int64_t items = (count + GPB - 1) / GPB;
    // thread 0 counts what the block decided and changed; one atomic per block and counter at
    // the end (atomics on one device address are served one after the other)
    unsigned blk_changed = 0u, blk_done = 0u;
    for (int64_t item = blockIdx.x; item < items; item += gridDim.x) {
        const int64_t base = item * GPB;
        const int c_begin = 0, c_end = csize;
        __syncthreads();
        if (threadIdx.x < GPB) {
            int64_t j = base + threadIdx.x;
            int n = j < count ? list[j] : -1;
            if (n < 0 || n >= N) n = -1;
            s_group[threadIdx.x] = n;
            s_scale[threadIdx.x] = n >= 0 ? scales[n / gpr] : 0.0f;
            s_prev[threadIdx.x] = n >= 0 ? (int)(codes[n] & (csize - 1)) : 0;
        }
        __syncthreads();
        for (int e = threadIdx.x; e < GPB * g; e += kBlock) {
            int q = e / g, i = e - q * g;
            int n = s_group[q];
            s_t[q][i] = n >= 0 ? T[(int64_t)n * g + i] : 0.0f;
            s_cprev[q][i] = codebook[(int64_t)s_prev[q] * g + i];
        }
        __syncthreads();
        best_t best[GPB];
#pragma unroll
        for (int q = 0; q < GPB; ++q) {
            best[q].obj = kInf;
            best[q].idx = 0x7fffffff;
        }
        if constexpr (G > 0) {
            double sc[GPB], tt[GPB][GS];
#pragma unroll
            for (int q = 0; q < GPB; ++q) {
                sc[q] = (double)s_scale[q];
#pragma unroll
                for (int i = 0; i < GS; ++i) tt[q][i] = (double)s_t[q][i];
            }
            // kBatch codewords per step: all their loads are issued before the arithmetic, so a
            // step costs one memory round trip (this kernel runs on few groups: latency bound)
            constexpr int kBatch = GS <= 8 ? 4 : 2;   // keeps the register count at two waves per SIMD
            for (int c0 = c_begin + threadIdx.x; c0 < c_end; c0 += kBlock * kBatch) {
                pv_f4 cv[kBatch][GS / 4];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int c = c0 + u * kBlock;
                    const pv_f4 *cw4 = reinterpret_cast<const pv_f4 *>(
                        codebook + (int64_t)(c < c_end ? c : c_begin) * GS);
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
                                // s * c is exact in double (two 24-bit factors), so the fused form
                                // rounds exactly like the product followed by the subtraction
                                double r = fma(sc[q], acc, -tt[q][v4 * 4 + e]);
                                obj[q] = obj[q] + r * r;
                            }
                        }
                    }
                    if (c < c_end) {
#pragma unroll
                        for (int q = 0; q < GPB; ++q)
                            if (obj[q] < best[q].obj) {
                                best[q].obj = obj[q];
                                best[q].idx = c;
                            }
                    }
                }
            }
        } else {
            for (int c = c_begin + threadIdx.x; c < c_end; c += kBlock) {
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
                for (int q = 0; q < GPB; ++q)
                    if (obj[q] < best[q].obj) {
                        best[q].obj = obj[q];
                        best[q].idx = c;
                    }
            }
        }
        best_t mine[GPB];
#pragma unroll
        for (int q = 0; q < GPB; ++q) mine[q] = block_min(best[q], s_obj, s_idx);  // valid in thread 0
        if (threadIdx.x == 0) {
#pragma unroll
            for (int q = 0; q < GPB; ++q) {
                if (s_group[q] < 0) continue;
                const int n = s_group[q];
                const int prev = s_prev[q];
                double o_prev = 0.0;
                for (int i = 0; i < g; ++i) {
                    double acc = (double)s_cprev[q][i];
                    double r = (double)s_scale[q] * acc - (double)s_t[q][i];
                    o_prev = o_prev + r * r;
                }
                int pick = mine[q].idx;
                if (o_prev == mine[q].obj || pick == 0x7fffffff) pick = prev;
                if (pick != prev) {
                    codes[n] = (uint16_t)pick;
                    ++blk_changed;
                }
                ++blk_done;
            }
        }
    }
    if (threadIdx.x == 0) {
        if (blk_changed && num_changed) atomicAdd(num_changed, (unsigned long long)blk_changed);
        if (blk_done && stat_counter) atomicAdd(stat_counter, (unsigned long long)blk_done);
    }
}

// ------------------------------------------------------------------ beam search
//
// One block per listed group.  The beam (tuples + objectives) and the pool of
// candidate objectives live in LDS.  At codebook m, candidate (e, c) is beam
// entry e with its m-th code replaced by c.  Candidates are ranked by
// (objective, tuple in lexicographic order); since all candidates of one step
// agree on positions > m, the tuple order is (rank of entry e's prefix, c).
// The best `keep` candidates are extracted one block-wide argmin at a time.
constexpr int kMaxM = 8;
constexpr int kMaxBeam = 64;
constexpr int kMaxPool = 4096;

__device__ __forceinline__ double beam_objective(const float *__restrict__ codebooks, int M,
                                                 int csize, int g, const uint16_t *tuple,
                                                 int replace_m, int replace_c, float s,
                                                 const float *t)
{
    double obj = 0.0;
    for (int i = 0; i < g; ++i) {
        int c0 = replace_m == 0 ? replace_c : tuple[0];
        double acc = (double)codebooks[((int64_t)c0) * g + i];
        for (int m = 1; m < M; ++m) {
            int cm = replace_m == m ? replace_c : tuple[m];
            acc = acc + (double)codebooks[((int64_t)m * csize + cm) * g + i];
        }
        double r = (double)s * acc - (double)t[i];
        obj = obj + r * r;
    }
    return obj;
}

__global__ __launch_bounds__(kBlock) void k_beam(
    const float *__restrict__ T, const float *__restrict__ codebooks,
    const float *__restrict__ scales, const int32_t *__restrict__ group_idx, int64_t k,
    int beam_width, uint16_t *__restrict__ codes, unsigned long long *__restrict__ num_changed,
    unsigned long long *__restrict__ stat_counter, int g, int M, int nbits, int gpr, int N)
{
    __shared__ double s_pool[kMaxPool];
    __shared__ unsigned char s_taken[kMaxPool];
    __shared__ double s_beam_obj[2][kMaxBeam];
    __shared__ uint16_t s_beam[2][kMaxBeam][kMaxM];
    __shared__ int s_rank[kMaxBeam], s_inv[kMaxBeam];
    __shared__ float s_t[kMaxG];
    __shared__ double s_obj[kBlock / 64];
    __shared__ int s_idx[kBlock / 64];
    __shared__ int s_pick;
    const int csize = 1 << nbits;
    unsigned blk_changed = 0u, blk_done = 0u;   // thread 0's counts, one atomic each at the end
    for (int64_t j = blockIdx.x; j < k; j += gridDim.x) {
        const int n = group_idx[j];
        if (n < 0 || n >= N) continue;  // uniform over the block
        __syncthreads();
        const float s = scales[n / gpr];
        if ((int)threadIdx.x < g) s_t[threadIdx.x] = T[(int64_t)n * g + threadIdx.x];
        if ((int)threadIdx.x < M)
            s_beam[0][0][threadIdx.x] = codes[(int64_t)n * M + threadIdx.x] & (csize - 1);
        __syncthreads();
        if (threadIdx.x == 0)
            s_beam_obj[0][0] = beam_objective(codebooks, M, csize, g, s_beam[0][0], -1, 0, s, s_t);
        __syncthreads();
        const double o_prev = s_beam_obj[0][0];
        int ncur = 1, cur = 0;
        for (int m = 0; m < M && ncur > 0; ++m) {
            // rank of each beam entry's prefix [0, m) in lexicographic order, and its inverse
            if ((int)threadIdx.x < ncur) {
                int r = 0;
                for (int e = 0; e < ncur; ++e) {
                    bool less = false;
                    for (int p = 0; p < m; ++p) {
                        uint16_t a = s_beam[cur][e][p], b = s_beam[cur][threadIdx.x][p];
                        if (a != b) {
                            less = a < b;
                            break;
                        }
                    }
                    r += less;
                }
                s_rank[threadIdx.x] = r;
                s_inv[r] = threadIdx.x;
            }
            const int npool = ncur * csize;
            for (int q = threadIdx.x; q < npool; q += kBlock) {
                int e = q / csize, c = q - e * csize;
                s_pool[q] = beam_objective(codebooks, M, csize, g, s_beam[cur][e], m, c, s, s_t);
                s_taken[q] = 0;
            }
            __syncthreads();
            const int keep = (m == M - 1) ? 1 : (npool < beam_width ? npool : beam_width);
            int got = 0;
            for (int r = 0; r < keep; ++r) {
                best_t b;
                b.obj = kInf;
                b.idx = 0x7fffffff;
                for (int q = threadIdx.x; q < npool; q += kBlock) {
                    if (s_taken[q]) continue;
                    int e = q / csize, c = q - e * csize;
                    int tie = s_rank[e] * csize + c;
                    double o = s_pool[q];
                    if (better(o, tie, b.obj, b.idx)) {  // false for NaN objectives
                        b.obj = o;
                        b.idx = tie;
                    }
                }
                b = block_min(b, s_obj, s_idx);
                if (threadIdx.x == 0) {
                    s_pick = b.idx;
                    if (b.idx != 0x7fffffff) {
                        int e = s_inv[b.idx / csize], c = b.idx % csize;
                        for (int p = 0; p < M; ++p)
                            s_beam[cur ^ 1][r][p] = (p == m) ? (uint16_t)c : s_beam[cur][e][p];
                        s_beam_obj[cur ^ 1][r] = b.obj;
                        s_taken[e * csize + c] = 1;
                    }
                }
                __syncthreads();
                if (s_pick == 0x7fffffff) break;  // nothing comparable left (uniform)
                got = r + 1;
            }
            __syncthreads();
            ncur = got;
            cur ^= 1;
        }
        if (threadIdx.x == 0) {
            if (ncur > 0 && s_beam_obj[cur][0] < o_prev) {
                for (int p = 0; p < M; ++p) codes[(int64_t)n * M + p] = s_beam[cur][0][p];
                ++blk_changed;
            }
            ++blk_done;
        }
    }
    if (threadIdx.x == 0) {
        if (blk_changed && num_changed) atomicAdd(num_changed, (unsigned long long)blk_changed);
        if (blk_done && stat_counter) atomicAdd(stat_counter, (unsigned long long)blk_done);
    }
}

// ------------------------------------------------------------------ beam search, 2 x 256 codewords
//
// The paper's additive configuration (two 8-bit codebooks, beam 8): one WAVE per
// listed group, both codebooks in LDS, no block-wide synchronisation per group.
// Step 0: lane l scores code0 = l, l+64, l+128, l+192 with code1 held; the best
// `beam_width` by (objective, code0) are extracted one wave-wide argmin at a
// time.  Step 1: every lane scores its four code1 values against every kept
// code0 and keeps the best by (objective, code0, code1); one wave-wide argmin
// gives the winner, which replaces the current pair only if strictly better.
// Objectives use the same double-precision chain as everywhere else.
constexpr int kBeam2Max = 8;

// Smallest value over the 64 lanes, in every lane: data-parallel-primitive shifts inside rows
// of 16 lanes, two row broadcasts, then the last lane's value is read out.
__device__ __forceinline__ unsigned wave_min_u32(unsigned v)
{
    constexpr unsigned kId = 0xFFFFFFFFu;   // lanes without a source keep the identity
    v = min(v, (unsigned)__builtin_amdgcn_update_dpp((int)kId, (int)v, 0x111, 0xf, 0xf, false));  // row_shr:1
    v = min(v, (unsigned)__builtin_amdgcn_update_dpp((int)kId, (int)v, 0x112, 0xf, 0xf, false));  // row_shr:2
    v = min(v, (unsigned)__builtin_amdgcn_update_dpp((int)kId, (int)v, 0x114, 0xf, 0xf, false));  // row_shr:4
    v = min(v, (unsigned)__builtin_amdgcn_update_dpp((int)kId, (int)v, 0x118, 0xf, 0xf, false));  // row_shr:8
    v = min(v, (unsigned)__builtin_amdgcn_update_dpp((int)kId, (int)v, 0x142, 0xa, 0xf, false));  // row_bcast:15
    v = min(v, (unsigned)__builtin_amdgcn_update_dpp((int)kId, (int)v, 0x143, 0xc, 0xf, false));  // row_bcast:31
    return (unsigned)__builtin_amdgcn_readlane((int)v, 63);
}

// Lexicographic minimum of (objective, index) over the wave, identical in every lane.
// Objectives are non-negative doubles, so their bit patterns order like unsigned integers:
// three 32-bit reductions (high word, low word among the lanes that hold the smallest high
// word, index among the lanes that hold the smallest objective).
__device__ __forceinline__ best_t wave_argmin_all(best_t b)
{
    const unsigned long long bits = (unsigned long long)__double_as_longlong(b.obj);
    const unsigned hi = (unsigned)(bits >> 32), lo = (unsigned)bits;
    const unsigned mhi = wave_min_u32(hi);
    const unsigned mlo = wave_min_u32(hi == mhi ? lo : 0xFFFFFFFFu);
    const bool mine = hi == mhi && lo == mlo;
    const unsigned midx = wave_min_u32(mine ? (unsigned)b.idx : 0xFFFFFFFFu);
    best_t r;
    r.obj = __longlong_as_double((long long)(((unsigned long long)mhi << 32) | mlo));
    r.idx = (int)midx;
    return r;
}

// One listed group, one wave, the reference arithmetic throughout.  cb0: first codebook
// (floats, row c at c * G); cb1(c, i): entry i of codeword c of the second codebook as a
// double.  Returns (in every lane) whether the pair changed; lane 0 writes the codes.
template <int G, class CB1>
__device__ __forceinline__ bool beam2_group_exact(int lane, int n, const float *__restrict__ T,
                                                  double s, const float *cb0, CB1 cb1,
                                                  int beam_width, uint16_t *__restrict__ codes)
{
    double t[G];
    {
        const pv_f4 *t4 = reinterpret_cast<const pv_f4 *>(T + (int64_t)n * G);
#pragma unroll
        for (int v = 0; v < G / 4; ++v) {
            pv_f4 x = t4[v];
#pragma unroll
            for (int e = 0; e < 4; ++e) t[v * 4 + e] = (double)x[e];
        }
    }
    const int p0 = codes[(int64_t)n * 2] & 255, p1 = codes[(int64_t)n * 2 + 1] & 255;
    // objective of the current pair, and step 0 (code1 = p1 held)
    double fixed[G];
#pragma unroll
    for (int i = 0; i < G; ++i) fixed[i] = cb1(p1, i);
    auto objective0 = [&](int c0) {
        double obj = 0.0;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            double acc = (double)cb0[c0 * G + i];
            acc = acc + fixed[i];
            double r = s * acc - t[i];
            obj = obj + r * r;
        }
        return obj;
    };
    const double o_prev = objective0(p0);
    double o0[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) o0[q] = objective0(lane + 64 * q);
    int beam_code[kBeam2Max];
    int nbeam = 0;
    unsigned taken = 0;
#pragma unroll
    for (int r = 0; r < kBeam2Max; ++r) {
        if (r < beam_width) {        // uniform
            best_t b;
            b.obj = kInf;
            b.idx = 0x7fffffff;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (!((taken >> q) & 1u) && better(o0[q], lane + 64 * q, b.obj, b.idx)) {
                    b.obj = o0[q];
                    b.idx = lane + 64 * q;
                }
            b = wave_argmin_all(b);
            beam_code[r] = b.idx;
            if (b.idx != 0x7fffffff) {
                nbeam = r + 1;
                if ((b.idx & 63) == lane) taken |= 1u << (b.idx >> 6);
            }
        } else {
            beam_code[r] = 0x7fffffff;
        }
    }
    // step 1: code1 over all 256 values for every kept code0
    double c1v[4][G];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < G; ++i) c1v[q][i] = cb1(lane + 64 * q, i);
    best_t w;
    w.obj = kInf;
    w.idx = 0x7fffffff;
#pragma unroll
    for (int e = 0; e < kBeam2Max; ++e) {
        if (e < nbeam && beam_code[e] != 0x7fffffff) {   // uniform (a dropped entry ends the list)
            const int c0 = beam_code[e];
            double c0v[G];
#pragma unroll
            for (int i = 0; i < G; ++i) c0v[i] = (double)cb0[c0 * G + i];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                double obj = 0.0;
#pragma unroll
                for (int i = 0; i < G; ++i) {
                    double acc = c0v[i] + c1v[q][i];
                    double r = s * acc - t[i];
                    obj = obj + r * r;
                }
                const int tie = c0 * 256 + lane + 64 * q;
                if (better(obj, tie, w.obj, w.idx)) {
                    w.obj = obj;
                    w.idx = tie;
                }
            }
        }
    }
    w = wave_argmin_all(w);
    const bool change = w.idx != 0x7fffffff && w.obj < o_prev;
    if (change && lane == 0) {
        codes[(int64_t)n * 2] = (uint16_t)(w.idx >> 8);
        codes[(int64_t)n * 2 + 1] = (uint16_t)(w.idx & 255);
    }
    return change;
}

template <int G>
__global__ __launch_bounds__(kBlock) void k_beam_2x8(
    const float *__restrict__ T, const float *__restrict__ codebooks,
    const float *__restrict__ scales, const int32_t *__restrict__ group_idx, int64_t k,
    int beam_width, uint16_t *__restrict__ codes, unsigned long long *__restrict__ num_changed,
    unsigned long long *__restrict__ stat_counter, int gpr, int N,
    const unsigned long long *__restrict__ d_count)
{
    // d_count: the list length when an earlier kernel of the stream wrote the list
    if (d_count) {
        const int64_t c = (int64_t)*d_count;
        if (c < k) k = c;
    }
    if ((int64_t)blockIdx.x * (kBlock / 64) >= k) return;   // before the tables are loaded
    __shared__ float s_cb[2 * 256 * G];
    for (int i = threadIdx.x; i < 2 * 256 * G / 4; i += kBlock)
        reinterpret_cast<pv_f4 *>(s_cb)[i] = reinterpret_cast<const pv_f4 *>(codebooks)[i];
    __syncthreads();
    const float *cb0 = s_cb, *cb1 = s_cb + 256 * G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned changed = 0, done = 0;
    auto second = [cb1](int c, int i) { return (double)cb1[c * G + i]; };
    for (int64_t j = (int64_t)blockIdx.x * (kBlock / 64) + wave; j < k;
         j += (int64_t)gridDim.x * (kBlock / 64)) {
        const int n = group_idx[j];
        if (n < 0 || n >= N) continue;   // uniform over the wave
        const double s = (double)scales[n / gpr];
        changed += beam2_group_exact<G>(lane, n, T, s, cb0, second, beam_width, codes) ? 1u : 0u;
        ++done;
    }
    // one atomic per block and counter: atomics on one device address are served one after the
    // other (about 10 ns each), and a kernel lasts until the last of them has been served
    __shared__ unsigned s_changed, s_done;
    if (threadIdx.x == 0) s_changed = s_done = 0u;
    __syncthreads();
    if (lane == 0) {
        if (changed) atomicAdd(&s_changed, changed);
        if (done) atomicAdd(&s_done, done);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (s_changed && num_changed) atomicAdd(num_changed, (unsigned long long)s_changed);
        if (s_done && stat_counter) atomicAdd(stat_counter, (unsigned long long)s_done);
    }
}

// ------------------------------------------------------------------ the same search on the matrix cores
//
// App. D's expansion  ||s (c0 + c1) - t||^2 = s^2 ||c1||^2 - 2 s <c1, r> + ||r||^2  with
// r = t - s c0  turns step 1 (every second code against every kept first code) into a
// 256 x G by G x 8 product per group: rows c1[0..G), columns -2 s r_e[0..G), and
// s^2 ||c1||^2 as the accumulator's initial value.  One wave takes TWO groups, so the 16
// columns of the fp64 16x16x4 matrix instruction are all used; the vector ALU only keeps
// the two smallest of the 64 results per lane.  Step 0 (256 candidates per group) uses the same
// expansion on the vector ALU, one group per half wave.
//
// The expanded form rounds differently from the reference chain, so it only FILTERS:
//  - step 0 ranks 24-bit truncations of the expanded objective (the code in the low 8 bits
//    makes the keys unique); the kept set is accepted when the first dropped candidate lies
//    above the last kept one by more than the truncation plus twice the rounding bound E;
//  - step 1 is accepted when the runner-up lies more than 2 E above the winner.
// Then the reference ordering must agree, the winner is re-evaluated with the reference
// chain and compared with the current pair as everywhere else.  A group that fails either
// test is appended to a list that k_beam_2x8 works through afterwards.  E = 2^-44 (|s| 2 cmax + ||t||)^2 bounds the rounding
// of both forms (at most G + 10 roundings of relative size 2^-53 on terms below that
// square) and the 6 index bits written into the low mantissa bits of a step-1 value.
typedef double d4v __attribute__((ext_vector_type(4)));
constexpr int kBeamBlock = 512;
constexpr int kExtra = 3;   // candidates beyond the beam that the step-0 boundary check may pull in

// smallest value over the 32 lanes of each half wave, in every lane of that half: exchanges
// inside quads, inside groups of 8 and of 16 lanes, then rows 0/1 and 2/3 swapped
__device__ __forceinline__ unsigned half_min_u32(unsigned v)
{
    v = min(v, (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xf, 0xf, false));   // lane ^ 1
    v = min(v, (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xf, 0xf, false));   // lane ^ 2
    v = min(v, (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x141, 0xf, 0xf, false));  // row_half_mirror
    v = min(v, (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x140, 0xf, 0xf, false));  // row_mirror
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return min(r[0], r[1]);
}

__device__ __forceinline__ double dpp_quad_f64(double v, int ctrl_sel)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    if (ctrl_sel == 0) {          // lane ^ 1
        lo = __builtin_amdgcn_update_dpp(lo, lo, 0xB1, 0xf, 0xf, false);
        hi = __builtin_amdgcn_update_dpp(hi, hi, 0xB1, 0xf, 0xf, false);
    } else if (ctrl_sel == 1) {   // lane ^ 2
        lo = __builtin_amdgcn_update_dpp(lo, lo, 0x4E, 0xf, 0xf, false);
        hi = __builtin_amdgcn_update_dpp(hi, hi, 0x4E, 0xf, 0xf, false);
    } else {                      // mirror inside groups of 8 lanes
        lo = __builtin_amdgcn_update_dpp(lo, lo, 0x141, 0xf, 0xf, false);
        hi = __builtin_amdgcn_update_dpp(hi, hi, 0x141, 0xf, 0xf, false);
    }
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double column_group_min(double v)
{
    v = fmin(v, dpp_quad_f64(v, 0));
    v = fmin(v, dpp_quad_f64(v, 1));
    v = fmin(v, dpp_quad_f64(v, 2));
    v = fmin(v, __shfl_xor(v, 16));
    v = fmin(v, __shfl_xor(v, 32));
    return v;
}

// running smallest (b1) and second smallest (b2) of a stream of finite values.  (Assembly: the
// compiler's fmin/fmax add an instruction per operand to quiet signalling NaNs.  The caller
// builds v with ordinary code from a matrix result, so the wait the hardware needs after the
// matrix instruction is already in place when these run.)
__device__ __forceinline__ void keep_two(double &b1, double &b2, double v)
{
    double hi;
    asm("v_max_f64 %0, %1, %2" : "=v"(hi) : "v"(b1), "v"(v));
    asm("v_min_f64 %0, %1, %2" : "=v"(b2) : "v"(b2), "v"(hi));
    asm("v_min_f64 %0, %1, %2" : "=v"(b1) : "v"(b1), "v"(v));
}

template <int G>
__global__ __launch_bounds__(kBeamBlock, 4) void k_beam_2x8_mfma(
    const float *__restrict__ T, const float *__restrict__ codebooks,
    const float *__restrict__ scales, const int32_t *__restrict__ group_idx, int64_t k,
    int beam_width, uint16_t *__restrict__ codes, unsigned long long *__restrict__ num_changed,
    unsigned long long *__restrict__ stat_fast, int32_t *__restrict__ redo_list,
    unsigned long long *__restrict__ redo_count, int gpr, int N)
{
    constexpr int KS = G / 4;        // matrix steps that carry coordinates
    constexpr int KP = G + 4;        // operand row: G coordinates, the squared norm, 3 zeros
    constexpr int kWaves = kBeamBlock / 64;   // the tables are shared by 8 waves
    // first codebook: doubles when they fit beside the operand table (no conversions in the
    // inner products), floats for the wider group
    typedef typename std::conditional<G == 8, double, float>::type c0_t;
    __shared__ c0_t s_cb0[256 * G];
    __shared__ double s_a1[256 * KP];
    __shared__ double s_n0[256];
    __shared__ double s_max[4];
    __shared__ int s_bad[4];
    __shared__ double s_wt[kWaves][2][G];
    __shared__ double s_ws[kWaves][2];
    __shared__ int s_wb[kWaves][2][kBeam2Max];
    __shared__ double s_xo[kWaves][2][kBeam2Max + kExtra];   // rare path: exact objectives and codes
    __shared__ int s_xc[kWaves][2][kBeam2Max + kExtra];      // of the candidates around the boundary

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x < 256) {
        // thread c: codeword c of both codebooks
        const int c = threadIdx.x;
        double n0 = 0.0, n1 = 0.0;
        bool bad = false;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const float a = codebooks[c * G + i], b = codebooks[(256 + c) * G + i];
            bad |= !(fabsf(a) <= 3.0e38f) || !(fabsf(b) <= 3.0e38f);
            s_cb0[c * G + i] = (c0_t)a;
            s_a1[c * KP + i] = (double)b;
            n0 = fma((double)a, (double)a, n0);
            n1 = fma((double)b, (double)b, n1);
        }
        s_a1[c * KP + G] = n1;
        s_a1[c * KP + G + 1] = 0.0;
        s_a1[c * KP + G + 2] = 0.0;
        s_a1[c * KP + G + 3] = 0.0;
        s_n0[c] = n0;
        double m = fmax(n0, n1);
        for (int off = 32; off > 0; off >>= 1) m = fmax(m, __shfl_down(m, off));
        const unsigned long long anybad = __ballot(bad);
        if (lane == 0) {
            s_max[wave] = m;
            s_bad[wave] = anybad != 0ull;
        }
    }
    __syncthreads();
    double cmax = 0.0;
    bool tables_ok = true;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        cmax = fmax(cmax, s_max[w]);
        tables_ok = tables_ok && s_bad[w] == 0;
    }
    cmax = sqrt(cmax) * 1.000001;    // largest codeword norm of either codebook

    const int h = lane >> 5, hl = lane & 31;             // step 0: half wave h takes group h of the pair
    const int col = lane & 15, kq = lane >> 4;           // step 1: column and k index of the matrix operands
    const int grp = col >> 3, e = col & 7;
    const int keep = beam_width < kBeam2Max ? beam_width : kBeam2Max;
    unsigned changed = 0, fast = 0;
    const int64_t pairs = (k + 1) / 2;
    for (int64_t pi = (int64_t)blockIdx.x * kWaves + wave; pi < pairs; pi += (int64_t)gridDim.x * kWaves) {
        // ---------------- step 0, one group per half wave
        const int64_t j = 2 * pi + h;
        int n = j < k ? group_idx[j] : -1;
        const bool valid = n >= 0 && n < N;
        if (!valid) n = 0;
        const double s = valid ? (double)scales[n / gpr] : 0.0;
        double t[G];
        {
            const pv_f4 *t4 = reinterpret_cast<const pv_f4 *>(T + (int64_t)n * G);
#pragma unroll
            for (int v = 0; v < G / 4; ++v) {
                pv_f4 x = t4[v];
#pragma unroll
                for (int u = 0; u < 4; ++u) t[v * 4 + u] = valid ? (double)x[u] : 0.0;
            }
        }
        const int p0 = codes[(int64_t)n * 2] & 255, p1 = codes[(int64_t)n * 2 + 1] & 255;
        double o_prev = 0.0;
        double r[G];
        double rr = 0.0, tt = 0.0;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const double c1 = s_a1[p1 * KP + i];
            double acc = (double)s_cb0[p0 * G + i];
            acc = acc + c1;
            const double d = s * acc - t[i];
            o_prev = o_prev + d * d;                 // the reference chain
            r[i] = fma(-s, c1, t[i]);
            rr = fma(r[i], r[i], rr);
            tt = fma(t[i], t[i], tt);
        }
        const double reach = fabs(s) * 2.0 * cmax + sqrt(tt);
        const double E = ldexp(reach * reach, -44);
        bool bad = !tables_ok || !(E < kInf);
        const double s2 = s * s, m2s = -2.0 * s;
        unsigned key[8];
        {
            double v[8];
            unsigned top = 0xFFFFFFFFu;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int c0 = hl + 32 * q;
                double dot = 0.0;
#pragma unroll
                for (int i = 0; i < G; ++i) dot = fma((double)s_cb0[c0 * G + i], r[i], dot);
                v[q] = fma(m2s, dot, s2 * s_n0[c0]) + rr;
                bad |= !(v[q] >= 0.0) || !(v[q] < kInf);
                top = min(top, (unsigned)__double2hiint(v[q]));
            }
            // keys carry the distance above (a lower bound of) the smallest candidate: the 12
            // mantissa bits that fit beside the code then resolve the gaps between the best few
            const double floor_v = __hiloint2double((int)(half_min_u32(top) & ~0xFFu), 0);
#pragma unroll
            for (int q = 0; q < 8; ++q)
                key[q] = ((unsigned)__double2hiint(v[q] - floor_v) & ~0xFFu) | (unsigned)(hl + 32 * q);
        }
        unsigned base = 0, k_last = 0, k_next = 0;
#pragma unroll
        for (int rnd = 0; rnd <= kBeam2Max; ++rnd) {
            if (rnd <= keep) {               // uniform
                // keys are unique within the half: the ones already taken are <= base - 1 and
                // wrap around to the top of the range
                unsigned head = umin3(key[0] - base, key[1] - base, key[2] - base);
                head = umin3(head, key[3] - base, key[4] - base);
                head = umin3(head, key[5] - base, key[6] - base);
                head = min(head, key[7] - base);
                const unsigned m = half_min_u32(head) + base;
                if (rnd < keep) {
                    if (hl == 0) s_wb[wave][h][rnd] = (int)(m & 0xFFu);
                    k_last = m;
                } else {
                    k_next = m;
                }
                base = m + 1u;
            }
        }
        // every dropped candidate is at least lower_of(its key), every kept one below
        // upper_of(its key): the kept set is certain when the two are more than 2 E apart
        auto lower_of = [](unsigned kk) { return __hiloint2double((int)(kk & ~0xFFu), 0); };
        auto upper_of = [](unsigned kk) { return __hiloint2double((int)((kk & ~0xFFu) + 0x100u), 0); };
        bool open = !bad && !(lower_of(k_next) - upper_of(k_last) > 2.0 * E);
        if (__ballot(open) != 0ull) {
            // Rare (a fraction of a percent of the groups): the boundary falls inside the
            // truncation.  Up to kExtra more candidates are extracted until a clear gap
            // follows; the kept ones and these are then ranked with the reference chain
            // (objective, code) and the best `keep` stay.  Both halves run the code, a half
            // whose set was certain ignores the outcome.
            unsigned extra[kExtra + 1];
            extra[0] = k_next;
            int taken_extra = 0;
#pragma unroll
            for (int x = 1; x <= kExtra; ++x) {
                unsigned head = umin3(key[0] - base, key[1] - base, key[2] - base);
                head = umin3(head, key[3] - base, key[4] - base);
                head = umin3(head, key[5] - base, key[6] - base);
                head = min(head, key[7] - base);
                const unsigned m = half_min_u32(head) + base;
                base = m + 1u;
                extra[x] = m;
                if (taken_extra == 0 && lower_of(m) - upper_of(extra[x - 1]) > 2.0 * E) taken_extra = x;
            }
            const int nc = keep + taken_extra;          // candidates to rank, if a gap was found
            int code = 0;
            if (hl < keep) code = s_wb[wave][h][hl < kBeam2Max ? hl : 0];
#pragma unroll
            for (int x = 0; x < kExtra; ++x)
                if (hl == keep + x) code = (int)(extra[x] & 0xFFu);
            double obj = 0.0;
#pragma unroll
            for (int i = 0; i < G; ++i) {
                double acc = (double)s_cb0[code * G + i];
                acc = acc + s_a1[p1 * KP + i];
                const double d = s * acc - t[i];
                obj = obj + d * d;
            }
            if (hl < kBeam2Max + kExtra) {
                s_xo[wave][h][hl] = obj;
                s_xc[wave][h][hl] = code;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            int rank = 0;
            for (int j = 0; j < kBeam2Max + kExtra; ++j)
                if (j < nc && better(s_xo[wave][h][j], s_xc[wave][h][j], obj, code)) ++rank;
            __builtin_amdgcn_wave_barrier();
            if (open && taken_extra > 0 && hl < nc && rank < keep) s_wb[wave][h][rank] = code;
            if (taken_extra > 0) open = false;
        }
        bad |= open;
        if (hl == 0) {
#pragma unroll
            for (int i = 0; i < G; ++i) s_wt[wave][h][i] = t[i];
            s_ws[wave][h] = s;
        }
        const unsigned long long badmask = __ballot(bad);
        const bool skipA = (badmask & 0xFFFFFFFFull) != 0ull, skipB = (badmask >> 32) != 0ull;
        const bool validA = __builtin_amdgcn_readlane((int)valid, 0) != 0;
        const bool validB = __builtin_amdgcn_readlane((int)valid, 32) != 0;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---------------- step 1, both groups in one matrix product
        const bool col_on = (grp ? (validB && !skipB) : (validA && !skipA)) && e < keep;
        const double sg = s_ws[wave][grp];
        const int c0e = col_on ? s_wb[wave][grp][e] : 0;
        double bop[KS];
        double rre = 0.0;
#pragma unroll
        for (int st = 0; st < KS; ++st) {
            const int kk = kq + 4 * st;
            const double re = fma(-sg, (double)s_cb0[c0e * G + kk], s_wt[wave][grp][kk]);
            rre = fma(re, re, rre);
            bop[st] = (-2.0 * sg) * re;
        }
        rre = rre + __shfl_xor(rre, 16);
        rre = rre + __shfl_xor(rre, 32);
        double b1 = kInf, b2 = kInf;
        const double sg2 = sg * sg;
        auto product = [&](int b) {
            d4v acc;
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = sg2 * s_a1[(16 * b + 4 * q + kq) * KP + G];
#pragma unroll
            for (int st = 0; st < KS; ++st)
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(s_a1[(16 * b + col) * KP + kq + 4 * st],
                                                           bop[st], acc, 0, 0, 0);
            return acc;
        };
        // the products of block b + 1 are issued before the results of block b are folded
        d4v cur = product(0);
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            d4v nxt = cur;
            if (b + 1 < 16) nxt = product(b + 1);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // result q of block b is codeword 16 b + 4 q + kq; its number goes into the low bits
                const unsigned lo = ((unsigned)__double2loint(cur[q]) & ~63u) | (unsigned)(b * 4 + q);
                keep_two(b1, b2, __hiloint2double(__double2hiint(cur[q]), (int)lo));
            }
            cur = nxt;
        }
        const int id1 = __double2loint(b1) & 63;
        const int tuple = (c0e << 8) | (16 * (id1 >> 2) + 4 * (id1 & 3) + kq);
        const double o1 = col_on ? b1 + rre : kInf, o2 = col_on ? b2 + rre : kInf;
        const double m1 = column_group_min(o1);
        const bool mine = col_on && o1 == m1;
        const unsigned long long wmask = __ballot(mine);
        const double m2 = column_group_min(mine ? o2 : o1);
        const unsigned long long maskA = 0x00FF00FF00FF00FFull;
        const unsigned long long winA = wmask & maskA, winB = wmask & ~maskA;
        const double EA = __shfl(E, 0), EB = __shfl(E, 32);
        const bool sure = m2 - m1 > 2.0 * (grp ? EB : EA);
        const bool sureA = __builtin_amdgcn_readlane((int)sure, 0) != 0;
        const bool sureB = __builtin_amdgcn_readlane((int)sure, 8) != 0;
        const bool fastA = validA && !skipA && sureA && __popcll(winA) == 1;
        const bool fastB = validB && !skipB && sureB && __popcll(winB) == 1;
        const int laneA = fastA ? __ffsll((long long)winA) - 1 : 0;
        const int laneB = fastB ? __ffsll((long long)winB) - 1 : 0;
        const int tupA = __builtin_amdgcn_readlane(tuple, laneA);
        const int tupB = __builtin_amdgcn_readlane(tuple, laneB);

        // ---------------- accept or keep, in the reference arithmetic
        const bool fast_h = h ? fastB : fastA;
        if (fast_h) {
            const int tup = h ? tupB : tupA;
            const int w0 = tup >> 8, w1 = tup & 255;
            double w = 0.0;
#pragma unroll
            for (int i = 0; i < G; ++i) {
                double acc = (double)s_cb0[w0 * G + i];
                acc = acc + s_a1[w1 * KP + i];
                const double d = s * acc - t[i];
                w = w + d * d;
            }
            if (hl == 0) {
                if (w < o_prev) {
                    codes[(int64_t)n * 2] = (uint16_t)w0;
                    codes[(int64_t)n * 2 + 1] = (uint16_t)w1;
                    ++changed;
                }
                ++fast;
            }
        }
        // groups the filter could not decide go to the list of the exact kernel
        if (valid && !fast_h && hl == 0) redo_list[atomicAdd(redo_count, 1ull)] = n;
        // the next pair overwrites the per-wave staging: every lane is done reading it
        __builtin_amdgcn_wave_barrier();
    }
    // lanes 0 and 32 hold the counters of their halves; one atomic per block and counter
    __shared__ unsigned s_changed, s_fast;
    if (threadIdx.x == 0) s_changed = s_fast = 0u;
    __syncthreads();
    if (hl == 0) {
        if (changed) atomicAdd(&s_changed, (unsigned)changed);
        if (fast) atomicAdd(&s_fast, (unsigned)fast);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (s_changed && num_changed) atomicAdd(num_changed, (unsigned long long)s_changed);
        if (s_fast && stat_fast) atomicAdd(stat_fast, (unsigned long long)s_fast);
    }
}

}  // namespace

pv_status pv_launch_exact_scan(pv_ctx *ctx, const pv_layout *l, const float *T,
                               const float *codebooks, const float *scales, const int32_t *list,
                               const uint32_t *d_count, int64_t max_count, uint16_t *codes,
                               int64_t *num_changed, int64_t *d_stat_counter)
{
    pv_timed t(ctx, PV_K_EXACT_SCAN);
    const int g = l->group_size;
    const int gpr = (int)(l->in_features / g);
    const int N = (int)pv_num_groups(l);
    int64_t blocks = (max_count + GPB - 1) / GPB;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    auto nc = reinterpret_cast<unsigned long long *>(num_changed);
    auto sc = reinterpret_cast<unsigned long long *>(d_stat_counter);
#define PV_SCAN(G_)                                                                               \
    hipLaunchKernelGGL(k_exact_scan<G_>, dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream, T,   \
                       codebooks, scales, list, d_count, max_count, codes, nc, sc, g, l->nbits, gpr, \
                       N)
    if (g == 8) PV_SCAN(8);
    else if (g == 16) PV_SCAN(16);
    else PV_SCAN(0);
#undef PV_SCAN
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

pv_status pv_launch_beam(pv_ctx *ctx, const pv_layout *l, const float *T, const float *codebooks,
                         const float *scales, const int32_t *group_idx, int64_t k,
                         int32_t beam_width, uint16_t *codes, int64_t *num_changed)
{
    pv_timed t(ctx, PV_K_BEAM);
    const int g = l->group_size;
    const int gpr = (int)(l->in_features / g);
    const int N = (int)pv_num_groups(l);
    int64_t *stat = static_cast<int64_t *>(ctx->stats.ptr) + 3;
    if (l->num_codebooks == 2 && l->nbits == 8 && beam_width <= kBeam2Max && (g == 8 || g == 16)) {
        int64_t wblocks = (k + kBlock / 64 - 1) / (kBlock / 64);
        if (wblocks > 2048) wblocks = 2048;
        auto nc = reinterpret_cast<unsigned long long *>(num_changed);
        auto sc = reinterpret_cast<unsigned long long *>(stat);
        if (ctx->search_mode == 0) {
            // matrix-core filter; stats[0] = groups it decided, stats[1] = groups redone exactly,
            // stats[4] = length of the redo list (all cleared by the caller's fill)
            pv_status est = pv_ensure(ctx, ctx->fb_list, (size_t)k * sizeof(int32_t) + 16);
            if (est != PV_OK) return est;
            int32_t *redo = reinterpret_cast<int32_t *>(static_cast<char *>(ctx->fb_list.ptr) + 16);
            auto st0 = reinterpret_cast<unsigned long long *>(stat - 3);
            int64_t pblocks = ((k + 1) / 2 + kBeamBlock / 64 - 1) / (kBeamBlock / 64);
            if (pblocks > 512) pblocks = 512;
            int64_t rblocks = wblocks < 1024 ? wblocks : 1024;
#define PV_BEAM2(G_)                                                                             \
    hipLaunchKernelGGL(k_beam_2x8_mfma<G_>, dim3((unsigned)pblocks), dim3(kBeamBlock), 0, ctx->stream, \
                       T, codebooks, scales, group_idx, k, beam_width, codes, nc, st0, redo,       \
                       st0 + 4, gpr, N);                                                           \
    hipLaunchKernelGGL(k_beam_2x8<G_>, dim3((unsigned)rblocks), dim3(kBlock), 0, ctx->stream, T,   \
                       codebooks, scales, redo, k, beam_width, codes, nc, st0 + 1, gpr, N, st0 + 4)
            if (g == 8) {
                // fp32 / fp16 filter (pv_beam.hip), then the exact kernel on what it leaves
                pv_launch_beam_2x8_f16(ctx, T, codebooks, scales, group_idx, k, beam_width, codes,
                                       num_changed, st0, redo, st0 + 4, gpr, N);
                hipLaunchKernelGGL(k_beam_2x8<8>, dim3((unsigned)rblocks), dim3(kBlock), 0, ctx->stream,
                                   T, codebooks, scales, redo, k, beam_width, codes, nc, st0 + 1, gpr, N,
                                   st0 + 4);
            } else {
                PV_BEAM2(16);
            }
#undef PV_BEAM2
            PV_HIP(ctx, hipGetLastError());
            return PV_OK;
        }
        if (g == 8)
            hipLaunchKernelGGL(k_beam_2x8<8>, dim3((unsigned)wblocks), dim3(kBlock), 0, ctx->stream, T,
                               codebooks, scales, group_idx, k, beam_width, codes, nc, sc, gpr, N,
                               (const unsigned long long *)nullptr);
        else
            hipLaunchKernelGGL(k_beam_2x8<16>, dim3((unsigned)wblocks), dim3(kBlock), 0, ctx->stream, T,
                               codebooks, scales, group_idx, k, beam_width, codes, nc, sc, gpr, N,
                               (const unsigned long long *)nullptr);
        PV_HIP(ctx, hipGetLastError());
        return PV_OK;
    }
    int64_t blocks = k < 16384 ? k : 16384;
    hipLaunchKernelGGL(k_beam, dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream, T, codebooks,
                       scales, group_idx, k, beam_width, codes,
                       reinterpret_cast<unsigned long long *>(num_changed),
                       reinterpret_cast<unsigned long long *>(stat), g, l->num_codebooks, l->nbits,
                       gpr, N);
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

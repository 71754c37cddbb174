// Nearest-codeword search for one codebook (M = 1) on the matrix cores.
//
// The decision "which codeword minimises || s * C[c] - t ||^2" (Eq. 7 argmin,
// App. K "try every code") is taken in double precision, exactly as the plain
// definition does.  The matrix cores only FILTER: by App. D's identity
//     || c - x ||^2 = ||c||^2 - 2 <c, x> + ||x||^2 ,   x = t / s ,
// the distance of every codeword to every selected group is one dense
// contraction.  It is evaluated on fp16 MFMA (fp32 accumulate) for fp16-rounded
// copies c_hi, x_hi of the operands, scaled by a power of two P so that the
// largest codebook entry lies in [16, 32).  The spare K slots of the
// 32x32x16 instruction carry ||c_hi||^2 and ||x_hi||^2 (each split into three
// fp16 pieces, times 1), so an accumulator IS the approximate squared distance
//     D~(c) = || c_hi - x_hi ||^2 + off        (+- E1 of fp32 accumulation),
// a positive float whose bit pattern orders like an unsigned integer.
//
// Running minimum (per lane, in registers): the 16 accumulators of a lane
// belong to one group (column) and to 16 consecutive codewords (a "half
// tile"); they are reduced with v_min3_u32, the low 11 bits of the minimum are
// replaced by the tile number, and the lane keeps the smallest and the second
// smallest such key per partition.  A partition is (codeword range of the
// workgroup) x (half wave) x (tile residue class).
//
// Exact re-rank + certificate (k_rerank): the 16 codewords of the best half
// tile and the previous code are evaluated in double -> E*.  A codeword that
// was not evaluated lies in a half tile whose key is at least the partition's
// runner-up key (or the best key of a partition that was not evaluated), and
//     | ||P C[c] - P x|| - ||c_hi - x_hi|| | <= dC + dx        (triangle inequality)
// with dC = max_c ||P C[c] - c_hi|| and dx = ||P x - x_hi|| (+ division
// rounding), so any codeword that could still reach E* has
//     key value < Vcut = (P sqrt(E*)/|s| + dC + dx)^2 + off + E1 .
// Every best-key half tile below Vcut is evaluated as well; if a runner-up key
// lies below Vcut the group cannot be certified and goes to the exact scan.
// Hence the chosen code is the double-precision argmin with the tie rule of
// the definition, whatever the fp16 rounding did.
#include <type_traits>

#include "pv_internal.h"

// Launch shape of the contraction kernel (tunable at build time).
#ifndef PV_STAGE
#define PV_STAGE 32   // KiB of operand A per LDS stage
#endif
#ifndef PV_STAGE2
#define PV_STAGE2 48  // the same for two k-steps per tile (g = 16): longer stages pay there even
                      // though only one block then fits a compute unit's LDS
#endif
#ifndef PV_NBX
#define PV_NBX 2      // group tiles (32 groups) per wave
#endif
#ifndef PV_WAVES
#define PV_WAVES 8    // waves per block
#endif
#ifndef PV_OCC
#define PV_OCC 2      // blocks per compute unit the register / LDS budget allows
#endif

namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int kBlock = 256;
constexpr int kResidues = 4;         // tile residue classes tracked separately per lane
constexpr unsigned kTileMask = 0x7FFu;
constexpr float kHalfMinNormal = 6.103515625e-05f;  // 2^-14
constexpr float kGamma = 7.62939453125e-06f;        // 2^-17: fp32 accumulation bound per unit of sum|terms|

// cb_meta layout (unsigned[8]): [0] bits of max|C|, [1] bits of max ||c_hi||^2,
// [2] bits of max ||P c - c_hi||^2, [3] bad-codebook flag
// x_meta layout (float[4] per selected group): off, E1, dx, flag (1 = skip the filter)

__device__ __forceinline__ float scale_from_maxabs(unsigned maxbits, bool *ok)
{
    float m = __uint_as_float(maxbits);
    *ok = (m > 0.0f) && (m < 3.0e38f) && (m >= 1.0e-30f);
    if (!*ok) return 1.0f;
    int ex;
    (void)frexpf(m, &ex);          // m = f * 2^ex, f in [0.5, 1)
    return ldexpf(1.0f, 5 - ex);   // m * P in [16, 32)
}

__device__ __forceinline__ _Float16 to_half_flush(float v)
{
    return fabsf(v) < kHalfMinNormal ? (_Float16)0.0f : (_Float16)v;
}

// value -> three fp16 pieces p1 + p2 + p3 ~= v (pieces below the normal range dropped)
__device__ __forceinline__ void split3(float v, _Float16 *p)
{
    p[0] = to_half_flush(v);
    float r = v - (float)p[0];
    p[1] = to_half_flush(r);
    r = r - (float)p[1];
    p[2] = to_half_flush(r);
}

// Largest |entry| of the codebook (fixes the common scale P).  Block 0 also
// clears the per-call counters, which only later launches touch.
__global__ __launch_bounds__(kBlock) void k_cb_absmax(const float *__restrict__ cb, int64_t n,
                                                      unsigned *__restrict__ meta,
                                                      unsigned long long *__restrict__ stats,
                                                      unsigned *__restrict__ fb_count,
                                                      unsigned long long *__restrict__ num_changed)
{
    if (blockIdx.x == 0) {
        if (threadIdx.x < 8) stats[threadIdx.x] = 0ull;
        if (threadIdx.x < 4) fb_count[threadIdx.x] = 0u;
        if (threadIdx.x == 0 && num_changed) *num_changed = 0ull;
    }
    float m = 0.0f;
    bool bad = false;
    const pv_f4 *cb4 = reinterpret_cast<const pv_f4 *>(cb);
    const int64_t n4 = n >> 2;   // the codebook holds 2^B * g floats with g a multiple of 8
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (int64_t)gridDim.x * kBlock) {
        pv_f4 v = cb4[i];
        float a = fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w)));
        bad |= !(fabsf(v.x) <= 3.0e38f) || !(fabsf(v.y) <= 3.0e38f) || !(fabsf(v.z) <= 3.0e38f) ||
               !(fabsf(v.w) <= 3.0e38f);
        m = fmaxf(m, a);
    }
    __shared__ float s_m[kBlock / 64];
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_down(m, off));
    if ((threadIdx.x & 63) == 0) s_m[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {   // one atomic per block: same-address atomics serialise
#pragma unroll
        for (int w = 1; w < kBlock / 64; ++w) m = fmaxf(m, s_m[w]);
        atomicMax(&meta[0], __float_as_uint(m));
    }
    if (bad) atomicMax(&meta[3], 1u);
}

// Operand preparation, one launch for both sides.
//
// Blocks [0, cb_blocks): one thread per codeword -> fp16 operand rows in MFMA
// order + the rounding bound dC.  Operand A of tile t (32 codewords), k-step j,
// k-half h, row r is the 16-byte chunk A[((t * NK + j) * 2 + h) * 32 + r].
// Codeword c sits in tile c / 32 at row 8*(q/4) + 4*hw + q%4 with
// hw = (c/16)%2, q = c%16, so that accumulator q of half wave hw is codeword
// 32*t + 16*hw + q.
//
// Remaining blocks: one thread per selected group (position j in the list):
// x = t / s, its fp16 copy in MFMA operand order, per-group bounds.  Operand B
// of group tile gt, k-step j, k-half h, column col is the chunk
// X[((gt * NK + j) * 2 + h) * 32 + col].
template <int G>
__global__ __launch_bounds__(kBlock) void k_prep(const float *__restrict__ cb, int csize,
                                                 int cb_blocks, unsigned *__restrict__ meta,
                                                 h8 *__restrict__ A, const float *__restrict__ T,
                                                 const float *__restrict__ scales,
                                                 const int32_t *__restrict__ group_idx, int k,
                                                 int k_pad, int gpr, int N, h8 *__restrict__ X,
                                                 float *__restrict__ x_meta)
{
    constexpr int NK = G / 8;
    bool ok;
    const float P = scale_from_maxabs(meta[0], &ok);
    h8 chunk[2 * NK];
#pragma unroll
    for (int u = 0; u < 2 * NK; ++u)
#pragma unroll
        for (int e = 0; e < 8; ++e) chunk[u][e] = (_Float16)0.0f;

    if ((int)blockIdx.x < cb_blocks) {
        const int c = blockIdx.x * kBlock + threadIdx.x;
        float d2 = 0.0f;
        if (c < csize) {
            float n2 = 0.0f;
            const pv_f4 *src = reinterpret_cast<const pv_f4 *>(cb + (int64_t)c * G);
#pragma unroll
            for (int v4 = 0; v4 < G / 4; ++v4) {
                pv_f4 raw = src[v4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = v4 * 4 + e;
                    float v = ok ? P * raw[e] : 0.0f;
                    _Float16 hv = to_half_flush(v);
                    float hf = (float)hv;
                    n2 = fmaf(hf, hf, n2);
                    float d = v - hf;
                    d2 = fmaf(d, d, d2);
                    chunk[i >> 3][i & 7] = (_Float16)(-2.0f * hf);
                }
            }
            _Float16 pieces[3];
            split3(n2, pieces);
            chunk[NK][0] = pieces[0];
            chunk[NK][1] = pieces[1];
            chunk[NK][2] = pieces[2];
            chunk[NK][3] = (_Float16)1.0f;
            chunk[NK][4] = (_Float16)1.0f;
            chunk[NK][5] = (_Float16)1.0f;
            const int tile = c >> 5, hw = (c >> 4) & 1, q = c & 15;
            const int row = 8 * (q >> 2) + 4 * hw + (q & 3);
#pragma unroll
            for (int u = 0; u < 2 * NK; ++u) A[((int64_t)tile * NK * 2 + u) * 32 + row] = chunk[u];
        }
        __shared__ float s_d[kBlock / 64];
        for (int off = 32; off > 0; off >>= 1) d2 = fmaxf(d2, __shfl_down(d2, off));
        if ((threadIdx.x & 63) == 0) s_d[threadIdx.x >> 6] = d2;
        __syncthreads();
        if (threadIdx.x == 0) {
#pragma unroll
            for (int w = 1; w < kBlock / 64; ++w) d2 = fmaxf(d2, s_d[w]);
            atomicMax(&meta[2], __float_as_uint(d2));
        }
        return;
    }

    const int j = ((int)blockIdx.x - cb_blocks) * kBlock + threadIdx.x;
    if (j >= k_pad) return;
    ok = ok && meta[3] == 0u;
    // ||c_hi|| <= sqrt(G) * 32 because every scaled codebook entry is below 32 in magnitude
    const float cmax = 32.0f * (G == 8 ? 2.8285f : 4.0004f);
    float off = 0.0f, e1 = 0.0f, dx = 0.0f, flag = 1.0f;
    const int n = j < k ? group_idx[j] : -1;
    if (n >= 0 && n < N && ok) {
        const float s = scales[n / gpr];
        bool fits = (s != 0.0f) && (fabsf(s) < 3.0e38f);
        const float div = fits ? s : 1.0f;
        float xx = 0.0f, d2 = 0.0f, u2 = 0.0f;
        const pv_f4 *src = reinterpret_cast<const pv_f4 *>(T + (int64_t)n * G);
#pragma unroll
        for (int v4 = 0; v4 < G / 4; ++v4) {
            pv_f4 raw = src[v4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = v4 * 4 + e;
                float u = P * (raw[e] / div);
                if (!(fabsf(u) < 240.0f)) fits = false;   // also catches NaN / inf
                _Float16 hv = to_half_flush(fits ? u : 0.0f);
                float hf = (float)hv;
                xx = fmaf(hf, hf, xx);
                float d = u - hf;
                d2 = fmaf(d, d, d2);
                u2 = fmaf(u, u, u2);
                chunk[i >> 3][i & 7] = hv;
            }
        }
        if (fits && xx < 57000.0f) {
            const float xn = sqrtf(xx) * 1.0001f;
            // bound of the fp32 accumulation error of one accumulator, plus dropped fp16 pieces
            const float e1p = kGamma * (cmax + xn) * (cmax + xn) * 1.01f + 2.5e-4f;
            off = 4.0f * e1p;
            e1 = 1.01f * e1p;
            // rounding of x to fp16, plus the fp32 division and scaling roundings (2^-22 ||u||)
            dx = sqrtf(d2) * 1.0001f + 2.4e-7f * sqrtf(u2) + 1.0e-30f;
            flag = 0.0f;
            _Float16 pieces[3];
            split3(xx + off, pieces);
            chunk[NK][0] = (_Float16)1.0f;
            chunk[NK][1] = (_Float16)1.0f;
            chunk[NK][2] = (_Float16)1.0f;
            chunk[NK][3] = pieces[0];
            chunk[NK][4] = pieces[1];
            chunk[NK][5] = pieces[2];
        } else {
#pragma unroll
            for (int u = 0; u < 2 * NK; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) chunk[u][e] = (_Float16)0.0f;
        }
    }
    const int gt = j >> 5, col = j & 31;
#pragma unroll
    for (int u = 0; u < 2 * NK; ++u) X[((int64_t)gt * NK * 2 + u) * 32 + col] = chunk[u];
    pv_f4 m;
    m.x = off;
    m.y = e1;
    m.z = dx;
    m.w = flag;
    reinterpret_cast<pv_f4 *>(x_meta)[j] = m;
}

// Plain C so that the compiler sees the reads of MFMA results and inserts the
// wait states the hardware requires between a matrix instruction and a vector
// read of its destination (it does not look inside inline assembly).  It folds
// the pair of mins into one v_min3_u32.
__device__ __forceinline__ unsigned umin3(unsigned a, unsigned b, unsigned c)
{
    return min(min(a, b), c);
}

// (m & mask) | tile in one instruction; operands are ordinary vector results.
__device__ __forceinline__ unsigned and_or(unsigned m, unsigned vmask, unsigned tile)
{
    unsigned r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(m), "v"(vmask), "s"(tile));
    return r;
}

__device__ __forceinline__ unsigned umed3(unsigned a, unsigned b, unsigned c)
{
    unsigned r;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Smallest of the 16 accumulators (positive floats compared as integers).  A single chain:
// a tree of independent v_min3 measured no faster here (the waves of a SIMD interleave).
__device__ __forceinline__ unsigned acc_min(const f16v &acc)
{
    unsigned m = umin3(__float_as_uint(acc[0]), __float_as_uint(acc[1]), __float_as_uint(acc[2]));
    m = umin3(m, __float_as_uint(acc[3]), __float_as_uint(acc[4]));
    m = umin3(m, __float_as_uint(acc[5]), __float_as_uint(acc[6]));
    m = umin3(m, __float_as_uint(acc[7]), __float_as_uint(acc[8]));
    m = umin3(m, __float_as_uint(acc[9]), __float_as_uint(acc[10]));
    m = umin3(m, __float_as_uint(acc[11]), __float_as_uint(acc[12]));
    m = umin3(m, __float_as_uint(acc[13]), __float_as_uint(acc[14]));
    return min(m, __float_as_uint(acc[15]));
}

// The distance contraction.  Block = 4 waves; wave w owns NB group tiles (32
// groups each) whose B operands stay in registers; the block streams the
// codeword tiles [t_begin, t_end) of its split through a double-buffered LDS
// stage shared by the 4 waves.  A stage is filled with direct global->LDS
// loads (no staging registers) one stage ahead of its use.  Inside a stage the
// loop is software pipelined: the MFMAs of tile t are issued, then the
// accumulators of tile t-1 are reduced on the vector ALU while the matrix core
// works.  Output: for every group and partition the smallest and second
// smallest key.
template <int NK, int NB>
__global__ __launch_bounds__(PV_WAVES * 64, (PV_OCC * PV_WAVES) / 4) void k_score_mfma(const h8 *__restrict__ A,
                                                          const h8 *__restrict__ X,
                                                          uint2 *__restrict__ partials, int ntiles,
                                                          int nsplit, int P, int merge,
                                                          int gblocks, unsigned *__restrict__ next_item)
{
    constexpr int S = (NK == 1 ? PV_STAGE : PV_STAGE2) / NK;       // tiles per stage
    constexpr int kStageChunks = S * NK * 64;                      // 16-byte chunks per stage
    constexpr int kW = PV_WAVES;                                   // waves per block
    constexpr int kRounds = (kStageChunks / 64 + kW - 1) / kW;     // 64-chunk rows per wave
    static_assert(S % kResidues == 0, "stage must hold whole residue cycles");
    // two stages in SEPARATE arrays (+ one tile of padding each): the compiler then knows that
    // the asynchronous fill of one does not alias the reads of the other and does not wait
    // for the fill before every read
    __shared__ h8 lds0[kStageChunks + NK * 64];
    __shared__ h8 lds1[kStageChunks + NK * 64];
    __shared__ unsigned s_item;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned vmask = ~kTileMask;
    asm volatile("" : "+v"(vmask));   // keep the mask in a vector register
    // Work items = (group block, codeword split).  A block starts with item blockIdx.x; when
    // there are more items than blocks the rest is handed out through a counter, so the
    // blocks in flight stay busy until the items run out (every block leaves when its next
    // item number passes the item count).
    const unsigned items = (unsigned)gblocks * (unsigned)nsplit;
    for (unsigned item = blockIdx.x; item < items;) {
    const int gb = (int)(item % (unsigned)gblocks), split = (int)(item / (unsigned)gblocks);
    const int gtile0 = (gb * kW + wave) * NB;
    const int t_begin = (int)((int64_t)split * ntiles / nsplit);
    const int t_end = (int)((int64_t)(split + 1) * ntiles / nsplit);

    h8 b[NB][NK];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int j = 0; j < NK; ++j) b[nb][j] = X[((int64_t)(gtile0 + nb) * NK + j) * 64 + lane];

    unsigned best[NB][kResidues], second[NB][kResidues];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < kResidues; ++r) best[nb][r] = second[nb][r] = 0xFFFFFFFFu;

    // rows of 64 chunks (1 KiB) are copied by one wave each: lane i -> chunk row + i
    auto fetch = [&](int t0, h8 *dst) {
        const int valid = (t_end - t0 < S ? t_end - t0 : S) * NK * 64;
        const h8 *src = A + (int64_t)t0 * NK * 64;
#pragma unroll
        for (int u = 0; u < kRounds; ++u) {
            const int row = (u * kW + wave) * 64;   // uniform over the wave
            if (row < valid && row < kStageChunks)
                __builtin_amdgcn_global_load_lds(
                    (const void *)(src + row + lane),
                    (__attribute__((address_space(3))) void *)(&dst[row]), 16, 0, 0);
        }
    };

    // While the matrix core works on unit (tile, nb) the vector ALU reduces the unit before
    // it.  One accumulator set per nb (two by tile parity when NB == 1), so a set is rewritten
    // a whole tile after it was last read.
    constexpr int kSets = NB >= 2 ? NB : 2;
    f16v acc[kSets];
    h8 a_cur[NK], a_nxt[NK];
    auto load_a = [&](const h8 *buf, int ts, h8 *a) {
#pragma unroll
        for (int j = 0; j < NK; ++j) a[j] = buf[(ts * NK + j) * 64 + lane];
    };
    auto issue = [&](int nb, int set) {
        f16v c = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < NK; ++j)
            c = __builtin_amdgcn_mfma_f32_32x32x16_f16(a_cur[j], b[nb][j], c, 0, 0, 0);
        acc[set] = c;
    };
    auto reduce = [&](unsigned tile, int nb, int set, int r) {
        const unsigned key = and_or(acc_min(acc[set]), vmask, tile);
        second[nb][r] = umed3(best[nb][r], second[nb][r], key);
        best[nb][r] = min(best[nb][r], key);
    };
    // One stage of `cnt` tiles (FULL: cnt == S, no per-tile guards).
    auto run_stage = [&](const h8 *buf, int t0, int cnt, auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        load_a(buf, 0, a_cur);
#pragma unroll 1
        for (int q4 = 0; q4 < S; q4 += kResidues) {
#pragma unroll
            for (int u = 0; u < kResidues; ++u) {
                const int ts = q4 + u;
                if (FULL || ts + 1 < cnt) load_a(buf, ts + 1, a_nxt);   // one spare tile pads the LDS array
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int set = NB >= 2 ? nb : (u & 1);
                    const int prev_set = NB >= 2 ? (nb + NB - 1) % NB : ((u + 1) & 1);
                    if (FULL || ts < cnt) issue(nb, set);
                    if (nb > 0) {
                        if (FULL || ts < cnt) reduce((unsigned)(t0 + ts), nb - 1, prev_set, u);
                    } else if (ts >= 1 && (FULL || ts - 1 < cnt)) {
                        reduce((unsigned)(t0 + ts - 1), NB - 1, prev_set, (u + kResidues - 1) % kResidues);
                    }
                }
#pragma unroll
                for (int j = 0; j < NK; ++j) a_cur[j] = a_nxt[j];
            }
        }
        if (FULL || cnt == S)
            reduce((unsigned)(t0 + S - 1), NB - 1, NB >= 2 ? NB - 1 : ((kResidues - 1) & 1), kResidues - 1);
    };

    if (t_begin < t_end) fetch(t_begin, lds0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    // stages alternate between the two arrays; each half of the loop body names its arrays
    // statically
    for (int t0 = t_begin; t0 < t_end; t0 += 2 * S) {
        {
            if (t0 + S < t_end) fetch(t0 + S, lds1);
            const int cnt = t_end - t0 < S ? t_end - t0 : S;      // uniform
            if (cnt == S) run_stage(lds0, t0, cnt, std::true_type{});
            else run_stage(lds0, t0, cnt, std::false_type{});
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        }
        const int t1 = t0 + S;
        if (t1 < t_end) {
            if (t1 + S < t_end) fetch(t1 + S, lds0);
            const int cnt = t_end - t1 < S ? t_end - t1 : S;
            if (cnt == S) run_stage(lds1, t1, cnt, std::true_type{});
            else run_stage(lds1, t1, cnt, std::false_type{});
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        }
    }

    const int col = lane & 31, hw = lane >> 5;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int64_t jpos = (int64_t)(gtile0 + nb) * 32 + col;
        if (merge) {
            unsigned b1 = best[nb][0], b2 = second[nb][0];
#pragma unroll
            for (int r = 1; r < kResidues; ++r) {
                // two smallest of {b1, b2, best[r], second[r]} (b1 <= b2, best <= second)
                unsigned lo = min(b1, best[nb][r]);
                unsigned hi = max(b1, best[nb][r]);
                b2 = min(min(b2, second[nb][r]), hi);
                b1 = lo;
            }
            partials[jpos * P + (split * 2 + hw)] = make_uint2(b1, b2);
        } else {
#pragma unroll
            for (int r = 0; r < kResidues; ++r)
                partials[jpos * P + (split * 2 + hw) * kResidues + r] =
                    make_uint2(best[nb][r], second[nb][r]);
        }
    }
    if (items <= gridDim.x) break;          // one item per block: nothing to fetch
    __syncthreads();                        // every wave is done with the LDS stages
    if (threadIdx.x == 0) s_item = gridDim.x + atomicAdd(next_item, 1u);
    __syncthreads();
    item = s_item;                          // uniform over the block
    }
}

// ---------------------------------------------------------------- exact re-rank

struct cand_t {
    double obj;
    int idx;
};

__device__ __forceinline__ bool cand_better(double o1, int i1, double o2, int i2)
{
    return o1 < o2 || (o1 == o2 && i1 < i2);
}

template <int G>
__device__ __forceinline__ double exact_obj(const float *__restrict__ cw, float s, const float *t)
{
    const pv_f4 *c4 = reinterpret_cast<const pv_f4 *>(cw);
    double obj = 0.0;
#pragma unroll
    for (int v4 = 0; v4 < G / 4; ++v4) {
        pv_f4 c = c4[v4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            double acc = (double)c[e];
            // s * c is exact in double (two 24-bit factors): the fused form rounds exactly
            // like the product followed by the subtraction
            double r = fma((double)s, acc, -(double)t[v4 * 4 + e]);
            obj = obj + r * r;
        }
    }
    return obj;
}

// A group the re-rank kernel could not decide alone: the partitions whose codewords must all
// be evaluated (bit p = partition p), and the best candidate found so far.
struct fb_rec_t {
    double obj;
    unsigned long long mask;
    int idx;
    int n;
};

// the same objective on a codeword already in registers
template <int G>
__device__ __forceinline__ double exact_obj_v(const pv_f4 (&c)[G / 4], float s, const float *t)
{
    double obj = 0.0;
#pragma unroll
    for (int v4 = 0; v4 < G / 4; ++v4) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            double acc = (double)c[v4][e];
            double r = fma((double)s, acc, -(double)t[v4 * 4 + e]);
            obj = obj + r * r;
        }
    }
    return obj;
}

// 16 lanes ("team") per selected group; lane q scores codeword q of a half tile.
template <int G>
__global__ __launch_bounds__(kBlock) void k_rerank(
    const float *__restrict__ T, const float *__restrict__ codebook,
    const float *__restrict__ scales, const int32_t *__restrict__ group_idx, int k,
    const uint2 *__restrict__ partials, int P, int per_half, const float *__restrict__ x_meta,
    const unsigned *__restrict__ cb_meta, uint16_t *__restrict__ codes,
    unsigned *__restrict__ block_counts, fb_rec_t *__restrict__ fb_rec,
    unsigned *__restrict__ fb_count, int gpr, int N, int nbits)
{
    __shared__ unsigned s_cnt[3];   // groups decided here, codes changed, candidates evaluated
    if (threadIdx.x < 3) s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const int gid = blockIdx.x * kBlock + threadIdx.x;
    const int j = gid >> 4, q = gid & 15;
    const int n = j < k ? group_idx[j] : -1;
    bool live = n >= 0 && n < N;             // whole 16-lane teams agree on every branch below
    pv_f4 meta = {0.f, 0.f, 0.f, 1.f};
    if (live) meta = reinterpret_cast<const pv_f4 *>(x_meta)[j];
    if (live && meta.w != 0.0f) {            // the filter was skipped for this group: every partition
        if (q == 0) {
            fb_rec_t r;
            r.obj = __builtin_huge_val();
            r.mask = P >= 64 ? ~0ull : ((1ull << P) - 1ull);
            r.idx = 0x7fffffff;
            r.n = n;
            fb_rec[atomicAdd(fb_count, 1u)] = r;
        }
        live = false;
    }
    if (live) {
        const int csize = 1 << nbits;
        const float s = scales[n / gpr];
        float t[G];
        {
            const pv_f4 *t4 = reinterpret_cast<const pv_f4 *>(T + (int64_t)n * G);
#pragma unroll
            for (int v4 = 0; v4 < G / 4; ++v4) {
                pv_f4 v = t4[v4];
                t[v4 * 4 + 0] = v.x;
                t[v4 * 4 + 1] = v.y;
                t[v4 * 4 + 2] = v.z;
                t[v4 * 4 + 3] = v.w;
            }
        }
        // the previous code and the filter's records are fetched side by side: their round
        // trips to memory overlap
        const int prev = codes[n] & (csize - 1);
        constexpr int kMaxRec = 4;           // P <= 64
        uint2 rec[kMaxRec];
#pragma unroll
        for (int u = 0; u < kMaxRec; ++u) {
            int p = q + 16 * u;
            rec[u] = p < P ? partials[(int64_t)j * P + p] : make_uint2(0xFFFFFFFFu, 0xFFFFFFFFu);
        }
        const double o_prev = exact_obj<G>(codebook + (int64_t)prev * G, s, t);
        // best key over all partitions, with its partition
        unsigned long long bk = ~0ull;
#pragma unroll
        for (int u = 0; u < kMaxRec; ++u) {
            int p = q + 16 * u;
            unsigned long long v = ((unsigned long long)rec[u].x << 32) | (unsigned)p;
            bk = v < bk ? v : bk;
        }
#pragma unroll
        for (int m = 8; m > 0; m >>= 1) {
            unsigned long long o = __shfl_xor(bk, m, 16);
            bk = o < bk ? o : bk;
        }
        const unsigned best_key = (unsigned)(bk >> 32);
        const int best_p = (int)(bk & 0xFFFFFFFFu);

        auto eval_half_tile = [&](unsigned key, int p, cand_t &c) {
            const int tile = (int)(key & kTileMask);
            const int hw = (p / per_half) & 1;
            const int cw = tile * 32 + hw * 16 + q;
            double o = exact_obj<G>(codebook + (int64_t)cw * G, s, t);
            if (cand_better(o, cw, c.obj, c.idx)) {
                c.obj = o;
                c.idx = cw;
            }
        };
        auto team_min = [&](cand_t c) {
#pragma unroll
            for (int m = 8; m > 0; m >>= 1) {
                double o = __shfl_xor(c.obj, m, 16);
                int i = __shfl_xor(c.idx, m, 16);
                if (cand_better(o, i, c.obj, c.idx)) {
                    c.obj = o;
                    c.idx = i;
                }
            }
            return c;
        };

        cand_t mine;
        mine.obj = __builtin_huge_val();
        mine.idx = 0x7fffffff;
        eval_half_tile(best_key, best_p, mine);
        cand_t first = team_min(mine);
        if (o_prev < first.obj) first.obj = o_prev;   // the previous code is a candidate too

        // every codeword that was not evaluated and could still reach E* has a key value below vcut
        bool okP;
        const float Pscale = scale_from_maxabs(cb_meta[0], &okP);
        const double dC = sqrt((double)__uint_as_float(cb_meta[2])) * 1.0001 + 1e-30;
        const double dstar = sqrt(first.obj) * (double)Pscale / fabs((double)s) * (1.0 + 1e-9);
        const double reach = dstar + dC + (double)meta.z;
        const double vcut_d = (reach * reach + (double)meta.x + (double)meta.y) * (1.0 + 1e-6);
        const float vcut = __double2float_ru(vcut_d);
        const bool no_bound = !(vcut_d < 3.0e38);     // also true for NaN: nothing can be excluded
        unsigned pending = 0;                         // bit u: rec[u].x needs evaluation
        unsigned long long open = 0;                  // partitions with a second key below vcut
#pragma unroll
        for (int u = 0; u < kMaxRec; ++u) {
            int p = q + 16 * u;
            if (p < P) {
                if (no_bound || __uint_as_float(rec[u].y & ~kTileMask) < vcut) open |= 1ull << p;
                if (p != best_p && __uint_as_float(rec[u].x & ~kTileMask) < vcut) pending |= 1u << u;
            }
        }
#pragma unroll
        for (int m = 8; m > 0; m >>= 1) open |= __shfl_xor(open, m, 16);
        const int team_shift = (threadIdx.x & 63) & ~15;
        // the best key of every other partition below vcut: its half tile is evaluated here
        unsigned extra = 0;
        for (;;) {
            const unsigned long long pb = __ballot(pending != 0);
            const unsigned team = (unsigned)((pb >> team_shift) & 0xFFFFull);
            if (!team) break;
            const int src = __ffs(team) - 1;      // lane of the team with work
            const unsigned their = __shfl(pending, src, 16);
            const int u = __ffs(their) - 1;
            unsigned key = 0;
#pragma unroll
            for (int uu = 0; uu < kMaxRec; ++uu)
                if (uu == u) key = rec[uu].x;
            key = __shfl(key, src, 16);
            eval_half_tile(key, src + 16 * u, mine);
            if (q == src) pending &= ~(1u << u);
            ++extra;
        }
        const cand_t win = team_min(mine);
        if (q == 0) {
            if (open) {
                // a partition may hide further codewords below vcut: all of its codewords are
                // evaluated by the partition scan, which also takes the decision
                fb_rec_t r;
                r.obj = win.obj;
                r.mask = open;
                r.idx = win.idx;
                r.n = n;
                fb_rec[atomicAdd(fb_count, 1u)] = r;
            } else {
                int pick = win.idx;
                if (o_prev <= win.obj || pick == 0x7fffffff) pick = prev;
                if (pick != prev) {
                    codes[n] = (uint16_t)pick;
                    atomicAdd(&s_cnt[1], 1u);
                }
                atomicAdd(&s_cnt[0], 1u);
            }
            atomicAdd(&s_cnt[2], 16u * (1u + extra) + 1u);
        }
    }
    __syncthreads();
    // per-block totals; the last kernel of the call adds them up (no same-address atomics here)
    if (threadIdx.x < 3) block_counts[3 * blockIdx.x + threadIdx.x] = s_cnt[threadIdx.x];
}

// One block per undecided group: every codeword of the group's open partitions is evaluated
// exactly (thread = one codeword position q of 16 tile slots per pass), the lexicographic
// minimum joins the candidate the re-rank kernel found, and the usual rule decides: the
// previous code on an exact tie, else the lowest index.  Partition p = (codeword split,
// half wave, tile residue) as the scoring kernel numbers them.  As the last kernel of a call
// it also clears the filter's codebook statistics and adds up the re-rank counters.
template <int G>
__global__ __launch_bounds__(kBlock) void k_partition_scan(
    const float *__restrict__ T, const float *__restrict__ codebook,
    const float *__restrict__ scales, const fb_rec_t *__restrict__ fb_rec,
    const unsigned *__restrict__ fb_count, uint16_t *__restrict__ codes, int ntiles, int nsplit,
    int per_half, int gpr, int nbits, unsigned long long *__restrict__ num_changed,
    unsigned long long *__restrict__ stats, unsigned *__restrict__ reset_meta,
    const unsigned *__restrict__ rr_counts, int rr_blocks)
{
    __shared__ double s_obj[kBlock / 64];
    __shared__ int s_idx[kBlock / 64];
    const unsigned count = *fb_count;
    const int csize = 1 << nbits;
    const int q = threadIdx.x & 15, slot = threadIdx.x >> 4;
    constexpr int kSlots = kBlock / 16;
    const int stride = per_half == 1 ? 1 : kResidues;     // merged records cover every residue
    unsigned changed = 0;
    for (unsigned item = blockIdx.x; item < count; item += gridDim.x) {
        const fb_rec_t rec = fb_rec[item];
        const int n = rec.n;
        const float s = scales[n / gpr];
        float t[G];
        {
            const pv_f4 *t4 = reinterpret_cast<const pv_f4 *>(T + (int64_t)n * G);
#pragma unroll
            for (int v4 = 0; v4 < G / 4; ++v4) {
                pv_f4 v = t4[v4];
                t[v4 * 4 + 0] = v.x;
                t[v4 * 4 + 1] = v.y;
                t[v4 * 4 + 2] = v.z;
                t[v4 * 4 + 3] = v.w;
            }
        }
        const int prev = codes[n] & (csize - 1);
        cand_t mine;
        mine.obj = __builtin_huge_val();
        mine.idx = 0x7fffffff;
        for (unsigned long long left = rec.mask; left; left &= left - 1) {   // uniform over the block
            const int p = __ffsll((long long)left) - 1;
            const int hw = (p / per_half) & 1;
            const int split = p / (2 * per_half);
            const int t_begin = (int)((int64_t)split * ntiles / nsplit);
            const int t_end = (int)((int64_t)(split + 1) * ntiles / nsplit);
            const int first = t_begin + (per_half == 1 ? 0 : p % per_half);
            // kAhead codewords per thread in flight (their loads first, then the arithmetic in
            // ascending codeword order)
            constexpr int kAhead = G <= 8 ? 4 : 2;
            const int step = kSlots * stride;
            for (int tile = first + slot * stride; tile < t_end; tile += step * kAhead) {
                pv_f4 c[kAhead][G / 4];
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    const int tu = tile + u * step < t_end ? tile + u * step : tile;
                    const pv_f4 *c4 = reinterpret_cast<const pv_f4 *>(
                        codebook + (int64_t)(tu * 32 + hw * 16 + q) * G);
#pragma unroll
                    for (int v4 = 0; v4 < G / 4; ++v4) c[u][v4] = c4[v4];
                }
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    if (tile + u * step < t_end) {
                        const int cw = (tile + u * step) * 32 + hw * 16 + q;
                        const double o = exact_obj_v<G>(c[u], s, t);
                        if (cand_better(o, cw, mine.obj, mine.idx)) {
                            mine.obj = o;
                            mine.idx = cw;
                        }
                    }
                }
            }
        }
        // block-wide lexicographic minimum
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            double o = __shfl_down(mine.obj, off);
            int i = __shfl_down(mine.idx, off);
            if (cand_better(o, i, mine.obj, mine.idx)) {
                mine.obj = o;
                mine.idx = i;
            }
        }
        __syncthreads();
        if ((threadIdx.x & 63) == 0) {
            s_obj[threadIdx.x >> 6] = mine.obj;
            s_idx[threadIdx.x >> 6] = mine.idx;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            cand_t win;
            win.obj = rec.obj;
            win.idx = rec.idx;
            for (int w = 0; w < kBlock / 64; ++w)
                if (cand_better(s_obj[w], s_idx[w], win.obj, win.idx)) {
                    win.obj = s_obj[w];
                    win.idx = s_idx[w];
                }
            const double o_prev = exact_obj<G>(codebook + (int64_t)prev * G, s, t);
            int pick = win.idx;
            if (o_prev <= win.obj || pick == 0x7fffffff) pick = prev;
            if (pick != prev) {
                codes[n] = (uint16_t)pick;
                ++changed;
            }
        }
    }
    if (threadIdx.x == 0 && changed && num_changed) atomicAdd(num_changed, (unsigned long long)changed);
    if (blockIdx.x == 0 && threadIdx.x == 0 && count) atomicAdd(&stats[1], (unsigned long long)count);
    // the filter's codebook statistics are dead once this (last) kernel of a call runs
    if (blockIdx.x == 0 && threadIdx.x < 8) reset_meta[threadIdx.x] = 0u;
    // fold the re-rank kernel's per-block counters (decided, changed, candidates) into the totals
    if (blockIdx.x == gridDim.x - 1) {
        unsigned long long c0 = 0, c1 = 0, c2 = 0;
        constexpr int kU = 4;            // independent loads in flight per thread
        for (int b0 = threadIdx.x; b0 < rr_blocks; b0 += kBlock * kU) {
            unsigned v[kU][3];
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const int b = b0 + u * kBlock;
#pragma unroll
                for (int e = 0; e < 3; ++e) v[u][e] = b < rr_blocks ? rr_counts[3 * b + e] : 0u;
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                c0 += v[u][0];
                c1 += v[u][1];
                c2 += v[u][2];
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            c0 += __shfl_down(c0, off);
            c1 += __shfl_down(c1, off);
            c2 += __shfl_down(c2, off);
        }
        if ((threadIdx.x & 63) == 0) {
            if (c0) atomicAdd(&stats[0], c0);
            if (c2) atomicAdd(&stats[2], c2);
            if (c1 && num_changed) atomicAdd(num_changed, c1);
        }
    }
}

__global__ void k_fill_u32(unsigned *p, int n, unsigned v)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

struct plan_t {
    int NK, NB, k_pad, gblocks, nsplit, P, per_half, merge, ntiles;
};

plan_t make_plan(const pv_layout *l, int64_t k)
{
    plan_t p;
    p.NK = l->group_size / 8;
    p.ntiles = (1 << l->nbits) / 32;
    p.NB = k >= 4096 ? PV_NBX : 1;
    const int per_block = PV_WAVES * p.NB * 32;
    p.gblocks = (int)((k + per_block - 1) / per_block);
    p.k_pad = p.gblocks * per_block;
    // PV_OCC blocks per compute unit fit (registers, LDS).  Few group blocks: cut the
    // codeword range so that the items fill those slots in ONE round (a 13th split that
    // spills 21 blocks into a second round costs 25 %).  Many group blocks: several short
    // items per slot, handed out dynamically, so the tail is one short item.
    const int slots = 256 * PV_OCC;
    int want = slots / p.gblocks;
    if (want < 4) want = (4 * slots + p.gblocks - 1) / p.gblocks;
    if (want > 8 && slots / p.gblocks < 4) want = 8;
    int max_split = p.ntiles / 8;
    if (max_split < 1) max_split = 1;
    if (want > max_split) want = max_split;
    if (want > 32) want = 32;
    if (want < 1) want = 1;
    p.nsplit = want;
    // keep all residue classes apart while the record count per group stays small
    p.merge = (p.nsplit * 2 * kResidues > 32) ? 1 : 0;
    p.per_half = p.merge ? 1 : kResidues;
    p.P = p.nsplit * 2 * p.per_half;
    return p;
}

// Nothing but matrix instructions: four independent accumulators per wave, four waves per
// SIMD over the whole chip (the matrix-core ceiling of the box at its current clock).
constexpr int kProbeBlocks = 256 * 4;
__global__ __launch_bounds__(kBlock, 4) void k_probe_mfma(float *__restrict__ sink, int64_t iters)
{
    const int lane = threadIdx.x & 63;
    h8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (_Float16)(0.001f * (float)(lane + e));
        b[e] = (_Float16)(0.5f + 0.01f * (float)e);
    }
    f16v acc[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[n][r] = 0.0f;
    for (int64_t it = 0; it + 4 <= iters; it += 4) {
#pragma unroll
        for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[n], 0, 0, 0);
    }
    if (blockIdx.x < 256) {
        float s = 0.0f;
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += acc[n][r];
        sink[((int64_t)blockIdx.x * 16 + (threadIdx.x >> 6)) * 64 + lane] = s;
    }
}

}  // namespace

pv_status pv_launch_probe_mfma(pv_ctx *ctx, int64_t iters, float *sink, int64_t *waves_out)
{
    pv_timed t(ctx, PV_K_PROBE_MFMA);
    hipLaunchKernelGGL(k_probe_mfma, dim3(kProbeBlocks), dim3(kBlock), 0, ctx->stream, sink, iters);
    PV_HIP(ctx, hipGetLastError());
    if (waves_out) *waves_out = (int64_t)kProbeBlocks * (kBlock / 64);
    return PV_OK;
}

bool pv_mfma_supported(const pv_layout *l)
{
    return l->num_codebooks == 1 && (l->group_size == 8 || l->group_size == 16) && l->nbits >= 5;
}

pv_status pv_launch_mfma_search(pv_ctx *ctx, const pv_layout *l, const float *T,
                                const float *codebooks, const float *scales,
                                const int32_t *group_idx, int64_t k, uint16_t *codes,
                                int64_t *num_changed)
{
    const plan_t p = make_plan(l, k);
    const int g = l->group_size;
    const int csize = 1 << l->nbits;
    const int gpr = (int)(l->in_features / g);
    const int N = (int)pv_num_groups(l);
    pv_status st;
    if ((st = pv_ensure(ctx, ctx->cb_f16, (size_t)csize * p.NK * 32)) != PV_OK) return st;
    if ((st = pv_ensure(ctx, ctx->cb_meta, 8 * sizeof(unsigned), /*zero_new=*/true)) != PV_OK) return st;
    if ((st = pv_ensure(ctx, ctx->x_f16, (size_t)p.k_pad * p.NK * 32)) != PV_OK) return st;
    if ((st = pv_ensure(ctx, ctx->x_meta, (size_t)p.k_pad * 4 * sizeof(float))) != PV_OK) return st;
    if ((st = pv_ensure(ctx, ctx->partials, (size_t)p.k_pad * p.P * sizeof(uint2))) != PV_OK) return st;
    if ((st = pv_ensure(ctx, ctx->fb_list, 4 * sizeof(int32_t) + (size_t)k * sizeof(fb_rec_t) + 64)) != PV_OK)
        return st;
    const int rr_blocks = (int)((k * 16 + kBlock - 1) / kBlock);
    if ((st = pv_ensure(ctx, ctx->rr_counts, (size_t)rr_blocks * 3 * sizeof(unsigned))) != PV_OK) return st;
    unsigned *rr_counts = static_cast<unsigned *>(ctx->rr_counts.ptr);
    h8 *A = static_cast<h8 *>(ctx->cb_f16.ptr);
    h8 *X = static_cast<h8 *>(ctx->x_f16.ptr);
    unsigned *cb_meta = static_cast<unsigned *>(ctx->cb_meta.ptr);
    float *x_meta = static_cast<float *>(ctx->x_meta.ptr);
    uint2 *partials = static_cast<uint2 *>(ctx->partials.ptr);
    unsigned *fb_count = reinterpret_cast<unsigned *>(ctx->fb_list.ptr);       // 4 counters, then the records
    fb_rec_t *fb_rec = reinterpret_cast<fb_rec_t *>(static_cast<char *>(ctx->fb_list.ptr) + 16);
    unsigned long long *stats = static_cast<unsigned long long *>(ctx->stats.ptr);
    hipStream_t sm = ctx->stream;
    if (ctx->meta_dirty) {   // a previous call did not run to its last kernel
        hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, sm, cb_meta, 8, 0u);
    }
    ctx->meta_dirty = true;
    {
        pv_timed t(ctx, PV_K_PREP);
        const int64_t ncb = (int64_t)csize * g;
        int blocks = (int)((ncb / 4 + kBlock * 4 - 1) / (kBlock * 4));
        if (blocks > 128) blocks = 128;
        hipLaunchKernelGGL(k_cb_absmax, dim3(blocks), dim3(kBlock), 0, sm, codebooks, ncb, cb_meta,
                           stats, fb_count, reinterpret_cast<unsigned long long *>(num_changed));
        const int cb_blocks = (csize + kBlock - 1) / kBlock;
        const int x_blocks = (p.k_pad + kBlock - 1) / kBlock;
        if (g == 8)
            hipLaunchKernelGGL(k_prep<8>, dim3(cb_blocks + x_blocks), dim3(kBlock), 0, sm, codebooks,
                               csize, cb_blocks, cb_meta, A, T, scales, group_idx, (int)k, p.k_pad,
                               gpr, N, X, x_meta);
        else
            hipLaunchKernelGGL(k_prep<16>, dim3(cb_blocks + x_blocks), dim3(kBlock), 0, sm,
                               codebooks, csize, cb_blocks, cb_meta, A, T, scales, group_idx, (int)k,
                               p.k_pad, gpr, N, X, x_meta);
    }
    {
        pv_timed t(ctx, PV_K_SCORE_MFMA);
        const int items = p.gblocks * p.nsplit;
        dim3 grid(items < 256 * PV_OCC ? items : 256 * PV_OCC);
#define PV_SCORE(NK_, NB_)                                                                     \
    hipLaunchKernelGGL((k_score_mfma<NK_, NB_>), grid, dim3(PV_WAVES * 64), 0, sm, A, X, partials,    \
                       p.ntiles, p.nsplit, p.P, p.merge, p.gblocks, fb_count + 1)
        if (p.NK == 1) {
            if (p.NB == PV_NBX) PV_SCORE(1, PV_NBX);
            else PV_SCORE(1, 1);
        } else {
            if (p.NB == PV_NBX) PV_SCORE(2, PV_NBX);
            else PV_SCORE(2, 1);
        }
#undef PV_SCORE
    }
    {
        pv_timed t(ctx, PV_K_RERANK);
        const dim3 rgrid((unsigned)rr_blocks);
        if (g == 8)
            hipLaunchKernelGGL(k_rerank<8>, rgrid, dim3(kBlock), 0, sm, T, codebooks, scales,
                               group_idx, (int)k, partials, p.P, p.per_half, x_meta, cb_meta, codes,
                               rr_counts, fb_rec, fb_count, gpr, N, l->nbits);
        else
            hipLaunchKernelGGL(k_rerank<16>, rgrid, dim3(kBlock), 0, sm, T, codebooks, scales,
                               group_idx, (int)k, partials, p.P, p.per_half, x_meta, cb_meta, codes,
                               rr_counts, fb_rec, fb_count, gpr, N, l->nbits);
    }
    {
        pv_timed t(ctx, PV_K_EXACT_SCAN);
        const unsigned sblocks = (unsigned)(k < 2048 ? k : 2048);
        auto nc = reinterpret_cast<unsigned long long *>(num_changed);
        if (g == 8)
            hipLaunchKernelGGL(k_partition_scan<8>, dim3(sblocks), dim3(kBlock), 0, sm, T, codebooks,
                               scales, fb_rec, fb_count, codes, p.ntiles, p.nsplit, p.per_half, gpr,
                               l->nbits, nc, stats, cb_meta, rr_counts, rr_blocks);
        else
            hipLaunchKernelGGL(k_partition_scan<16>, dim3(sblocks), dim3(kBlock), 0, sm, T, codebooks,
                               scales, fb_rec, fb_count, codes, p.ntiles, p.nsplit, p.per_half, gpr,
                               l->nbits, nc, stats, cb_meta, rr_counts, rr_blocks);
    }
    PV_HIP(ctx, hipGetLastError());
    ctx->meta_dirty = false;
    return PV_OK;
}

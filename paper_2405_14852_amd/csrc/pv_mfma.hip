// Nearest-codeword search for one codebook (M = 1) on the matrix cores.
//
// The decision "which codeword minimises || s * C[c] - t ||^2" (Eq. 7 argmin,
// App. K "try every code") is taken in double precision, exactly as the plain
// definition does.  The matrix cores only FILTER: by App. D's identity
//     || c - x ||^2 = ||c||^2 - 2 <c, x> + ||x||^2 ,   x = t / s ,
// the distance of every codeword to every selected group is one dense
// contraction.  It is evaluated on fp16 MFMA (fp32 accumulate) for fp16-rounded
// copies c_hi, x_hi of the operands, scaled by a power of two P so that the
// largest codebook entry lies in [16, 32), in the form of a "closeness"
//     kv(c) = SHIFT + 2 <c_hi, x_hi> - ||c_hi||^2  =  SHIFT + ||x_hi||^2 - || c_hi - x_hi ||^2
// which is LARGE for near codewords.  SHIFT = (||x_hi|| + min_c ||c|| + margin)^2 is a constant
// of the group that makes kv non-negative for at least the smallest codeword, so a negative kv
// marks a codeword farther away than that one.
//   g = 8:  the spare K slots of the 32x32x16 instruction carry -||c_hi||^2 (three fp16
//           pieces against -1) and SHIFT (three pieces against 1): the accumulator IS kv.
//   g = 16: all 16 K slots carry data, so the accumulator is 2 <c_hi, x_hi> alone.  The
//           codebook is laid out in ascending order of ||c_hi||^2, so that the norms of the
//           32 U codewords behind one key differ by next to nothing: after the maximum of the
//           products was taken (never below zero, which can only raise it), the smallest of
//           those norms is subtracted (again raising the key at most) and SHIFT added.
//
// Running maximum (per lane, in registers): the 16 accumulators of a lane belong to one group
// (column) and to 16 consecutive codeword positions (a "half tile"); they are reduced with
// v_max3_i32 on the float bits (correct whenever the maximum is non-negative; if every value
// is negative the result is some negative value, which is all that is needed), the chain runs
// on over the U tiles of a "super-unit", the low 11 bits of the result are replaced by the
// super-unit number, and the lane keeps the largest and second largest such key per partition.
// A partition is (codeword range of the work item) x (half wave) x (super-unit residue class).
//
// Exact re-rank + certificate (k_rerank): the 16 U codewords behind the best key and the
// previous code are evaluated in double -> E*.  With the triangle inequality
//     | ||P C[c] - P x|| - ||c_hi - x_hi|| | <= dC + dx
// (dC = max_c ||P C[c] - c_hi||, dx = ||P x - x_hi|| + division rounding) a codeword can reach
// E* only if  kv(c) >= SHIFT + ||x_hi||^2 - (P sqrt(E*)/|s| + dC + dx)^2, and the key behind
// which it sits is at least kv(c) - E1 (fp32 accumulation, dropped pieces, truncation).  Every
// best key at or above that cut is evaluated as well; a partition whose runner-up key reaches
// the cut may hide further codewords and is scanned completely, in the same kernel.  Hence the
// chosen code is the double-precision argmin with the tie rule of the definition, whatever the
// fp16 rounding did.
#include "pv_internal.h"
#include "pv_dpp.h"

// Launch shape of the contraction kernel (tunable at build time).
#ifndef PV_STAGE
#define PV_STAGE 32   // KiB of operand A per LDS stage (= codeword tiles per stage)
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
#ifndef PV_SUPER
#define PV_SUPER 2    // codeword tiles behind one key (a super-unit)
#endif
#ifndef PV_TEAM
#define PV_TEAM 8     // lanes of the re-rank kernel that share one group at g = 8 (twice as many at g = 16: measured)
#endif
constexpr int rerank_team(int g) { return g == 16 && PV_TEAM < 16 ? 2 * PV_TEAM : PV_TEAM; }
#ifndef PV_DEPTH
#define PV_DEPTH 2    // units (matrix instructions) in flight before a unit's accumulators are reduced
#endif

namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int kBlock = 256;
constexpr int kU = PV_SUPER;
constexpr int kResidues = 4;         // super-unit residue classes tracked separately per lane
constexpr unsigned kKeyMask = 0x7FFu;
constexpr int kNoKey = (int)0x80000000;             // "no key": below every key a lane can form
constexpr float kHalfMinNormal = 6.103515625e-05f;  // 2^-14
constexpr float kGamma = 7.62939453125e-06f;        // 2^-17: fp32 accumulation bound per unit of sum|terms|
constexpr float kNormMargin = 0.04f;                // >= max_c | ||c_hi|| - ||P c|| | (half an fp16 ulp below 32, 16 dims)
constexpr int kNormBins = 65536;                    // buckets of the norm ordering (g = 16)

// cb_meta layout (unsigned[8]): [0] bits of max|C|, [1] ~bits of min_c ||c||^2 (unscaled),
// [2] bits of max ||P c - c_hi||^2, [3] bad-codebook flag, [4] blocks of the re-rank kernel done,
// [5] bits of max_c ||c||^2 (unscaled)
// x_meta layout (float[4] per selected group): SHIFT as the kernel adds it, ||x_hi||^2, E1,
// dx (negative: the filter is skipped for this group)

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

// Bucket of a squared norm of scaled fp16 codeword entries (at most 16 * 32^2): the 32 octaves
// below 2^15, 2048 buckets each; ascending in the norm.
__device__ __forceinline__ int norm_bucket(float n2)
{
    const int e = (int)(__float_as_uint(n2) >> 12);
    const int top = (int)(0x47000000u >> 12);      // bits of 32768.0f
    const int key = e - (top - (kNormBins - 1));
    return key < 0 ? 0 : (key > kNormBins - 1 ? kNormBins - 1 : key);
}

// Residue cycles of the table owned by codeword split `split` of `nsplit`: cycles are dealt to
// the splits round robin by rank (for g = 16 the rank is the norm order, so every split sees
// every norm band: codewords near a target have similar norms, and they should fall into
// different partitions), and a split's cycles lie next to each other in memory.
__device__ __host__ __forceinline__ int split_count(int split, int ncyc, int nsplit)
{
    return (ncyc - split + nsplit - 1) / nsplit;
}
__device__ __host__ __forceinline__ int split_begin(int split, int ncyc, int nsplit)
{
    // sum of split_count over the splits before: the first ncyc % nsplit splits hold one more
    const int q = ncyc / nsplit, r = ncyc % nsplit;
    return split * q + (split < r ? split : r);
}

// fp16 copy of one scaled codeword: c_hi (as floats), its squared norm, the squared rounding error
template <int G>
__device__ __forceinline__ void round_codeword(const float *__restrict__ cw, float P, bool ok,
                                               float (&hf)[G], float &n2, float &d2)
{
    n2 = 0.0f;
    d2 = 0.0f;
    const pv_f4 *src = reinterpret_cast<const pv_f4 *>(cw);
#pragma unroll
    for (int v4 = 0; v4 < G / 4; ++v4) {
        pv_f4 raw = src[v4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = v4 * 4 + e;
            float v = ok ? P * raw[e] : 0.0f;
            hf[i] = (float)to_half_flush(v);
            n2 = fmaf(hf[i], hf[i], n2);
            float d = v - hf[i];
            d2 = fmaf(d, d, d2);
        }
    }
}

// Codebook statistics, one thread per codeword: largest |entry| (fixes the common scale P),
// smallest squared norm, non-finite entries.  Block 0 also clears the per-call counters, and
// the grid clears the tables of the norm ordering (g = 16), which only later launches touch.
// The statistics live in one of two slots, alternating from call to call: this kernel clears
// the slot of the next call (nothing of this call reads it), so no kernel has to run last.
template <int G>
__global__ __launch_bounds__(kBlock) void k_cb_stats(const float *__restrict__ cb, int csize,
                                                     unsigned *__restrict__ meta,
                                                     unsigned *__restrict__ meta_next,
                                                     unsigned long long *__restrict__ stats,
                                                     unsigned *__restrict__ fb_count,
                                                     unsigned long long *__restrict__ num_changed,
                                                     unsigned *__restrict__ hist,
                                                     unsigned *__restrict__ nmin_bits, int nsu_alloc,
                                                     unsigned long long *__restrict__ change_slots,
                                                     int nslots)
{
    for (int i = blockIdx.x * kBlock + threadIdx.x; i < nslots; i += gridDim.x * kBlock) change_slots[i] = 0ull;
    if (blockIdx.x == 0) {
        if (threadIdx.x < 8) stats[threadIdx.x] = 0ull;
        if (threadIdx.x < 8) meta_next[threadIdx.x] = 0u;   // the statistics slot of the next call
        if (threadIdx.x < 4) fb_count[threadIdx.x] = 0u;
        if (threadIdx.x == 0 && num_changed) *num_changed = 0ull;
    }
    const int tid = blockIdx.x * kBlock + threadIdx.x, nthreads = gridDim.x * kBlock;
    if (hist) {
        for (int i = tid; i < kNormBins; i += nthreads) hist[i] = 0u;
        for (int i = tid; i < nsu_alloc; i += nthreads) nmin_bits[i] = 0x7F800000u;   // +inf
    }
    float m = 0.0f, nmin = __builtin_huge_valf(), nmax = 0.0f;
    bool bad = false;
    for (int c = tid; c < csize; c += nthreads) {
        const pv_f4 *src = reinterpret_cast<const pv_f4 *>(cb + (int64_t)c * G);
        float n2 = 0.0f;
#pragma unroll
        for (int v4 = 0; v4 < G / 4; ++v4) {
            pv_f4 v = src[v4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float a = fabsf(v[e]);
                bad |= !(a <= 3.0e38f);
                m = fmaxf(m, a);
                n2 = fmaf(v[e], v[e], n2);
            }
        }
        nmin = fminf(nmin, n2);
        nmax = fmaxf(nmax, n2);
    }
    __shared__ float s_m[kBlock / 64], s_n[kBlock / 64], s_x[kBlock / 64];
    for (int off = 32; off > 0; off >>= 1) {
        m = fmaxf(m, __shfl_down(m, off));
        nmin = fminf(nmin, __shfl_down(nmin, off));
        nmax = fmaxf(nmax, __shfl_down(nmax, off));
    }
    if ((threadIdx.x & 63) == 0) {
        s_m[threadIdx.x >> 6] = m;
        s_n[threadIdx.x >> 6] = nmin;
        s_x[threadIdx.x >> 6] = nmax;
    }
    __syncthreads();
    if (threadIdx.x == 0) {   // one atomic per block: same-address atomics serialise
#pragma unroll
        for (int w = 1; w < kBlock / 64; ++w) {
            m = fmaxf(m, s_m[w]);
            nmin = fminf(nmin, s_n[w]);
            nmax = fmaxf(nmax, s_x[w]);
        }
        atomicMax(&meta[0], __float_as_uint(m));
        if (nmin >= 0.0f && nmin < 3.0e38f) atomicMax(&meta[1], ~__float_as_uint(nmin));
        if (nmax >= 0.0f && nmax < 3.0e38f) atomicMax(&meta[5], __float_as_uint(nmax));
        else bad = true;
    }
    if (bad) atomicMax(&meta[3], 1u);
}

// Norm ordering, step 1 (g = 16): bucket of every codeword's ||c_hi||^2 and the bucket counts.
template <int G>
__global__ __launch_bounds__(kBlock) void k_cb_bucket(const float *__restrict__ cb, int csize,
                                                      const unsigned *__restrict__ meta,
                                                      uint16_t *__restrict__ bucket,
                                                      unsigned *__restrict__ hist)
{
    bool ok;
    const float P = scale_from_maxabs(meta[0], &ok);
    const int c = blockIdx.x * kBlock + threadIdx.x;
    if (c >= csize) return;
    float hf[G], n2, d2;
    round_codeword<G>(cb + (int64_t)c * G, P, ok, hf, n2, d2);
    const int b = norm_bucket(n2);
    bucket[c] = (uint16_t)b;
    atomicAdd(&hist[b], 1u);
}

// Step 2: exclusive prefix sum of the bucket counts.  Block b owns 1024 buckets; it adds up
// everything before them itself (coalesced reads of a table that sits in L2: cheaper than any
// exchange between blocks) and scans its own.
constexpr int kScanBlock = 1024;
__global__ __launch_bounds__(kScanBlock) void k_cb_scan(const unsigned *__restrict__ hist,
                                                        unsigned *__restrict__ offsets)
{
    __shared__ unsigned s_w[kScanBlock / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int first = blockIdx.x * kScanBlock;
    unsigned before = 0;
    for (int i0 = 0; i0 < first; i0 += 8 * kScanBlock) {   // eight loads in flight per thread
        unsigned v8[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * kScanBlock + threadIdx.x;
            v8[u] = i < first ? hist[i] : 0u;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) before += v8[u];
    }
    for (int off = 32; off > 0; off >>= 1) before += __shfl_xor(before, off);
    if (lane == 0) s_w[wave] = before;
    __syncthreads();
    unsigned base = 0;
#pragma unroll
    for (int w = 0; w < kScanBlock / 64; ++w) base += s_w[w];
    __syncthreads();
    const unsigned v = hist[first + threadIdx.x];
    unsigned inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        unsigned u = __shfl_up(inc, off);
        if (lane >= off) inc += u;
    }
    if (lane == 63) s_w[wave] = inc;
    __syncthreads();
    for (int w = 0; w < wave; ++w) base += s_w[w];
    offsets[first + threadIdx.x] = base + inc - v;
}

// Operand preparation, one launch for both sides.
//
// Blocks [0, cb_blocks): one thread per codeword position of the padded table.  A codeword is
// placed at position pos (g = 8: its own index; g = 16: the next free rank of its norm bucket,
// ranks ascending in ||c_hi||^2 up to the bucket width, and the residue cycles of the ranking
// dealt round robin to the codeword splits), perm[pos] names it.  The 32 U
// positions of super-unit su are split in two runs of 16 U, one per half wave hw, each run in
// U pieces of 16, one per tile: position pos = ((su * 2 + hw) * U + uu) * 16 + q sits in tile
// su * U + uu at row 8*(q/4) + 4*hw + q%4, so that accumulator q of half wave hw is that
// position, and the 16 U positions behind one key of a lane are consecutive (for g = 16: in
// norm order, their smallest norm is nmin[su * 2 + hw]).  Operand A of tile t, k-half h, row r
// is the 16-byte chunk A[(t * 2 + h) * 32 + r]:
//   g = 8:  k-half 0 = 2 c_hi, k-half 1 = { three pieces of ||c_hi||^2, 1, 1, 1, 0, 0 }
//   g = 16: k-half 0 = 2 c_hi[0..8), k-half 1 = 2 c_hi[8..16)
// Positions past the codebook's end (padding up to whole super-units) are zero rows.
//
// Remaining blocks: one thread per selected group (position j in the list): x = t / s, its
// fp16 copy, per-group bounds.  Operand B of group tile gt, k-half h, column col is the chunk
// X[(gt * 2 + h) * 32 + col]:
//   g = 8:  k-half 0 = x_hi, k-half 1 = { -1, -1, -1, three pieces of SHIFT, 0, 0 }
//   g = 16: the two halves of x_hi (SHIFT travels in x_meta)
// and x_stage[j] = { the g target values, the row scale, the current code, the group id } is
// what the re-rank kernel needs of the group, in one place (its loads then depend on nothing
// but the list position).
#ifndef PV_CB_PER
#define PV_CB_PER 4
#endif
constexpr int kCbPer = PV_CB_PER;   // codeword positions a thread of the codebook part
template <int G>
__global__ __launch_bounds__(kBlock) void k_prep(const float *__restrict__ cb, int csize, int cpad,
                                                 int cb_blocks, unsigned *__restrict__ meta,
                                                 h8 *__restrict__ A, uint16_t *__restrict__ perm,
                                                 const uint16_t *__restrict__ bucket,
                                                 unsigned *__restrict__ bucket_next,
                                                 unsigned *__restrict__ nmin_bits,
                                                 float *__restrict__ cnorm,
                                                 const float *__restrict__ T,
                                                 const float *__restrict__ scales,
                                                 const int32_t *__restrict__ group_idx, int k,
                                                 int k_pad, int gpr, int N, h8 *__restrict__ X,
                                                 float *__restrict__ x_meta,
                                                 const uint16_t *__restrict__ codes, int csize_mask,
                                                 float *__restrict__ x_stage, int ncyc, int nsplit)
{
    bool ok;
    const float P = scale_from_maxabs(meta[0], &ok);
    h8 chunk[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int e = 0; e < 8; ++e) chunk[u][e] = (_Float16)0.0f;

    if ((int)blockIdx.x < cb_blocks) {
        float d2 = 0.0f;
        // kCbPer codeword positions a thread: a quarter of the blocks, and of the atomics on the
        // one address that takes the largest rounding error
#pragma unroll 1
        for (int rep = 0; rep < kCbPer; ++rep) {
        const int c = (blockIdx.x * kCbPer + rep) * kBlock + threadIdx.x;
        if (rep > 0) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) chunk[u][e] = (_Float16)0.0f;
        }
        if (c < cpad) {
            int pos = c;
            if (c < csize) {
                float hf[G], n2, d2c;
                round_codeword<G>(cb + (int64_t)c * G, P, ok, hf, n2, d2c);
                d2 = fmaxf(d2, d2c);
#pragma unroll
                for (int i = 0; i < G; ++i) chunk[i >> 3][i & 7] = (_Float16)(2.0f * hf[i]);
                if (G == 8) {
                    _Float16 pieces[3];
                    split3(n2, pieces);
                    chunk[1][0] = pieces[0];
                    chunk[1][1] = pieces[1];
                    chunk[1][2] = pieces[2];
                    chunk[1][3] = (_Float16)1.0f;
                    chunk[1][4] = (_Float16)1.0f;
                    chunk[1][5] = (_Float16)1.0f;
                } else {
                    // rank in norm order -> place in memory: cycle rc of the ranking is cycle
                    // rc / nsplit of split rc % nsplit
                    const int rank = (int)atomicAdd(&bucket_next[bucket[c]], 1u);
                    constexpr int per_cycle = 32 * kU * kResidues;
                    const int rc = rank / per_cycle;
                    pos = (split_begin(rc % nsplit, ncyc, nsplit) + rc / nsplit) * per_cycle + rank % per_cycle;
                    atomicMin(&nmin_bits[pos / (16 * kU)], __float_as_uint(n2));
                    cnorm[pos] = n2;           // for the re-rank kernel's cheap distances
                }
                perm[pos] = (uint16_t)c;
            } else if (G == 16) {
                atomicMin(&nmin_bits[pos / (16 * kU)], 0u);   // padding rows count as norm 0
                cnorm[pos] = 0.0f;
            }
            const int q = pos & 15, uu = (pos >> 4) % kU, hw = (pos / (16 * kU)) & 1;
            const int tile = (pos / (32 * kU)) * kU + uu;
            const int row = 8 * (q >> 2) + 4 * hw + (q & 3);
#pragma unroll
            for (int u = 0; u < 2; ++u) A[((int64_t)tile * 2 + u) * 32 + row] = chunk[u];
        }
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
    ok = ok && meta[3] == 0u && meta[1] != 0u;
    // ||c_hi|| <= P max_c ||c|| + rounding
    const float cmax = P * sqrtf(__uint_as_float(meta[5])) * 1.0001f + kNormMargin;
    float shift = 0.0f, xx = 0.0f, e1 = 0.0f, dx = -1.0f;
    int n = j < k ? group_idx[j] : -1;
    if (n >= N) n = -1;
    pv_f4 *stage = reinterpret_cast<pv_f4 *>(x_stage + (int64_t)j * (G + 4));
    {
        pv_f4 tail = {0.0f, 0.0f, 0.0f, 0.0f};
        if (n >= 0) {
            tail.x = scales[n / gpr];
            tail.y = __int_as_float((int)codes[n] & csize_mask);
        }
        tail.z = __int_as_float(n);
        stage[G / 4] = tail;
    }
    if (n >= 0) {
        const pv_f4 *src = reinterpret_cast<const pv_f4 *>(T + (int64_t)n * G);
#pragma unroll
        for (int v4 = 0; v4 < G / 4; ++v4) stage[v4] = src[v4];
    }
    if (n >= 0 && ok) {
        const float s = scales[n / gpr];
        bool fits = (s != 0.0f) && (fabsf(s) < 3.0e38f);
        const float div = fits ? s : 1.0f;
        float d2 = 0.0f, u2 = 0.0f;
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
        const float xn = sqrtf(xx) * 1.0001f;
        // the smallest codeword, scaled: kv of that codeword is then non-negative
        const float cn0 = P * sqrtf(__uint_as_float(~meta[1])) * 1.0001f + kNormMargin;
        const float want = (xn + cn0) * (xn + cn0) * 1.0001f + 1.0e-3f;
        if (fits && xx < 57000.0f && want < 60000.0f) {
            // bound of the fp32 accumulation error of one accumulator (g = 8: products, norm
            // pieces and SHIFT add up to at most 2 (cmax + xn)^2 in magnitude; g = 16: the
            // products alone, then two fp32 additions on the vector ALU), plus dropped fp16 pieces
            const float e1p = (G == 8 ? 2.0f : 1.0f) * kGamma * (cmax + xn) * (cmax + xn) * 1.01f +
                              (G == 8 ? 5.0e-4f : 4.0e-7f * (cmax + xn) * (cmax + xn));
            e1 = 1.01f * e1p;
            // rounding of x to fp16, plus the fp32 division and scaling roundings (2^-22 ||u||)
            dx = sqrtf(d2) * 1.0001f + 2.4e-7f * sqrtf(u2) + 1.0e-30f;
            if (G == 8) {
                _Float16 pieces[3];
                split3(want, pieces);
                shift = ((float)pieces[0] + (float)pieces[1]) + (float)pieces[2];
                chunk[1][0] = (_Float16)-1.0f;
                chunk[1][1] = (_Float16)-1.0f;
                chunk[1][2] = (_Float16)-1.0f;
                chunk[1][3] = pieces[0];
                chunk[1][4] = pieces[1];
                chunk[1][5] = pieces[2];
            } else {
                shift = want;
            }
        } else {
            xx = 0.0f;
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) chunk[u][e] = (_Float16)0.0f;
        }
    }
    const int gt = j >> 5, col = j & 31;
#pragma unroll
    for (int u = 0; u < 2; ++u) X[((int64_t)gt * 2 + u) * 32 + col] = chunk[u];
    pv_f4 m;
    m.x = shift;
    m.y = xx;
    m.z = e1;
    m.w = dx;
    reinterpret_cast<pv_f4 *>(x_meta)[j] = m;
}

// Plain C so that the compiler sees the reads of MFMA results and inserts the
// wait states the hardware requires between a matrix instruction and a vector
// read of its destination (it does not look inside inline assembly).  It folds
// the pair of maxima into one v_max3_i32.
__device__ __forceinline__ int imax3(int a, int b, int c)
{
    return max(max(a, b), c);
}

// (m & mask) | unit in one instruction; operands are ordinary vector results.
__device__ __forceinline__ int and_or(int m, unsigned vmask, unsigned unit)
{
    int r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(m), "v"(vmask), "s"(unit));
    return r;
}

__device__ __forceinline__ int imed3(int a, int b, int c)
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Largest of a running value and the 16 accumulators (float bits compared as signed integers:
// the order of non-negative floats; a negative float lies below every non-negative one).
// A single chain: a tree of independent v_max3 measured no faster here (the waves of a SIMD
// interleave).
template <bool FIRST>
__device__ __forceinline__ int acc_max(const f16v &acc, int run)
{
    int m;
    if (FIRST && run == kNoKey) {
        m = imax3(__float_as_int(acc[0]), __float_as_int(acc[1]), __float_as_int(acc[2]));
        m = imax3(m, __float_as_int(acc[3]), __float_as_int(acc[4]));
        m = imax3(m, __float_as_int(acc[5]), __float_as_int(acc[6]));
        m = imax3(m, __float_as_int(acc[7]), __float_as_int(acc[8]));
        m = imax3(m, __float_as_int(acc[9]), __float_as_int(acc[10]));
        m = imax3(m, __float_as_int(acc[11]), __float_as_int(acc[12]));
        m = imax3(m, __float_as_int(acc[13]), __float_as_int(acc[14]));
        return max(m, __float_as_int(acc[15]));
    }
    m = imax3(run, __float_as_int(acc[0]), __float_as_int(acc[1]));
    m = imax3(m, __float_as_int(acc[2]), __float_as_int(acc[3]));
    m = imax3(m, __float_as_int(acc[4]), __float_as_int(acc[5]));
    m = imax3(m, __float_as_int(acc[6]), __float_as_int(acc[7]));
    m = imax3(m, __float_as_int(acc[8]), __float_as_int(acc[9]));
    m = imax3(m, __float_as_int(acc[10]), __float_as_int(acc[11]));
    m = imax3(m, __float_as_int(acc[12]), __float_as_int(acc[13]));
    return imax3(m, __float_as_int(acc[14]), __float_as_int(acc[15]));
}

// place of the record of (partition p, list position j)
__device__ __forceinline__ int64_t rec_at(int p, int64_t j, int P, int k_pad)
{
    (void)P;
    return (int64_t)p * k_pad + j;
}

// The distance contraction.  Block = PV_WAVES waves; wave w owns NB group tiles (32 groups
// each) whose B operands stay in registers; the block streams the codeword tiles of its split
// through a double-buffered LDS stage shared by its waves.  A stage is filled with direct
// global->LDS loads (no staging registers) one stage ahead of its use.  Inside a stage the
// loop is software pipelined: the MFMA of unit (tile, group tile) is issued, then the
// accumulators of the unit before it are reduced on the vector ALU while the matrix core
// works.  Output: for every group and partition the largest and second largest key.
template <int G, int NB>
__global__ __launch_bounds__(PV_WAVES * 64, (PV_OCC * PV_WAVES) / 4) void k_score_mfma(
    const h8 *__restrict__ A, const h8 *__restrict__ X, const float *__restrict__ x_meta,
    const float *__restrict__ nmin, int2 *__restrict__ partials, int ncyc, int nsplit, int per_half,
    int gblocks, int k_pad, unsigned *__restrict__ next_item)
{
    constexpr int S = PV_STAGE;                                    // tiles per stage
    constexpr int kStageChunks = S * 64;                           // 16-byte chunks per stage
    constexpr int kW = PV_WAVES;                                   // waves per block
    constexpr int kRounds = (kStageChunks / 64 + kW - 1) / kW;     // 64-chunk rows per wave
    constexpr int kSuStage = S / kU;                               // super-units per stage
    constexpr int kCycle = kResidues * kU;                         // tiles per residue cycle
    static_assert(S % kCycle == 0, "stage must hold whole residue cycles");
    static_assert(2 * kSuStage <= 64, "one lane per staged norm");
    // two stages in SEPARATE arrays (+ one tile of padding each): the compiler then knows that
    // the asynchronous fill of one does not alias the reads of the other and does not wait
    // for the fill before every read
    __shared__ h8 lds0[kStageChunks + 64];
    __shared__ h8 lds1[kStageChunks + 64];
    __shared__ float ldn0[64], ldn1[64];     // smallest norm behind each key of the stage (g = 16)
    __shared__ unsigned s_item;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned vmask = ~kKeyMask;
    asm volatile("" : "+v"(vmask));   // keep the mask in a vector register
    // Work items = (group block, codeword split).  A block starts with item blockIdx.x; when
    // there are more items than blocks the rest is handed out through a counter, so the
    // blocks in flight stay busy until the items run out (every block leaves when its next
    // item number passes the item count).
    const unsigned items = (unsigned)gblocks * (unsigned)nsplit;
    for (unsigned item = blockIdx.x; item < items;) {
    const int gb = (int)(item % (unsigned)gblocks), split = (int)(item / (unsigned)gblocks);
    const int gtile0 = (gb * kW + wave) * NB;
    // a split is a whole number of residue cycles (the table is padded to one)
    const int t_begin = split_begin(split, ncyc, nsplit) * kCycle;
    const int t_end = t_begin + split_count(split, ncyc, nsplit) * kCycle;

    h8 b[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) b[nb] = X[(int64_t)(gtile0 + nb) * 64 + lane];
    // g = 16: SHIFT of the lane's group (added to the key on the vector ALU)
    float shift[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
        shift[nb] = G == 16 ? x_meta[((int64_t)(gtile0 + nb) * 32 + (lane & 31)) * 4] : 0.0f;

    int best[NB][kResidues], second[NB][kResidues], run[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        run[nb] = kNoKey;
#pragma unroll
        for (int r = 0; r < kResidues; ++r) best[nb][r] = second[nb][r] = kNoKey;
    }

    // rows of 64 chunks (1 KiB) are copied by one wave each: lane i -> chunk row + i
    auto fetch = [&](int t0, h8 *dst, float *dstn) {
        const int valid = (t_end - t0 < S ? t_end - t0 : S) * 64;
        const h8 *src = A + (int64_t)t0 * 64;
#pragma unroll
        for (int u = 0; u < kRounds; ++u) {
            const int row = (u * kW + wave) * 64;   // uniform over the wave
            if (row < valid && row < kStageChunks)
                __builtin_amdgcn_global_load_lds(
                    (const void *)(src + row + lane),
                    (__attribute__((address_space(3))) void *)(&dst[row]), 16, 0, 0);
        }
        if (G == 16 && wave == kW - 1)   // the norm table is padded: reads past the split's end are harmless
            __builtin_amdgcn_global_load_lds((const void *)(nmin + (t0 / kU) * 2 + lane),
                                             (__attribute__((address_space(3))) void *)(&dstn[0]), 4,
                                             0, 0);
    };

    // Units (tile, nb) are issued in order; while the matrix core works on the last kD of them
    // the vector ALU reduces the unit kD back.  Four accumulator sets, used round robin, so a
    // set is rewritten three units after it was last read.
    constexpr int kD = PV_DEPTH;
    constexpr int kSets = 4;
    constexpr int kUnitsCycle = NB * kCycle;            // units per residue cycle (unrolled)
    static_assert(kUnitsCycle % kSets == 0 && kD >= 1 && kD < kSets, "accumulator sets must line up");
    f16v acc[kSets];
    h8 a_cur, a_nxt;
    auto issue = [&](int nb, int set) {
        const f16v z = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        acc[set] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a_cur, b[nb], z, 0, 0, 0);
    };
    // rel: the tile's place in its residue cycle (a constant after unrolling: it picks the
    // registers); su_stage: its super-unit within the stage.  The key is closed at the last
    // tile of a super-unit.
    auto reduce = [&](const float *bufn, int t0, int su_stage, int rel, int nb, int set) {
        const int uu = rel % kU;
        // g = 16: the chain starts at zero (the products can be negative, and a negative
        // maximum would not come out of the integer comparison: zero bounds it from above)
        if (uu == 0) run[nb] = G == 16 ? acc_max<false>(acc[set], 0) : acc_max<true>(acc[set], kNoKey);
        else run[nb] = acc_max<false>(acc[set], run[nb]);
        if (uu == kU - 1) {
            const int r = rel / kU;
            int kv = run[nb];
            if (G == 16) kv = __float_as_int((__int_as_float(kv) - bufn[su_stage * 2 + (lane >> 5)]) + shift[nb]);
            const int key = and_or(kv, vmask, (unsigned)(t0 / kU + su_stage));
            second[nb][r] = imed3(best[nb][r], second[nb][r], key);
            best[nb][r] = max(best[nb][r], key);
        }
    };
    // One stage of `cnt` tiles (a whole number of residue cycles).
    auto run_stage = [&](const h8 *buf, const float *bufn, int t0, int cnt) {
        a_cur = buf[lane];
#pragma unroll 1
        for (int q4 = 0; q4 < cnt; q4 += kCycle) {
#pragma unroll
            for (int vr = 0; vr < kUnitsCycle; ++vr) {
                const int u = vr / NB, nb = vr % NB, ts = q4 + u;
                if (nb == 0) a_nxt = buf[(ts + 1) * 64 + lane];   // one spare tile pads the LDS array
                // g = 16: the wave asks for priority while it hands its matrix instruction over
                // (measured: 408 -> 399 us on 183 500 groups; at g = 8 it costs 2 %)
                if (G == 16) __builtin_amdgcn_s_setprio(3);
                issue(nb, vr % kSets);
                if (G == 16) __builtin_amdgcn_s_setprio(0);
                // the unit kD back: tile q4 + dq (dq may point into the cycle before), group tile wnb
                const int dq = (vr - kD >= 0) ? (vr - kD) / NB : -((kD - vr + NB - 1) / NB);
                const int wnb = ((vr - kD) % NB + NB) % NB;
                if (q4 > 0 || vr >= kD)
                    reduce(bufn, t0, (q4 + dq) / kU, (dq + kCycle) % kCycle, wnb,
                           ((vr - kD) % kSets + kSets) % kSets);
                // keep this order: left to itself the scheduler moves a unit's reduction up
                // behind its own matrix instruction, and the wave then waits out that
                // instruction's whole latency instead of working on older units
                __builtin_amdgcn_sched_barrier(0);
                if (nb == NB - 1) a_cur = a_nxt;
            }
        }
        // the last kD units of the stage (its last residue cycle)
#pragma unroll
        for (int w = kUnitsCycle - kD; w < kUnitsCycle; ++w)
            reduce(bufn, t0, (cnt - kCycle + w / NB) / kU, w / NB, w % NB, w % kSets);
    };

    if (t_begin < t_end) fetch(t_begin, lds0, ldn0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    // stages alternate between the two arrays; each half of the loop body names its arrays
    // statically
    for (int t0 = t_begin; t0 < t_end; t0 += 2 * S) {
        {
            if (t0 + S < t_end) fetch(t0 + S, lds1, ldn1);
            run_stage(lds0, ldn0, t0, t_end - t0 < S ? t_end - t0 : S);      // uniform
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        }
        const int t1 = t0 + S;
        if (t1 < t_end) {
            if (t1 + S < t_end) fetch(t1 + S, lds0, ldn0);
            run_stage(lds1, ldn1, t1, t_end - t1 < S ? t_end - t1 : S);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        }
    }

    // records: partials[p * k_pad + j], so that the 32 lanes of a half wave write 256
    // consecutive bytes
    const int col = lane & 31, hw = lane >> 5;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int64_t jpos = (int64_t)(gtile0 + nb) * 32 + col;
        // the two largest of two (largest, second largest) pairs
        auto join = [](int &b1, int &b2, int c1, int c2) {
            const int hi = max(b1, c1), lo = min(b1, c1);
            b2 = max(max(b2, c2), lo);
            b1 = hi;
        };
        if (per_half == 1) {          // all residue classes in one record
            int b1 = best[nb][0], b2 = second[nb][0];
#pragma unroll
            for (int r = 1; r < kResidues; ++r) join(b1, b2, best[nb][r], second[nb][r]);
            partials[rec_at(split * 2 + hw, jpos, nsplit * 2, k_pad)] = make_int2(b1, b2);
        } else if (per_half == 2) {   // classes r and r + 2 share a record
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                int b1 = best[nb][r], b2 = second[nb][r];
                join(b1, b2, best[nb][r + 2], second[nb][r + 2]);
                partials[rec_at((split * 2 + hw) * 2 + r, jpos, nsplit * 4, k_pad)] = make_int2(b1, b2);
            }
        } else {
#pragma unroll
            for (int r = 0; r < kResidues; ++r)
                partials[rec_at((split * 2 + hw) * kResidues + r, jpos, nsplit * 2 * kResidues, k_pad)] =
                    make_int2(best[nb][r], second[nb][r]);
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

// largest value a key can stand for: the super-unit bits replaced by ones; a negative key
// (every value behind it negative) is bounded by zero
__device__ __forceinline__ float key_upper(int key)
{
    return key < 0 ? 0.0f : __int_as_float(key | (int)kKeyMask);
}

// || c_hi - x_hi ||^2 of one table position as || x_hi ||^2 + || c_hi ||^2 - <2 c_hi, x_hi>: the
// product straight from the fp16 operands the matrix cores saw, two terms per instruction
// (v_dot2c_f32_f16, fp32 accumulate), the codeword's norm from the operand row (g = 8: its
// three pieces) or from the table k_prep keeps in position order (g = 16).  The three terms
// cancel, so the error is absolute: (G + 4) 2^-24 (|| c_hi || + || x_hi ||)^2 bounds the
// roundings of the two norms, of the G / 2 accumulation steps and of the final sum; kDdAbs
// times that square covers it eight times over.  The value is only ever compared from below
// (value - bound <= reach), so a generous bound costs a few needless exact evaluations.
constexpr float kDdAbs = 1.0e-5f;
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
template <int G>
__device__ __forceinline__ float approx_dd(const h8 *__restrict__ A, const float *__restrict__ cnorm,
                                           int tile, int row, int pos, const h8 (&xq)[G / 8], float xx)
{
    float dot = 0.0f;
#pragma unroll
    for (int h = 0; h < G / 8; ++h) {
        const h8 a = A[((int64_t)tile * 2 + h) * 32 + row];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const h2 av = {a[2 * e], a[2 * e + 1]};
            const h2 xv = {xq[h][2 * e], xq[h][2 * e + 1]};
            dot = __builtin_amdgcn_fdot2(av, xv, dot, false);
        }
    }
    float cc;
    if (G == 8) {
        const h8 nrm = A[((int64_t)tile * 2 + 1) * 32 + row];
        cc = ((float)nrm[0] + (float)nrm[1]) + (float)nrm[2];
    } else {
        cc = cnorm[pos];
    }
    return fmaxf((xx + cc) - dot, 0.0f);
}

// A group the team could not decide alone: the partitions whose codewords must all be
// evaluated (bit p = partition p), and the best candidate found so far.
struct open_rec_t {
    double obj;
    float reach2;              // a codeword can reach obj only if ||c_hi - x_hi||^2 <= reach2
    unsigned long long mask;
    int idx;
    int n;
    int j;                     // position in the list (names the group's fp16 operand)
};

// A team of kTeam lanes per selected group; a lane scores 16 / kTeam positions of each half tile
// behind a key.  Groups
// with a partition left open are finished by the whole block afterwards, one at a time: for
// every position of the open partitions || c_hi - x_hi ||^2 is formed from the fp16 operands
// the matrix cores saw and the codewords that can still reach the best objective found are
// evaluated.  Every block leaves its counters in block_counts (summed by
// whoever asks for the call's statistics) and passes its changed codes on through atomics; no
// block waits for another and none publishes plain stores to another (a device-wide release
// costs a write-back of the whole L2 of the block's die).
#ifndef PV_RR_OCC
#define PV_RR_OCC 4   // blocks of the re-rank kernel per compute unit the register budget must allow (g = 16: 149 -> 128 registers, four waves per SIMD instead of three; five would spill)
#endif
// v_sqrt_f32 and v_rcp_f32 as they are (1 ulp each; the library's sqrtf and the division add a
// dozen instructions apiece to round correctly and to scale denormal arguments).  Every use
// multiplies the result by a margin far above the few ulps that leaves open; a vanishing or
// denormal scale gives an infinite reciprocal, with which nothing is excluded.
__device__ __forceinline__ float fast_sqrt(float v) { return __builtin_amdgcn_sqrtf(v); }
__device__ __forceinline__ float fast_rcp(float v) { return __builtin_amdgcn_rcpf(v); }
// an upper bound of a non-negative double as a float: rounding to nearest is off by at most
// 2^-24 of the value, the factor makes up for that; below the smallest normal float the floor
// applied before the root takes over
__device__ __forceinline__ float float_above(double v) { return (float)v * 1.0000002f; }

template <int G>
__global__ __launch_bounds__(kBlock, PV_RR_OCC) void k_rerank(
    const float *__restrict__ x_stage, const float *__restrict__ codebook, int k, int k_pad,
    const int2 *__restrict__ partials, int P, int per_half, int ncyc, int nsplit,
    const float *__restrict__ x_meta, const unsigned *__restrict__ cb_meta, const h8 *__restrict__ A,
    const float *__restrict__ cnorm, const h8 *__restrict__ X, const uint16_t *__restrict__ perm,
    uint16_t *__restrict__ codes,
    unsigned *__restrict__ block_counts, unsigned long long *__restrict__ change_slots,
    unsigned long long *__restrict__ num_changed, int nbits)
{
    constexpr int kTeam = rerank_team(G);          // lanes per group
    constexpr int kTeams = kBlock / kTeam;         // groups per block
    constexpr int kPer = 16 / kTeam;               // positions of a half tile per lane
    static_assert(kTeam == 8 || kTeam == 16, "a team is 8 or 16 consecutive lanes");
    __shared__ unsigned s_cnt[4];   // groups decided by the teams, codes changed, candidates evaluated, groups scanned
    __shared__ open_rec_t s_open[kTeams];
    __shared__ unsigned s_nopen;
    if (threadIdx.x < 4) s_cnt[threadIdx.x] = 0;
    if (threadIdx.x == 0) s_nopen = 0;
    __syncthreads();
    const int csize = 1 << nbits;
    const int gid = blockIdx.x * kBlock + threadIdx.x;
    const int j = gid / kTeam, q = gid % kTeam;
    // everything the team needs of its group sits at the list position: one round of loads
    const bool inlist = j < k;
    const pv_f4 *stage = reinterpret_cast<const pv_f4 *>(x_stage + (int64_t)(inlist ? j : 0) * (G + 4));
    const pv_f4 tail = stage[G / 4];
    pv_f4 meta = reinterpret_cast<const pv_f4 *>(x_meta)[inlist ? j : 0];
    const int n = inlist ? __float_as_int(tail.z) : -1;
    bool live = n >= 0;                      // whole teams agree on every branch below
    if (!live) meta.w = -1.0f;
    if (live && meta.w < 0.0f) {             // the filter was skipped for this group: every partition
        if (q == 0) {
            open_rec_t r;
            r.obj = __builtin_huge_val();
            r.reach2 = __builtin_huge_valf();      // no operand to test against: every codeword
            r.mask = P >= 64 ? ~0ull : ((1ull << P) - 1ull);
            r.idx = 0x7fffffff;
            r.n = n;
            r.j = j;
            s_open[atomicAdd(&s_nopen, 1u)] = r;
        }
        live = false;
    }
    if (live) {
        const float s = tail.x;
        float t[G];
#pragma unroll
        for (int v4 = 0; v4 < G / 4; ++v4) {
            pv_f4 v = stage[v4];
            t[v4 * 4 + 0] = v.x;
            t[v4 * 4 + 1] = v.y;
            t[v4 * 4 + 2] = v.z;
            t[v4 * 4 + 3] = v.w;
        }
        const int prev = __float_as_int(tail.y);
        constexpr int kMaxRec = 64 / kTeam;  // P <= 64
        int2 rec[kMaxRec];
#pragma unroll
        for (int u = 0; u < kMaxRec; ++u) {
            int p = q + kTeam * u;
            rec[u] = p < P ? partials[rec_at(p, j, P, k_pad)] : make_int2(kNoKey, kNoKey);
        }
        const double o_prev = exact_obj<G>(codebook + (int64_t)prev * G, s, t);
        // best key over all partitions, with its partition
        long long bk = (long long)0x8000000000000000ull;
#pragma unroll
        for (int u = 0; u < kMaxRec; ++u) {
            int p = q + kTeam * u;
            long long v = ((long long)rec[u].x << 32) | (long long)(unsigned)(63 - p);
            bk = v > bk ? v : bk;
        }
        bk = pv_team_max_i64<kTeam>(bk);
        const int best_key = (int)(bk >> 32);
        const int best_p = 63 - (int)(bk & 0xFFFFFFFFll);

        // the group's fp16 operand as the matrix cores saw it
        h8 xq[G / 8];
        {
            const int gt = j >> 5, col = j & 31;
#pragma unroll
            for (int h = 0; h < G / 8; ++h) xq[h] = X[((int64_t)gt * 2 + h) * 32 + col];
        }
        bool okP;
        const float Pscale = scale_from_maxabs(cb_meta[0], &okP);
        // what the cheap distance may be off by, at most (see approx_dd)
        const float nsum = Pscale * fast_sqrt(__uint_as_float(cb_meta[5])) * 1.0001f + kNormMargin +
                           fast_sqrt(meta.y) * 1.0001f;
        const float dabs = kDdAbs * nsum * nsum;
        const float dC = fast_sqrt(__uint_as_float(cb_meta[2])) * 1.0001f + 1e-30f;
        const float p_over_s = Pscale * fast_rcp(fabsf(s));   // inf for a vanishing scale: nothing is excluded then
        // The 16 U positions behind a key (lane q takes positions q, q + kTeam, ... of each of the
        // U half tiles) are looked at in two levels: || c_hi - x_hi ||^2 from the fp16 operand rows (cheap,
        // consecutive rows), and the exact objective only for positions that can still reach
        // the best objective known: || c_hi - x_hi || <= P sqrt(E) / |s| + dC + dx.
        constexpr int kMine = kU * kPer;               // positions of a key per lane
        auto level1 = [&](int key, int p, float (&dd)[kMine], int (&pos)[kMine], int (&cwd)[kMine]) {
            const int su = key & (int)kKeyMask;
            const int hw = (p / per_half) & 1;
#pragma unroll
            for (int uu = 0; uu < kU; ++uu)
#pragma unroll
                for (int e = 0; e < kPer; ++e) {
                    const int qq = q + kTeam * e;
                    const int row = 8 * (qq >> 2) + 4 * hw + (qq & 3);
                    pos[uu * kPer + e] = ((su * 2 + hw) * kU + uu) * 16 + qq;
                    // unconditional (the padded table has the row), so that the loads of all the
                    // lane's positions are in flight together
                    dd[uu * kPer + e] = approx_dd<G>(A, cnorm, su * kU + uu, row, pos[uu * kPer + e], xq, meta.y);
                    // the codeword behind the position comes along (g = 8: positions are
                    // codewords), so that an exact evaluation is one more round trip, not two
                    cwd[uu * kPer + e] = G == 8 ? pos[uu * kPer + e] : (int)perm[pos[uu * kPer + e]];
                }
#pragma unroll
            for (int i = 0; i < kMine; ++i)
                if (pos[i] >= csize) dd[i] = __builtin_huge_valf();
        };
        auto exact_at = [&](int cw, cand_t &c) {
            const double o = exact_obj<G>(codebook + (int64_t)cw * G, s, t);
            if (cand_better(o, cw, c.obj, c.idx)) {
                c.obj = o;
                c.idx = cw;
            }
        };
        // upper bound, in fp32 with every rounding covered, of (P sqrt(E) / |s| + dC + dx)^2
        auto reach2_of = [&](double e_star) {
            const float ef = float_above(e_star);
            // (a NaN passes the floor and the root, and is caught below)
            const float rr = fast_sqrt(ef < 1.2e-38f ? 1.2e-38f : ef) * p_over_s * 1.000002f + dC + meta.w;
            const float r2 = rr * rr * 1.000002f;
            return r2 == r2 ? r2 : __builtin_huge_valf();   // NaN: nothing can be excluded
        };
        auto team_min = [&](cand_t c) {
            pv_team_stages<kTeam>([&](auto ctrl) {
                constexpr int C = decltype(ctrl)::value;
                const double o = pv_dpp_f64<C>(c.obj);
                const int i = pv_dpp<C>(c.idx);
                if (cand_better(o, i, c.obj, c.idx)) {
                    c.obj = o;
                    c.idx = i;
                }
            });
            return c;
        };

        cand_t mine;
        mine.obj = __builtin_huge_val();
        mine.idx = 0x7fffffff;
        unsigned exact_evals = 1;                      // the previous code
        double e_star = o_prev;
        if (best_key != kNoKey) {
            float dd[kMine];
            int pos[kMine], cwd[kMine];
            level1(best_key, best_p, dd, pos, cwd);
            // the position that looks nearest is evaluated first: it fixes the reach for the rest
            int wu = 0;
            float dmin = dd[0];
#pragma unroll
            for (int uu = 1; uu < kMine; ++uu)
                if (dd[uu] < dmin) {
                    dmin = dd[uu];
                    wu = uu;
                }
            unsigned long long pick = ((unsigned long long)__float_as_uint(dmin) << 32) | (unsigned)q;
            pick = pv_team_min_u64<kTeam>(pick);
            const bool chosen = (int)(pick & 15u) == q && dmin < 3.0e38f;
            if (chosen) {
                int pw = cwd[0];                   // cwd[wu] without dynamic register indexing
#pragma unroll
                for (int uu = 1; uu < kMine; ++uu)
                    if (uu == wu) pw = cwd[uu];
                exact_at(pw, mine);
            }
            const double o0 = __shfl(mine.obj, (int)(pick & 15u), kTeam);
            if (o0 < e_star) e_star = o0;
            const float r2f = reach2_of(e_star);
#pragma unroll
            for (int uu = 0; uu < kMine; ++uu)
                if (!(chosen && uu == wu) && dd[uu] - dabs <= r2f && pos[uu] < csize) {
                    exact_at(cwd[uu], mine);
                    ++exact_evals;
                }
            if (chosen) ++exact_evals;
        }
        cand_t first = team_min(mine);
        if (first.obj < e_star) e_star = first.obj;

        // every codeword that was not evaluated and could still reach E* sits behind a key
        // whose upper bound is at least kcut
        const float reach2f = reach2_of(e_star);
        // lower bound of SHIFT + ||x_hi||^2 - reach2 - E1 (fp32, every rounding covered)
        const float base = meta.x + meta.y;
        const float kcut = (base * 0.999999f - reach2f * 1.000001f) - meta.z - 1.0e-6f * (base + reach2f);
        const bool no_bound = !(kcut > -3.0e38f);      // also true for NaN: nothing can be excluded
        unsigned pending = 0;                         // bit u: rec[u].x needs evaluation
        unsigned long long open = 0;                  // partitions with a second key at or above kcut
#pragma unroll
        for (int u = 0; u < kMaxRec; ++u) {
            int p = q + kTeam * u;
            if (p < P) {
                if (rec[u].y != kNoKey && (no_bound || key_upper(rec[u].y) >= kcut)) open |= 1ull << p;
                if (p != best_p && rec[u].x != kNoKey && (no_bound || key_upper(rec[u].x) >= kcut))
                    pending |= 1u << u;
            }
        }
        open = pv_team_or_u64<kTeam>(open);
        const int team_shift = (threadIdx.x & 63) & ~(kTeam - 1);
        // the best key of every other partition at or above kcut: its positions are evaluated here
        unsigned extra = 0;
        for (;;) {
            const unsigned long long pb = __ballot(pending != 0);
            const unsigned team = (unsigned)((pb >> team_shift) & ((1ull << kTeam) - 1ull));
            if (!team) break;
            const int src = __ffs(team) - 1;      // lane of the team with work
            const unsigned their = __shfl(pending, src, kTeam);
            const int u = __ffs(their) - 1;
            int key = 0;
#pragma unroll
            for (int uu = 0; uu < kMaxRec; ++uu)
                if (uu == u) key = rec[uu].x;
            key = __shfl(key, src, kTeam);
            {
                float dd[kMine];
                int pos[kMine], cwd[kMine];
                level1(key, src + kTeam * u, dd, pos, cwd);
#pragma unroll
                for (int uu = 0; uu < kMine; ++uu)
                    if (dd[uu] - dabs <= reach2f && pos[uu] < csize) {
                        exact_at(cwd[uu], mine);
                        ++exact_evals;
                    }
            }
            if (q == src) pending &= ~(1u << u);
            ++extra;
        }
        (void)extra;
        exact_evals = pv_team_sum_u32<kTeam>(exact_evals);
        const cand_t win = team_min(mine);
        if (q == 0) {
            if (open) {
                // a partition may hide further codewords at or above kcut: all of its
                // positions are evaluated by the block, which also takes the decision
                open_rec_t r;
                r.obj = win.obj;
                r.reach2 = no_bound ? __builtin_huge_valf() : reach2_of(o_prev < win.obj ? o_prev : win.obj);
                r.mask = open;
                r.idx = win.idx;
                r.n = n;
                r.j = j;
                s_open[atomicAdd(&s_nopen, 1u)] = r;
            } else {
                int pick = win.idx;
                if (o_prev <= win.obj || pick == 0x7fffffff) pick = prev;
                if (pick != prev) {
                    codes[n] = (uint16_t)pick;
                    atomicAdd(&s_cnt[1], 1u);
                }
                atomicAdd(&s_cnt[0], 1u);
            }
            atomicAdd(&s_cnt[2], exact_evals - (unsigned)(kTeam - 1));   // the previous code was counted by every lane
        }
    }
    __syncthreads();

    // ---- groups left open: every position of their open partitions, by the whole block, one
    // group at a time.
    // Partition p = (codeword split, half wave, residue class) as the scoring kernel numbers them.
    const unsigned nopen = s_nopen;
    __shared__ double s_obj[kBlock / 64];
    __shared__ int s_idx[kBlock / 64];
    for (unsigned item = 0; item < nopen; ++item) {
        const open_rec_t rec = s_open[item];
        const int n2 = rec.n;
        const pv_f4 *stage2 = reinterpret_cast<const pv_f4 *>(x_stage + (int64_t)rec.j * (G + 4));
        const pv_f4 tail2 = stage2[G / 4];
        const float s = tail2.x;
        float t[G];
#pragma unroll
        for (int v4 = 0; v4 < G / 4; ++v4) {
            pv_f4 v = stage2[v4];
            t[v4 * 4 + 0] = v.x;
            t[v4 * 4 + 1] = v.y;
            t[v4 * 4 + 2] = v.z;
            t[v4 * 4 + 3] = v.w;
        }
        const int prev = __float_as_int(tail2.y);
        const int lane = threadIdx.x & 63;
        const int qq = threadIdx.x & 15, slot = threadIdx.x >> 4;
        constexpr int kSlots = kBlock / 16;
        // the group's fp16 operand as the matrix cores saw it
        h8 xq[G / 8];
        {
            const int gt = rec.j >> 5, col = rec.j & 31;
#pragma unroll
            for (int h = 0; h < G / 8; ++h) xq[h] = X[((int64_t)gt * 2 + h) * 32 + col];
        }
        const float xx = x_meta[(int64_t)rec.j * 4 + 1];
        bool okP2;
        const float nsum = scale_from_maxabs(cb_meta[0], &okP2) * fast_sqrt(__uint_as_float(cb_meta[5])) * 1.0001f +
                           kNormMargin + fast_sqrt(xx) * 1.0001f;
        const float dabs = kDdAbs * nsum * nsum;
        const bool test = rec.reach2 < 3.0e38f;
        const float r2f = rec.reach2;
        cand_t mine;
        mine.obj = __builtin_huge_val();
        mine.idx = 0x7fffffff;
        for (unsigned long long left = rec.mask; left; left &= left - 1) {   // uniform over the block
            const int p = __ffsll((long long)left) - 1;
            const int hw = (p / per_half) & 1;
            const int split = p / (2 * per_half);
            const int su_begin = split_begin(split, ncyc, nsplit) * kResidues;
            const int su_end = su_begin + split_count(split, ncyc, nsplit) * kResidues;
            const int row = 8 * (qq >> 2) + 4 * hw + (qq & 3);
            // the classes of the record: p % per_half, + per_half, ... (relative to the split's
            // start); kBatch super-units per lane at a time, so that their operand rows are in
            // flight together
            constexpr int kBatch = 2;
            for (int rel0 = (p % per_half) + slot * per_half; su_begin + rel0 < su_end;
                 rel0 += kSlots * per_half * kBatch) {
                float dd[kBatch][kU];
#pragma unroll
                for (int bb = 0; bb < kBatch; ++bb) {
                    // unconditional loads (a row of the split's last super-unit stands in past its
                    // end), so that the whole batch is in flight together
                    const int su = su_begin + rel0 + bb * kSlots * per_half;
                    const int su_c = su < su_end ? su : su_end - 1;
#pragma unroll
                    for (int uu = 0; uu < kU; ++uu)
                        dd[bb][uu] = approx_dd<G>(A, cnorm, su_c * kU + uu, row,
                                                  ((su_c * 2 + hw) * kU + uu) * 16 + qq, xq, xx);
                }
#pragma unroll
                for (int bb = 0; bb < kBatch; ++bb) {
                    const int su = su_begin + rel0 + bb * kSlots * per_half;
#pragma unroll
                    for (int uu = 0; uu < kU; ++uu) {
                        const int pos = ((su * 2 + hw) * kU + uu) * 16 + qq;
                        if (su < su_end && pos < csize && (!test || dd[bb][uu] - dabs <= r2f)) {
                            const int cw = G == 8 ? pos : (int)perm[pos];
                            const double obj = exact_obj<G>(codebook + (int64_t)cw * G, s, t);
                            if (cand_better(obj, cw, mine.obj, mine.idx)) {
                                mine.obj = obj;
                                mine.idx = cw;
                            }
                        }
                    }
                }
            }
        }
        // block-wide lexicographic minimum
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            double o = __shfl_xor(mine.obj, off);
            int i = __shfl_xor(mine.idx, off);
            if (cand_better(o, i, mine.obj, mine.idx)) {
                mine.obj = o;
                mine.idx = i;
            }
        }
        __syncthreads();
        if (lane == 0) {
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
                codes[n2] = (uint16_t)pick;
                atomicAdd(&s_cnt[1], 1u);
            }
            atomicAdd(&s_cnt[3], 1u);
        }
    }
    __syncthreads();
    // per-block totals: groups decided by the teams, codes changed, candidates evaluated, groups scanned
    if (threadIdx.x < 4) block_counts[4 * blockIdx.x + threadIdx.x] = s_cnt[threadIdx.x];
    // *num_changed: thousands of atomics on one address would queue for longer than the kernel
    // runs, so 64 blocks share a slot that carries (arrivals << 40 | sum); the block that finds
    // all others arrived passes the sum on
    if (threadIdx.x == 0 && num_changed) {
        const unsigned first = (blockIdx.x >> 6) << 6;
        const unsigned members = gridDim.x - first < 64u ? gridDim.x - first : 64u;
        const unsigned long long old =
            atomicAdd(&change_slots[blockIdx.x >> 6], (1ull << 40) | (unsigned long long)s_cnt[1]);
        if ((unsigned)(old >> 40) == members - 1u) {
            const unsigned long long total = (old & ((1ull << 40) - 1ull)) + s_cnt[1];
            if (total) atomicAdd(num_changed, total);
        }
    }
}

// ------------------------------------------------ stochastic rounding over the two nearest
//
// The same filter serves App. F's rounding over the TWO nearest codewords: the certificate is
// the one of k_rerank with the best objective replaced by the second best found so far, E2.
// A codeword that was not evaluated can belong to the two nearest only if its objective
// reaches E2, hence only if its key is at least the cut taken from E2; every best key at or
// above that cut has its 16 U positions looked at (cheap distance first, exact objective for
// those within reach of E2), and a partition whose runner-up key reaches the cut is scanned
// completely by the block.  The two nearest (objective, then index) go to pv_round_pick.
struct two_t {
    double o1, o2;
    int i1, i2;
};

__device__ __forceinline__ void two_clear(two_t &b)
{
    b.o1 = b.o2 = __builtin_huge_val();
    b.i1 = b.i2 = kPvNoCode;
}

__device__ __forceinline__ void two_insert(two_t &b, double o, int c)
{
    if (cand_better(o, c, b.o1, b.i1)) {
        b.o2 = b.o1; b.i2 = b.i1;
        b.o1 = o; b.i1 = c;
    } else if (cand_better(o, c, b.o2, b.i2)) {
        b.o2 = o; b.i2 = c;
    }
}

// the two smallest of the union of two such pairs (a codeword sits in at most one of them)
__device__ __forceinline__ two_t two_merge(two_t a, const two_t &b)
{
    if (b.i1 != kPvNoCode) two_insert(a, b.o1, b.i1);
    if (b.i2 != kPvNoCode) two_insert(a, b.o2, b.i2);
    return a;
}

template <int WIDTH>
__device__ __forceinline__ two_t two_reduce(two_t b)
{
#pragma unroll
    for (int m = WIDTH / 2; m > 0; m >>= 1) {
        two_t o;
        o.o1 = __shfl_xor(b.o1, m, WIDTH);
        o.o2 = __shfl_xor(b.o2, m, WIDTH);
        o.i1 = __shfl_xor(b.i1, m, WIDTH);
        o.i2 = __shfl_xor(b.i2, m, WIDTH);
        b = two_merge(b, o);
    }
    return b;
}

struct open2_t {
    two_t best;
    float reach2;
    unsigned long long mask;
    int n;
    int j;
};

template <int G>
__global__ __launch_bounds__(kBlock) void k_round_top2(
    const float *__restrict__ x_stage, const float *__restrict__ codebook, int k, int k_pad,
    const int2 *__restrict__ partials, int P, int per_half, int ncyc, int nsplit,
    const float *__restrict__ x_meta, const unsigned *__restrict__ cb_meta, const h8 *__restrict__ A,
    const float *__restrict__ cnorm, const h8 *__restrict__ X, const uint16_t *__restrict__ perm,
    uint16_t *__restrict__ codes, unsigned *__restrict__ block_counts,
    unsigned long long *__restrict__ change_slots, unsigned long long *__restrict__ num_changed,
    int nbits, int power, unsigned long long seed)
{
    constexpr int kTeam = rerank_team(G);
    constexpr int kTeams = kBlock / kTeam;
    constexpr int kPer = 16 / kTeam;
    __shared__ unsigned s_cnt[4];   // groups decided by the teams, codes changed, candidates evaluated, groups scanned
    __shared__ open2_t s_open[kTeams];
    __shared__ unsigned s_nopen;
    if (threadIdx.x < 4) s_cnt[threadIdx.x] = 0;
    if (threadIdx.x == 0) s_nopen = 0;
    __syncthreads();
    const int csize = 1 << nbits;
    const int gid = blockIdx.x * kBlock + threadIdx.x;
    const int j = gid / kTeam, q = gid % kTeam;
    const bool inlist = j < k;
    const pv_f4 *stage = reinterpret_cast<const pv_f4 *>(x_stage + (int64_t)(inlist ? j : 0) * (G + 4));
    const pv_f4 tail = stage[G / 4];
    pv_f4 meta = reinterpret_cast<const pv_f4 *>(x_meta)[inlist ? j : 0];
    const int n = inlist ? __float_as_int(tail.z) : -1;
    bool live = n >= 0;                      // whole teams agree on every branch below
    if (!live) meta.w = -1.0f;
    bool okP;
    const float Pscale = scale_from_maxabs(cb_meta[0], &okP);
    const float cmaxn = Pscale * fast_sqrt(__uint_as_float(cb_meta[5])) * 1.0001f + kNormMargin;
    auto decide = [&](const two_t &b, int group, int prev) {
        int pick = prev;                     // nothing could be evaluated (non-finite input): keep
        if (b.i1 != kPvNoCode) pick = pv_round_pick(b.o1, b.i1, b.o2, b.i2, power, seed, (unsigned long long)group);
        if (pick != prev) {
            codes[group] = (uint16_t)pick;
            atomicAdd(&s_cnt[1], 1u);
        }
    };
    if (live && meta.w < 0.0f) {             // the filter was skipped for this group: every partition
        if (q == 0) {
            open2_t r;
            two_clear(r.best);
            r.reach2 = __builtin_huge_valf();
            r.mask = P >= 64 ? ~0ull : ((1ull << P) - 1ull);
            r.n = n;
            r.j = j;
            s_open[atomicAdd(&s_nopen, 1u)] = r;
        }
        live = false;
    }
    if (live) {
        const float s = tail.x;
        float t[G];
#pragma unroll
        for (int v4 = 0; v4 < G / 4; ++v4) {
            pv_f4 v = stage[v4];
            t[v4 * 4 + 0] = v.x;
            t[v4 * 4 + 1] = v.y;
            t[v4 * 4 + 2] = v.z;
            t[v4 * 4 + 3] = v.w;
        }
        const int prev = __float_as_int(tail.y);
        constexpr int kMaxRec = 64 / kTeam;  // P <= 64
        int2 rec[kMaxRec];
#pragma unroll
        for (int u = 0; u < kMaxRec; ++u) {
            int p = q + kTeam * u;
            rec[u] = p < P ? partials[rec_at(p, j, P, k_pad)] : make_int2(kNoKey, kNoKey);
        }
        // the two largest keys over all partitions, runner-up keys included: entry = key, partition,
        // whether it is the partition's best (low bit) - the largest key is always a best one
        auto entry = [](int key, int p, int is_best) {
            return ((long long)key << 32) | (long long)(unsigned)(((63 - p) << 1) | is_best);
        };
        long long bk = (long long)0x8000000000000000ull;
#pragma unroll
        for (int u = 0; u < kMaxRec; ++u) {
            const long long v = entry(rec[u].x, q + kTeam * u, 1);
            bk = v > bk ? v : bk;
        }
#pragma unroll
        for (int m = kTeam / 2; m > 0; m >>= 1) {
            long long o = __shfl_xor(bk, m, kTeam);
            bk = o > bk ? o : bk;
        }
        long long bk2 = (long long)0x8000000000000000ull;
#pragma unroll
        for (int u = 0; u < kMaxRec; ++u) {
            const long long vx = entry(rec[u].x, q + kTeam * u, 1), vy = entry(rec[u].y, q + kTeam * u, 0);
            if (vx != bk && vx > bk2) bk2 = vx;
            if (vy > bk2) bk2 = vy;
        }
#pragma unroll
        for (int m = kTeam / 2; m > 0; m >>= 1) {
            long long o = __shfl_xor(bk2, m, kTeam);
            bk2 = o > bk2 ? o : bk2;
        }
        const int best_key = (int)(bk >> 32);
        const int best_p = 63 - (int)((bk & 0xFFFFFFFFll) >> 1);
        const int next_key = (int)(bk2 >> 32);
        const int next_p = 63 - (int)((bk2 & 0xFFFFFFFFll) >> 1);
        const bool next_is_best = (bk2 & 1ll) != 0;      // the best key of its partition (else its runner-up)
        h8 xq[G / 8];
        {
            const int gt = j >> 5, col = j & 31;
#pragma unroll
            for (int h = 0; h < G / 8; ++h) xq[h] = X[((int64_t)gt * 2 + h) * 32 + col];
        }
        const float nsum = cmaxn + fast_sqrt(meta.y) * 1.0001f;
        const float dabs = kDdAbs * nsum * nsum;
        const float p_over_s = Pscale * fast_rcp(fabsf(s));
        const float dC = fast_sqrt(__uint_as_float(cb_meta[2])) * 1.0001f + 1e-30f;
        auto reach2_of = [&](double e) {
            const float ef = float_above(e);   // a NaN passes the floor and the root, and is caught below
            const float rr = fast_sqrt(ef < 1.2e-38f ? 1.2e-38f : ef) * p_over_s * 1.000002f + dC + meta.w;
            const float r2 = rr * rr * 1.000002f;
            return r2 == r2 ? r2 : __builtin_huge_valf();
        };
        two_t mine;
        two_clear(mine);
        unsigned exact_evals = 0;
        // the positions behind a key: cheap distance first, exact objective for those within reach
        auto eval_key = [&](int key, int p, float reach2) {
            const int su = key & (int)kKeyMask;
            const int hw = (p / per_half) & 1;
#pragma unroll
            for (int uu = 0; uu < kU; ++uu)
#pragma unroll
                for (int e = 0; e < kPer; ++e) {
                    const int qq = q + kTeam * e;
                    const int row = 8 * (qq >> 2) + 4 * hw + (qq & 3);
                    const int pos = ((su * 2 + hw) * kU + uu) * 16 + qq;
                    const float dd = approx_dd<G>(A, cnorm, su * kU + uu, row, pos, xq, meta.y);
                    if (pos < csize && dd - dabs <= reach2) {
                        const int cw = G == 8 ? pos : (int)perm[pos];
                        two_insert(mine, exact_obj<G>(codebook + (int64_t)cw * G, s, t), cw);
                        ++exact_evals;
                    }
                }
        };
        if (best_key != kNoKey) eval_key(best_key, best_p, __builtin_huge_valf());
        // The second nearest usually sits behind the second largest key, not among the neighbours
        // of the nearest: that key is evaluated before the cut is taken, else the cut would come
        // from a poor second objective and leave nearly every partition open.
        if (next_key != kNoKey && next_p < P) {
            const two_t sofar = two_reduce<kTeam>(mine);
            eval_key(next_key, next_p, sofar.i2 == kPvNoCode ? __builtin_huge_valf() : reach2_of(sofar.o2));
        }
        const two_t first = two_reduce<kTeam>(mine);
        // every codeword that was not evaluated and could still reach E2 sits behind a key at or above kcut
        const float reach2f = first.i2 == kPvNoCode ? __builtin_huge_valf() : reach2_of(first.o2);
        const float base = meta.x + meta.y;
        const float kcut = (base * 0.999999f - reach2f * 1.000001f) - meta.z - 1.0e-6f * (base + reach2f);
        const bool no_bound = !(kcut > -3.0e38f);
        unsigned pending = 0;
        unsigned long long open = 0;
#pragma unroll
        for (int u = 0; u < kMaxRec; ++u) {
            int p = q + kTeam * u;
            if (p < P) {
                if (rec[u].y != kNoKey && (no_bound || key_upper(rec[u].y) >= kcut)) open |= 1ull << p;
                if (p != best_p && !(next_is_best && p == next_p) && rec[u].x != kNoKey &&
                    (no_bound || key_upper(rec[u].x) >= kcut))
                    pending |= 1u << u;
            }
        }
#pragma unroll
        for (int m = kTeam / 2; m > 0; m >>= 1) open |= __shfl_xor(open, m, kTeam);
        const int team_shift = (threadIdx.x & 63) & ~(kTeam - 1);
        for (;;) {
            const unsigned long long pb = __ballot(pending != 0);
            const unsigned team = (unsigned)((pb >> team_shift) & ((1ull << kTeam) - 1ull));
            if (!team) break;
            const int src = __ffs(team) - 1;
            const unsigned their = __shfl(pending, src, kTeam);
            const int u = __ffs(their) - 1;
            int key = 0;
#pragma unroll
            for (int uu = 0; uu < kMaxRec; ++uu)
                if (uu == u) key = rec[uu].x;
            key = __shfl(key, src, kTeam);
            eval_key(key, src + kTeam * u, reach2f);
            if (q == src) pending &= ~(1u << u);
        }
#pragma unroll
        for (int m = kTeam / 2; m > 0; m >>= 1) exact_evals += __shfl_xor(exact_evals, m, kTeam);
        const two_t win = two_reduce<kTeam>(mine);
        if (q == 0) {
            if (open) {
                open2_t r;
                r.best = win;
                r.reach2 = (no_bound || win.i2 == kPvNoCode) ? __builtin_huge_valf() : reach2_of(win.o2);
                r.mask = open;
                r.n = n;
                r.j = j;
                s_open[atomicAdd(&s_nopen, 1u)] = r;
            } else {
                decide(win, n, prev);
                atomicAdd(&s_cnt[0], 1u);
            }
            atomicAdd(&s_cnt[2], exact_evals);
        }
    }
    __syncthreads();

    // ---- groups left open: every position of their open partitions, by the whole block
    const unsigned nopen = s_nopen;
    __shared__ two_t s_two[kBlock / 64];
    for (unsigned item = 0; item < nopen; ++item) {
        const open2_t rec = s_open[item];
        const pv_f4 *stage2 = reinterpret_cast<const pv_f4 *>(x_stage + (int64_t)rec.j * (G + 4));
        const pv_f4 tail2 = stage2[G / 4];
        const float s = tail2.x;
        float t[G];
#pragma unroll
        for (int v4 = 0; v4 < G / 4; ++v4) {
            pv_f4 v = stage2[v4];
            t[v4 * 4 + 0] = v.x;
            t[v4 * 4 + 1] = v.y;
            t[v4 * 4 + 2] = v.z;
            t[v4 * 4 + 3] = v.w;
        }
        const int prev = __float_as_int(tail2.y);
        const int lane = threadIdx.x & 63;
        const int qq = threadIdx.x & 15, slot = threadIdx.x >> 4;
        constexpr int kSlots = kBlock / 16;
        h8 xq[G / 8];
        {
            const int gt = rec.j >> 5, col = rec.j & 31;
#pragma unroll
            for (int h = 0; h < G / 8; ++h) xq[h] = X[((int64_t)gt * 2 + h) * 32 + col];
        }
        const float xx = x_meta[(int64_t)rec.j * 4 + 1];
        const float nsum = cmaxn + fast_sqrt(xx) * 1.0001f;
        const float dabs = kDdAbs * nsum * nsum;
        const bool test = rec.reach2 < 3.0e38f;
        const float r2f = rec.reach2;
        two_t mine;
        two_clear(mine);
        for (unsigned long long left = rec.mask; left; left &= left - 1) {   // uniform over the block
            const int p = __ffsll((long long)left) - 1;
            const int hw = (p / per_half) & 1;
            const int split = p / (2 * per_half);
            const int su_begin = split_begin(split, ncyc, nsplit) * kResidues;
            const int su_end = su_begin + split_count(split, ncyc, nsplit) * kResidues;
            const int row = 8 * (qq >> 2) + 4 * hw + (qq & 3);
            constexpr int kBatch = 2;
            for (int rel0 = (p % per_half) + slot * per_half; su_begin + rel0 < su_end;
                 rel0 += kSlots * per_half * kBatch) {
                float dd[kBatch][kU];
#pragma unroll
                for (int bb = 0; bb < kBatch; ++bb) {
                    const int su = su_begin + rel0 + bb * kSlots * per_half;
                    const int su_c = su < su_end ? su : su_end - 1;
#pragma unroll
                    for (int uu = 0; uu < kU; ++uu)
                        dd[bb][uu] = approx_dd<G>(A, cnorm, su_c * kU + uu, row,
                                                  ((su_c * 2 + hw) * kU + uu) * 16 + qq, xq, xx);
                }
#pragma unroll
                for (int bb = 0; bb < kBatch; ++bb) {
                    const int su = su_begin + rel0 + bb * kSlots * per_half;
#pragma unroll
                    for (int uu = 0; uu < kU; ++uu) {
                        const int pos = ((su * 2 + hw) * kU + uu) * 16 + qq;
                        if (su < su_end && pos < csize && (!test || dd[bb][uu] - dabs <= r2f)) {
                            const int cw = G == 8 ? pos : (int)perm[pos];
                            two_insert(mine, exact_obj<G>(codebook + (int64_t)cw * G, s, t), cw);
                        }
                    }
                }
            }
        }
        mine = two_reduce<64>(mine);
        __syncthreads();
        if (lane == 0) s_two[threadIdx.x >> 6] = mine;
        __syncthreads();
        if (threadIdx.x == 0) {
            // a codeword of an open partition may already sit in the team's pair (it was behind an
            // evaluated key): the same index is not taken twice
            two_t win = rec.best;
            for (int w = 0; w < kBlock / 64; ++w) {
                const two_t o = s_two[w];
                if (o.i1 != kPvNoCode && o.i1 != win.i1 && o.i1 != win.i2) two_insert(win, o.o1, o.i1);
                if (o.i2 != kPvNoCode && o.i2 != win.i1 && o.i2 != win.i2) two_insert(win, o.o2, o.i2);
            }
            decide(win, rec.n, prev);
            atomicAdd(&s_cnt[3], 1u);
        }
    }
    __syncthreads();
    if (threadIdx.x < 4) block_counts[4 * blockIdx.x + threadIdx.x] = s_cnt[threadIdx.x];
    // *num_changed through the slots 64 blocks share (see k_rerank)
    if (threadIdx.x == 0 && num_changed) {
        const unsigned first = (blockIdx.x >> 6) << 6;
        const unsigned members = gridDim.x - first < 64u ? gridDim.x - first : 64u;
        const unsigned long long old =
            atomicAdd(&change_slots[blockIdx.x >> 6], (1ull << 40) | (unsigned long long)s_cnt[1]);
        if ((unsigned)(old >> 40) == members - 1u) {
            const unsigned long long total = (old & ((1ull << 40) - 1ull)) + s_cnt[1];
            if (total) atomicAdd(num_changed, total);
        }
    }
}

struct plan_t {
    int NB, k_pad, gblocks, nsplit, P, per_half, ntiles, ncyc, nsu, cpad;
};

plan_t make_plan(const pv_layout *l, int64_t k, bool two_nearest)
{
    plan_t p;
    p.ntiles = (1 << l->nbits) / 32;
    constexpr int cycle = kResidues * kU;    // tiles per residue cycle
    p.ncyc = (p.ntiles + cycle - 1) / cycle; // whole cycles: the table is padded with zero rows
    p.nsu = p.ncyc * kResidues;
    p.cpad = p.nsu * kU * 32;
    p.NB = k >= 4096 ? PV_NBX : 1;
    const int per_block = PV_WAVES * p.NB * 32;
    p.gblocks = (int)((k + per_block - 1) / per_block);
    p.k_pad = p.gblocks * per_block;
    // PV_OCC blocks per compute unit fit (registers, LDS).  Few group blocks: cut the
    // codeword range so that the items fill those slots in ONE round (a 13th split that
    // spills 21 blocks into a second round costs 25 %).  Many group blocks: several short
    // items per slot, handed out dynamically, so the tail is one short item - two to four of
    // them, and a power of two of splits: the splits then cover equal numbers of residue cycles,
    // and the re-rank reads 32 records a group instead of 48 (14336 x 4096 at g = 16, 183 500
    // groups: 4 splits against 6 leave the scoring as it is and take 10 us off the re-rank;
    // 3 and 5 splits cost the scoring 25 to 37 us).
    const int slots = 256 * PV_OCC;
    int want = slots / p.gblocks;
    // The rounding over the two nearest codewords keeps the finer cut (4 items a slot): its
    // cut comes from the second best objective, more keys reach it, and with 32 records a group
    // a third more groups were left to the block-wide scan (352 against 338 us there).
    if (want < 4 && two_nearest) want = (4 * slots + p.gblocks - 1) / p.gblocks;
    if (want < 4) {
        const int least = (2 * slots + p.gblocks - 1) / p.gblocks;
        want = 4;
        while (want < least) want *= 2;
    }
    if (want > 8 && slots / p.gblocks < 4) want = 8;
    int max_split = p.nsu * kU / 8;
    if (max_split > p.ncyc) max_split = p.ncyc;
    if (max_split < 1) max_split = 1;
    if (want > max_split) want = max_split;
    if (want > 32) want = 32;
    if (want < 1) want = 1;
    p.nsplit = want;
    // as many residue classes apart as 64 records per group allow: the more partitions, the
    // fewer groups have two keys above the cut in one of them
    p.per_half = kResidues;
    while (p.per_half > 1 && p.nsplit * 2 * p.per_half > 64) p.per_half >>= 1;
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
                                int64_t *num_changed, int32_t power, uint64_t seed)
{
    const plan_t p = make_plan(l, k, power > 0);
    const int g = l->group_size;
    const int csize = 1 << l->nbits;
    const int gpr = (int)(l->in_features / g);
    const int N = (int)pv_num_groups(l);
    const int nsu_alloc = 2 * p.nsu + 64;    // two norms per super-unit; the scoring kernel stages 64 at a time
    pv_status st;
    // codebook operand, then: position -> codeword, norm buckets, bucket counts / offsets,
    // smallest norm per super-unit
    const size_t a_bytes = (size_t)p.cpad * 32;
    const size_t perm_off = a_bytes, bucket_off = perm_off + (size_t)p.cpad * 2;
    const size_t hist_off = (bucket_off + (size_t)csize * 2 + 255) & ~(size_t)255;
    const size_t offs_off = hist_off + (size_t)kNormBins * 4;
    const size_t nmin_off = offs_off + (size_t)kNormBins * 4;
    const size_t cnorm_off = (nmin_off + (size_t)nsu_alloc * 4 + 255) & ~(size_t)255;   // g = 16: norm per position
    if ((st = pv_ensure(ctx, ctx->cb_f16, cnorm_off + (size_t)p.cpad * 4)) != PV_OK) return st;
    if ((st = pv_ensure(ctx, ctx->cb_meta, 16 * sizeof(unsigned), /*zero_new=*/true)) != PV_OK) return st;
    if ((st = pv_ensure(ctx, ctx->x_f16, (size_t)p.k_pad * 32)) != PV_OK) return st;
    // per-group bounds, then the staged targets / scale / code / id of each group
    const size_t stage_off = (size_t)p.k_pad * 4 * sizeof(float);
    if ((st = pv_ensure(ctx, ctx->x_meta, stage_off + (size_t)p.k_pad * (g + 4) * sizeof(float))) != PV_OK)
        return st;
    if ((st = pv_ensure(ctx, ctx->partials, (size_t)p.k_pad * p.P * sizeof(int2))) != PV_OK) return st;
    if ((st = pv_ensure(ctx, ctx->fb_list, 64)) != PV_OK) return st;
    const int rr_blocks = (int)((k * rerank_team(l->group_size) + kBlock - 1) / kBlock);
    const int nslots = (rr_blocks + 63) / 64;
    if ((st = pv_ensure(ctx, ctx->rr_counts, (size_t)rr_blocks * 4 * sizeof(unsigned) + (size_t)nslots * 8 + 16)) != PV_OK)
        return st;
    unsigned *rr_counts = static_cast<unsigned *>(ctx->rr_counts.ptr);
    unsigned long long *change_slots = reinterpret_cast<unsigned long long *>(
        static_cast<char *>(ctx->rr_counts.ptr) + (((size_t)rr_blocks * 4 * sizeof(unsigned) + 7) & ~(size_t)7));
    char *cbase = static_cast<char *>(ctx->cb_f16.ptr);
    h8 *A = reinterpret_cast<h8 *>(cbase);
    uint16_t *perm = reinterpret_cast<uint16_t *>(cbase + perm_off);
    uint16_t *bucket = reinterpret_cast<uint16_t *>(cbase + bucket_off);
    unsigned *hist = reinterpret_cast<unsigned *>(cbase + hist_off);
    unsigned *offsets = reinterpret_cast<unsigned *>(cbase + offs_off);
    unsigned *nmin_bits = reinterpret_cast<unsigned *>(cbase + nmin_off);
    float *cnorm = reinterpret_cast<float *>(cbase + cnorm_off);
    h8 *X = static_cast<h8 *>(ctx->x_f16.ptr);
    unsigned *cb_meta = static_cast<unsigned *>(ctx->cb_meta.ptr);
    float *x_meta = static_cast<float *>(ctx->x_meta.ptr);
    float *x_stage = x_meta + (size_t)p.k_pad * 4;
    int2 *partials = static_cast<int2 *>(ctx->partials.ptr);
    unsigned *fb_count = reinterpret_cast<unsigned *>(ctx->fb_list.ptr);       // 4 counters
    unsigned long long *stats = static_cast<unsigned long long *>(ctx->stats.ptr);
    auto nc = reinterpret_cast<unsigned long long *>(num_changed);
    hipStream_t sm = ctx->stream;
    // two statistics slots, used alternately (the first kernel of a call clears the other one)
    unsigned *cb_meta_next = cb_meta + (ctx->meta_phase ? 0 : 8);
    cb_meta += ctx->meta_phase ? 8 : 0;
    ctx->meta_phase ^= 1;
    {
        // Under graph capture the slots do not alternate from replay to replay (the graph keeps
        // the pointers of the captured call), so the slot this call accumulates into still holds
        // what the last replay left: clear it first (a fill kernel, not a memset node).
        hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
        PV_HIP(ctx, hipStreamIsCapturing(sm, &capturing));
        if (capturing != hipStreamCaptureStatusNone) {
            pv_status fs = pv_launch_fill_f32(ctx, reinterpret_cast<float *>(cb_meta), 8, 0.0f);
            if (fs != PV_OK) return fs;
        }
    }
    ctx->rr_blocks_last = rr_blocks;
    {
        pv_timed t(ctx, PV_K_PREP);
        int blocks = (csize + kBlock - 1) / kBlock;
        // every block ends with three atomics, each on one address: 64 blocks measured best (32
        // are as good, 128 cost 1.6 us more, 256 another 4)
        if (blocks > 64) blocks = 64;
        const int cb_blocks = (p.cpad + kBlock * kCbPer - 1) / (kBlock * kCbPer);
        const int x_blocks = (p.k_pad + kBlock - 1) / kBlock;
        if (g == 8) {
            hipLaunchKernelGGL(k_cb_stats<8>, dim3(blocks), dim3(kBlock), 0, sm, codebooks, csize,
                               cb_meta, cb_meta_next, stats, fb_count, nc, (unsigned *)nullptr,
                               (unsigned *)nullptr, 0, change_slots, nslots);
            hipLaunchKernelGGL(k_prep<8>, dim3(cb_blocks + x_blocks), dim3(kBlock), 0, sm, codebooks,
                               csize, p.cpad, cb_blocks, cb_meta, A, perm, bucket, hist, nmin_bits, cnorm, T,
                               scales, group_idx, (int)k, p.k_pad, gpr, N, X, x_meta, codes, csize - 1,
                               x_stage, p.ncyc, p.nsplit);
        } else {
            hipLaunchKernelGGL(k_cb_stats<16>, dim3(blocks), dim3(kBlock), 0, sm, codebooks, csize,
                               cb_meta, cb_meta_next, stats, fb_count, nc, hist, nmin_bits, nsu_alloc,
                               change_slots, nslots);
            hipLaunchKernelGGL(k_cb_bucket<16>, dim3((csize + kBlock - 1) / kBlock), dim3(kBlock), 0,
                               sm, codebooks, csize, cb_meta, bucket, hist);
            hipLaunchKernelGGL(k_cb_scan, dim3(kNormBins / kScanBlock), dim3(kScanBlock), 0, sm, hist, offsets);
            hipLaunchKernelGGL(k_prep<16>, dim3(cb_blocks + x_blocks), dim3(kBlock), 0, sm,
                               codebooks, csize, p.cpad, cb_blocks, cb_meta, A, perm, bucket, offsets,
                               nmin_bits, cnorm, T, scales, group_idx, (int)k, p.k_pad, gpr, N, X, x_meta,
                               codes, csize - 1, x_stage, p.ncyc, p.nsplit);
        }
    }
    {
        pv_timed t(ctx, PV_K_SCORE_MFMA);
        const int items = p.gblocks * p.nsplit;
        dim3 grid(items < 256 * PV_OCC ? items : 256 * PV_OCC);
        const float *nmin = reinterpret_cast<const float *>(nmin_bits);
#define PV_SCORE(G_, NB_)                                                                          \
    hipLaunchKernelGGL((k_score_mfma<G_, NB_>), grid, dim3(PV_WAVES * 64), 0, sm, A, X, x_meta, nmin, \
                       partials, p.ncyc, p.nsplit, p.per_half, p.gblocks, p.k_pad, fb_count + 1)
        if (g == 8) {
            if (p.NB == PV_NBX) PV_SCORE(8, PV_NBX);
            else PV_SCORE(8, 1);
        } else {
            if (p.NB == PV_NBX) PV_SCORE(16, PV_NBX);
            else PV_SCORE(16, 1);
        }
#undef PV_SCORE
    }
    {
        pv_timed t(ctx, PV_K_RERANK);
        const dim3 rgrid((unsigned)rr_blocks);
        if (power > 0) {
#define PV_ROUND2(G_)                                                                              \
    hipLaunchKernelGGL(k_round_top2<G_>, rgrid, dim3(kBlock), 0, sm, x_stage, codebooks, (int)k,    \
                       p.k_pad, partials, p.P, p.per_half, p.ncyc, p.nsplit, x_meta, cb_meta, A,    \
                       cnorm, X, perm, codes, rr_counts, change_slots, nc, l->nbits, (int)power,    \
                       (unsigned long long)seed)
            if (g == 8) PV_ROUND2(8);
            else PV_ROUND2(16);
#undef PV_ROUND2
        } else if (g == 8)
            hipLaunchKernelGGL(k_rerank<8>, rgrid, dim3(kBlock), 0, sm, x_stage, codebooks, (int)k,
                               p.k_pad, partials, p.P, p.per_half, p.ncyc, p.nsplit, x_meta, cb_meta, A,
                               cnorm, X, perm, codes, rr_counts, change_slots, nc, l->nbits);
        else
            hipLaunchKernelGGL(k_rerank<16>, rgrid, dim3(kBlock), 0, sm, x_stage, codebooks, (int)k,
                               p.k_pad, partials, p.P, p.per_half, p.ncyc, p.nsplit, x_meta, cb_meta, A,
                               cnorm, X, perm, codes, rr_counts, change_slots, nc, l->nbits);
    }
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

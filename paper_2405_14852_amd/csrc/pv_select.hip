// Group scores and top-k selection (Alg. 2 line 5, per matrix as in Sec. 3.4).
//
// score_n = sum_i (T[n,i] - W[n,i])^2 as an fp32 fused-multiply-add chain in
// index order, so that every implementation of this rule gives the same bits.
// Scores are non-negative floats, so their bit patterns order like unsigned
// integers.  The k-th largest key is found by a 3-digit radix select (11 + 12 +
// 8 bits below the sign, most significant first); groups above the threshold are taken, groups
// equal to it are taken lowest id first, and the ids are written in ascending
// order through a two-level prefix sum.  Nothing returns to the host.
//
// Launches: [scores + digit-0 histogram] [digit-1 histogram] [digit-2 histogram]
// [per-chunk counts] [ordered write].  Digit 0 (exponent and three mantissa bits: an
// eighth of an octave - the later passes pay one atomic on device memory for each key
// that shares the chosen one, the sweep one for each populated bin of each block) is counted in an LDS histogram inside
// the streaming score kernel, whose
// blocks are persistent so that clearing and flushing it is paid once per block;
// the later digits usually see only the few per cent of keys that share the
// chosen digit 0, but a narrow score distribution (updates of one size, as an
// optimiser's sign-like step produces) sends nearly all keys there, so they are
// counted in per-block LDS histograms as well.  Each launch resolves the digit of the histogram before it and
// publishes it for the launches that follow.
#include "pv_internal.h"

#ifndef PV_VOTE_ROUNDS
#define PV_VOTE_ROUNDS 1   // wave-wide merges before per-lane LDS atomics (guards degenerate inputs)
#endif

#ifndef PV_LATE_VOTE_ROUNDS
#define PV_LATE_VOTE_ROUNDS 0   // the same for the later digits: plain LDS atomics are faster on spread-out scores and on the narrow ones of an Adam step; only when EVERY score is equal would the merge win (5.6 M groups: 139 against 157 us for sweep + selection)
#endif

namespace {

constexpr int kBlock = 256;
#ifndef PV_REST_BITS
#define PV_REST_BITS 20
#endif
constexpr int kRestBits = PV_REST_BITS;         // bits of a key below digit 0
#ifndef PV_MID_BITS
#define PV_MID_BITS (PV_REST_BITS - 8)
#endif
constexpr int kMidBits = PV_MID_BITS;
constexpr int kSlots = 4096;                    // slots of every histogram in device memory
constexpr int kFirstBins = 1 << (31 - kRestBits);      // digit 0: exponent and 3 mantissa bits (keys are clamped below 2^31)
constexpr int kBins = 1 << kMidBits;                   // digit 1: the next mantissa bits
constexpr int kLastBins = 1 << (kRestBits - kMidBits + 1); // digit 2: the remaining low mantissa bits (at most)
static_assert(kFirstBins <= kSlots && kBins <= kSlots && kLastBins <= kSlots, "a histogram fits its slots");
constexpr int kItems = 8;                      // groups per thread in the compaction kernels
constexpr int kChunk = kBlock * kItems;        // groups per chunk there
static_assert(kChunk < 65536, "the compaction packs two per-chunk counts into 32 bits");
#ifndef PV_SEL_BLOCKS
#define PV_SEL_BLOCKS 512
#endif
constexpr int kMaxBlocks = PV_SEL_BLOCKS;      // persistent grid of the streaming kernels: two blocks per compute unit (1024 cost 1 us on 2 M groups and 4 to 6 us on 3.7 to 5.6 M, 256 lose a sixth of the bandwidth)
constexpr int kCompactBlocks = 1024;           // grid of the two compaction kernels

// The key of a score: its bits, which order like the values because scores are sums of squares
// (never negative); a pattern with the sign bit set can only be a NaN and is clamped to the
// largest key, so that digit 0 needs no bit for the sign.
__device__ __forceinline__ unsigned score_key(float s) { return min(__float_as_uint(s), 0x7FFFFFFFu); }

// `mid`: the width of digit 1, which every call fixes when digit 0 is known (see k_hist_next).
__device__ __forceinline__ int digit_of(unsigned key, int pass, int mid = kMidBits)
{
    return pass == 0 ? (int)(key >> kRestBits)
                     : pass == 1 ? (int)((key >> (kRestBits - mid)) & ((1u << mid) - 1u))
                                 : (int)(key & ((1u << (kRestBits - mid)) - 1u));
}

// Add one count per valid lane to an LDS histogram.  Lanes of a wave that hit
// the same bin as the first pending lane are merged first (catches the
// dominant bins of a narrow score distribution); the rest use one atomic each.
template <int ROUNDS>
__device__ __forceinline__ void hist_add(unsigned *hist, int bin, bool valid)
{
    const int lane = threadIdx.x & 63;
    if (ROUNDS > 0) {
        unsigned long long todo = __ballot(valid);
#pragma unroll 1
        for (int round = 0; round < ROUNDS && todo; ++round) {
            int leader = __ffsll((long long)todo) - 1;
            int lb = __shfl(bin, leader);
            unsigned long long same = __ballot(valid && bin == lb);
            if (lane == leader) atomicAdd(&hist[lb], (unsigned)__popcll(same));
            if (valid && bin == lb) valid = false;
            todo &= ~same;
        }
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

// Global histograms are stored so that the scan below reads them coalesced:
// digit d of a `bins`-digit histogram has rank r = bins - 1 - d from the top and
// lives at slot (r % kPer) * 256 + r / kPer with kPer = kSlots / 256 ranks per scan thread;
// thread t of the scan owns ranks [kPer t, kPer t + kPer), i.e. slots t, t + 256, ...
// Every histogram occupies kSlots slots.
constexpr int kPer = kSlots / kBlock;
// The first histogram is fed by every block of the scoring sweep at about the same moment, and
// most of the counts fall on a dozen bins: its atomics would queue on a dozen addresses (5 to
// 14 us on 2 M groups, depending on where the scores fall).  It is kept in kSub copies (two
// already take the queue below the kernel's streaming time; more only cost the readers), block
// b adds to copy b % kSub, the reader adds the copies.
#ifndef PV_HIST_COPIES
#define PV_HIST_COPIES 2
#endif
constexpr int kSub = PV_HIST_COPIES;
constexpr int kHist1 = kSub * kSlots;         // offsets of the second and third histogram
constexpr int kHist2 = kHist1 + kSlots;
constexpr int kHistTotal = kHist2 + kSlots;
__device__ __forceinline__ int hist_slot(int digit, int bins)
{
    const int r = bins - 1 - digit;
    return (r % kPer) * kBlock + (r / kPer);
}

// Given a histogram of `bins` digits and the rank `kk` (1-based, counted from the
// largest digit), find the digit d with  count(> d) < kk <= count(>= d)  and
// return kk - count(> d).  All threads of the block call this; the result goes
// to all, with the count of that digit if `count` is given.  `tmp` is kBlock + 3 unsigneds of LDS.
template <int COPIES = 1>
__device__ void pick_digit(const unsigned *__restrict__ ghist, int bins, unsigned kk,
                           unsigned *tmp, int *digit, unsigned *kk_rem, unsigned *count = nullptr)
{
    constexpr int per = kPer;            // ranks per thread; thread 0 owns the TOP digits
    const int tid = threadIdx.x;
    unsigned cnt[per];
    unsigned sum = 0;
#pragma unroll
    for (int j = 0; j < per; ++j) {
        unsigned part[COPIES];     // all loads of the copies in flight together
#pragma unroll
        for (int c = 0; c < COPIES; ++c)
            part[c] = ghist[c * kSlots + j * kBlock + tid];   // ranks beyond `bins`: slots that stay zero
        cnt[j] = 0u;
#pragma unroll
        for (int c = 0; c < COPIES; ++c) cnt[j] += part[c];
        sum += cnt[j];
    }
    unsigned total;
    unsigned above = block_excl_scan(sum, tmp, &total);
#pragma unroll
    for (int j = 0; j < per; ++j) {
        if (above < kk && kk <= above + cnt[j]) {
            tmp[kBlock] = (unsigned)(bins - 1 - (tid * per + j));
            tmp[kBlock + 1] = kk - above;
            tmp[kBlock + 2] = cnt[j];
        }
        above += cnt[j];
    }
    __syncthreads();
    *digit = (int)tmp[kBlock];
    *kk_rem = tmp[kBlock + 1];
    if (count) *count = tmp[kBlock + 2];
    __syncthreads();
}

__device__ __forceinline__ void flush_hist(const unsigned *lh, unsigned *__restrict__ gh, int bins)
{
    for (int b = threadIdx.x; b < bins; b += kBlock) {
        unsigned v = lh[b];
        if (v) atomicAdd(&gh[hist_slot(b, bins)], v);
    }
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

// Pass 0, any group size: one thread per group.
__global__ __launch_bounds__(kBlock) void k_scores_hist0(const float *__restrict__ T,
                                                         const float *__restrict__ W,
                                                         float *__restrict__ scores,
                                                         unsigned *__restrict__ hist0, int N, int g,
                                                         int want_hist)
{
    __shared__ unsigned lh[kFirstBins];
    if (want_hist)
        for (int b = threadIdx.x; b < kFirstBins; b += kBlock) lh[b] = 0;
    __syncthreads();
    for (int64_t base = (int64_t)blockIdx.x * kBlock; base < N; base += (int64_t)gridDim.x * kBlock) {
        const int64_t n = base + threadIdx.x;
        const bool valid = n < N;
        unsigned key = 0;
        if (valid) {
            float s = score_group(T + n * g, W + n * g, g);
            scores[n] = s;
            key = score_key(s);
        }
        if (want_hist) hist_add<PV_VOTE_ROUNDS>(lh, digit_of(key, 0), valid);
    }
    __syncthreads();
    if (want_hist) flush_hist(lh, hist0 + (blockIdx.x % kSub) * kSlots, kFirstBins);
}

// Pass 0 for g = 4 * PARTS (PARTS a power of two): every lane loads one 16-byte
// vector of T and of W, so a wave reads two contiguous 1 KiB runs per step.
// The fused-multiply-add chain of a group runs over PARTS neighbouring lanes in
// index order: each lane folds its four differences onto the partial sum of
// the lane before it; the last lane of the group holds the score.
constexpr int kVecUnroll = 4;

// NORM: the sweep also adds up (scales[row] * codeword element)^2 over the dequantised weights
// of the codes (one codebook; lane `part` of a group takes the same 16-byte piece of its
// codeword as of its target), in double, every thread in the order of its loop, the block
// in the fixed order of the reduction below: partial[block].
struct norm_args {
    const uint16_t *codes;
    const pv_f4 *cb4;
    const float *scales;
    double *partial;
    unsigned mask;
    double inv_gpr;
};

template <int PARTS, bool NORM>
__global__ __launch_bounds__(kBlock) void k_scores_hist0_vec(const float *__restrict__ T,
                                                             const float *__restrict__ W,
                                                             float *__restrict__ scores,
                                                             unsigned *__restrict__ hist0,
                                                             int64_t nvec, int want_hist, norm_args na)
{
    __shared__ unsigned lh[kFirstBins];
    double nacc = 0.0;
    if (want_hist)
        for (int b = threadIdx.x; b < kFirstBins; b += kBlock) lh[b] = 0;
    __syncthreads();
    const pv_f4 *T4 = reinterpret_cast<const pv_f4 *>(T);
    const pv_f4 *W4 = reinterpret_cast<const pv_f4 *>(W);
    const int part = threadIdx.x & (PARTS - 1);   // kBlock and every stride are multiples of PARTS
    for (int64_t cbase = (int64_t)blockIdx.x * (kBlock * kVecUnroll); cbase < nvec;
         cbase += (int64_t)gridDim.x * (kBlock * kVecUnroll)) {
        const int64_t base = cbase + threadIdx.x;
        pv_f4 a[kVecUnroll], b[kVecUnroll];
#pragma unroll
        for (int u = 0; u < kVecUnroll; ++u) {
            const int64_t i = base + (int64_t)u * kBlock;
            if (i < nvec) {
                a[u] = __builtin_nontemporal_load(&T4[i]);
                b[u] = __builtin_nontemporal_load(&W4[i]);
            } else {
                a[u] = pv_f4{0.f, 0.f, 0.f, 0.f};
                b[u] = a[u];
            }
        }
        // (requesting the codes a chunk ahead, so that the pieces go out with the chunk's targets
        // and weights, measured 3 us slower on 2 M groups)
        pv_f4 cw[kVecUnroll];
        float sc[kVecUnroll];
        if constexpr (NORM) {
            unsigned code[kVecUnroll];
#pragma unroll
            for (int u = 0; u < kVecUnroll; ++u) {      // codes and scales first, all in flight ...
                const int64_t i = base + (int64_t)u * kBlock;
                const unsigned n = (unsigned)((i < nvec ? i : 0) / PARTS);
                code[u] = na.codes[n] & na.mask;
                sc[u] = i < nvec ? na.scales[pv_row_of(n, na.inv_gpr)] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < kVecUnroll; ++u)        // ... then the codeword pieces
                cw[u] = na.cb4[(int64_t)code[u] * PARTS + part];
        }
#pragma unroll
        for (int u = 0; u < kVecUnroll; ++u) {
            const int64_t i = base + (int64_t)u * kBlock;
            if constexpr (NORM) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const double w = (double)(sc[u] * cw[u][e]);
                    nacc = nacc + w * w;
                }
            }
            const float d0 = a[u].x - b[u].x, d1 = a[u].y - b[u].y;
            const float d2 = a[u].z - b[u].z, d3 = a[u].w - b[u].w;
            float s = 0.0f;
#pragma unroll
            for (int r = 0; r < PARTS; ++r) {
                // after round r the lanes with part <= r hold their final prefix
                float in = r == 0 ? 0.0f : __shfl_up(s, 1);
                if (part >= r) {
                    float c = part == 0 ? 0.0f : in;
                    c = fmaf(d0, d0, c);
                    c = fmaf(d1, d1, c);
                    c = fmaf(d2, d2, c);
                    c = fmaf(d3, d3, c);
                    if (part == r) s = c;
                }
            }
            const bool valid = i < nvec && part == PARTS - 1;
            if (valid) scores[i / PARTS] = s;
            if (want_hist) hist_add<PV_VOTE_ROUNDS>(lh, digit_of(score_key(s), 0), valid);
        }
    }
    __syncthreads();
    if (want_hist) flush_hist(lh, hist0 + (blockIdx.x % kSub) * kSlots, kFirstBins);
    if constexpr (NORM) {
        __shared__ double ntmp[kBlock / 64];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) nacc = nacc + __shfl_down(nacc, off);
        if ((threadIdx.x & 63) == 0) ntmp[threadIdx.x >> 6] = nacc;
        __syncthreads();
        if (threadIdx.x == 0) {
            double t = 0.0;
            for (int w = 0; w < kBlock / 64; ++w) t = t + ntmp[w];
            na.partial[blockIdx.x] = t;
        }
    }
}

// Targets and pass 0 in one sweep (g = 4 * PARTS): T = W - alpha * G is formed and stored, and
// the scores and the digit-0 histogram are taken from the same registers, so T and W are
// not read back from memory.  The arithmetic is the one of the separate kernels: one fused
// multiply-add per element of T, then the subtraction T - W and the chain above.
template <int PARTS, bool ADAM>
__global__ __launch_bounds__(kBlock) void k_targets_scores_hist0_vec(const float *W, const float *G,
                                                                     float alpha, float *T,
                                                                     float *__restrict__ scores,
                                                                     unsigned *__restrict__ hist0,
                                                                     int64_t nvec, int want_hist,
                                                                     pv_adam_t adam, float *m, float *v)
{
    __shared__ unsigned lh[kFirstBins];
    if (want_hist)
        for (int b = threadIdx.x; b < kFirstBins; b += kBlock) lh[b] = 0;
    __syncthreads();
    const pv_f4 *W4 = reinterpret_cast<const pv_f4 *>(W);
    const pv_f4 *G4 = reinterpret_cast<const pv_f4 *>(G);
    pv_f4 *T4 = reinterpret_cast<pv_f4 *>(T);
    const int part = threadIdx.x & (PARTS - 1);
    const int64_t step = (int64_t)gridDim.x * (kBlock * kVecUnroll);
    pv_f4 *M4 = reinterpret_cast<pv_f4 *>(m);
    pv_f4 *V4 = reinterpret_cast<pv_f4 *>(v);
    pv_f4 w[kVecUnroll], gr[kVecUnroll], wn[kVecUnroll], gn[kVecUnroll];
    auto load = [&](int64_t cbase, pv_f4 *pw, pv_f4 *pg) {
#pragma unroll
        for (int u = 0; u < kVecUnroll; ++u) {
            const int64_t i = cbase + threadIdx.x + (int64_t)u * kBlock;
            if (i < nvec) {
                pw[u] = __builtin_nontemporal_load(&W4[i]);
                pg[u] = __builtin_nontemporal_load(&G4[i]);
            } else {
                pw[u] = pv_f4{0.f, 0.f, 0.f, 0.f};
                pg[u] = pw[u];
            }
        }
    };
    int64_t cbase = (int64_t)blockIdx.x * (kBlock * kVecUnroll);
    if (cbase < nvec) load(cbase, w, gr);
    for (; cbase < nvec; cbase += step) {
        // the loads of the next chunk are in flight while this one is scored
        if (cbase + step < nvec) load(cbase + step, wn, gn);
        const int64_t base = cbase + threadIdx.x;
#pragma unroll
        for (int u = 0; u < kVecUnroll; ++u) {
            const int64_t i = base + (int64_t)u * kBlock;
            pv_f4 t;
            if constexpr (ADAM) {
                pv_f4 mm = pv_f4{0.f, 0.f, 0.f, 0.f}, vv = mm;
                if (i < nvec) {
                    mm = __builtin_nontemporal_load(&M4[i]);
                    vv = __builtin_nontemporal_load(&V4[i]);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float mi = mm[e], vi = vv[e];
                    t[e] = pv_adam_one(w[u][e], gr[u][e], mi, vi, adam);
                    mm[e] = mi;
                    vv[e] = vi;
                }
                if (i < nvec) {
                    M4[i] = mm;
                    V4[i] = vv;
                }
            } else {
                t.x = fmaf(-alpha, gr[u].x, w[u].x);
                t.y = fmaf(-alpha, gr[u].y, w[u].y);
                t.z = fmaf(-alpha, gr[u].z, w[u].z);
                t.w = fmaf(-alpha, gr[u].w, w[u].w);
            }
            if (i < nvec) __builtin_nontemporal_store(t, &T4[i]);
            const float d0 = t.x - w[u].x, d1 = t.y - w[u].y;
            const float d2 = t.z - w[u].z, d3 = t.w - w[u].w;
            float s = 0.0f;
#pragma unroll
            for (int r = 0; r < PARTS; ++r) {
                float in = r == 0 ? 0.0f : __shfl_up(s, 1);
                if (part >= r) {
                    float c = part == 0 ? 0.0f : in;
                    c = fmaf(d0, d0, c);
                    c = fmaf(d1, d1, c);
                    c = fmaf(d2, d2, c);
                    c = fmaf(d3, d3, c);
                    if (part == r) s = c;
                }
            }
            const bool valid = i < nvec && part == PARTS - 1;
            if (valid) scores[i / PARTS] = s;
            if (want_hist) hist_add<PV_VOTE_ROUNDS>(lh, digit_of(score_key(s), 0), valid);
        }
#pragma unroll
        for (int u = 0; u < kVecUnroll; ++u) {
            w[u] = wn[u];
            gr[u] = gn[u];
        }
    }
    __syncthreads();
    if (want_hist) flush_hist(lh, hist0 + (blockIdx.x % kSub) * kSlots, kFirstBins);
}

// The same sweep for group sizes 1 and 2: a 16-byte vector holds 4 / GS whole groups and every
// lane scores its own (no exchange between lanes).  The last nelem % 4 elements, which fill
// no vector, are left to thread 0 of block 0.
template <int GS>
__global__ __launch_bounds__(kBlock) void k_targets_scores_hist0_sub(const float *W, const float *G,
                                                                     float alpha, float *T,
                                                                     float *__restrict__ scores,
                                                                     unsigned *__restrict__ hist0,
                                                                     int64_t nelem, int want_hist)
{
    constexpr int kPerVec = 4 / GS;               // groups per vector
    __shared__ unsigned lh[kFirstBins];
    if (want_hist)
        for (int b = threadIdx.x; b < kFirstBins; b += kBlock) lh[b] = 0;
    __syncthreads();
    const pv_f4 *W4 = reinterpret_cast<const pv_f4 *>(W);
    const pv_f4 *G4 = reinterpret_cast<const pv_f4 *>(G);
    pv_f4 *T4 = reinterpret_cast<pv_f4 *>(T);
    const int64_t nvec = nelem >> 2;
    // whole blocks stay in the loop together (the histogram update uses wave-wide votes)
    for (int64_t cbase = (int64_t)blockIdx.x * (kBlock * kVecUnroll); cbase < nvec;
         cbase += (int64_t)gridDim.x * (kBlock * kVecUnroll)) {
        pv_f4 w[kVecUnroll], gr[kVecUnroll];
#pragma unroll
        for (int u = 0; u < kVecUnroll; ++u) {
            const int64_t i = cbase + threadIdx.x + (int64_t)u * kBlock;
            if (i < nvec) {
                w[u] = __builtin_nontemporal_load(&W4[i]);
                gr[u] = __builtin_nontemporal_load(&G4[i]);
            } else {
                w[u] = pv_f4{0.f, 0.f, 0.f, 0.f};
                gr[u] = w[u];
            }
        }
#pragma unroll
        for (int u = 0; u < kVecUnroll; ++u) {
            const int64_t i = cbase + threadIdx.x + (int64_t)u * kBlock;
            const bool valid = i < nvec;
            pv_f4 t;
            float sc[kPerVec];
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = fmaf(-alpha, gr[u][e], w[u][e]);
#pragma unroll
            for (int q = 0; q < kPerVec; ++q) {
                float s = 0.0f;
#pragma unroll
                for (int e = 0; e < GS; ++e) {
                    const float d = t[q * GS + e] - w[u][q * GS + e];
                    s = fmaf(d, d, s);
                }
                sc[q] = s;
            }
            if (valid) {
                __builtin_nontemporal_store(t, &T4[i]);
#pragma unroll
                for (int q = 0; q < kPerVec; ++q) scores[i * kPerVec + q] = sc[q];
            }
            if (want_hist) {
#pragma unroll
                for (int q = 0; q < kPerVec; ++q)
                    hist_add<PV_VOTE_ROUNDS>(lh, digit_of(score_key(sc[q]), 0), valid);
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        // the elements after the last whole vector: whole groups, since nelem is a multiple of GS
        for (int64_t i = nvec << 2; i < nelem; i += GS) {
            float s = 0.0f;
            for (int e = 0; e < GS; ++e) {
                const float tv = fmaf(-alpha, G[i + e], W[i + e]);
                T[i + e] = tv;
                const float d = tv - W[i + e];
                s = fmaf(d, d, s);
            }
            scores[i / GS] = s;
            if (want_hist) atomicAdd(&lh[digit_of(score_key(s), 0)], 1u);
        }
    }
    __syncthreads();
    if (want_hist) flush_hist(lh, hist0 + (blockIdx.x % kSub) * kSlots, kFirstBins);
}

// Passes 1 and 2: histogram of the next digit among keys that match the digits
// chosen so far.  Each launch resolves the digit of the previous histogram and
// block 0 publishes it in `state` for the launches that follow:
// state[4] = digit 0, state[5] = digit 1, state[6] = rank left after digit 0,
// state[7] = rank left after digit 1, state[2] = width of digit 1.
// The width of digit 1 is fixed when digit 0 is known: kMidBits when few keys share digit 0 (a
// spread-out distribution: every such key costs an atomic on device memory in the flush, and a
// wide digit 1 leaves few for the last pass), one bit less when more than an eighth of all keys
// do (a narrow one, as after a sign-like optimiser step: the keys then fall on half as many bins
// of digit 1 and merge in the block histograms).
constexpr int kHistBlock = 512;   // measured against 256 and 1024 threads on 2 M and 5.6 M groups
__global__ __launch_bounds__(kHistBlock) void k_hist_next(const float *__restrict__ scores,
                                                      const unsigned *__restrict__ hist_all,
                                                      unsigned *__restrict__ hist_out,
                                                      unsigned *__restrict__ state, int N,
                                                      unsigned k, int pass)
{
    __shared__ unsigned tmp[kBlock + 3];
    __shared__ unsigned lh[kBins];
    int d0, d1 = 0, mid;
    unsigned kk;
    if (pass == 1) {
        unsigned share;
        pick_digit<kSub>(hist_all, kFirstBins, k, tmp, &d0, &kk, &share);
        mid = share > (unsigned)N / 8u ? kMidBits - 1 : kMidBits;
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            state[4] = (unsigned)d0;
            state[6] = kk;
            state[2] = (unsigned)mid;
        }
    } else {
        d0 = (int)state[4];
        mid = (int)state[2];
        pick_digit(hist_all + kHist1, 1 << mid, state[6], tmp, &d1, &kk);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            state[5] = (unsigned)d1;
            state[7] = kk;
        }
    }
    const int bins = pass == 1 ? (1 << mid) : (1 << (kRestBits - mid));
    // Per-block histogram in LDS, flushed once: a narrow score distribution (all updates of
    // one size, as after a sign-like optimiser step) puts most keys into a few bins, and that
    // many atomics on a few global addresses would serialise.
    for (int b = threadIdx.x; b < bins; b += kHistBlock) lh[b] = 0;
    __syncthreads();
    const pv_f4 *s4 = reinterpret_cast<const pv_f4 *>(scores);
    const int64_t n4 = N >> 2;
    const int64_t stride = (int64_t)gridDim.x * kHistBlock;
    // four vectors per thread in flight: with many groups (single-weight units) the loop is
    // otherwise one memory round trip per vector
    constexpr int kAhead = 4;
    for (int64_t base = (int64_t)blockIdx.x * kHistBlock; base < n4; base += stride * kAhead) {
        pv_f4 v[kAhead];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int64_t i = base + u * stride + threadIdx.x;
            v[u] = i < n4 ? s4[i] : pv_f4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int64_t i = base + u * stride + threadIdx.x;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                unsigned key = score_key(v[u][e]);
                bool valid = i < n4 && digit_of(key, 0) == d0 && (pass == 1 || digit_of(key, 1, mid) == d1);
                hist_add<PV_LATE_VOTE_ROUNDS>(lh, digit_of(key, pass, mid), valid);
            }
        }
    }
    if (blockIdx.x == 0 && (int)threadIdx.x < (N & 3)) {
        unsigned key = score_key(scores[(n4 << 2) + threadIdx.x]);
        if (digit_of(key, 0) == d0 && (pass == 1 || digit_of(key, 1, mid) == d1))
            atomicAdd(&lh[digit_of(key, pass, mid)], 1u);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < bins; b += kHistBlock) {
        unsigned v = lh[b];
        if (v) atomicAdd(&hist_out[hist_slot(b, bins)], v);
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

// Threshold key and number of ties to take, then per-chunk (greater, equal) counts.
__global__ __launch_bounds__(kBlock) void k_chunk_counts(const float *__restrict__ scores,
                                                         const unsigned *__restrict__ hist_all,
                                                         unsigned *state,
                                                         unsigned *__restrict__ chunk_counts, int N,
                                                         int nchunks)
{
    __shared__ unsigned tmp[kBlock + 3];
    const int d0 = (int)state[4], d1 = (int)state[5], mid = (int)state[2];
    int d2;
    unsigned kk;
    pick_digit(hist_all + kHist2, 1 << (kRestBits - mid), state[7], tmp, &d2, &kk);
    const unsigned thr = ((unsigned)d0 << kRestBits) | ((unsigned)d1 << (kRestBits - mid)) | (unsigned)d2;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        state[0] = thr;
        state[1] = kk;  // how many keys equal to thr are selected (lowest ids first)
    }
    for (int c = blockIdx.x; c < nchunks; c += gridDim.x) {
        const int64_t base = (int64_t)c * kChunk + (int64_t)threadIdx.x * kItems;
        unsigned gt = 0, eq = 0;
        if (base + kItems <= N) {
            const pv_f4 *s4 = reinterpret_cast<const pv_f4 *>(scores + base);
#pragma unroll
            for (int v = 0; v < kItems / 4; ++v) {
                pv_f4 x = s4[v];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    unsigned key = score_key(x[e]);
                    gt += key > thr;
                    eq += key == thr;
                }
            }
        } else {
            for (int j = 0; j < kItems; ++j)
                if (base + j < N) {
                    unsigned key = score_key(scores[base + j]);
                    gt += key > thr;
                    eq += key == thr;
                }
        }
        gt = block_sum(gt, tmp);
        eq = block_sum(eq, tmp);
        if (threadIdx.x == 0) {
            chunk_counts[2 * c] = gt;
            chunk_counts[2 * c + 1] = eq;
        }
    }
}

// Ordered write: position of a selected group = (#greater with a lower id) +
// min(#equal with a lower id, ties to take).  Also re-zeroes the histograms for
// the next call.
__global__ __launch_bounds__(kBlock) void k_compact_write(const float *__restrict__ scores,
                                                          const unsigned *__restrict__ state,
                                                          const unsigned *__restrict__ chunk_counts,
                                                          unsigned *__restrict__ hist_all,
                                                          int32_t *__restrict__ out_idx, int N,
                                                          int nchunks)
{
    __shared__ unsigned tmp[kBlock + 3];
    const unsigned thr = state[0], need_eq = state[1];
    // counts of all earlier chunks: [0, done) is already in (pg, pe), a block that takes several
    // chunks only adds the ones in between
    unsigned pg = 0, pe = 0;
    int done = 0;
    const uint2 *cc2 = reinterpret_cast<const uint2 *>(chunk_counts);
    for (int c = blockIdx.x; c < nchunks; c += gridDim.x) {
        unsigned ag = 0, ae = 0;
        for (int b = done + threadIdx.x; b < c; b += kBlock) {
            const uint2 v = cc2[b];
            ag += v.x;
            ae += v.y;
        }
        pg += block_sum(ag, tmp);
        pe += block_sum(ae, tmp);
        done = c;
        const int64_t base = (int64_t)c * kChunk + (int64_t)threadIdx.x * kItems;
        unsigned keys[kItems];
        unsigned gt = 0, eq = 0;
        if (base + kItems <= N) {
            const pv_f4 *s4 = reinterpret_cast<const pv_f4 *>(scores + base);
#pragma unroll
            for (int v = 0; v < kItems / 4; ++v) {
                const pv_f4 x = s4[v];
#pragma unroll
                for (int e = 0; e < 4; ++e) keys[v * 4 + e] = score_key(x[e]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < kItems; ++j) keys[j] = base + j < N ? score_key(scores[base + j]) : 0u;
        }
#pragma unroll
        for (int j = 0; j < kItems; ++j)
            if (base + j < N) {
                gt += keys[j] > thr;
                eq += keys[j] == thr;
            }
        // one scan for both counts: a chunk holds kChunk = 2048 keys, so each fits 16 bits
        unsigned tot;
        const unsigned both = block_excl_scan(gt | (eq << 16), tmp, &tot);
        unsigned rg = pg + (both & 0xFFFFu);   // greater keys before this thread's items
        unsigned re = pe + (both >> 16);       // equal keys before them
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
    }
    // leave the histograms zero for the next call (all their readers ran in earlier launches)
    for (int64_t z = (int64_t)blockIdx.x * kBlock + threadIdx.x; z < kHistTotal;
         z += (int64_t)gridDim.x * kBlock)
        hist_all[z] = 0;
}

}  // namespace

// The scratch memory of one selection: every group's score (unless the caller keeps them),
// the radix-select histograms (all zero when a call starts, left zero when it ends), the
// per-chunk counts of the compaction, the digits and threshold found so far.
struct sel_bufs {
    float *scores;
    unsigned *hist, *cc, *state;
    pv_norm_req *norm = nullptr;
};

__global__ void k_sel_clear(unsigned *p, int n)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0u;
}

static pv_status select_run(pv_ctx *ctx, const pv_layout *l, const float *T, const float *W,
                            int64_t k, int32_t *out_idx, const sel_bufs &bufs, const float *G,
                            float alpha, const pv_adam_t *adam, float *m, float *v);

// G != nullptr: T is an OUTPUT, formed here as W - alpha * G in the same pass that scores it.
pv_status pv_launch_select(pv_ctx *ctx, const pv_layout *l, const float *T, const float *W,
                           int64_t k, int32_t *out_idx, float *scores, const float *G, float alpha,
                           const pv_adam_t *adam, float *m, float *v, pv_norm_req *norm)
{
    const int N = (int)pv_num_groups(l);
    pv_status st;
    if (norm && (G || !pv_select_norm_supported(l)))
        return pv_fail(ctx, PV_ERR_UNSUPPORTED, "norm request: scores-only sweep, one codebook, g = 8 or 16");
    if (!scores) {
        st = pv_ensure(ctx, ctx->sel_scores, (size_t)N * sizeof(float) + 16);
        if (st != PV_OK) return st;
        scores = static_cast<float *>(ctx->sel_scores.ptr);
    }
    const int nchunks = (N + kChunk - 1) / kChunk;
    st = pv_ensure(ctx, ctx->sel_hist, (size_t)kHistTotal * sizeof(unsigned), /*zero_new=*/true);
    if (st != PV_OK) return st;
    st = pv_ensure(ctx, ctx->sel_blocks, (size_t)nchunks * 2 * sizeof(unsigned));
    if (st != PV_OK) return st;
    st = pv_ensure(ctx, ctx->sel_state, 8 * sizeof(unsigned));
    if (st != PV_OK) return st;
    sel_bufs bufs;
    bufs.scores = scores;
    bufs.hist = static_cast<unsigned *>(ctx->sel_hist.ptr);
    bufs.cc = static_cast<unsigned *>(ctx->sel_blocks.ptr);
    bufs.state = static_cast<unsigned *>(ctx->sel_state.ptr);
    bufs.norm = norm;
    return select_run(ctx, l, T, W, k, out_idx, bufs, G, alpha, adam, m, v);
}

bool pv_select_norm_supported(const pv_layout *l)
{
    return l->num_codebooks == 1 && (l->group_size == 8 || l->group_size == 16);
}

int pv_select_norm_parts() { return kMaxBlocks; }

// ---------------------------------------------------------------- selection without allocation
// For callers that cannot allocate device memory (code under HIP graph capture, tight serving
// loops, harnesses that forbid it): the same selection with its scratch in one static device
// array.  Each GPU holds its own copy of the array for the life of the process; every call on
// a GPU shares it, so calls that overlap on one GPU (two streams, two contexts) race.
constexpr int64_t kStaticMaxGroups = INT64_C(1) << 22;            // 4 194 304 groups
constexpr size_t kStaticScoresOff = 0;
constexpr size_t kStaticHistOff = kStaticScoresOff + (size_t)kStaticMaxGroups * sizeof(float) + 256;
constexpr size_t kStaticCcOff = kStaticHistOff + (size_t)kHistTotal * sizeof(unsigned);
constexpr size_t kStaticStateOff =
    kStaticCcOff + (size_t)((kStaticMaxGroups + kChunk - 1) / kChunk) * 2 * sizeof(unsigned);
constexpr size_t kStaticBytes = kStaticStateOff + 256;            // about 16.1 MiB
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

// In host code `scratch` is only a stand-in for the symbol: the memory is reached through the
// address the runtime reports for it on each device.
constexpr int kMaxDevices = 64;
static unsigned char *g_static_ptr[kMaxDevices] = {nullptr};

// The device must be current.  Called by pv_create (once per context) and again by the entry
// point itself; the first call on a device asks the runtime, later ones return the kept address.
pv_status pv_static_scratch_init(pv_ctx *ctx, int device)
{
    if (device < 0 || device >= kMaxDevices)
        return pv_fail(ctx, PV_ERR_INVALID_ARG, "device %d outside 0..%d", device, kMaxDevices - 1);
    unsigned char *p = __atomic_load_n(&g_static_ptr[device], __ATOMIC_ACQUIRE);
    if (p) return PV_OK;
    void *sym = nullptr;
    hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !sym) {
        (void)hipGetLastError();
        return pv_fail(ctx, PV_ERR_DEVICE, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    }
    __atomic_store_n(&g_static_ptr[device], static_cast<unsigned char *>(sym), __ATOMIC_RELEASE);
    return PV_OK;
}

int64_t pv_static_max_groups() { return kStaticMaxGroups; }

pv_status pv_launch_select_static(pv_ctx *ctx, const pv_layout *l, const float *T, const float *W,
                                  int64_t k, int32_t *out_idx, float *scores)
{
    pv_status st = pv_static_scratch_init(ctx, ctx->device);
    if (st != PV_OK) return st;
    unsigned char *base = __atomic_load_n(&g_static_ptr[ctx->device], __ATOMIC_ACQUIRE);
    sel_bufs bufs;
    bufs.scores = scores ? scores : reinterpret_cast<float *>(base + kStaticScoresOff);
    bufs.hist = reinterpret_cast<unsigned *>(base + kStaticHistOff);
    bufs.cc = reinterpret_cast<unsigned *>(base + kStaticCcOff);
    bufs.state = reinterpret_cast<unsigned *>(base + kStaticStateOff);
    // the array keeps what the last call (of any context) left: the histograms must start at
    // zero whatever that was (a fill kernel, which a capturing caller may record)
    hipLaunchKernelGGL(k_sel_clear, dim3(16), dim3(kBlock), 0, ctx->stream, bufs.hist, kHistTotal);
    const bool timing = ctx->timing;   // timing brackets create events: not in this call
    ctx->timing = false;
    st = select_run(ctx, l, T, W, k, out_idx, bufs, nullptr, 0.0f, nullptr, nullptr, nullptr);
    ctx->timing = timing;
    return st;
}

static pv_status select_run(pv_ctx *ctx, const pv_layout *l, const float *T, const float *W,
                            int64_t k, int32_t *out_idx, const sel_bufs &bufs, const float *G,
                            float alpha, const pv_adam_t *adam, float *m, float *v)
{
    const int N = (int)pv_num_groups(l);
    const int g = l->group_size;
    const int nchunks = (N + kChunk - 1) / kChunk;
    pv_status st;
    float *scores = bufs.scores;
    unsigned *hist = bufs.hist;
    unsigned *cc = bufs.cc;
    unsigned *state = bufs.state;
    const int want_hist = k > 0 ? 1 : 0;
    const bool vec_g = g == 4 || g == 8 || g == 16 || g == 32 || g == 64;
    if (G && !adam && (g == 1 || g == 2)) {
        pv_timed t(ctx, PV_K_ENCODE_TARGETS);
        const int64_t nelem = (int64_t)N * g;
        int64_t vb = ((nelem >> 2) + kBlock * kVecUnroll - 1) / (kBlock * kVecUnroll);
        const unsigned vblocks = (unsigned)(vb < 1 ? 1 : (vb < kMaxBlocks ? vb : kMaxBlocks));
        float *Tw = const_cast<float *>(T);
        if (g == 1)
            hipLaunchKernelGGL(k_targets_scores_hist0_sub<1>, dim3(vblocks), dim3(kBlock), 0, ctx->stream,
                               W, G, alpha, Tw, scores, hist, nelem, want_hist);
        else
            hipLaunchKernelGGL(k_targets_scores_hist0_sub<2>, dim3(vblocks), dim3(kBlock), 0, ctx->stream,
                               W, G, alpha, Tw, scores, hist, nelem, want_hist);
    } else {
    if (G && !vec_g) {   // no fused kernel for this group size: form T first
        // (the Adam variant reaches this launcher only for the group sizes that have one)
        st = pv_launch_encode_targets(ctx, W, G, alpha, const_cast<float *>(T),
                                      l->out_features * l->in_features);
        if (st != PV_OK) return st;
        G = nullptr;
    }
    if (G) {
        pv_timed t(ctx, PV_K_ENCODE_TARGETS);
        const int64_t nvec = (int64_t)N * (g / 4);
        int64_t vb = (nvec + kBlock * kVecUnroll - 1) / (kBlock * kVecUnroll);
        const unsigned vblocks = (unsigned)(vb < kMaxBlocks ? vb : kMaxBlocks);
        float *Tw = const_cast<float *>(T);
        const pv_adam_t a = adam ? *adam : pv_adam_t{};
#define PV_FUSED(PARTS_)                                                                            \
    do {                                                                                            \
        if (adam)                                                                                   \
            hipLaunchKernelGGL((k_targets_scores_hist0_vec<PARTS_, true>), dim3(vblocks), dim3(kBlock), \
                               0, ctx->stream, W, G, alpha, Tw, scores, hist, nvec, want_hist, a, m, v); \
        else                                                                                        \
            hipLaunchKernelGGL((k_targets_scores_hist0_vec<PARTS_, false>), dim3(vblocks),          \
                               dim3(kBlock), 0, ctx->stream, W, G, alpha, Tw, scores, hist, nvec,   \
                               want_hist, a, m, v);                                                 \
    } while (0)
        if (g == 4) PV_FUSED(1);
        else if (g == 8) PV_FUSED(2);
        else if (g == 16) PV_FUSED(4);
        else if (g == 32) PV_FUSED(8);
        else PV_FUSED(16);
#undef PV_FUSED
    } else {
        pv_timed t(ctx, PV_K_GROUP_SCORES);
        const int64_t nvec = (int64_t)N * (g / 4);
        int64_t vb = (nvec + kBlock * kVecUnroll - 1) / (kBlock * kVecUnroll);
        const unsigned vblocks = (unsigned)(vb < kMaxBlocks ? vb : kMaxBlocks);
        int64_t sb = ((int64_t)N + kBlock - 1) / kBlock;
        const unsigned sblocks = (unsigned)(sb < kMaxBlocks ? sb : kMaxBlocks);
        norm_args na{};
        if (bufs.norm) {
            na.codes = bufs.norm->codes;
            na.cb4 = reinterpret_cast<const pv_f4 *>(bufs.norm->codebooks);
            na.scales = bufs.norm->scales;
            na.partial = bufs.norm->partial;
            na.mask = (1u << l->nbits) - 1u;
            na.inv_gpr = 1.0 / (double)(l->in_features / g);
            bufs.norm->parts = (int)vblocks;
        }
#define PV_SCORES(PARTS_)                                                                          \
    do {                                                                                           \
        if (bufs.norm)                                                                             \
            hipLaunchKernelGGL((k_scores_hist0_vec<PARTS_, true>), dim3(vblocks), dim3(kBlock), 0, \
                               ctx->stream, T, W, scores, hist, nvec, want_hist, na);              \
        else                                                                                       \
            hipLaunchKernelGGL((k_scores_hist0_vec<PARTS_, false>), dim3(vblocks), dim3(kBlock), 0, \
                               ctx->stream, T, W, scores, hist, nvec, want_hist, na);              \
    } while (0)
        if (g == 4) PV_SCORES(1);
        else if (g == 8) PV_SCORES(2);
        else if (g == 16) PV_SCORES(4);
        else if (g == 32) PV_SCORES(8);
        else if (g == 64) PV_SCORES(16);
        else
            hipLaunchKernelGGL(k_scores_hist0, dim3(sblocks), dim3(kBlock), 0, ctx->stream, T, W,
                               scores, hist, N, g, want_hist);
#undef PV_SCORES
    }
    }   // group sizes other than 1 and 2
    if (k > 0) {
        pv_timed t(ctx, PV_K_SELECT);
        int64_t hb = ((int64_t)(N >> 2) + kHistBlock - 1) / kHistBlock;
        const unsigned hblocks = (unsigned)(hb < 512 ? (hb < 1 ? 1 : hb) : 512);
        const unsigned cblocks = (unsigned)(nchunks < kCompactBlocks ? nchunks : kCompactBlocks);
        hipLaunchKernelGGL(k_hist_next, dim3(hblocks), dim3(kHistBlock), 0, ctx->stream, scores, hist,
                           hist + kHist1, state, N, (unsigned)k, 1);
        hipLaunchKernelGGL(k_hist_next, dim3(hblocks), dim3(kHistBlock), 0, ctx->stream, scores, hist,
                           hist + kHist2, state, N, (unsigned)k, 2);
        hipLaunchKernelGGL(k_chunk_counts, dim3(cblocks), dim3(kBlock), 0, ctx->stream, scores, hist,
                           state, cc, N, nchunks);
        hipLaunchKernelGGL(k_compact_write, dim3(cblocks), dim3(kBlock), 0, ctx->stream, scores,
                           state, cc, hist, out_idx, N, nchunks);
    }
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

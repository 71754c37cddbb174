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
//   ranked candidates (radix select, then a stable descending sort of the k_max
//   selected keys: inside one block's LDS when they fit, else the four-pass
//   device-wide radix sort) -> all candidates re-encoded in place (previous codes saved) ->
//   squared change per candidate -> prefix sums in rank order -> first prefix
//   that breaks the bound -> codes of the candidates behind it restored.
// Everything stays on the device; the kept count is written to device memory.
//
// Arithmetic: a group's change is the sum over its weights of
// (double(w_new) - double(w_old))^2 with w the fp32 dequantised weights; the
// prefix sums and ||x^k||^2 are double sums in a fixed (launch-independent)
// association, so a run is reproducible; they differ from a sequential sum by
// rounding only.
#include "pv_internal.h"
#include "pv_radix.h"

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

// Ranking of up to kSmallMax candidates in two kernels.  First every block sorts one tile of
// kRankTile candidates in LDS: a stable radix sort of the complemented keys (descending
// scores, equal scores in the order they came in, i.e. ascending ids), four passes of 8 bits,
// the (key, position) pairs held in registers between passes - wave w holds the consecutive
// run w * kRankRounds * 64 .., 64 pairs a round - and written through LDS once per pass to
// the slot their digit rank gives them.  Slots beyond k are padded with the largest key and
// positions >= k, so they stay behind.  Then k_tr_merge_ranks places every candidate among
// the other tiles by bisection.
constexpr int kRankRounds = 1;
constexpr int kRankTile = kSortBlock * kRankRounds;      // 1024
constexpr int kRankTilesMax = 32;
constexpr int kSmallMax = kRankTile * kRankTilesMax;     // 32768
// The kernel also does what k_tr_gather does for the device-wide route: the keys are read
// straight from the scores of the selected groups, the candidates' codes are saved, and block 0
// adds up the partial norms and resets the state.
__global__ __launch_bounds__(kSortBlock) void k_tr_sort_tiles(
    const int32_t *__restrict__ idx, const float *__restrict__ scores, int k,
    const uint16_t *__restrict__ codes, int M, uint16_t *__restrict__ old_codes,
    const double *__restrict__ norm_partial, int norm_parts, tr_state *__restrict__ state,
    unsigned *__restrict__ tile_keys, int32_t *__restrict__ tile_pos)
{
    __shared__ unsigned s_key[kRankTile];
    __shared__ unsigned s_pos[kRankTile];
    __shared__ unsigned wcnt[kSortWaves][256];
    __shared__ unsigned s_first[256];
    __shared__ unsigned s_w4[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tile0 = blockIdx.x * kRankTile;
    unsigned key[kRankRounds], pos[kRankRounds], rank[kRankRounds];
#pragma unroll
    for (int j = 0; j < kRankRounds; ++j) {
        const int e = tile0 + (wave * kRankRounds + j) * 64 + lane;
        pos[j] = (unsigned)e;
        key[j] = 0xFFFFFFFFu;
        if (e < k) {
            const int64_t n = idx[e];
            key[j] = ~__float_as_uint(scores[n]);   // scores are >= +0: the bits order like the values
            for (int m = 0; m < M; ++m) old_codes[(int64_t)e * M + m] = codes[n * M + m];
        }
    }
    if (blockIdx.x == 0) {                // the partial norms, added as k_tr_gather adds them
        __shared__ double s_norm[kBlock / 64];
        double acc = 0.0;
        if (threadIdx.x < kBlock) {
            for (int i = threadIdx.x; i < norm_parts; i += kBlock) acc = acc + norm_partial[i];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) acc = acc + __shfl_down(acc, off);
            if (lane == 0) s_norm[wave] = acc;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            double t = 0.0;
            for (int w = 0; w < kBlock / 64; ++w) t = t + s_norm[w];
            state->normsq = t;
            state->first_violation = kNone;
            state->first_moved = kNone;
            state->kept = 0;
        }
    }
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int shift = 0; shift < 32; shift += 8) {
        for (int w = threadIdx.x; w < kSortWaves * 256; w += kSortBlock) (&wcnt[0][0])[w] = 0u;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kRankRounds; ++j) {
            const unsigned d = (key[j] >> shift) & 255u;
            unsigned long long same = ~0ull;
#pragma unroll
            for (int bit = 0; bit < 8; ++bit) {
                const unsigned long long has = __ballot((d >> bit) & 1u);
                same &= ((d >> bit) & 1u) ? has : ~has;
            }
            const unsigned before = wcnt[wave][d];
            rank[j] = before + (unsigned)__popcll(same & below);
            if (lane == 63 - __clzll(same)) wcnt[wave][d] = before + (unsigned)__popcll(same);
        }
        __syncthreads();
        unsigned cnt = 0;
        if (threadIdx.x < 256) {          // one digit each: offsets of the waves, then of the digits
            unsigned c[kSortWaves];
#pragma unroll
            for (int w = 0; w < kSortWaves; ++w) c[w] = wcnt[w][threadIdx.x];
#pragma unroll
            for (int w = 0; w < kSortWaves; ++w) {
                wcnt[w][threadIdx.x] = cnt;
                cnt += c[w];
            }
            unsigned a = cnt;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const unsigned oa = __shfl_up(a, off);
                if (lane >= off) a += oa;
            }
            if (lane == 63) s_w4[wave] = a;
            cnt = a - cnt;                // exclusive inside the wave
        }
        __syncthreads();
        if (threadIdx.x < 256) {
            unsigned a = 0;
            for (int w = 0; w < wave; ++w) a += s_w4[w];
            s_first[threadIdx.x] = cnt + a;
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kRankRounds; ++j) {
            const unsigned d = (key[j] >> shift) & 255u;
            const unsigned slot = s_first[d] + wcnt[wave][d] + rank[j];
            s_key[slot] = key[j];
            s_pos[slot] = pos[j];
        }
        __syncthreads();
        if (shift < 24) {
#pragma unroll
            for (int j = 0; j < kRankRounds; ++j) {
                const int e = (wave * kRankRounds + j) * 64 + lane;
                key[j] = s_key[e];
                pos[j] = s_pos[e];
            }
        }
    }
    for (int r = threadIdx.x; r < kRankTile && tile0 + r < k; r += kSortBlock) {
        tile_keys[tile0 + r] = s_key[r];
        tile_pos[tile0 + r] = (int32_t)s_pos[r];
    }
}

// Rank of every candidate among all tiles: its place in its own sorted tile plus, for every
// other tile, the number of that tile's (complemented) keys that come before it - keys that
// are smaller, and in the tiles before its own also the equal ones, whose ids are lower.
// All tiles' keys sit in LDS; the bisections of one candidate over the tiles advance together.
constexpr int kMergeParts = 8;                                  // threads per candidate
constexpr int kMergeCands = kSortBlock / kMergeParts;           // candidates per block
__global__ __launch_bounds__(kSortBlock) void k_tr_merge_ranks(const unsigned *__restrict__ tile_keys,
                                                               const int32_t *__restrict__ tile_pos,
                                                               int k, int32_t *__restrict__ order)
{
    __shared__ unsigned s_all[kSmallMax];
    {   // all keys into LDS, 16 bytes a load, every load of a thread in flight together (the
        // array is padded to 256 bytes, so the last vector may reach past k)
        typedef unsigned u4 __attribute__((ext_vector_type(4)));
        const u4 *src = reinterpret_cast<const u4 *>(tile_keys);
        const int nvec = (k + 3) >> 2;
        constexpr int kVecs = kSmallMax / 4 / kSortBlock;       // 8 vectors a thread at most
        u4 buf[kVecs];
#pragma unroll
        for (int u = 0; u < kVecs; ++u) {
            const int v = u * kSortBlock + threadIdx.x;
            buf[u] = src[v < nvec ? v : 0];
        }
#pragma unroll
        for (int u = 0; u < kVecs; ++u) {
            const int v = u * kSortBlock + threadIdx.x;
            if (v < nvec) reinterpret_cast<u4 *>(s_all)[v] = buf[u];
        }
    }
    __syncthreads();
    const int tiles = (k + kRankTile - 1) / kRankTile;
    const int part = threadIdx.x % kMergeParts;                 // this thread's tiles: part, part + 8, ..
    const int e = blockIdx.x * kMergeCands + threadIdx.x / kMergeParts;
    const int ec = e < k ? e : k - 1;
    const int own = ec / kRankTile, local = ec - own * kRankTile;
    const unsigned key = s_all[ec];
    constexpr int kSlots = kRankTilesMax / kMergeParts;
    int lo[kSlots], len[kSlots];
#pragma unroll
    for (int q = 0; q < kSlots; ++q) {
        const int b = part + q * kMergeParts;
        lo[q] = 0;
        const int left = k - b * kRankTile;
        len[q] = (b < tiles && b != own) ? (left < kRankTile ? left : kRankTile) : 0;
    }
    // lo[q] = number of keys of that tile that come before this one, by halving the range
    for (int step = 0; step < 11; ++step) {
#pragma unroll
        for (int q = 0; q < kSlots; ++q) {
            const int b = part + q * kMergeParts;
            const int half = len[q] >> 1;
            const int at = b * kRankTile + lo[q] + half;
            const unsigned probe = s_all[len[q] > 0 ? at : 0];
            const bool before = b < own ? probe <= key : probe < key;
            const bool go = len[q] > 0 && before;
            lo[q] = go ? lo[q] + half + 1 : lo[q];
            len[q] = len[q] > 0 ? (before ? len[q] - half - 1 : half) : 0;
        }
    }
    int rank = 0;
#pragma unroll
    for (int q = 0; q < kSlots; ++q) rank += lo[q];
#pragma unroll
    for (int off = 1; off < kMergeParts; off <<= 1) rank += __shfl_xor(rank, off);
    if (part == 0 && e < k) order[local + rank] = tile_pos[e];
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

// ||x^k||^2 for one codebook and g = 4 * LPG (8 or 16): LPG neighbouring lanes share a group
// and read neighbouring 16-byte pieces of its codeword, so that one request to L2 brings the
// whole codeword (the kernel is bound by the number of such requests: the codebook is L2
// resident, the rows are picked at random).  Block b sums the groups
// [b * per_block, (b + 1) * per_block); a thread adds the squares of its four weights of the
// groups t / LPG, t / LPG + 256 / LPG, ..., in that order, kGroups groups in flight.
template <int LPG>
__global__ __launch_bounds__(kBlock) void k_tr_normsq_rows(const uint16_t *__restrict__ codes,
                                                           const float *__restrict__ codebooks,
                                                           const float *__restrict__ scales, int64_t N,
                                                           int64_t per_block, int nbits, int gpr,
                                                           double *__restrict__ partial)
{
    __shared__ double tmp[kBlock / 64];
    constexpr int kGroups = 8;
    constexpr int kStride = kBlock / LPG;
    const unsigned mask = (1u << nbits) - 1u;
    const int64_t lo = (int64_t)blockIdx.x * per_block;
    const int64_t hi = lo + per_block < N ? lo + per_block : N;
    const int piece = threadIdx.x % LPG;
    const pv_f4 *cb4 = reinterpret_cast<const pv_f4 *>(codebooks);
    double acc = 0.0;
    for (int64_t n0 = lo + threadIdx.x / LPG; n0 < hi; n0 += (int64_t)kStride * kGroups) {
        unsigned code[kGroups];
        float s[kGroups];
#pragma unroll
        for (int u = 0; u < kGroups; ++u) {
            const int64_t n = n0 + (int64_t)u * kStride;
            code[u] = n < hi ? (codes[n] & mask) : 0u;
            s[u] = n < hi ? scales[n / gpr] : 0.0f;
        }
        pv_f4 c[kGroups];
#pragma unroll
        for (int u = 0; u < kGroups; ++u) c[u] = cb4[(int64_t)code[u] * LPG + piece];
#pragma unroll
        for (int u = 0; u < kGroups; ++u) {
            if (n0 + (int64_t)u * kStride < hi) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    double w = (double)(s[u] * c[u][e]);
                    acc = acc + w * w;
                }
            }
        }
    }
    acc = block_sum(acc, tmp);
    if (threadIdx.x == 0) partial[blockIdx.x] = acc;
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
                                                      bool offsets_ready /* else: tile sums */,
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
    double before_tile = 0.0;
    if (offsets_ready) {
        before_tile = tile_off[blockIdx.x];
    } else {              // few tiles: the sums of the tiles before this one, added in tile order
        for (int t = 0; t < (int)blockIdx.x; ++t) before_tile = before_tile + tile_off[t];
    }
    const double off = before_tile + tile_exclusive(mine, s_wave, &total);
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
    int norm_blocks = (int)((N + 1023) / 1024);       // a round of gathers per thread: latency, not volume, sets the time
    if (norm_blocks > 4096) norm_blocks = 4096;
    if (norm_blocks < 1) norm_blocks = 1;
    const int64_t per_block = (N + norm_blocks - 1) / norm_blocks;

    const int sort_tiles = (k + kSortTile - 1) / kSortTile;      // tiles of a device-wide sorting pass
    const bool small_sort = k <= kSmallMax;
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
    size_t o_keys3 = o_norm + align_up((size_t)(norm_blocks > pv_select_norm_parts() ? norm_blocks : pv_select_norm_parts()) * 8);
    size_t o_vals2 = o_keys3 + align_up(small_sort ? 0 : kk * 4);
    size_t o_hist = o_vals2 + align_up(small_sort ? 0 : kk * 4);
    size_t o_rowpre = o_hist + align_up(small_sort ? 0 : (size_t)sort_tiles * 256 * 4);
    size_t o_totals = o_rowpre + align_up(small_sort ? 0 : (size_t)sort_tiles * 256 * 4);
    size_t total = o_totals + 1024;
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
    unsigned *keys3 = reinterpret_cast<unsigned *>(base + o_keys3);
    int32_t *vals2 = reinterpret_cast<int32_t *>(base + o_vals2);
    unsigned *hist = reinterpret_cast<unsigned *>(base + o_hist);
    unsigned *rowpre = reinterpret_cast<unsigned *>(base + o_rowpre);
    unsigned *totals = reinterpret_cast<unsigned *>(base + o_totals);
    float *scores = static_cast<float *>(ctx->sel_scores.ptr);
    hipStream_t sm = ctx->stream;

    // ||x^k||^2 of the codes as they are now (partial sums; the gather kernel adds them up).
    // One codebook and g = 8 or 16: the scoring sweep of the selection takes it on its way.
    pv_norm_req norm_req{codes, codebooks, scales, norm_partial, 0};
    const bool fused_norm = pv_select_norm_supported(l);
    if (!fused_norm) {
        pv_timed t(ctx, PV_K_TRUST_RATIO);
        if (M == 1 && g == 8)
            hipLaunchKernelGGL(k_tr_normsq_rows<2>, dim3(norm_blocks), dim3(kBlock), 0, sm, codes, codebooks,
                               scales, N, per_block, l->nbits, gpr, norm_partial);
        else if (M == 1 && g == 16)
            hipLaunchKernelGGL(k_tr_normsq_rows<4>, dim3(norm_blocks), dim3(kBlock), 0, sm, codes, codebooks,
                               scales, N, per_block, l->nbits, gpr, norm_partial);
        else if (M == 1 && g % 4 == 0)
            hipLaunchKernelGGL((k_tr_normsq<1, true>), dim3(norm_blocks), dim3(kBlock), 0, sm, codes,
                               codebooks, scales, N, per_block, g, M, l->nbits, gpr, norm_partial);
        else
            hipLaunchKernelGGL((k_tr_normsq<0, false>), dim3(norm_blocks), dim3(kBlock), 0, sm, codes,
                               codebooks, scales, N, per_block, g, M, l->nbits, gpr, norm_partial);
    }
    // candidates: the k_max groups of the selection rule (ascending ids) and every score
    st = pv_launch_select(ctx, l, T, W, k, idx, scores, nullptr, 0.0f, nullptr, nullptr, nullptr,
                          fused_norm ? &norm_req : nullptr);
    if (st != PV_OK) return st;
    if (fused_norm) norm_blocks = norm_req.parts;
    const unsigned kblocks = (unsigned)((k + kBlock - 1) / kBlock);
    {
        pv_timed t(ctx, PV_K_TRUST_RATIO);
        if (!(k > 0 && small_sort))
            hipLaunchKernelGGL(k_tr_gather, dim3(kblocks > 0 ? kblocks : 1), dim3(kBlock), 0, sm, idx, k,
                               scores, codes, M, old_codes, keys, pos, norm_partial, norm_blocks, state);
        // descending keys; equal keys keep their order (ascending ids): the sort is stable
        if (k > 0 && small_sort) {
            const unsigned rtiles = (unsigned)((k + kRankTile - 1) / kRankTile);
            hipLaunchKernelGGL(k_tr_sort_tiles, dim3(rtiles), dim3(kSortBlock), 0, sm, idx, scores, k, codes,
                               M, old_codes, norm_partial, norm_blocks, state, keys2, pos);
            hipLaunchKernelGGL(k_tr_merge_ranks, dim3((unsigned)((k + kMergeCands - 1) / kMergeCands)),
                               dim3(kSortBlock), 0, sm, keys2, pos, k, order);
        } else if (k > 0) {
            // four passes over the complemented keys; (keys2, pos) and (keys3, vals2) take turns
            for (int pass = 0; pass < 4; ++pass) {
                unsigned *k_out = (pass & 1) ? keys3 : keys2;
                int32_t *v_out = pass == 3 ? order : ((pass & 1) ? vals2 : pos);
                const unsigned *k_in = (pass & 1) ? keys2 : keys3;
                const int32_t *v_in = (pass & 1) ? pos : vals2;
                if (pass == 0) {
                    const descending_keys dk{keys};
                    hipLaunchKernelGGL(k_digit_hist<descending_keys>, dim3(sort_tiles), dim3(kSortBlock),
                                       0, sm, dk, (int64_t)k, 0, sort_tiles, hist);
                    hipLaunchKernelGGL(k_row_scan, dim3(256), dim3(kRadixBlock), 0, sm, hist, sort_tiles,
                                       rowpre, totals);
                    hipLaunchKernelGGL((k_digit_scatter<descending_keys, unsigned>), dim3(sort_tiles),
                                       dim3(kSortBlock), 0, sm, dk, (const int32_t *)nullptr, (int64_t)k, 0,
                                       sort_tiles, rowpre, totals, k_out, v_out);
                } else {
                    const plain_keys<unsigned> pk{k_in};
                    hipLaunchKernelGGL(k_digit_hist<plain_keys<unsigned>>, dim3(sort_tiles),
                                       dim3(kSortBlock), 0, sm, pk, (int64_t)k, 8 * pass, sort_tiles, hist);
                    hipLaunchKernelGGL(k_row_scan, dim3(256), dim3(kRadixBlock), 0, sm, hist, sort_tiles,
                                       rowpre, totals);
                    hipLaunchKernelGGL((k_digit_scatter<plain_keys<unsigned>, unsigned>), dim3(sort_tiles),
                                       dim3(kSortBlock), 0, sm, pk, v_in, (int64_t)k, 8 * pass, sort_tiles,
                                       rowpre, totals, k_out, v_out);
                }
            }
        }
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
            const bool few = tiles <= 256;   // then every block adds the earlier tile sums itself
            if (!few)
                hipLaunchKernelGGL(k_tr_tile_offsets, dim3(1), dim3(kBlock), 0, sm, tile_sum, tiles);
            hipLaunchKernelGGL(k_tr_prefix, dim3(tiles), dim3(kBlock), 0, sm, delta, moved, k,
                               (const double *)tile_sum, !few, ratio, prefix, state);
        }
        hipLaunchKernelGGL(k_tr_rollback, dim3(kblocks > 0 ? kblocks : 1), dim3(kBlock), 0, sm, idx,
                           order, k, old_codes, codes, M, state, prefix, chunk, rank_idx, num_applied,
                           stats);
    }
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

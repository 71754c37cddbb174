// Gradients of the continuous parameters for the P step (Alg. 3, P step: "backprop";
// App. K: codebooks and per-channel scales): the chain rule through
//     W[o, j*g + i] = s_o * sum_m C_m[b(o,j,m), i]
// applied to G = d phi / d W:
//     d phi / d C_m[c, i] = sum over groups n = (o, j) with b(o,j,m) = c of  s_o * G[n, i]
//     d phi / d s_o       = sum_j sum_i G[o, j*g + i] * (C_0[b_0, i] + C_1[b_1, i] + ...)
//
// The codebook gradient is a scatter-add of N * g values into 2^B * g sums.  Floating-point
// atomics would serialise on popular codewords and give run-dependent roundings (and atomics
// on device memory are slow on a part whose L2 is split over several dies); instead the
// groups are SORTED by code with a stable radix sort written for this key width - 8 bits a
// pass, so at most two passes of histogram, prefix sum and scatter, with ranks taken from
// wave ballots and per-wave counters in LDS so that equal codes keep ascending group order
// and no atomic touches device memory - and every codeword's segment is summed by g
// lanes in that order, in double, with exact products: the same sum, in the same order, as a
// plain loop over the groups.  Segments longer than kLong groups are cut into pieces of kLong
// that are summed by the teams of one block and added in piece order (a different
// association from the plain loop: reproducible from run to run, but no longer the sequential
// rounding).  Small codebooks take another route (k_pg_small below).  The scale gradient is
// one block-wide tree sum per row.
#include "pv_internal.h"
#include "pv_radix.h"

namespace {

constexpr int kBlock = 256;
constexpr int kLong = 128;       // groups per piece: a segment up to this long is summed by one team alone
// the codes of codebook m as sort keys, masked to B bits
struct code_keys {
    const uint16_t *codes;
    int M, m;
    unsigned mask;
    __device__ __forceinline__ unsigned operator()(int64_t e) const
    {
        return (unsigned)(codes[e * M + m] & mask);
    }
};

// start[c] = first position of code c in the sorted order (= position of the next present
// code when c is absent); start[csize] = N.  Also clears the length of the list of long segments.
__global__ __launch_bounds__(kBlock) void k_pg_starts(const uint16_t *__restrict__ sorted, int64_t N,
                                                      int csize, int32_t *__restrict__ start,
                                                      unsigned *__restrict__ nlong)
{
    const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (r == 0) *nlong = 0u;
    if (r >= N) return;
    const int cur = sorted[r];
    const int prev = r == 0 ? -1 : (int)sorted[r - 1];
    for (int c = prev + 1; c <= cur; ++c) start[c] = (int32_t)r;
    if (r == N - 1)
        for (int c = cur + 1; c <= csize; ++c) start[c] = (int32_t)N;
}

// Sum of s_o * G[n, i] over ids[a .. b) in that order, kInFlight gathers issued together.
constexpr int kInFlight = 8;
template <bool HAVE_SCALES, class IDS>
__device__ __forceinline__ double ordered_sum(IDS ids, const float *__restrict__ s_of,
                                              const float *__restrict__ G,
                                              const float *__restrict__ scales, int gpr, int g,
                                              int i, int a, int b, double acc = 0.0)
{
    for (int r0 = a; r0 < b; r0 += kInFlight) {
        float gv[kInFlight], sv[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const int r = r0 + u < b ? r0 + u : b - 1;
            const int n = ids[r];
            gv[u] = G[(int64_t)n * g + i];
            sv[u] = HAVE_SCALES ? s_of[r] : scales[n / gpr];
        }
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const double next = acc + (double)sv[u] * (double)gv[u];
            acc = r0 + u < b ? next : acc;
        }
    }
    return acc;
}

// Segments of up to kLong groups: one team of TEAM lanes per codeword (TEAM = the group size
// rounded up to a power of two, at least 8).  The team stages the segment's ids and row
// scales in LDS, then lane i sums dimension i in segment order.  A longer segment is put on
// the list for k_pg_long.
template <int TEAM>
__global__ __launch_bounds__(kBlock) void k_pg_short(const int32_t *__restrict__ start,
                                                     const int32_t *__restrict__ order,
                                                     const float *__restrict__ G,
                                                     const float *__restrict__ scales, int gpr, int g,
                                                     int csize, int32_t *__restrict__ long_list,
                                                     unsigned *__restrict__ nlong,
                                                     float *__restrict__ out)
{
    constexpr int kTeams = kBlock / TEAM;
    __shared__ int s_id[kTeams][kLong];
    __shared__ float s_s[kTeams][kLong];
    const int team = threadIdx.x / TEAM, i = threadIdx.x % TEAM;
    const int c = blockIdx.x * kTeams + team;
    int lo = 0, len = 0;
    bool mine = false;
    if (c < csize) {
        lo = start[c];
        len = start[c + 1] - lo;
        mine = len <= kLong;
        if (!mine) {
            len = 0;
            if (i == 0) long_list[atomicAdd(nlong, 1u)] = c;
        }
    }
    for (int r = i; r < len; r += TEAM) s_id[team][r] = order[lo + r];
    __syncthreads();
    // the first kFirst gathers of G and the row scales of the whole segment are requested
    // together: a typical segment costs one round trip here, not one per few groups
    constexpr int kFirst = 32;
    float gv[kFirst];
    const int ii = i < g ? i : 0;
    if (len > 0) {
#pragma unroll
        for (int u = 0; u < kFirst; ++u)
            gv[u] = G[(int64_t)s_id[team][u < len ? u : len - 1] * g + ii];
    }
    for (int r = i; r < len; r += TEAM) s_s[team][r] = scales[s_id[team][r] / gpr];
    __syncthreads();
    if (mine && i < g) {
        double acc = 0.0;
        if (len > 0) {
#pragma unroll
            for (int u = 0; u < kFirst; ++u) {
                const double next = acc + (double)s_s[team][u < len ? u : len - 1] * (double)gv[u];
                acc = u < len ? next : acc;
            }
            if (len > kFirst)
                acc = ordered_sum<true>(s_id[team], s_s[team], G, scales, gpr, g, i, kFirst, len, acc);
        }
        out[(int64_t)c * g + i] = (float)acc;
    }
}

// Segments longer than kLong: one block per segment.  Its teams sum pieces of kLong ids in
// order (piece p of the segment that starts at sorted position lo keeps its sum in
// partial[lo / kLong + p], p >= 1: the ranges of different segments cannot meet; piece 0 stays
// in LDS), and the first g threads add the piece sums in piece order.
template <int TEAM>
__global__ __launch_bounds__(kBlock) void k_pg_long(const int32_t *__restrict__ long_list,
                                                    const unsigned *__restrict__ nlong,
                                                    const int32_t *__restrict__ start,
                                                    const int32_t *__restrict__ order,
                                                    const float *__restrict__ G,
                                                    const float *__restrict__ scales, int gpr, int g,
                                                    double *partial, float *__restrict__ out)
{
    constexpr int kTeams = kBlock / TEAM;
    __shared__ double s_first[64];
    const int team = threadIdx.x / TEAM, i = threadIdx.x % TEAM;
    const int count = (int)*nlong;
    for (int li = blockIdx.x; li < count; li += gridDim.x) {
        const int c = long_list[li];
        const int lo = start[c], len = start[c + 1] - lo;
        const int32_t *ids = order + lo;
        const int pieces = (len + kLong - 1) / kLong;
        double *mine = partial + (int64_t)(lo / kLong) * g;
        for (int p = team; p < pieces; p += kTeams) {
            const int a = p * kLong, b = a + kLong < len ? a + kLong : len;
            if (i < g) {
                const double acc = ordered_sum<false>(ids, nullptr, G, scales, gpr, g, i, a, b);
                if (p == 0) s_first[i] = acc;
                else mine[(int64_t)p * g + i] = acc;
            }
        }
        __syncthreads();
        if ((int)threadIdx.x < g) {
            double acc = s_first[threadIdx.x];
            int p = 1;
            for (; p + 4 <= pieces; p += 4) {          // four loads in flight, added in piece order
                double v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = mine[(int64_t)(p + u) * g + threadIdx.x];
#pragma unroll
                for (int u = 0; u < 4; ++u) acc = acc + v[u];
            }
            for (; p < pieces; ++p) acc = acc + mine[(int64_t)p * g + threadIdx.x];
            out[(int64_t)c * g + threadIdx.x] = (float)acc;
        }
        __syncthreads();
    }
}

// Small codebooks (all M * 2^B * g sums fit one block's LDS): every codeword is shared by
// thousands of groups, so sorting buys nothing.  Each block sweeps a contiguous range of
// groups once, 16 bytes of G per thread, and adds s_o * G into its own LDS table with LDS
// atomics.  To make the result independent of the order in which the atomics land, the
// table is kept in 64-bit FIXED POINT: with X = max|s| * max|G| (both maxima are taken
// beforehand, the product of two floats is exact in double) every term is scaled by a power
// of two that leaves `headroom` bits for the number of terms one block can add, and rounded
// to an integer once; integer addition is associative, so a table is a function of the
// block's inputs only.  The tables are added over the blocks as integers too (exactly) and
// the total is scaled back and rounded to fp32.  A term keeps min(62 - headroom, 50) bits
// below X (>= 39 for the largest matrices), so a sum differs from the exact one by far less
// than the rounding of a sequential double loop does.  Gradients or scales that are not
// finite make every entry NaN.  The kernel is bound by the LDS atomics (sixteen per group and
// codebook), not by reading G: indices are kept in 32 bits relative to the block's range and
// the conversion to an integer is one addition, so that the vector ALU stays out of the way.
constexpr int kSmallBlock = 1024;                         // one table serves sixteen waves
constexpr int kSmallAhead = 2;                            // vectors of a thread in flight
// The power of two that turns a term s_o * G into a 64-bit integer (see k_pg_small): from the
// largest |scale| and the largest |G| (as bits: NaN > inf > every finite value), leaving
// `headroom` bits for the terms one block adds to an entry.  Block 0 leaves the inverse factor
// and the poison flag (some input not finite) in meta[0], meta[1].  All threads of a
// kSmallBlock-wide block call this; s_max is 2 * kSmallBlock / 64 unsigneds of LDS.
__device__ __forceinline__ double fixed_point_unit(const float *__restrict__ scales, int out_features,
                                                   const unsigned *__restrict__ gmax_bits, int nmax,
                                                   int headroom, unsigned *s_max,
                                                   double *__restrict__ meta)
{
    constexpr int kW = kSmallBlock / 64;
    unsigned sb = 0u, gb = 0u;
    for (int o = threadIdx.x; o < out_features; o += kSmallBlock) sb = max(sb, __float_as_uint(fabsf(scales[o])));
    for (int o = threadIdx.x; o < nmax; o += kSmallBlock) gb = max(gb, gmax_bits[o]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        sb = max(sb, (unsigned)__shfl_down(sb, off));
        gb = max(gb, (unsigned)__shfl_down(gb, off));
    }
    if ((threadIdx.x & 63) == 0) {
        s_max[threadIdx.x >> 6] = sb;
        s_max[kW + (threadIdx.x >> 6)] = gb;
    }
    __syncthreads();
    sb = gb = 0u;
#pragma unroll
    for (int w = 0; w < kW; ++w) {
        sb = max(sb, s_max[w]);
        gb = max(gb, s_max[kW + w]);
    }
    const double X = (double)__uint_as_float(sb) * (double)__uint_as_float(gb);
    const bool poison = !(X < __builtin_huge_val());
    int ex = 0;
    (void)frexp(X, &ex);                                  // X < 2^ex
    const int kbits = 62 - headroom < 50 ? 62 - headroom : 50;   // bits of a term below 2^ex
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        meta[0] = (X > 0.0 && !poison) ? ldexp(1.0, -(kbits - ex)) : 0.0;
        meta[1] = poison ? 1.0 : 0.0;
    }
    return (X > 0.0 && !poison) ? ldexp(1.0, kbits - ex) : 0.0;
}

// x + 1.5 * 2^52 holds the integer nearest to x (ties to even) in its low mantissa bits for
// |x| < 2^51; the terms stay below 2^50
__device__ __forceinline__ unsigned long long fixed_point_term(double x)
{
    constexpr double kMagic = 6755399441055744.0;
    return (unsigned long long)(__double_as_longlong(x + kMagic) - __double_as_longlong(kMagic));
}

// VPG: 16-byte vectors per group when that is 1, 2 or 4 (a shift finds the group), else 0
template <int VPG>
__global__ __launch_bounds__(kSmallBlock) void k_pg_small(
    const float *__restrict__ G, const uint16_t *__restrict__ codes,
    const float *__restrict__ scales, int64_t N, int64_t per_block, int g, int M, int nbits,
    int gpr, int out_features, const unsigned *__restrict__ gmax_bits, int nmax, int headroom,
    long long *__restrict__ partial, double *__restrict__ meta)
{
    extern __shared__ unsigned long long tab[];         // [M][2^B][g]
    __shared__ unsigned s_max[2 * (kSmallBlock / 64)];
    const int csize = 1 << nbits;
    const unsigned mask = (unsigned)csize - 1u;
    const int entries = M * csize * g;
    for (int e = threadIdx.x; e < entries; e += kSmallBlock) tab[e] = 0ull;
    const double up = fixed_point_unit(scales, out_features, gmax_bits, nmax, headroom, s_max, meta);
    const unsigned vpg = VPG > 0 ? (unsigned)VPG : (unsigned)(g / 4);   // 16-byte vectors per group
    const int64_t lo = (int64_t)blockIdx.x * per_block;
    const int64_t hi = lo + per_block < N ? lo + per_block : N;
    // everything inside the block's range is counted from its first group in 32 bits
    const unsigned nvec = hi > lo ? (unsigned)(hi - lo) * vpg : 0u;
    const unsigned row0 = (unsigned)(lo / gpr), rem0 = (unsigned)(lo - (int64_t)row0 * gpr);
    const double inv_gpr = 1.0 / (double)gpr;
    const pv_f4 *G4 = reinterpret_cast<const pv_f4 *>(G) + lo * vpg;
    const uint16_t *codes0 = codes + lo * M;
    // Within a codeword's row the elements are permuted by bits of the code (power-of-two
    // groups): for a given element the 64 lanes of an atomic then spread over all LDS banks
    // instead of the few that a row stride of 8 g bytes leaves them.
    const unsigned swm = (g & (g - 1)) == 0 ? (unsigned)g - 1u : 0u;
    for (unsigned v0 = threadIdx.x; v0 < nvec; v0 += kSmallBlock * kSmallAhead) {
        pv_f4 gv[kSmallAhead];
        float sf[kSmallAhead];
        unsigned nl[kSmallAhead], q4[kSmallAhead], c01[kSmallAhead][2];
#pragma unroll
        for (int u = 0; u < kSmallAhead; ++u) {
            const unsigned v = v0 + (unsigned)u * kSmallBlock;
            const unsigned vc = v < nvec ? v : nvec - 1u;   // clamped: the loads of a batch go out together
            nl[u] = vc / vpg;
            q4[u] = vc - nl[u] * vpg;
            gv[u] = __builtin_nontemporal_load(&G4[vc]);
            sf[u] = scales[row0 + pv_row_of(rem0 + nl[u], inv_gpr)];
#pragma unroll
            for (int m = 0; m < 2; ++m) c01[u][m] = m < M ? codes0[(size_t)nl[u] * M + m] & mask : 0u;
        }
#pragma unroll
        for (int u = 0; u < kSmallAhead; ++u) {
            if (v0 + (unsigned)u * kSmallBlock >= nvec) break;
            const double ss = (double)sf[u] * up;           // a power of two: exact
            unsigned long long term[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                term[e] = fixed_point_term(ss * (double)gv[u][e]);
            for (int m = 0; m < M; ++m) {
                const unsigned c = m < 2 ? c01[u][m] : codes0[(size_t)nl[u] * M + m] & mask;
                unsigned long long *row = tab + ((size_t)m * csize + c) * g;
                const unsigned sw = (c >> 2) & swm;
#pragma unroll
                for (int e = 0; e < 4; ++e) atomicAdd(&row[(q4[u] * 4u + e) ^ sw], term[e]);
            }
        }
    }
    __syncthreads();
    long long *out = partial + (int64_t)blockIdx.x * entries;
    for (int e = threadIdx.x; e < entries; e += kSmallBlock) {
        const unsigned sw = ((((unsigned)e / (unsigned)g) & mask) >> 2) & swm;   // the code within its codebook, as on the way in
        out[e] = (long long)tab[(unsigned)e ^ sw];
    }
}

// adds the per-block tables as integers (16 threads per entry, each a slice of the blocks),
// scales back and rounds once
constexpr int kSlices = 16;
__global__ __launch_bounds__(kBlock) void k_pg_small_final(const long long *__restrict__ partial,
                                                           int blocks, int entries,
                                                           const double *__restrict__ meta,
                                                           float *__restrict__ out)
{
    __shared__ long long s_hi[kSlices][kBlock / kSlices];
    __shared__ long long s_lo[kSlices][kBlock / kSlices];
    const int col = threadIdx.x % (kBlock / kSlices), sl = threadIdx.x / (kBlock / kSlices);
    const int e = blockIdx.x * (kBlock / kSlices) + col;
    long long hi = 0, lo = 0;                           // total = hi * 2^32 + lo
    if (e < entries) {
        for (int b0 = sl; b0 < blocks; b0 += kSlices * 4) {
            long long p[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int b = b0 + u * kSlices;
                p[u] = b < blocks ? partial[(int64_t)b * entries + e] : 0;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                hi += p[u] >> 32;
                lo += p[u] & 0xffffffffll;
            }
        }
    }
    s_hi[sl][col] = hi;
    s_lo[sl][col] = lo;
    __syncthreads();
    if (sl == 0 && e < entries) {
        for (int q = 1; q < kSlices; ++q) {
            hi += s_hi[q][col];
            lo += s_lo[q][col];
        }
        // |hi| < 2^40 and 0 <= lo < 2^41: both conversions are exact, the sum rounds once
        const double total = (double)hi * 4294967296.0 + (double)lo;
        out[e] = meta[1] != 0.0 ? __builtin_nanf("") : (float)(total * meta[0]);
    }
}

// largest |G| seen by each block, as bits, for callers that do not ask for the scale gradient
// (whose kernel takes the maximum of each row on its way)
__global__ __launch_bounds__(kBlock) void k_pg_absmax(const float *__restrict__ G, int64_t n4,
                                                      unsigned *__restrict__ gmax_bits)
{
    const pv_f4 *G4 = reinterpret_cast<const pv_f4 *>(G);
    unsigned mb = 0u;
    for (int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x; v < n4; v += (int64_t)gridDim.x * kBlock) {
        const pv_f4 x = G4[v];
#pragma unroll
        for (int e = 0; e < 4; ++e) mb = max(mb, __float_as_uint(fabsf(x[e])));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mb = max(mb, (unsigned)__shfl_down(mb, off));
    __shared__ unsigned tmp_max[kBlock / 64];
    if ((threadIdx.x & 63) == 0) tmp_max[threadIdx.x >> 6] = mb;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / 64; ++w) mb = max(mb, tmp_max[w]);
        gmax_bits[blockIdx.x] = mb;
    }
}

// one block per output row; VEC: g % 4 == 0, a thread takes 16-byte vectors
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_pg_scales(const float *__restrict__ G,
                                                      const uint16_t *__restrict__ codes,
                                                      const float *__restrict__ codebooks, int g,
                                                      int M, int nbits, int gpr,
                                                      float *__restrict__ grad_scales,
                                                      unsigned *__restrict__ gmax_bits /* [rows], NULL ok */)
{
    __shared__ double tmp[kBlock / 64];
    unsigned mb = 0u;                     // largest |G| of the row, as bits
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
        // kAhead vectors of a thread at a time: their codes, then their codewords, are in flight
        // together (a row is only a few vectors per thread: one at a time the kernel is a chain
        // of round trips); the terms are still added in index order
        constexpr int kAhead = 4;
        for (int64_t e0 = threadIdx.x; e0 < nv; e0 += (int64_t)kBlock * kAhead) {
            pv_f4 gv[kAhead], q[kAhead];
            unsigned code[kAhead];
            int q4[kAhead];
            int64_t n[kAhead];
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                const int64_t e = e0 + (int64_t)u * kBlock;
                const int64_t ec = e < nv ? e : nv - 1;
                n[u] = o * gpr + ec / vpg;
                q4[u] = (int)(ec % vpg);
                gv[u] = __builtin_nontemporal_load(&G4[ec]);
                code[u] = codes[n[u] * M] & mask;
            }
#pragma unroll
            for (int u = 0; u < kAhead; ++u) q[u] = C4[((int64_t)code[u] * g) / 4 + q4[u]];
            for (int m = 1; m < M; ++m) {
                pv_f4 c[kAhead];
#pragma unroll
                for (int u = 0; u < kAhead; ++u)
                    c[u] = C4[((m * csize + (codes[n[u] * M + m] & mask)) * g) / 4 + q4[u]];
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    q[u].x = q[u].x + c[u].x;
                    q[u].y = q[u].y + c[u].y;
                    q[u].z = q[u].z + c[u].z;
                    q[u].w = q[u].w + c[u].w;
                }
            }
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                if (e0 + (int64_t)u * kBlock < nv) {
                    acc = acc + (double)gv[u].x * (double)q[u].x;
                    acc = acc + (double)gv[u].y * (double)q[u].y;
                    acc = acc + (double)gv[u].z * (double)q[u].z;
                    acc = acc + (double)gv[u].w * (double)q[u].w;
                    mb = max(max(mb, __float_as_uint(fabsf(gv[u].x))), __float_as_uint(fabsf(gv[u].y)));
                    mb = max(max(mb, __float_as_uint(fabsf(gv[u].z))), __float_as_uint(fabsf(gv[u].w)));
                }
            }
        }
    } else {
        for (int64_t e = threadIdx.x; e < in_features; e += kBlock) {
            const int64_t n = o * gpr + e / g;
            const int i = (int)(e % g);
            float q = codebooks[(int64_t)(codes[n * M] & mask) * g + i];
            for (int m = 1; m < M; ++m)
                q = q + codebooks[(m * csize + (codes[n * M + m] & mask)) * g + i];
            const float gv = G[o * in_features + e];
            acc = acc + (double)gv * (double)q;
            mb = max(mb, __float_as_uint(fabsf(gv)));
        }
    }
    __shared__ unsigned tmp_max[kBlock / 64];
    if (gmax_bits) {     // one plain store per row: atomics on one device address would queue up
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mb = max(mb, (unsigned)__shfl_down(mb, off));
        if ((threadIdx.x & 63) == 0) tmp_max[threadIdx.x >> 6] = mb;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc = acc + __shfl_down(acc, off);
    if ((threadIdx.x & 63) == 0) tmp[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < kBlock / 64; ++w) t = t + tmp[w];
        grad_scales[o] = (float)t;
        if (gmax_bits) {
            unsigned m4 = 0u;
            for (int w = 0; w < kBlock / 64; ++w) m4 = max(m4, tmp_max[w]);
            gmax_bits[o] = m4;
        }
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
        int headroom = 1;                                 // 2^headroom > terms one block adds to an entry
        while (((int64_t)1 << headroom) <= per_block) ++headroom;
        const int64_t n4 = N * g / 4;
        int64_t mblocks = (n4 + kBlock * 8 - 1) / (kBlock * 8);
        if (mblocks > 2048) mblocks = 2048;
        const int nmax = grad_scales ? (int)l->out_features : (int)mblocks;
        const size_t o_meta = align_up((size_t)blocks * entries * 8);
        const size_t o_gmax = o_meta + 256;
        pv_status st2 = pv_ensure(ctx, ctx->pstep, o_gmax + (size_t)nmax * 4);
        if (st2 != PV_OK) return st2;
        long long *partial = static_cast<long long *>(ctx->pstep.ptr);
        double *meta = reinterpret_cast<double *>(static_cast<char *>(ctx->pstep.ptr) + o_meta);
        unsigned *gmax = reinterpret_cast<unsigned *>(static_cast<char *>(ctx->pstep.ptr) + o_gmax);
        pv_timed t(ctx, PV_K_PSTEP);
        if (grad_scales)     // first: it reads all of G anyway and takes max|G| of each row on its way
            hipLaunchKernelGGL(k_pg_scales<true>, dim3((unsigned)l->out_features), dim3(kBlock), 0, sm,
                               G, codes, codebooks, g, M, l->nbits, gpr, grad_scales, gmax);
        else
            hipLaunchKernelGGL(k_pg_absmax, dim3((unsigned)mblocks), dim3(kBlock), 0, sm, G, n4, gmax);
#define PV_SMALL(V_)                                                                             \
    hipLaunchKernelGGL(k_pg_small<V_>, dim3(blocks), dim3(kSmallBlock), (size_t)entries * 8, sm, G, \
                       codes, scales, N, per_block, g, M, l->nbits, gpr, (int)l->out_features,  \
                       gmax, nmax, headroom, partial, meta)
        if (g == 8) PV_SMALL(2);
        else if (g == 16) PV_SMALL(4);
        else if (g == 4) PV_SMALL(1);
        else PV_SMALL(0);
#undef PV_SMALL
        hipLaunchKernelGGL(k_pg_small_final,
                           dim3((unsigned)((entries + kBlock / kSlices - 1) / (kBlock / kSlices))),
                           dim3(kBlock), 0, sm, partial, blocks, (int)entries, meta, grad_codebooks);
        PV_HIP(ctx, hipGetLastError());
        return PV_OK;
    }

    const size_t nn = (size_t)N;
    const int nblocks = (int)((N + kSortTile - 1) / kSortTile);           // tiles of a sorting pass
    const int hist_n = 256 * nblocks;
    size_t o_start = 0;
    size_t o_long = o_start + align_up((size_t)(csize + 1) * 4);
    size_t o_nlong = o_long + align_up((size_t)csize * 4);
    size_t o_total = o_nlong + 256;
    size_t o_hist = o_total + 1024;
    size_t o_base = o_hist + align_up((size_t)hist_n * 4);
    size_t o_keys_a = o_base + align_up((size_t)hist_n * 4);
    size_t o_keys_b = o_keys_a + align_up(nn * 2);
    size_t o_vals_a = o_keys_b + align_up(nn * 2);
    size_t o_order = o_vals_a + align_up(nn * 4);
    size_t o_part = o_order + align_up(nn * 4);
    size_t total = o_part + align_up((size_t)(N / kLong + 2) * g * 8);
    pv_status st = pv_ensure(ctx, ctx->pstep, total);
    if (st != PV_OK) return st;
    char *base = static_cast<char *>(ctx->pstep.ptr);
    int32_t *start = reinterpret_cast<int32_t *>(base + o_start);
    int32_t *long_list = reinterpret_cast<int32_t *>(base + o_long);
    unsigned *nlong = reinterpret_cast<unsigned *>(base + o_nlong);
    unsigned *dig_totals = reinterpret_cast<unsigned *>(base + o_total);
    unsigned *hist = reinterpret_cast<unsigned *>(base + o_hist);
    unsigned *hbase = reinterpret_cast<unsigned *>(base + o_base);
    uint16_t *keys_a = reinterpret_cast<uint16_t *>(base + o_keys_a);
    uint16_t *keys_b = reinterpret_cast<uint16_t *>(base + o_keys_b);
    int32_t *vals_a = reinterpret_cast<int32_t *>(base + o_vals_a);
    int32_t *order = reinterpret_cast<int32_t *>(base + o_order);
    double *partial = reinterpret_cast<double *>(base + o_part);

    pv_timed t(ctx, PV_K_PSTEP);
    int team = 8;
    while (team < g) team <<= 1;      // lanes per work item (g <= 64 checked by the caller)
    const int teams_per_block = kBlock / team;
    const unsigned sblocks = (unsigned)((csize + teams_per_block - 1) / teams_per_block);
    int64_t max_long = N / (kLong + 1);           // segments that can be longer than kLong
    if (max_long > csize) max_long = csize;
    if (max_long > 2048) max_long = 2048;         // blocks stride over the list
    const bool two = l->nbits > 8;
    for (int m = 0; m < M; ++m) {
        // pass over the low 8 bits of the codes (the only one when B <= 8) ...
        uint16_t *k1 = two ? keys_a : keys_b;
        int32_t *v1 = two ? vals_a : order;
        const code_keys ck{codes, M, m, mask};
        hipLaunchKernelGGL(k_digit_hist<code_keys>, dim3(nblocks), dim3(kSortBlock), 0, sm, ck, N, 0,
                           nblocks, hist);
        hipLaunchKernelGGL(k_row_scan, dim3(256), dim3(kRadixBlock), 0, sm, hist, nblocks, hbase, dig_totals);
        hipLaunchKernelGGL((k_digit_scatter<code_keys, uint16_t>), dim3(nblocks), dim3(kSortBlock), 0,
                           sm, ck, (const int32_t *)nullptr, N, 0, nblocks, hbase, dig_totals, k1, v1);
        if (two) {   // ... and over the high ones
            const plain_keys<uint16_t> pk{keys_a};
            hipLaunchKernelGGL(k_digit_hist<plain_keys<uint16_t>>, dim3(nblocks), dim3(kSortBlock), 0,
                               sm, pk, N, 8, nblocks, hist);
            hipLaunchKernelGGL(k_row_scan, dim3(256), dim3(kRadixBlock), 0, sm, hist, nblocks, hbase,
                               dig_totals);
            hipLaunchKernelGGL((k_digit_scatter<plain_keys<uint16_t>, uint16_t>), dim3(nblocks),
                               dim3(kSortBlock), 0, sm, pk, (const int32_t *)vals_a, N, 8, nblocks, hbase,
                               dig_totals, keys_b, order);
        }
        hipLaunchKernelGGL(k_pg_starts, dim3((unsigned)((N + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                           sm, keys_b, N, csize, start, nlong);
        float *out = grad_codebooks + (int64_t)m * csize * g;
#define PV_ACC(TEAM_)                                                                            \
    do {                                                                                         \
        hipLaunchKernelGGL(k_pg_short<TEAM_>, dim3(sblocks), dim3(kBlock), 0, sm, start, order, G, \
                           scales, gpr, g, csize, long_list, nlong, out);                         \
        if (max_long > 0)                                                                        \
            hipLaunchKernelGGL(k_pg_long<TEAM_>, dim3((unsigned)max_long), dim3(kBlock), 0, sm,   \
                               long_list, nlong, start, order, G, scales, gpr, g, partial, out);  \
    } while (0)
        switch (team) {
        case 8: PV_ACC(8); break;
        case 16: PV_ACC(16); break;
        case 32: PV_ACC(32); break;
        default: PV_ACC(64); break;
        }
#undef PV_ACC
    }
    if (grad_scales) {
        if (g % 4 == 0)
            hipLaunchKernelGGL(k_pg_scales<true>, dim3((unsigned)l->out_features), dim3(kBlock), 0, sm,
                               G, codes, codebooks, g, M, l->nbits, gpr, grad_scales, (unsigned *)nullptr);
        else
            hipLaunchKernelGGL(k_pg_scales<false>, dim3((unsigned)l->out_features), dim3(kBlock), 0, sm,
                               G, codes, codebooks, g, M, l->nbits, gpr, grad_scales, (unsigned *)nullptr);
    }
    PV_HIP(ctx, hipGetLastError());
    return PV_OK;
}

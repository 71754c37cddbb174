// Stable least-significant-digit radix sort of (key, value) pairs on the device, 8 bits a
// pass, written for the two places that need one: the 16-bit codes of the P step (Alg. 3)
// and the 32-bit update norms that rank the candidates of the trust-ratio rule (Sec. 4.3).
// A pass is three kernels - digit histogram per tile, prefix sums per digit row, scatter - and
// no atomic touches device memory: ranks come from wave ballots and per-wave counters in LDS,
// so keys with equal digits keep the order they came in.  Keys are read through a functor
// (KEYS: unsigned operator()(int64_t e) const), values are the element's index in the first
// pass (vals == nullptr) and carried afterwards.  Kernels live in an unnamed namespace: every
// file that includes this header instantiates its own.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int kRadixBlock = 256;          // threads of the row-scan kernel
constexpr int kSortBlock = 1024;          // threads of a sorting block: 16 waves
constexpr int kSortPer = 8;                   // rounds: keys per thread in a sorting pass
constexpr int kSortTile = kSortBlock * kSortPer;  // keys per block
constexpr int kSortWaves = kSortBlock / 64;

// the keys written by an earlier pass (or any plain array of keys)
template <class T>
struct plain_keys {
    const T *k;
    __device__ __forceinline__ unsigned operator()(int64_t e) const { return (unsigned)k[e]; }
};

// 32-bit keys in descending order: ascending order of the complement
struct descending_keys {
    const unsigned *k;
    __device__ __forceinline__ unsigned operator()(int64_t e) const { return ~k[e]; }
};

// Key j of this thread: wave w of the block owns the 64 * kSortPer consecutive keys that start at
// tile + w * 64 * kSortPer and takes them 64 at a time, so that (wave, round, lane) order is the
// order of the keys.
__device__ __forceinline__ int64_t sort_index(int j)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    return (int64_t)blockIdx.x * kSortTile + (int64_t)(wave * kSortPer + j) * 64 + lane;
}

// hist[d * nblocks + b] = keys of tile b whose digit is d
template <class KEYS>
__global__ __launch_bounds__(kSortBlock) void k_digit_hist(KEYS keys, int64_t N, int shift,
                                                           int nblocks, unsigned *__restrict__ hist)
{
    __shared__ unsigned h[256];
    if (threadIdx.x < 256) h[threadIdx.x] = 0u;
    unsigned k[kSortPer];
#pragma unroll
    for (int j = 0; j < kSortPer; ++j) {          // all loads in flight before the first is used
        const int64_t e = sort_index(j);
        k[j] = keys(e < N ? e : N - 1);
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kSortPer; ++j)
        if (sort_index(j) < N) atomicAdd(&h[(k[j] >> shift) & 255u], 1u);
    __syncthreads();
    if (threadIdx.x < 256) hist[(int64_t)threadIdx.x * nblocks + blockIdx.x] = h[threadIdx.x];
}

// Row d of the histogram (one block per digit): rowpre[d][b] = keys with digit d in the tiles
// before b, total[d] = keys with digit d.  The rows do not depend on one another; the offsets
// of the digits themselves (a prefix sum over 256 totals) are taken by every scatter block.
__global__ __launch_bounds__(kRadixBlock) void k_row_scan(const unsigned *__restrict__ hist, int nblocks,
                                                        unsigned *__restrict__ rowpre,
                                                        unsigned *__restrict__ total)
{
    __shared__ unsigned s_wave[kRadixBlock / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned *in = hist + (int64_t)blockIdx.x * nblocks;
    unsigned *out = rowpre + (int64_t)blockIdx.x * nblocks;
    unsigned carry = 0;
    for (int b0 = 0; b0 < nblocks; b0 += kRadixBlock) {
        const int b = b0 + threadIdx.x;
        const unsigned cnt = b < nblocks ? in[b] : 0u;
        unsigned incl = cnt;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const unsigned o = __shfl_up(incl, off);
            if (lane >= off) incl += o;
        }
        __syncthreads();                  // s_wave is reused from the previous round
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        unsigned before = 0, all = 0;
#pragma unroll
        for (int w = 0; w < kRadixBlock / 64; ++w) {
            before += w < wave ? s_wave[w] : 0u;
            all += s_wave[w];
        }
        if (b < nblocks) out[b] = carry + before + incl - cnt;
        carry += all;
    }
    if (threadIdx.x == 0) total[blockIdx.x] = carry;
}

// Stable scatter of tile b by this pass' digit.  In every round the 64 lanes of a wave find,
// with one ballot per digit bit, the lanes that hold the same digit; a key's rank is the
// wave's running count of that digit (wcnt[wave][d], kept in LDS by the last lane of each
// set) plus the number of such lanes below it.  The counts of the waves are then turned
// into offsets in wave order, so that keys with equal digits keep the order they came in.
// The tile is first put in digit order in LDS and written out from there: neighbouring
// threads then write neighbouring addresses (a run per digit) instead of one line each.
template <class KEYS, class KOUT>
__global__ __launch_bounds__(kSortBlock) void k_digit_scatter(
    KEYS keys, const int32_t *__restrict__ vals /* nullptr: the index itself */, int64_t N, int shift,
    int nblocks, const unsigned *__restrict__ rowpre, const unsigned *__restrict__ total,
    KOUT *__restrict__ keys_out, int32_t *__restrict__ vals_out)
{
    __shared__ unsigned wcnt[kSortWaves][256];
    __shared__ unsigned s_first[256];     // first slot of digit d inside the tile
    __shared__ unsigned s_dest[256];      // where that slot goes in the output
    __shared__ unsigned s_w4[8];
    __shared__ KOUT s_key[kSortTile];
    __shared__ int32_t s_val[kSortTile];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned k[kSortPer], rank[kSortPer];
    int32_t v[kSortPer];
#pragma unroll
    for (int j = 0; j < kSortPer; ++j) {
        const int64_t e = sort_index(j);
        const int64_t ec = e < N ? e : N - 1;
        k[j] = keys(ec);
        v[j] = vals ? vals[ec] : (int32_t)ec;
    }
    unsigned dig_total = 0, dig_pre = 0;
    if (threadIdx.x < 256) {
        dig_total = total[threadIdx.x];
        dig_pre = rowpre[(int64_t)threadIdx.x * nblocks + blockIdx.x];
    }
    for (int w = threadIdx.x; w < kSortWaves * 256; w += kSortBlock) (&wcnt[0][0])[w] = 0u;
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int j = 0; j < kSortPer; ++j) {
        const bool valid = sort_index(j) < N;
        const unsigned d = (k[j] >> shift) & 255u;
        unsigned long long same = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const unsigned long long has = __ballot((d >> bit) & 1u);
            same &= ((d >> bit) & 1u) ? has : ~has;
        }
        const unsigned before = wcnt[wave][d];
        rank[j] = before + (unsigned)__popcll(same & below);
        if (valid && lane == 63 - __clzll(same)) wcnt[wave][d] = before + (unsigned)__popcll(same);
    }
    __syncthreads();
    // threads 0..255 (four waves), one digit each: offsets of the waves inside the digit, then
    // two 256-entry prefix sums: of the tile's digit counts (slots in LDS) and of the global
    // digit totals (where each digit starts in the output)
    unsigned tile_cnt = 0;
    if (threadIdx.x < 256) {
        unsigned c[kSortWaves];
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) c[w] = wcnt[w][threadIdx.x];
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) {
            wcnt[w][threadIdx.x] = tile_cnt;
            tile_cnt += c[w];
        }
        unsigned a = tile_cnt, g2 = dig_total;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const unsigned oa = __shfl_up(a, off), og = __shfl_up(g2, off);
            if (lane >= off) {
                a += oa;
                g2 += og;
            }
        }
        if (lane == 63) {
            s_w4[wave] = a;
            s_w4[4 + wave] = g2;
        }
        tile_cnt = a - tile_cnt;          // exclusive inside the wave
        dig_total = g2 - dig_total;
    }
    __syncthreads();
    if (threadIdx.x < 256) {
        unsigned a = 0, g2 = 0;
        for (int w = 0; w < wave; ++w) {
            a += s_w4[w];
            g2 += s_w4[4 + w];
        }
        s_first[threadIdx.x] = tile_cnt + a;
        s_dest[threadIdx.x] = dig_total + g2 + dig_pre;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kSortPer; ++j) {
        if (sort_index(j) < N) {
            const unsigned d = (k[j] >> shift) & 255u;
            const unsigned slot = s_first[d] + wcnt[wave][d] + rank[j];
            s_key[slot] = (KOUT)k[j];
            s_val[slot] = v[j];
        }
    }
    __syncthreads();
    const int64_t left = N - (int64_t)blockIdx.x * kSortTile;
    const int in_tile = left < kSortTile ? (int)left : kSortTile;
#pragma unroll
    for (int j = 0; j < kSortPer; ++j) {
        const int slot = j * kSortBlock + threadIdx.x;
        if (slot < in_tile) {
            const unsigned key = s_key[slot];
            const unsigned d = (key >> shift) & 255u;
            const unsigned pos = s_dest[d] + ((unsigned)slot - s_first[d]);
            keys_out[pos] = (KOUT)key;
            vals_out[pos] = s_val[slot];
        }
    }
}

}  // namespace

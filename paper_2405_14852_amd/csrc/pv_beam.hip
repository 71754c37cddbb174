// Beam search over two 8-bit codebooks of 8-dimensional codewords (Sec. 4.2, App. K: beam 8;
// App. D: the expansion of the squared distance) as a FILTER in single and half precision,
// with the decision left to the reference arithmetic (double, the chain of the plain
// definition).  A group that cannot be certified goes to a list that the exact kernel
// (one wave per group, double throughout) works through afterwards.
//
// With x = t / s the objective of a pair is  s^2 || c0 + c1 - x ||^2.
//
// Step 0 (256 first codes against the current second code), 32 groups a wave, two lanes a
// group: with y0 = x - C1[p1] the matrix cores give the closeness of every first code to y0
// (as in step 1 below; the shift makes every closeness non-negative).  Each lane sees the 16
// codes of its half of each of the 8 tiles and keeps the largest closeness of each; the nine
// largest of a group's 16 such maxima belong to nine different codes, so the (beam + 1)-th
// largest of them bounds the (beam + 1)-th smallest distance from above, and a code can be among
// the beam + 1 nearest in the fp32 form below only if its closeness reaches a cut under that
// value (triangle inequality; the rounding of both operands, of the accumulation and of the form
// are in the cut).  A second round of the same matrix instructions marks those codes, a dozen a
// group, and only they go through
//     || c0 ||^2 - 2 <c0, y0> + || y0 ||^2   in fp32
// and the insertion into nine sorted values (the code in the low 8 bits); the two lanes merge
// their lists.  The kept set (the smallest beam_width) is accepted when the next value lies above
// the last kept one by more than twice the rounding bound of that form.
//
// Step 1 (256 second codes against each kept first code) is a dense contraction, done on
// the fp16 matrix cores exactly like the one-codebook filter: columns are (group, kept
// code) pairs, y1 = x - C0[c0], rows the second codebook, the spare K slots carry the
// squared norms and a shift, so an accumulator is a closeness
//     kv = SHIFT + 2 <c1_hi, y1_hi> - || c1_hi ||^2 = SHIFT + || y1_hi ||^2 - || c1_hi - y1_hi ||^2 .
// A lane keeps the largest and second largest key (tile number in the low bits) of its
// column and half.  The 16 lanes of a group then evaluate the 16 codewords behind the
// group's best key with the reference chain, which fixes the best objective E*; by the
// triangle inequality a pair can reach E* only if its key is at least
//     SHIFT + || y1_hi ||^2 - (P sqrt(E*) / |s| + dC + dy)^2 - E1 ,
// every best key at or above that cut is evaluated as well, and a second key at or above it
// sends the group to the list.  The winner among the evaluated pairs (objective, then pair)
// replaces the current pair if it is strictly better, as everywhere else.
#include "pv_internal.h"
#include "pv_dpp.h"

namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int G = 8;
constexpr int kKeep = 8;                            // largest beam the kernel takes
constexpr unsigned kKeyMask = 0x7FFu;
constexpr int kNoKey = (int)0x80000000;
constexpr float kHalfMinNormal = 6.103515625e-05f;  // 2^-14
constexpr float kGamma = 7.62939453125e-06f;        // 2^-17: fp32 accumulation bound per unit of sum|terms|
constexpr float kNormMargin = 0.04f;

__device__ __forceinline__ _Float16 to_half_flush(float v)
{
    return fabsf(v) < kHalfMinNormal ? (_Float16)0.0f : (_Float16)v;
}

__device__ __forceinline__ void split3(float v, _Float16 *p)
{
    p[0] = to_half_flush(v);
    float r = v - (float)p[0];
    p[1] = to_half_flush(r);
    r = r - (float)p[1];
    p[2] = to_half_flush(r);
}

__device__ __forceinline__ int imax3(int a, int b, int c) { return max(max(a, b), c); }

// v_sqrt_f32 as it is (1 ulp; the library's sqrtf adds a dozen instructions to round correctly and
// to scale denormal arguments).  Every use below multiplies the root by a margin far above one
// ulp, or feeds a bound with that much slack.
__device__ __forceinline__ float fast_sqrt(float v) { return __builtin_amdgcn_sqrtf(v); }

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

__device__ __forceinline__ unsigned umed3(unsigned a, unsigned b, unsigned c)
{
    unsigned r;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Sorting networks (19 exchanges for eight values, 25 for nine): descending integers, ascending
// unsigned keys.
__device__ __forceinline__ void sort8_desc(int (&a)[8])
{
    auto ce = [&](int i, int j) {
        const int hi = max(a[i], a[j]), lo = min(a[i], a[j]);
        a[i] = hi;
        a[j] = lo;
    };
    ce(0, 1); ce(2, 3); ce(4, 5); ce(6, 7);
    ce(0, 2); ce(1, 3); ce(4, 6); ce(5, 7);
    ce(1, 2); ce(5, 6); ce(0, 4); ce(3, 7);
    ce(1, 5); ce(2, 6);
    ce(1, 4); ce(3, 6);
    ce(2, 4); ce(3, 5);
    ce(3, 4);
}

__device__ __forceinline__ void sort9_asc(unsigned (&a)[9])
{
    auto ce = [&](int i, int j) {
        const unsigned lo = min(a[i], a[j]), hi = max(a[i], a[j]);
        a[i] = lo;
        a[j] = hi;
    };
    ce(0, 1); ce(3, 4); ce(6, 7);
    ce(1, 2); ce(4, 5); ce(7, 8);
    ce(0, 1); ce(3, 4); ce(6, 7);
    ce(0, 3); ce(3, 6); ce(0, 3);
    ce(1, 4); ce(4, 7); ce(1, 4);
    ce(2, 5); ce(5, 8); ce(2, 5);
    ce(1, 3); ce(5, 7);
    ce(2, 6); ce(4, 6); ce(2, 4);
    ce(2, 3); ce(5, 6);
}

__device__ __forceinline__ float key_upper(int key)
{
    return key < 0 ? 0.0f : __int_as_float(key | (int)kKeyMask);
}

__device__ __forceinline__ bool better(double o1, int i1, double o2, int i2)
{
    return o1 < o2 || (o1 == o2 && i1 < i2);
}

// Exchanges among the 16 lanes that work on one group in step 1 (8 consecutive lanes in each
// half of the wave): the stages of a team of 8, then the two halves of the wave.
__device__ __forceinline__ unsigned group16_min_u32(unsigned v)
{
    v = pv_team_min_u32<8>(v);
    const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);   // {lower half's, upper half's} in every lane
    return min(r[0], r[1]);
}

__device__ __forceinline__ unsigned long long group16_min_u64(unsigned long long v)
{
    v = pv_team_min_u64<8>(v);
    const unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
    const auto rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    const unsigned long long a = ((unsigned long long)rh[0] << 32) | rl[0];
    const unsigned long long b = ((unsigned long long)rh[1] << 32) | rl[1];
    return a < b ? a : b;
}

// an upper bound of a non-negative double as a float: rounding to nearest is off by at most
// 2^-24 of the value, the factor makes up for that (an infinity stays one; below the smallest
// normal float the caller's floor takes over)
__device__ __forceinline__ float float_above(double v) { return (float)v * 1.0000002f; }

// the reference chain for one pair
__device__ __forceinline__ double pair_objective(const float *c0, const float *c1, double s,
                                                 const float *t)
{
    double obj = 0.0;
#pragma unroll
    for (int i = 0; i < G; ++i) {
        double acc = (double)c0[i];
        acc = acc + (double)c1[i];
        const double r = s * acc - (double)t[i];
        obj = obj + r * r;
    }
    return obj;
}

struct tables_t {
    float c0[256 * G];      // first codebook
    float c1[256 * G];      // second codebook
    float n0[256];          // || c0 ||^2 (fp32 chain)
    h8 a0[8 * 64];          // first codebook as matrix operand: tile, k-half, row
    h8 a1[8 * 64];          // second codebook, the same
    float red[kWaves][8];
    float P, cmax0, cmaxu, cmax0h, cmax1, cmin1, dC0, dC1;
    int bad;
};

constexpr int kBatch = 32;  // groups a wave works on at a time: two lanes a group in step 0
struct wave_t {
    float x[kBatch][G];     // P t / s of the wave's groups (P: the power of two that scales the operands)
    float t[kBatch][G];
    float s[kBatch];
    float p_over_s[kBatch]; // P / |s|: objectives to distances of the scaled operands
    double o_prev[kBatch];
    float e_prev[kBatch];   // a float above o_prev
    int n[kBatch];
    unsigned char keep[kBatch][kKeep];   // kept first codes
    unsigned char prev[kBatch][2];
    unsigned char ok[kBatch];   // the group is still with the filter
};

__global__ __launch_bounds__(kBlock, 2) void k_beam_2x8_f16(
    const float *__restrict__ T, const float *__restrict__ codebooks,
    const float *__restrict__ scales, const int32_t *__restrict__ group_idx, int64_t k,
    int beam_width, uint16_t *__restrict__ codes, unsigned long long *__restrict__ num_changed,
    unsigned long long *__restrict__ stat_fast, int32_t *__restrict__ redo_list,
    unsigned long long *__restrict__ redo_count, int gpr, int N)
{
    __shared__ tables_t tb;
    __shared__ wave_t ws[kWaves];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    wave_t &w = ws[wave];

    // ---------------------------------------------------------------- tables (every block its own)
    {
        const int c = threadIdx.x;               // codeword c of both codebooks
        float m = 0.0f, nmax0 = 0.0f, nmax1 = 0.0f, nmin1 = __builtin_huge_valf();
        bool bad = false;
        float a[G], b[G];
        float n0 = 0.0f, n1 = 0.0f;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            a[i] = codebooks[c * G + i];
            b[i] = codebooks[(256 + c) * G + i];
            bad |= !(fabsf(a[i]) <= 3.0e38f) || !(fabsf(b[i]) <= 3.0e38f);
            tb.c0[c * G + i] = a[i];
            tb.c1[c * G + i] = b[i];
            m = fmaxf(m, fmaxf(fabsf(a[i]), fabsf(b[i])));
            n0 = fmaf(a[i], a[i], n0);
            n1 = fmaf(b[i], b[i], n1);
        }
        tb.n0[c] = n0;
        nmax0 = n0;
        nmax1 = n1;
        nmin1 = n1;
        for (int off = 32; off > 0; off >>= 1) {
            m = fmaxf(m, __shfl_xor(m, off));
            nmax0 = fmaxf(nmax0, __shfl_xor(nmax0, off));
            nmax1 = fmaxf(nmax1, __shfl_xor(nmax1, off));
            nmin1 = fminf(nmin1, __shfl_xor(nmin1, off));
        }
        const unsigned long long anybad = __ballot(bad);
        if (lane == 0) {
            tb.red[wave][0] = m;
            tb.red[wave][1] = nmax0;
            tb.red[wave][2] = nmax1;
            tb.red[wave][3] = nmin1;
            tb.red[wave][4] = anybad ? 1.0f : 0.0f;
        }
        __syncthreads();
        float M = 0.0f, X0 = 0.0f, X1 = 0.0f, N1 = __builtin_huge_valf(), B = 0.0f;
#pragma unroll
        for (int v = 0; v < kWaves; ++v) {
            M = fmaxf(M, tb.red[v][0]);
            X0 = fmaxf(X0, tb.red[v][1]);
            X1 = fmaxf(X1, tb.red[v][2]);
            N1 = fminf(N1, tb.red[v][3]);
            B = fmaxf(B, tb.red[v][4]);
        }
        const bool ok = (M > 0.0f) && (M < 3.0e38f) && (M >= 1.0e-30f) && B == 0.0f && X0 < 3.0e38f &&
                        X1 < 3.0e38f;
        float P = 1.0f;
        if (ok) {
            int ex;
            (void)frexpf(M, &ex);
            P = ldexpf(1.0f, 5 - ex);            // M * P in [16, 32)
        }
        // operand rows of codeword c of both codebooks: 2 c_hi | three pieces of ||c_hi||^2, 1, 1, 1
        float dmax[2], nhmax0 = 0.0f;
        auto rows_of = [&](const float *v8, h8 *table, float &d2out, float &nhout) {
            h8 ch0, ch1;
            float nh = 0.0f, d2 = 0.0f;
#pragma unroll
            for (int i = 0; i < G; ++i) {
                const float v = ok ? P * v8[i] : 0.0f;
                const float hf = (float)to_half_flush(v);
                nh = fmaf(hf, hf, nh);
                const float d = v - hf;
                d2 = fmaf(d, d, d2);
                ch0[i] = (_Float16)(2.0f * hf);
            }
            _Float16 pieces[3];
            split3(nh, pieces);
#pragma unroll
            for (int i = 0; i < 8; ++i) ch1[i] = (_Float16)0.0f;
            ch1[0] = pieces[0];
            ch1[1] = pieces[1];
            ch1[2] = pieces[2];
            ch1[3] = (_Float16)1.0f;
            ch1[4] = (_Float16)1.0f;
            ch1[5] = (_Float16)1.0f;
            const int tile = c >> 5, hw = (c >> 4) & 1, q = c & 15;
            const int row = 8 * (q >> 2) + 4 * hw + (q & 3);
            table[(tile * 2 + 0) * 32 + row] = ch0;
            table[(tile * 2 + 1) * 32 + row] = ch1;
            d2out = d2;
            nhout = nh;
        };
        float nh1;
        rows_of(a, tb.a0, dmax[0], nhmax0);
        rows_of(b, tb.a1, dmax[1], nh1);
        for (int off = 32; off > 0; off >>= 1) {
            dmax[0] = fmaxf(dmax[0], __shfl_xor(dmax[0], off));
            dmax[1] = fmaxf(dmax[1], __shfl_xor(dmax[1], off));
            nhmax0 = fmaxf(nhmax0, __shfl_xor(nhmax0, off));
        }
        __syncthreads();
        if (lane == 0) {
            tb.red[wave][5] = dmax[1];
            tb.red[wave][6] = dmax[0];
            tb.red[wave][7] = nhmax0;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            float D1 = 0.0f, D0 = 0.0f, H0 = 0.0f;
#pragma unroll
            for (int v = 0; v < kWaves; ++v) {
                D1 = fmaxf(D1, tb.red[v][5]);
                D0 = fmaxf(D0, tb.red[v][6]);
                H0 = fmaxf(H0, tb.red[v][7]);
            }
            tb.P = P;
            tb.cmax0 = sqrtf(X0) * 1.0001f;                        // unscaled
            tb.cmaxu = sqrtf(fmaxf(X0, X1)) * 1.0001f;             // unscaled, both codebooks
            tb.cmax0h = sqrtf(H0) * 1.0001f + kNormMargin;         // scaled, of the fp16 copy
            tb.cmax1 = P * sqrtf(X1) * 1.0001f + kNormMargin;      // scaled, of the fp16 copy
            tb.cmin1 = P * sqrtf(N1) * 1.0001f + kNormMargin;
            tb.dC0 = sqrtf(D0) * 1.0001f + 1.0e-30f;
            tb.dC1 = sqrtf(D1) * 1.0001f + 1.0e-30f;
            tb.bad = ok ? 0 : 1;
        }
        __syncthreads();
    }
    const float P = tb.P;
    const bool tables_ok = tb.bad == 0;
    const int keep = beam_width < kKeep ? beam_width : kKeep;
    unsigned vmask = ~kKeyMask;
    asm volatile("" : "+v"(vmask));
    unsigned low8 = ~0xFFu;
    asm volatile("" : "+v"(low8));                // in a register: the and-or takes no literal
    const int col = lane & 31, hw = lane >> 5;
    const f16v zacc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    unsigned changed = 0, fast = 0;
    const int64_t batches = (k + kBatch - 1) / kBatch;
    for (int64_t bi = (int64_t)blockIdx.x * kWaves + wave; bi < batches; bi += (int64_t)gridDim.x * kWaves) {
        // ------------------------------------------------------------ step 0: two lanes a group
        // Lanes col and col + 32 work on group col of the batch.  The matrix cores give the
        // closeness of all 256 first codes to y0 (column col, the lane's half of every tile of
        // 32 codes); the nine largest of the 16 (tile, half) maxima belong to nine different
        // codes, so the (keep + 1)-th largest of them, K, bounds the (keep + 1)-th smallest
        // distance from above, and by the triangle inequality a code can belong to the keep + 1
        // nearest in the fp32 form only if its closeness reaches a cut below K.  Only those codes
        // (a dozen) go through the fp32 form and the sorted insertion, each lane taking the ones
        // of its halves; the two lanes then merge their lists.
        {
            const int64_t j = bi * kBatch + col;
            int n = j < k ? group_idx[j] : -1;
            if (n >= N) n = -1;
            const bool valid = n >= 0;
            const int nn = valid ? n : 0;
            const float s = valid ? scales[nn / gpr] : 1.0f;
            float t[G];
            {
                const pv_f4 *t4 = reinterpret_cast<const pv_f4 *>(T + (int64_t)nn * G);
                const pv_f4 v0 = t4[0], v1 = t4[1];
                t[0] = v0.x; t[1] = v0.y; t[2] = v0.z; t[3] = v0.w;
                t[4] = v1.x; t[5] = v1.y; t[6] = v1.z; t[7] = v1.w;
            }
            const int p0 = codes[(int64_t)nn * 2] & 255, p1 = codes[(int64_t)nn * 2 + 1] & 255;
            bool ok = valid && tables_ok && (s != 0.0f) && (fabsf(s) < 3.0e38f);
            const float div = ok ? s : 1.0f;
            float x[G], y[G];
            float yy = 0.0f, xx = 0.0f;
#pragma unroll
            for (int i = 0; i < G; ++i) {
                x[i] = t[i] / div;
                y[i] = x[i] - tb.c1[p1 * G + i];
                yy = fmaf(y[i], y[i], yy);
                xx = fmaf(x[i], x[i], xx);
            }
            ok = ok && (xx < 1.0e30f) && (yy < 1.0e30f);   // also catches NaN
            const double o_prev = pair_objective(&tb.c0[p0 * G], &tb.c1[p1 * G], (double)s, t);
            // fp32 form of || c0 - y ||^2, never below zero by more than its rounding; a margin
            // keeps the bits ordered like integers
            const float span = tb.cmax0 + sqrtf(yy) + sqrtf(xx);
            const float e0 = 4.0e-6f * span * span;        // rounding bound of the form (4 * 2^-20)
            const float lift = yy * 1.00001f + e0;

            // operand column: P y0 as fp16, norms, shift (all closenesses non-negative:
            // SHIFT = (||y_hi|| + max ||c0_hi||)^2)
            float u[G], hf[G];
            float yyh = 0.0f, u2 = 0.0f;
#pragma unroll
            for (int i = 0; i < G; ++i) u[i] = P * y[i];
            const float umax = fmaxf(fmaxf(fmaxf(fabsf(u[0]), fabsf(u[1])), fmaxf(fabsf(u[2]), fabsf(u[3]))),
                                     fmaxf(fmaxf(fabsf(u[4]), fabsf(u[5])), fmaxf(fabsf(u[6]), fabsf(u[7]))));
            bool fits = ok && umax < 240.0f;
#pragma unroll
            for (int i = 0; i < G; ++i) {
                hf[i] = (float)to_half_flush(fits ? u[i] : 0.0f);
                yyh = fmaf(hf[i], hf[i], yyh);
                u2 = fmaf(u[i], u[i], u2);
            }
            const float d2 = fmaf(2.4e-7f, u2, 3.0e-8f);
            const float yn = fast_sqrt(yyh) * 1.0001f;
            const float want = (yn + tb.cmax0h) * (yn + tb.cmax0h) * 1.0001f + 1.0e-3f;
            fits = fits && yyh < 57000.0f && want < 60000.0f;
            _Float16 sp[3];
            split3(fits ? want : 0.0f, sp);
            const float shift = ((float)sp[0] + (float)sp[1]) + (float)sp[2];
            const float base = shift + yyh;
            const float e1 = 1.01f * (2.0f * kGamma * (tb.cmax0h + yn) * (tb.cmax0h + yn) * 1.01f + 5.0e-4f);
            // rounding of P y0 to fp16, plus the fp32 division, subtraction and scaling; and of the codebook
            const float delta = fast_sqrt(d2) * 1.0001f + 2.4e-7f * (fast_sqrt(u2) + 2.0f * P * tb.cmaxu) + 1.0e-30f +
                                tb.dC0;
            h8 bop;
            if (hw == 0) {
#pragma unroll
                for (int i = 0; i < G; ++i) bop[i] = (_Float16)(fits ? hf[i] : 0.0f);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) bop[i] = (_Float16)0.0f;
                if (fits) {
                    bop[0] = (_Float16)-1.0f;
                    bop[1] = (_Float16)-1.0f;
                    bop[2] = (_Float16)-1.0f;
                    bop[3] = sp[0];
                    bop[4] = sp[1];
                    bop[5] = sp[2];
                }
            }
            // round 1: the largest closeness of each (tile, half); the operand tiles of the first
            // codebook come from LDS as they are needed (held in registers they would cost a
            // wave of occupancy)
            auto aop = [&](int tl) { return tb.a0[tl * 64 + lane]; };
            int pm[8];
            {
                f16v acc[2];
                auto tile_max = [&](const f16v &a) {
                    int m = imax3(__float_as_int(a[0]), __float_as_int(a[1]), __float_as_int(a[2]));
                    m = imax3(m, __float_as_int(a[3]), __float_as_int(a[4]));
                    m = imax3(m, __float_as_int(a[5]), __float_as_int(a[6]));
                    m = imax3(m, __float_as_int(a[7]), __float_as_int(a[8]));
                    m = imax3(m, __float_as_int(a[9]), __float_as_int(a[10]));
                    m = imax3(m, __float_as_int(a[11]), __float_as_int(a[12]));
                    m = imax3(m, __float_as_int(a[13]), __float_as_int(a[14]));
                    return max(m, __float_as_int(a[15]));
                };
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop(0), bop, zacc, 0, 0, 0);
#pragma unroll
                for (int tl = 1; tl < 8; ++tl) {
                    acc[tl & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop(tl), bop, zacc, 0, 0, 0);
                    pm[tl - 1] = tile_max(acc[(tl - 1) & 1]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                pm[7] = tile_max(acc[1]);
            }
            // K: the (keep + 1)-th largest of the group's 16 maxima.  Both lanes sort their eight;
            // max(a[i], b[7 - i]) are then the eight largest of the sixteen and the largest of the
            // min(a[i], b[7 - i]) is the ninth.
            int K;
            {
                sort8_desc(pm);
                int other[8];
#pragma unroll
                for (int tl = 0; tl < 8; ++tl) {
                    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)pm[tl], (unsigned)pm[tl], false, false);
                    other[tl] = (int)(hw ? r[0] : r[1]);
                }
                if (keep == kKeep) {                     // uniform
                    K = min(pm[0], other[7]);
#pragma unroll
                    for (int i = 1; i < 8; ++i) K = max(K, min(pm[i], other[7 - i]));
                } else {
                    int big[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) big[i] = max(pm[i], other[7 - i]);
                    sort8_desc(big);
                    K = big[0];
#pragma unroll
                    for (int r = 1; r < kKeep; ++r)
                        if (r <= keep) K = big[r];
                }
            }
            // the cut: anchors (the codes behind the maxima down to K) lie within rho of y_hi; a
            // code of the keep + 1 nearest in the fp32 form lies within
            //     delta + sqrt((rho + delta)^2 + 2 e0 P^2)
            // of it (delta: what the fp16 operands are off by; e0: what the form is off by)
            fits = fits && K >= 0;
            const float rho2 = fmaxf((base - __int_as_float(K < 0 ? 0 : K)) * 1.000001f + e1 + 1.0e-6f * base, 0.0f);
            const float rho = fast_sqrt(rho2) * 1.000001f + delta;
            const float reach = delta + fast_sqrt(rho * rho * 1.000001f + 2.000001f * e0 * P * P) * 1.000001f;
            float reach2 = reach * reach * 1.000002f;
            if (!(reach2 == reach2)) reach2 = __builtin_huge_valf();
            const float kcut0 = (base * 0.999999f - reach2 * 1.000001f) - e1 - 1.0e-6f * (base + reach2);
            // round 2: the codes at or above the cut, one bit each (bit 16 (tile & 1) + a of word
            // tile / 2 for code 32 tile + 16 hw + a)
            unsigned cand[4] = {0u, 0u, 0u, 0u};
            asm volatile("" : "+v"(bop));   // a second round of its own: the 128 closenesses of round 1 are not kept
            {
                f16v acc[2];
                // closenesses and the cut are non-negative floats, so acc >= cut is the sign of
                // (cut - 1) - acc on their bits, shifted into the word from the right (a closeness
                // that rounding made negative may or may not get a bit: it lies far below the cut)
                const unsigned kc1 = __float_as_uint(kcut0) - 1u;
                auto mark = [&](const f16v &a, int tl) {
                    unsigned bits = 0u;
#pragma unroll
                    for (int e = 15; e >= 0; --e)
                        bits = __builtin_amdgcn_alignbit(bits, kc1 - __float_as_uint(a[e]), 31);
                    cand[tl >> 1] |= bits << (16 * (tl & 1));
                };
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop(0), bop, zacc, 0, 0, 0);
#pragma unroll
                for (int tl = 1; tl < 8; ++tl) {
                    acc[tl & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop(tl), bop, zacc, 0, 0, 0);
                    mark(acc[(tl - 1) & 1], tl - 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
                mark(acc[1], 7);
            }
            if (!(kcut0 > 0.0f)) cand[0] = cand[1] = cand[2] = cand[3] = ~0u;   // no bound: every code
            if (!fits) cand[0] = cand[1] = cand[2] = cand[3] = 0u;
            // the fp32 form and the sorted insertion for the lane's candidates
            unsigned top[kKeep + 1];
#pragma unroll
            for (int r = 0; r <= kKeep; ++r) top[r] = 0x7F800000u;          // +inf
            float ym2[G];                                 // -2 y: the products come out of the chain as they are needed
#pragma unroll
            for (int i = 0; i < G; ++i) ym2[i] = -2.0f * y[i];
            auto insert = [&](unsigned carry) {
#pragma unroll
                for (int r = 0; r + 1 <= kKeep; r += 2) {
                    const unsigned lo = min(top[r], carry);
                    const unsigned mid = umed3(top[r], top[r + 1], carry);
                    carry = max(top[r + 1], carry);
                    top[r] = lo;
                    top[r + 1] = mid;
                }
                top[kKeep] = min(top[kKeep], carry);
            };
            for (;;) {
                int wsel = -1;
                unsigned word = 0u;
#pragma unroll
                for (int q = 3; q >= 0; --q)
                    if (cand[q]) {
                        wsel = q;
                        word = cand[q];
                    }
                if (!__any(wsel >= 0)) break;
                const bool have = wsel >= 0;
                const int bit = have ? __ffs((int)word) - 1 : 0;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (q == wsel) cand[q] &= cand[q] - 1u;
                const int tile = 2 * (have ? wsel : 0) + (bit >> 4);
                const int c0 = tile * 32 + hw * 16 + (bit & 15);
                const pv_f4 r0 = *reinterpret_cast<const pv_f4 *>(&tb.c0[c0 * G]);
                const pv_f4 r1 = *reinterpret_cast<const pv_f4 *>(&tb.c0[c0 * G + 4]);
                // || c0 ||^2 + lift - 2 <c0, y>: every partial sum stays below span^2, nine roundings
                float d = tb.n0[c0] + lift;
                d = fmaf(r0.x, ym2[0], d);
                d = fmaf(r0.y, ym2[1], d);
                d = fmaf(r0.z, ym2[2], d);
                d = fmaf(r0.w, ym2[3], d);
                d = fmaf(r1.x, ym2[4], d);
                d = fmaf(r1.y, ym2[5], d);
                d = fmaf(r1.z, ym2[6], d);
                d = fmaf(r1.w, ym2[7], d);
                insert(have ? ((__float_as_uint(d) & low8) | (unsigned)c0) : 0x7F800000u);
            }
            // the other lane's list: min(a[i], b[8 - i]) are the nine smallest of the eighteen
            {
                static_assert(kKeep == 8, "the merge sorts nine values");
                unsigned theirs[kKeep + 1];
#pragma unroll
                for (int r = 0; r <= kKeep; ++r) {
                    const auto sw = __builtin_amdgcn_permlane32_swap(top[r], top[r], false, false);
                    theirs[r] = hw ? sw[0] : sw[1];
                }
#pragma unroll
                for (int r = 0; r <= kKeep; ++r) top[r] = min(top[r], theirs[kKeep - r]);
                sort9_asc(top);
            }
            ok = ok && fits;
            // the kept set is certain when the first dropped value clears the last kept one by
            // twice the rounding bound plus the 8 bits given to the code (a code that was not a
            // candidate lies above keep + 1 candidates, hence above the first dropped value)
            {
                unsigned last = top[0], next = top[1];
#pragma unroll
                for (int r = 1; r < kKeep; ++r)
                    if (r < keep) {
                        last = top[r];
                        next = top[r + 1];
                    }
                const float vl = __uint_as_float(last | 0xFFu), vn = __uint_as_float(next & ~0xFFu);
                ok = ok && (vn - vl > 2.0f * e0 + 1.0e-6f * vn);   // false for NaN
                ok = ok && next != 0x7F800000u;                    // keep + 1 candidates were there
            }
            if (hw == 0) {
                w.n[col] = valid ? n : -1;
                w.s[col] = s;
                w.p_over_s[col] = P / fabsf(div);
                w.o_prev[col] = o_prev;
                w.e_prev[col] = float_above(o_prev);
                w.ok[col] = ok ? 1 : 0;
                w.prev[col][0] = (unsigned char)p0;
                w.prev[col][1] = (unsigned char)p1;
#pragma unroll
                for (int i = 0; i < G; ++i) {
                    w.x[col][i] = P * x[i];
                    w.t[col][i] = t[i];
                }
#pragma unroll
                for (int r = 0; r < kKeep; ++r) w.keep[col][r] = (unsigned char)(top[r] & 0xFFu);
            }
        }
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_s_waitcnt(0);

        // ------------------------------------------------------------ step 1: 8 column tiles of 4 groups
        const int gq = col >> 3, e = col & 7;            // group of the tile, kept code
        h8 a1[8];
#pragma unroll
        for (int tl = 0; tl < 8; ++tl) a1[tl] = tb.a1[tl * 64 + lane];
#pragma unroll 1
        for (int ct = 0; ct < kBatch / 4; ++ct) {
            const int gl = ct * 4 + gq;                  // the group's lane of step 0
            const bool gok = w.ok[gl] != 0;
            const bool head = e == 0 && hw == 0 && w.n[gl] >= 0;   // the lane that speaks for the group
            if (!__any(gok)) {                           // nothing of this tile is with the filter
                if (head) redo_list[atomicAdd(redo_count, 1ull)] = w.n[gl];
                continue;
            }
            const bool live = gok && e < keep;
            const int c0e = w.keep[gl][e];
            const float s = w.s[gl];
            // operand column: y1 = P (x - C0[c0e]) as fp16, norms, shift
            float u[G], hf[G];
            float yy = 0.0f, u2 = 0.0f;
#pragma unroll
            // (one rounding, of P (x - c0): scaling by a power of two commutes with it)
            for (int i = 0; i < G; ++i) u[i] = fmaf(-P, tb.c0[c0e * G + i], w.x[gl][i]);
            // a column with an element of 240 or more does not fit and is dropped whole, so what the
            // lines below make of its elements is never used (x and the codebook are finite for a
            // live column, so u is a number or an infinity, never a NaN)
            const float umax = fmaxf(fmaxf(fmaxf(fabsf(u[0]), fabsf(u[1])), fmaxf(fabsf(u[2]), fabsf(u[3]))),
                                     fmaxf(fmaxf(fabsf(u[4]), fabsf(u[5])), fmaxf(fabsf(u[6]), fabsf(u[7]))));
            bool fits = live && umax < 240.0f;
#pragma unroll
            for (int i = 0; i < G; ++i) {
                // (no flush of a denormal half here: whether the matrix core keeps it or flushes
                // it, the operand stays within the bound below of u, and || hf ||^2 moves by less
                // than 3e-8)
                hf[i] = (float)(_Float16)u[i];
                yy = fmaf(hf[i], hf[i], yy);
                u2 = fmaf(u[i], u[i], u2);
            }
            // || u - hf ||^2: an element moves by at most 2^-11 of itself when it is rounded to
            // half precision and by less than 2^-14 when it is flushed to zero
            const float d2 = fmaf(2.4e-7f, u2, 3.0e-8f);
            const float yn = fast_sqrt(yy) * 1.0001f;
            const float want = (yn + tb.cmin1) * (yn + tb.cmin1) * 1.0001f + 1.0e-3f;
            fits = fits && yy < 57000.0f && want < 60000.0f;
            _Float16 sp[3];
            split3(fits ? want : 0.0f, sp);
            const float shift = ((float)sp[0] + (float)sp[1]) + (float)sp[2];
            const float base = shift + yy;
            const float e1 = 1.01f * (2.0f * kGamma * (tb.cmax1 + yn) * (tb.cmax1 + yn) * 1.01f + 5.01e-4f);
            // rounding of y1 to fp16, plus the fp32 division, subtraction and scaling
            const float dy = fast_sqrt(d2) * 1.0001f + 2.4e-7f * (fast_sqrt(u2) + 2.0f * P * tb.cmax0) + 1.0e-30f;
            h8 bop;
            if (hw == 0) {
#pragma unroll
                for (int i = 0; i < G; ++i) bop[i] = (_Float16)(fits ? hf[i] : 0.0f);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) bop[i] = (_Float16)0.0f;
                if (fits) {
                    bop[0] = (_Float16)-1.0f;
                    bop[1] = (_Float16)-1.0f;
                    bop[2] = (_Float16)-1.0f;
                    bop[3] = sp[0];
                    bop[4] = sp[1];
                    bop[5] = sp[2];
                }
            }
            // a column that does not fit takes its whole group out of the filter
            const bool colbad = live && !fits;
            // 8 row tiles; the unit before is reduced while the matrix core works
            int best = kNoKey, second = kNoKey;
            f16v acc[2];
            const f16v z = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            auto reduce = [&](const f16v &a, int tile) {
                int m = imax3(__float_as_int(a[0]), __float_as_int(a[1]), __float_as_int(a[2]));
                m = imax3(m, __float_as_int(a[3]), __float_as_int(a[4]));
                m = imax3(m, __float_as_int(a[5]), __float_as_int(a[6]));
                m = imax3(m, __float_as_int(a[7]), __float_as_int(a[8]));
                m = imax3(m, __float_as_int(a[9]), __float_as_int(a[10]));
                m = imax3(m, __float_as_int(a[11]), __float_as_int(a[12]));
                m = imax3(m, __float_as_int(a[13]), __float_as_int(a[14]));
                m = max(m, __float_as_int(a[15]));
                const int key = and_or(m, vmask, (unsigned)tile);
                second = imed3(best, second, key);
                best = max(best, key);
            };
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1[0], bop, z, 0, 0, 0);
#pragma unroll
            for (int tl = 1; tl < 8; ++tl) {
                acc[tl & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1[tl], bop, z, 0, 0, 0);
                reduce(acc[(tl - 1) & 1], tl - 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            reduce(acc[1], 7);
            if (!live || !fits) best = second = kNoKey;

            // ---- the group's 16 lanes: (col & ~7) + 0..7 in both halves
            // the lane whose best key stands for the smallest distance (keys of different columns
            // are closenesses relative to different bases: the distances are what compares)
            const float dist = best == kNoKey ? __builtin_huge_valf() : fmaxf(base - key_upper(best), 0.0f);
            // (which column is looked at first decides nothing but how much is left to evaluate
            // afterwards, so the low six bits of the distance make room for the lane)
            const unsigned bk = group16_min_u32((__float_as_uint(dist) & ~63u) | (unsigned)lane);
            const int glane = (int)(bk & 63u);
            const int gkey = __shfl(best, glane);
            unsigned gbad = colbad ? 1u : 0u;
            if (__any(colbad)) {                         // rare: the exchange is skipped by the whole wave
#pragma unroll
                for (int m = 1; m < 8; m <<= 1) gbad |= __shfl_xor(gbad, m);
                gbad |= __shfl_xor(gbad, 32);
            }
            bool open = gbad != 0u || gkey == kNoKey;   // filter left (or nothing to look at)
            // reference objective of the 16 pairs behind a key: lane (e, hw) takes codeword
            // e + 8 hw of the key's half tile
            const double sd = (double)s;
            float tt[G];
#pragma unroll
            for (int i = 0; i < G; ++i) tt[i] = w.t[gl][i];
            double wobj = __builtin_huge_val();
            int widx = 0x7fffffff;
            auto eval_key = [&](int key, int klane) {
                const int tile = key & (int)kKeyMask;
                const int khw = klane >> 5, ke = klane & 7;
                const int c0 = w.keep[gl][ke];
                const int c1 = tile * 32 + khw * 16 + e + 8 * hw;
                const double o = pair_objective(&tb.c0[c0 * G], &tb.c1[c1 * G], sd, tt);
                const int tie = c0 * 256 + c1;
                if (better(o, tie, wobj, widx)) {
                    wobj = o;
                    widx = tie;
                }
            };
            // smallest objective of the group's 16 lanes, then the smallest pair index among the
            // lanes that hold it (objectives are never negative and never NaN: their bits order
            // like integers)
            auto group_min = [&](double &o, int &i) {
                const unsigned long long mine_bits = (unsigned long long)__double_as_longlong(o);
                const unsigned long long m = group16_min_u64(mine_bits);
                i = (int)group16_min_u32(mine_bits == m ? (unsigned)i : 0x7fffffffu);
                o = __longlong_as_double((long long)m);
            };
            if (!open) eval_key(gkey, glane);
            const double o_prev = w.o_prev[gl];
            // E*: the smallest objective known for the group (a float above it; the exact minimum and
            // its pair are taken once, after everything has been evaluated)
            // (objectives are never negative, so their float bits order like integers; a NaN
            // sorts above everything and is dropped by the fminf)
            float e_star = __uint_as_float(group16_min_u32(__float_as_uint(float_above(wobj))));
            e_star = fminf(e_star, w.e_prev[gl]);
            // every pair that was not evaluated and could still reach E* sits behind a key whose
            // upper bound is at least kcut (fp32, every rounding covered)
            const float rr = fast_sqrt(e_star < 1.2e-38f ? 1.2e-38f : e_star) * w.p_over_s[gl] * 1.000002f + tb.dC1 + dy;
            float reach2 = rr * rr * 1.000002f;
            if (!(reach2 == reach2)) reach2 = __builtin_huge_valf();
            const float kcut = (base * 0.999999f - reach2 * 1.000001f) - e1 - 1.0e-6f * (base + reach2);
            const bool no_bound = !(kcut > -3.0e38f);
            bool pending = !open && live && fits && lane != glane && best != kNoKey &&
                           (no_bound || key_upper(best) >= kcut);
            bool lopen = !open && live && fits && second != kNoKey && (no_bound || key_upper(second) >= kcut);
            // keys of the other lanes at or above their cut: evaluated by the group as well
            const unsigned long long gmask = (0xFFull << (lane & 24)) | (0xFFull << (32 + (lane & 24)));
            if (__any(pending)) {
                for (;;) {
                    const unsigned long long pb = __ballot(pending) & gmask;
                    if (!__any(pb != 0ull)) break;
                    if (pb) {
                        const int src = __ffsll((long long)pb) - 1;
                        const int key = __shfl(best, src);
                        eval_key(key, src);
                        if (lane == src) pending = false;
                    }
                }
            }
            double gobj = wobj;
            int gidx = widx;
            group_min(gobj, gidx);
            if (__any(lopen)) {
                unsigned go = lopen ? 1u : 0u;
#pragma unroll
                for (int m = 1; m < 8; m <<= 1) go |= __shfl_xor(go, m);
                go |= __shfl_xor(go, 32);
                open = open || go != 0u;
            }
            if (head) {
                const int n = w.n[gl];
                if (!gok || open) {
                    const unsigned long long slot = atomicAdd(redo_count, 1ull);
                    redo_list[slot] = n;
                } else {
                    if (gidx != 0x7fffffff && gobj < o_prev) {
                        codes[(int64_t)n * 2] = (uint16_t)(gidx >> 8);
                        codes[(int64_t)n * 2 + 1] = (uint16_t)(gidx & 255);
                        ++changed;
                    }
                    ++fast;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    for (int off = 32; off > 0; off >>= 1) {
        changed += __shfl_xor(changed, off);
        fast += __shfl_xor(fast, off);
    }
    // one atomic per block and counter: atomics on one device address are served one after the
    // other, and all the waves finish at about the same time
    __shared__ unsigned s_changed, s_fast;
    if (threadIdx.x == 0) s_changed = s_fast = 0u;
    __syncthreads();
    if (lane == 0) {
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

pv_status pv_launch_beam_2x8_f16(pv_ctx *ctx, const float *T, const float *codebooks,
                                 const float *scales, const int32_t *group_idx, int64_t k,
                                 int32_t beam_width, uint16_t *codes, int64_t *num_changed,
                                 unsigned long long *stat_fast, int32_t *redo_list,
                                 unsigned long long *redo_count, int gpr, int N)
{
    int64_t blocks = (k + kBatch * kWaves - 1) / (kBatch * kWaves);
    if (blocks > 768) blocks = 768;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_beam_2x8_f16, dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream, T,
                       codebooks, scales, group_idx, k, beam_width, codes,
                       reinterpret_cast<unsigned long long *>(num_changed), stat_fast, redo_list,
                       redo_count, gpr, N);
    return PV_OK;
}

// Reductions over a team of 8 or 16 consecutive lanes (or 8 lanes in both halves of a wave)
// through the data-parallel-primitive paths of the vector unit instead of LDS: a __shfl_xor is
// an LDS permute with its latency on the critical path of the short, dependent chains these
// kernels consist of.  Stages, in this order: lane ^ 1 and lane ^ 2 inside quads, then the
// mirror image inside 8 lanes (quads are uniform by then, so the mirror brings the other
// quad's value), then the mirror image inside 16 lanes.  Valid for operations whose result does
// not depend on the order of the operands (min, max, or, sum, and a lexicographic minimum with
// a total order); every lane of the team ends with the team's result.  All lanes of a team must
// be active together.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>

constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppMirror8 = 0x141, kDppMirror16 = 0x140;

template <int CTRL>
__device__ __forceinline__ int pv_dpp(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}

template <int CTRL>
__device__ __forceinline__ unsigned long long pv_dpp_u64(unsigned long long v)
{
    const unsigned lo = (unsigned)pv_dpp<CTRL>((int)(unsigned)v);
    const unsigned hi = (unsigned)pv_dpp<CTRL>((int)(unsigned)(v >> 32));
    return ((unsigned long long)hi << 32) | lo;
}

template <int CTRL>
__device__ __forceinline__ double pv_dpp_f64(double v)
{
    return __hiloint2double(pv_dpp<CTRL>(__double2hiint(v)), pv_dpp<CTRL>(__double2loint(v)));
}

// f(integral_constant<int, control word>) once per stage of a TEAM of 8 or 16 lanes
template <int TEAM, class F>
__device__ __forceinline__ void pv_team_stages(F &&f)
{
    static_assert(TEAM == 8 || TEAM == 16, "teams of 8 or 16 lanes");
    f(std::integral_constant<int, kDppXor1>{});
    f(std::integral_constant<int, kDppXor2>{});
    f(std::integral_constant<int, kDppMirror8>{});
    if constexpr (TEAM == 16) f(std::integral_constant<int, kDppMirror16>{});
}

template <int TEAM>
__device__ __forceinline__ unsigned pv_team_min_u32(unsigned v)
{
    pv_team_stages<TEAM>([&](auto c) { v = min(v, (unsigned)pv_dpp<decltype(c)::value>((int)v)); });
    return v;
}

template <int TEAM>
__device__ __forceinline__ unsigned long long pv_team_min_u64(unsigned long long v)
{
    pv_team_stages<TEAM>([&](auto c) {
        const unsigned long long o = pv_dpp_u64<decltype(c)::value>(v);
        v = o < v ? o : v;
    });
    return v;
}

template <int TEAM>
__device__ __forceinline__ long long pv_team_max_i64(long long v)
{
    pv_team_stages<TEAM>([&](auto c) {
        const long long o = (long long)pv_dpp_u64<decltype(c)::value>((unsigned long long)v);
        v = o > v ? o : v;
    });
    return v;
}

template <int TEAM>
__device__ __forceinline__ unsigned long long pv_team_or_u64(unsigned long long v)
{
    pv_team_stages<TEAM>([&](auto c) { v |= pv_dpp_u64<decltype(c)::value>(v); });
    return v;
}

template <int TEAM>
__device__ __forceinline__ unsigned pv_team_sum_u32(unsigned v)
{
    pv_team_stages<TEAM>([&](auto c) { v += (unsigned)pv_dpp<decltype(c)::value>((int)v); });
    return v;
}

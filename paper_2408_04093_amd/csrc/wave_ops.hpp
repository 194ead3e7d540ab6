// Wavefront (64-lane) data-movement helpers for gfx950.  Device code only.
//
// A DPP "row" is 16 consecutive lanes.  Reductions inside a row use the DPP
// modifier of the VALU add/max itself (no extra move, no LDS); anything that
// crosses rows goes through ds_bpermute (__shfl_xor).
#pragma once
#include <hip/hip_runtime.h>

namespace ta {

constexpr int kWave = 64;

// DPP controls (gfx9 encoding)
constexpr int kDppXor1 = 0xB1;        // quad_perm:[1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm:[2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each 8 lanes
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each 16 lanes

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x) {
    long long b = __double_as_longlong(x);
    int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffLL), CTRL, 0xf, 0xf, true);
    int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xf, 0xf, true);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

template <int CTRL> __device__ __forceinline__ float dpp(float x) { return dpp_f32<CTRL>(x); }
template <int CTRL> __device__ __forceinline__ double dpp(double x) { return dpp_f64<CTRL>(x); }

// Sum over groups of LANES consecutive lanes (LANES in {8,16,32}); every lane
// of the group ends with the total.  After the two quad steps all four lanes
// of a quad agree, so the mirror steps pair up whole quads.
template <int LANES, typename F>
__device__ __forceinline__ F group_sum(F x) {
    x += dpp<kDppXor1>(x);
    x += dpp<kDppXor2>(x);
    x += dpp<kDppHalfMirror>(x);
    if constexpr (LANES >= 16) x += dpp<kDppMirror>(x);
    if constexpr (LANES >= 32) x += __shfl_xor(x, 16);
    return x;
}

// N sums at once over groups of LANES consecutive lanes (LANES in {8,16}, N in {1,2,4}), as a
// reduce-scatter: every lane ends with ONE of the N totals instead of all of them, at log2(LANES) + N - 1
// additions instead of N log2(LANES).  A lane's inputs are numbered by "slot": slot j of a lane is
// total (j ^ own), where own = scatter_own(lane in group) is the total the lane ends with (its slot 0).
// The exchange steps pair lanes whose `own` differ (by 3, then by 1, for N = 4), so each lane adds what
// its partner holds for the lane's own totals: no selects.  The remaining steps are plain sums among the
// LANES / N lanes that own the same total, all of which end with it.
template <int LANES, int N>
__device__ __forceinline__ int scatter_own(int lane_in_group) { return lane_in_group / (LANES / N); }

template <int LANES, int N, typename F>
__device__ __forceinline__ F scatter_sum(const F (&x)[N]) {
    static_assert((LANES == 8 || LANES == 16) && (N == 1 || N == 2 || N == 4), "unsupported shape");
    constexpr int kA = LANES == 16 ? kDppMirror : kDppHalfMirror;   // flips every bit of the lane index in the group
    if constexpr (N == 1) {
        return group_sum<LANES>(x[0]);
    } else if constexpr (N == 2) {       // own = top bit
        F y = x[0] + dpp<kA>(x[1]);
        y += dpp<kDppXor1>(y);
        y += dpp<kDppXor2>(y);
        if constexpr (LANES == 16) y += dpp<kDppHalfMirror>(y);
        return y;
    } else {                             // own = top two bits
        constexpr int kB = LANES == 16 ? kDppHalfMirror : kDppXor2;   // flips the second bit, keeps the top one
        const F y0 = x[0] + dpp<kA>(x[3]), y1 = x[1] + dpp<kA>(x[2]);
        F z = y0 + dpp<kB>(y1);
        z += dpp<kDppXor1>(z);
        if constexpr (LANES == 16) z += dpp<kDppXor2>(z);
        return z;
    }
}

// The inverse: every lane contributes the value of its own total and receives all N, in slot order.
template <int LANES, int N>
__device__ __forceinline__ void scatter_gather(float own, float (&p)[N]) {
    constexpr int kA = LANES == 16 ? kDppMirror : kDppHalfMirror;
    p[0] = own;
    if constexpr (N == 2) p[1] = dpp<kA>(own);
    if constexpr (N == 4) {
        constexpr int kB = LANES == 16 ? kDppHalfMirror : kDppXor2;
        p[1] = dpp<kB>(own);
        p[3] = dpp<kA>(own);
        p[2] = dpp<kA>(p[1]);
    }
}

// Reductions across the groups of a wave (lane distance >= LANES).
template <int LANES, typename F>
__device__ __forceinline__ F across_groups_max(F x) {
#pragma unroll
    for (int off = LANES; off < kWave; off <<= 1) x = fmax(x, __shfl_xor(x, off));
    return x;
}
template <int LANES, typename F>
__device__ __forceinline__ F across_groups_sum(F x) {
#pragma unroll
    for (int off = LANES; off < kWave; off <<= 1) x += __shfl_xor(x, off);
    return x;
}

// Whole-wave reductions (used by the combine kernel).
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
    return x;
}

// Maximum / sum over the four lanes l, l ^ 16, l ^ 32, l ^ 48 (the same column position in the
// four 16-lane rows of the wave), left in all four.  gfx950 swaps half-waves and 16-lane rows
// between two registers in the vector ALU (v_permlane32_swap: upper half of the first with lower
// half of the second; v_permlane16_swap: odd rows of the first with even rows of the second), so
// with both operands holding x, one swap and one max / add fold each pair: no LDS round trip as
// with ds_bpermute.
__device__ __forceinline__ float rows_max(float x) {
    const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float m = fmaxf(__uint_as_float(h[0]), __uint_as_float(h[1]));
    const auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(m), __float_as_uint(m), false, false);
    return fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
}
__device__ __forceinline__ float rows_sum(float x) {
    const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float m = __uint_as_float(h[0]) + __uint_as_float(h[1]);
    const auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(m), __float_as_uint(m), false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// 2^x on the hardware transcendental unit (v_exp_f32, about 1 ulp).
__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

// fp32 -> bf16 bits, round to nearest even.  Input must be finite or +-inf.
__device__ __forceinline__ unsigned short f32_to_bf16_rne(float x) {
    unsigned int u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

}  // namespace ta

// fp64 min-plus helpers shared by the kernels that relax whole rows of cost vectors against a 64 x 64 table staged
// in LDS (the interval table and its block route).  Costs are integers in [0, 2^52] and every sum stays below 2^53,
// so fp64 arithmetic is exact; inside these kernels "infeasible" is 2^52 - 1.
#pragma once
#include "kernels.h"

#include <type_traits>

namespace rh {
namespace {

constexpr double kInfD = 4503599627370495.0; // 2^52 - 1 stands for "infeasible" inside the kernel

__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Exact for 0 <= x < 2^52 - 1 (two full-rate instructions: the integer becomes the mantissa of 2^52 + x);
// anything from 2^52 - 1 up, which includes RH_INF, becomes the kernel's infeasible value.
__device__ __forceinline__ double to_f64(int64_t x) {
    uint32_t lo = (uint32_t)x, hi = (uint32_t)((uint64_t)x >> 32);
    const bool big = hi >= 0x100000u;
    lo = big ? 0xFFFFFFFFu : lo;
    hi = big ? 0xFFFFFu : hi;
    return __hiloint2double((int)(hi | 0x43300000u), (int)lo) - 4503599627370496.0;
}

// back to the interface's integers: infeasible is 2^52
__device__ __forceinline__ int64_t to_i64(double m) { return m >= kInfD ? kInf : (int64_t)m; }

__device__ __forceinline__ double bcast(double x, int lane) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), lane);
    return __hiloint2double(hi, lo);
}

// x of lane N of this lane's row of 16 lanes (one v_mov_b64_dpp)
template <int N>
__device__ __forceinline__ double row_bcast(double x) {
    const long long v = __double_as_longlong(x);
    return __longlong_as_double(__builtin_amdgcn_update_dpp(v, v, 0x150 + N, 0xF, 0xF, false));
}

// x of another lane of the wave
__device__ __forceinline__ double from_lane(double x, int lane) {
    const int lo = __builtin_amdgcn_ds_bpermute(lane << 2, __double2loint(x));
    const int hi = __builtin_amdgcn_ds_bpermute(lane << 2, __double2hiint(x));
    return __hiloint2double(hi, lo);
}

// Kp = 64, the whole table of an edge in one piece: acc[q][0] = min(acc[q][0], min_a V[q][a] + piece[a][lane]) for
// the first NA of the wave's two rows.  Lane 16 r + j: in step n its row of 16 lanes works on a = 4 n + r, and the
// lane relaxes columns j + 16 (k ^ r), k = 0..3 (the exclusive-or spreads the four rows of lanes over the LDS
// banks); its partial minimum for column j + 16 (k ^ r) is acc4[k].
template <int NA, int SLOTS>
__device__ __forceinline__ void relax_rows64(const double* __restrict__ piece, int lane, const double (&V)[SLOTS][1],
                                             double (&acc)[SLOTS][1]) {
    const int r = lane >> 4, j = lane & 15;
    double src[NA], acc4[NA][4];
#pragma unroll
    for (int q = 0; q < NA; ++q) {
        src[q] = from_lane(V[q][0], 4 * j + r);    // lane 16 r + n holds V[q][4 n + r]
#pragma unroll
        for (int k = 0; k < 4; ++k) acc4[q][k] = kInfD;
    }
    __builtin_amdgcn_sched_barrier(0);
    const double* base = piece + r * 64 + j;
    // The values of three steps are on their way from LDS while one step is worked on (a wave may have a SIMD to
    // itself here, so nothing else covers the trip): the registers of a step are refilled for three steps later
    // as soon as they have been used, and the scheduler is told to keep that order.
    double x[3][4];
    auto load = [&](double (&xs)[4], int n) {
#pragma unroll
        for (int k = 0; k < 4; ++k) xs[k] = base[(4 * n) * 64 + 16 * (k ^ r)];
    };
    auto step = [&](auto n_tag) {
        constexpr int N = decltype(n_tag)::value;
        double (&xs)[4] = x[N % 3];
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const double sv = row_bcast<N>(src[q]);
#pragma unroll
            for (int k = 0; k < 4; ++k) acc4[q][k] = __builtin_fmin(acc4[q][k], xs[k] + sv);
        }
        if constexpr (N + 3 < 16) load(xs, N + 3);
        __builtin_amdgcn_sched_barrier(0);
    };
    load(x[0], 0);
    load(x[1], 1);
    load(x[2], 2);
    __builtin_amdgcn_sched_barrier(0);
    step(std::integral_constant<int, 0>{});  step(std::integral_constant<int, 1>{});
    step(std::integral_constant<int, 2>{});  step(std::integral_constant<int, 3>{});
    step(std::integral_constant<int, 4>{});  step(std::integral_constant<int, 5>{});
    step(std::integral_constant<int, 6>{});  step(std::integral_constant<int, 7>{});
    step(std::integral_constant<int, 8>{});  step(std::integral_constant<int, 9>{});
    step(std::integral_constant<int, 10>{}); step(std::integral_constant<int, 11>{});
    step(std::integral_constant<int, 12>{}); step(std::integral_constant<int, 13>{});
    step(std::integral_constant<int, 14>{}); step(std::integral_constant<int, 15>{});
    // Column 16 r + j (this lane's own) is acc4[0] here, acc4[1] in the lane 16 further (its r differs in bit 0),
    // acc4[2] and acc4[3] in the lanes 32 and 48 further: fold the four rows of lanes.
#pragma unroll
    for (int q = 0; q < NA; ++q) {
        const double a0 = __builtin_fmin(acc4[q][0], from_lane(acc4[q][1], lane ^ 16));
        const double a2 = __builtin_fmin(acc4[q][2], from_lane(acc4[q][3], lane ^ 16));
        acc[q][0] = __builtin_fmin(acc[q][0], __builtin_fmin(a0, from_lane(a2, lane ^ 32)));
    }
}

}  // namespace
}  // namespace rh

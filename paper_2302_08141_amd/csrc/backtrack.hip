// Plan extraction: plan[N-1] = last, plan[i] = arg_i[plan[i+1]] -- the chosen strategy
// per operator (the X of Sec. 4.2 in index form).  A chain of N-1 dependent 2-byte
// reads per problem; one lane per problem.
#include "kernels.h"

namespace rh {
namespace {

__global__ void __launch_bounds__(64)
backtrack_kernel(int32_t B, int32_t N, int32_t Kp, const uint16_t* __restrict__ arg,
                 const int32_t* __restrict__ last, int32_t* __restrict__ plan) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= B) return;
    const uint16_t* ap = arg + (int64_t)p * (N - 1) * Kp;
    int32_t* pl = plan + (int64_t)p * N;
    int32_t x = last[p] & (Kp - 1);   // Kp is a power of two: stay inside the row whatever `last` holds
    pl[N - 1] = x;
    for (int i = N - 2; i >= 0; --i) {
        x = ap[(int64_t)i * Kp + x] & (Kp - 1);
        pl[i] = x;
    }
}

__global__ void __launch_bounds__(256)
check_costs_kernel(const int64_t* __restrict__ x, int64_t n, unsigned long long* violations) {
    unsigned long long bad = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t v = x[i];
        bad += !((v >= 0 && v < ((int64_t)1 << 36)) || v == kInf);
    }
    if (bad) atomicAdd(violations, bad);
}

}  // namespace

hipError_t launch_backtrack(int32_t B, int32_t N, int32_t Kp, const uint16_t* arg,
                            const int32_t* last, int32_t* plan, hipStream_t stream) {
    if (B == 0) return hipSuccess;
    hipLaunchKernelGGL(backtrack_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, B, N, Kp, arg, last,
                       plan);
    return hipGetLastError();
}

hipError_t launch_check_costs(const int64_t* x, int64_t n, int64_t* violations, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(check_costs_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, x, n,
                       reinterpret_cast<unsigned long long*>(violations));
    return hipGetLastError();
}

}  // namespace rh

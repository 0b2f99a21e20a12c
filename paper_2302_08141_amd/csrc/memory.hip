// Memory-constrained search (Sec. 4.4): parameters are ranked by size, the candidates that
// replicate one of the k largest are removed, the chain is solved again, and the smallest k
// whose plan fits the device memory wins.  The sweep over k is a batch of chain problems that
// share the edge tables; the kernels here build the masked node-cost tables, add up the
// parameter memory of the returned plans and pick the first feasible k.
#include "kernels.h"

namespace rh {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ int64_t block_sum(int64_t x, int64_t* scratch) {
    const int t = threadIdx.x;
    scratch[t] = x;
    __syncthreads();
    for (int s = kThreads / 2; s > 0; s >>= 1) {
        if (t < s) scratch[t] += scratch[t + s];
        __syncthreads();
    }
    const int64_t r = scratch[0];
    __syncthreads();
    return r;
}

// One workgroup per operator: its rank among the parameter sizes (largest first, equal sizes by
// operator index), then its row of every masked table.
__global__ void __launch_bounds__(kThreads)
mask_replicated_kernel(int32_t N, int32_t Kp, int32_t n_k, int32_t k0, const int64_t* __restrict__ c,
                       const int64_t* __restrict__ param_bytes, const uint8_t* __restrict__ repl,
                       int64_t* __restrict__ c_out) {
    __shared__ int64_t scratch[kThreads];
    const int i = blockIdx.x;
    const int64_t mine = param_bytes[i];
    int64_t ahead = 0;
    for (int l = threadIdx.x; l < N; l += kThreads) {
        const int64_t other = param_bytes[l];
        ahead += (other > mine) || (other == mine && l < i);
    }
    const int64_t rank = block_sum(ahead, scratch);
    for (int j = threadIdx.x; j < Kp; j += kThreads) {
        const int64_t cost = c[(int64_t)i * Kp + j];
        const bool replicates = mine > 0 && repl[(int64_t)i * Kp + j] != 0;
        for (int t = 0; t < n_k; ++t)
            c_out[((int64_t)t * N + i) * Kp + j] = (replicates && rank < k0 + t) ? kInf : cost;
    }
}

__global__ void __launch_bounds__(kThreads)
plan_memory_kernel(int32_t N, int32_t Kp, const int32_t* __restrict__ plan, const int64_t* __restrict__ mem,
                   int64_t* __restrict__ plan_mem) {
    __shared__ int64_t scratch[kThreads];
    const int b = blockIdx.x;
    int64_t s = 0;
    for (int i = threadIdx.x; i < N; i += kThreads) {
        const int x = plan[(int64_t)b * N + i] & (Kp - 1);   // Kp is a power of two: stay inside the row
        s += mem[(int64_t)i * Kp + x];
    }
    const int64_t total = block_sum(s, scratch);
    if (threadIdx.x == 0) plan_mem[b] = total;
}

__global__ void __launch_bounds__(kThreads)
first_feasible_kernel(int32_t B, const int64_t* __restrict__ total, const int64_t* __restrict__ plan_mem,
                      int64_t limit, int32_t* __restrict__ first) {
    __shared__ int32_t best[kThreads];
    int32_t mine = INT32_MAX;
    for (int b = threadIdx.x; b < B; b += kThreads)
        if (total[b] >= 0 && total[b] < kInf && plan_mem[b] <= limit) { mine = b; break; }   // b ascends per thread;
            // a negative total marks a problem whose search did not finish (rh_minplus_chain): never feasible
    best[threadIdx.x] = mine;
    __syncthreads();
    for (int s = kThreads / 2; s > 0; s >>= 1) {
        if (threadIdx.x < s && best[threadIdx.x + s] < best[threadIdx.x]) best[threadIdx.x] = best[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) *first = best[0] == INT32_MAX ? -1 : best[0];
}

}  // namespace

hipError_t launch_mask_replicated(int32_t N, int32_t Kp, int32_t n_k, int32_t k0, const int64_t* c,
                                  const int64_t* param_bytes, const uint8_t* repl, int64_t* c_out,
                                  hipStream_t stream) {
    if (n_k == 0) return hipSuccess;
    hipLaunchKernelGGL(mask_replicated_kernel, dim3(N), dim3(kThreads), 0, stream, N, Kp, n_k, k0, c, param_bytes,
                       repl, c_out);
    return hipGetLastError();
}

hipError_t launch_plan_memory(int32_t B, int32_t N, int32_t Kp, const int32_t* plan, const int64_t* mem,
                              const int64_t* total, int64_t limit, int64_t* plan_mem, int32_t* first,
                              hipStream_t stream) {
    if (B > 0)
        hipLaunchKernelGGL(plan_memory_kernel, dim3(B), dim3(kThreads), 0, stream, N, Kp, plan, mem, plan_mem);
    if (first != nullptr)
        hipLaunchKernelGGL(first_feasible_kernel, dim3(1), dim3(kThreads), 0, stream, B, total, plan_mem, limit,
                           first);
    return hipGetLastError();
}

}  // namespace rh

// Plan extraction: plan[N-1] = last, plan[i] = arg_i[plan[i+1]] -- the chosen strategy
// per operator (the X of Sec. 4.2 in index form).  A chain of N-1 dependent 2-byte reads per
// problem.  One wavefront per problem: the rows of arg are fetched 8 KiB at a time with
// coalesced 16-byte loads (the next chunk is already in registers while one lane walks the
// current one in LDS, so the dependent reads cost an LDS access instead of a trip to memory),
// and the plan goes out in coalesced pieces.
#include "kernels.h"

namespace rh {
namespace {

typedef int int4v __attribute__((ext_vector_type(4)));

constexpr int kBtWaves = 4;              // problems per workgroup
constexpr int kChunkBytes = 8192;        // of arg rows per wave in LDS
constexpr int kLoads = kChunkBytes / (64 * 16);

__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ void __launch_bounds__(kBtWaves * 64)
backtrack_kernel(int32_t B, int32_t N, int32_t Kp, int32_t lgKp, const uint16_t* __restrict__ arg,
                 const int32_t* __restrict__ last, int32_t* __restrict__ plan) {
    __shared__ int4v rows_all[kBtWaves][kChunkBytes / 16];
    __shared__ int32_t out_all[kBtWaves][kChunkBytes / 32];   // at most one plan entry per 32-byte row

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int p = blockIdx.x * kBtWaves + wave;
    if (p >= B) return;   // no workgroup barrier below
    int4v* rows = rows_all[wave];
    int32_t* out = out_all[wave];
    const uint16_t* rows16 = reinterpret_cast<const uint16_t*>(rows);
    int32_t* pl = plan + (int64_t)p * N;
    int32_t x = last[p] & (Kp - 1);   // Kp is a power of two: stay inside the row whatever `last` holds
    if (lane == 0) pl[N - 1] = x;
    if (N == 1) return;

    const int cr = kChunkBytes >> (lgKp + 1);                 // rows per chunk
    const int n_rows = N - 1;
    const int n_chunks = (n_rows + cr - 1) / cr;
    // chunk k (counted from the end of the chain) covers rows [hi - cr, hi) with hi = n_rows - k*cr, cut at 0
    const int4v* base = reinterpret_cast<const int4v*>(arg + (int64_t)p * n_rows * Kp);
    const int words_per_row = Kp >> 3;                        // 16-byte words
    int4v buf[kLoads];
    auto fetch = [&](int k) {
        const int hi = n_rows - k * cr;
        const int lo = hi - cr > 0 ? hi - cr : 0;
        const int n_words = (hi - lo) * words_per_row;
        const int4v* src = base + (int64_t)lo * words_per_row;
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int w = lane + 64 * j;
            buf[j] = w < n_words ? __builtin_nontemporal_load(src + w) : int4v{0, 0, 0, 0};
        }
    };
    fetch(0);
    for (int k = 0; k < n_chunks; ++k) {
        const int hi = n_rows - k * cr;
        const int lo = hi - cr > 0 ? hi - cr : 0;
#pragma unroll
        for (int j = 0; j < kLoads; ++j) rows[lane + 64 * j] = buf[j];
        if (k + 1 < n_chunks) fetch(k + 1);                   // in flight during the walk
        wave_sync();
        if (lane == 0) {
            for (int r = hi - lo - 1; r >= 0; --r) {
                x = rows16[(r << lgKp) + x] & (Kp - 1);
                out[r] = x;
            }
        }
        wave_sync();
        x = __builtin_amdgcn_readfirstlane(x);
        for (int r = lane; r < hi - lo; r += 64) pl[lo + r] = out[r];
        wave_sync();                                          // out and rows are reused by the next chunk
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
    int lgKp = 0;
    while ((1 << lgKp) < Kp) ++lgKp;
    hipLaunchKernelGGL(backtrack_kernel, dim3((B + kBtWaves - 1) / kBtWaves), dim3(kBtWaves * 64), 0, stream, B, N,
                       Kp, lgKp, arg, last, plan);
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

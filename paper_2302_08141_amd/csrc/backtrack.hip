// Plan extraction: plan[N-1] = last, plan[i] = arg_i[plan[i+1]] -- the chosen strategy
// per operator (the X of Sec. 4.2 in index form).  A chain of N-1 dependent 2-byte reads per
// problem.  One wavefront per problem: the rows of arg are fetched 8 KiB at a time with
// coalesced 16-byte loads (the next chunk is already in registers while one lane walks the
// current one in LDS, so the dependent reads cost an LDS access instead of a trip to memory),
// and the plan goes out in coalesced pieces.
//
// A few long chains are walked in blocks of rows, all blocks at once: (1) every block but the
// lowest maps each possible strategy at its upper end to the strategy at its lower end (Kp
// walks side by side, one per lane); (2) one workgroup chains the maps from `last` downwards and
// writes the plan entry at every block boundary; (3) every block is walked as above from its
// boundary entry.  The maps are parked inside the plan rows of their own blocks (overwritten
// by step 3), so no workspace is needed; a block must be long enough to hold its map.
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

// Problem p: rows of arg at arg + p (N-1) Kp, start strategy last[p * last_stride], plan at plan + p * plan_stride.
__global__ void __launch_bounds__(kBtWaves * 64)
backtrack_kernel(int32_t B, int32_t N, int32_t Kp, int32_t lgKp, const uint16_t* __restrict__ arg,
                 const int32_t* last, int64_t last_stride, int32_t* plan, int64_t plan_stride) {
    __shared__ int4v rows_all[kBtWaves][kChunkBytes / 16];
    __shared__ int32_t out_all[kBtWaves][kChunkBytes / 32];   // at most one plan entry per 32-byte row

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int p = blockIdx.x * kBtWaves + wave;
    if (p >= B) return;   // no workgroup barrier below
    int4v* rows = rows_all[wave];
    int32_t* out = out_all[wave];
    const uint16_t* rows16 = reinterpret_cast<const uint16_t*>(rows);
    int32_t* pl = plan + (int64_t)p * plan_stride;
    int32_t x = last[(int64_t)p * last_stride] & (Kp - 1);   // Kp is a power of two: stay inside the row whatever `last` holds
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

// ---- blocks of rows, for a few long chains ----------------------------------------------------------
// Rows 0..N-2 of a problem: block 0 = rows [0, len0), block b >= 1 = rows [len0 + (b-1) len, len0 + b len).
// The map of block b >= 1 (Kp entries of 16 bits) sits in plan[first row of b + 1 ...], 4-byte aligned.
constexpr int kMapChunkBytes = 8192;

__global__ void __launch_bounds__(1024)
backtrack_maps_kernel(int32_t N, int32_t Kp, int32_t lgKp, int32_t len0, int32_t len,
                      const uint16_t* __restrict__ arg, int32_t* __restrict__ plan) {
    __shared__ int4v rows[kMapChunkBytes / 16];
    const uint16_t* rows16 = reinterpret_cast<const uint16_t*>(rows);
    const int b = blockIdx.x + 1, p = blockIdx.y, t = threadIdx.x;       // Kp threads
    const int r0 = len0 + (b - 1) * len;                                  // rows [r0, r0 + len)
    const int4v* base = reinterpret_cast<const int4v*>(arg + ((int64_t)p * (N - 1) + r0) * Kp);
    const int words_per_row = Kp >> 3, cr = kMapChunkBytes >> (lgKp + 1); // rows per chunk
    int32_t x = t;
    for (int hi = len; hi > 0; hi -= cr) {
        const int lo = hi - cr > 0 ? hi - cr : 0;
        const int n_words = (hi - lo) * words_per_row;
        __syncthreads();                                                  // the chunk before has been walked
        for (int w = t; w < n_words; w += Kp) rows[w] = __builtin_nontemporal_load(base + (int64_t)lo * words_per_row + w);
        __syncthreads();
        for (int r = hi - lo - 1; r >= 0; --r) x = rows16[(r << lgKp) + x] & (Kp - 1);
    }
    uint16_t* map = reinterpret_cast<uint16_t*>(plan + (int64_t)p * N + r0 + 1);
    map[t] = (uint16_t)x;
}

__global__ void __launch_bounds__(256)
backtrack_compose_kernel(int32_t N, int32_t Kp, int32_t len0, int32_t len, int32_t nblk,
                         const int32_t* __restrict__ last, int32_t* __restrict__ plan) {
    __shared__ uint16_t maps[24576];                                      // (nblk - 1) * Kp entries at most
    const int p = blockIdx.x, t = threadIdx.x;
    int32_t* pl = plan + (int64_t)p * N;
    for (int b = 1; b < nblk; ++b) {
        const uint16_t* map = reinterpret_cast<const uint16_t*>(pl + len0 + (b - 1) * len + 1);
        for (int k = t; k < Kp; k += 256) maps[(b - 1) * Kp + k] = map[k];
    }
    __syncthreads();
    if (t == 0) {
        int32_t x = last[p] & (Kp - 1);
        for (int b = nblk - 1; b >= 1; --b) {
            pl[len0 + b * len] = x;                                       // upper end of block b (N-1 for the top one)
            x = maps[(b - 1) * Kp + x];
        }
        pl[len0] = x;                                                     // upper end of block 0
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
    // blocks for a few long chains: a block holds its map (Kp / 2 plan entries, after the boundary entry), the
    // maps of a problem fit the composing workgroup's LDS, and all walks together still fill the chip
    const int min_len = Kp / 2 + 2;
    int nblk = (N - 1) / min_len;
    if (nblk > 64) nblk = 64;
    if ((int64_t)(nblk - 1) * Kp > 24576) nblk = 24576 / Kp + 1;
    if (B <= 16 && Kp >= 64 && nblk >= 8) {
        const int len = (N - 1) / nblk, len0 = (N - 1) - (nblk - 1) * len;   // len0 in [len, len + nblk)
        hipLaunchKernelGGL(backtrack_maps_kernel, dim3(nblk - 1, B), dim3(Kp), 0, stream, N, Kp, lgKp, len0, len, arg,
                           plan);
        hipLaunchKernelGGL(backtrack_compose_kernel, dim3(B), dim3(256), 0, stream, N, Kp, len0, len, nblk, last,
                           plan);
        for (int p = 0; p < B; ++p) {
            const uint16_t* ap = arg + (int64_t)p * (N - 1) * Kp;
            int32_t* pp = plan + (int64_t)p * N;
            // block 0: rows [0, len0), start entry plan[len0]; blocks b >= 1 as nblk - 1 problems of len rows
            hipLaunchKernelGGL(backtrack_kernel, dim3(1), dim3(kBtWaves * 64), 0, stream, 1, len0 + 1, Kp, lgKp, ap,
                               pp + len0, (int64_t)0, pp, (int64_t)0);
            hipLaunchKernelGGL(backtrack_kernel, dim3((nblk - 1 + kBtWaves - 1) / kBtWaves), dim3(kBtWaves * 64), 0,
                               stream, nblk - 1, len + 1, Kp, lgKp, ap + (int64_t)len0 * Kp, pp + len0 + len,
                               (int64_t)len, pp + len0, (int64_t)len);
        }
        return hipGetLastError();
    }
    hipLaunchKernelGGL(backtrack_kernel, dim3((B + kBtWaves - 1) / kBtWaves), dim3(kBtWaves * 64), 0, stream, B, N,
                       Kp, lgKp, arg, last, (int64_t)1, plan, (int64_t)N);
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

// The plans of the chosen pipeline stages, all at once.  Sec. 3 plans every stage's subgraph on its own; once the
// stage search has fixed the boundaries, stage t of a chain holds the operators bounds[t] .. bounds[t+1]-1 and its
// plan is the minimiser of Sec. 4.2's objective over these operators and the edges between them -- the chain DP on
// the sub-chain, with the chain DP's tie rule (lowest minimiser at every step, so the plan returned is the smallest
// optimal one when plans are compared from the stage's last operator backwards).  The stage's total is the entry
// T[bounds[t]][bounds[t+1]] of the table of stage times.
//
// Stages have different lengths, so this is a ragged batch: one workgroup per (stage, problem) walks its sub-chain
// edge by edge (column b = t mod Kp, the rows of an edge table dealt to 512 / Kp slices whose (value, lowest a)
// candidates meet in LDS), leaves arg for the edges inside the stage, the stage's total and its last operator's
// strategy; then one wavefront per (stage, problem) walks arg backwards, 8 KiB of rows at a time through LDS.
// Edges that cross a stage boundary belong to no stage and are not looked at.
#include "kernels.h"

namespace rh {
namespace {

typedef int int4v __attribute__((ext_vector_type(4)));

constexpr int kSpThreads = 512;

__device__ __forceinline__ int64_t sat(int64_t x) { return x < kInf ? x : kInf; }

__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Operators f .. e1 - 1 of stage t of problem p, or f = e1 = -1 if the boundaries do not describe a stage
// (negative, decreasing, beyond the chain: what a search without a feasible split leaves).
__device__ __forceinline__ void stage_range(const int32_t* __restrict__ bounds, int32_t S, int32_t L, int p, int t,
                                            int* f, int* e1) {
    const int32_t a = bounds[(int64_t)p * (S + 1) + t], b = bounds[(int64_t)p * (S + 1) + t + 1];
    const bool ok = a >= 0 && b > a && b <= L;
    *f = ok ? a : -1;
    *e1 = ok ? b : -1;
}

template <int KP>
__global__ void __launch_bounds__(KP > kSpThreads ? KP : kSpThreads)
stage_chains_kernel(int32_t L, int32_t S, const int32_t* __restrict__ bounds, const int64_t* __restrict__ c,
                    const int64_t* __restrict__ R, uint16_t* __restrict__ arg, int64_t* __restrict__ stage_total,
                    int32_t* __restrict__ stage_last) {
    constexpr int T = KP > kSpThreads ? KP : kSpThreads;
    constexpr int SL = T / KP;                  // row slices
    __shared__ int64_t v[KP];
    __shared__ int64_t pv[SL][KP];
    __shared__ uint16_t pa[SL][KP];
    const int tid = threadIdx.x;
    const int b = tid % KP, slice = tid / KP;
    const int t = blockIdx.x, p = blockIdx.y;
    int f, e1;
    stage_range(bounds, S, L, p, t, &f, &e1);
    if (f < 0) {                                // (uniform over the workgroup)
        if (tid == 0) {
            stage_total[(int64_t)p * S + t] = kInf;
            stage_last[(int64_t)p * S + t] = 0;
        }
        return;
    }
    c += (int64_t)p * L * KP;
    R += (int64_t)p * (L - 1) * KP * KP;
    arg += (int64_t)p * (L - 1) * KP;
    // Narrow tables (at most 16 rows per thread): the rows of the next edge and the node cost that goes with them
    // wait in registers while this edge is relaxed -- a trip to memory takes longer than an edge.
    constexpr int NR = KP >= SL ? KP / SL : 1;  // rows of an edge table per thread (slices beyond KP rows idle)
    constexpr bool kAhead = NR <= 16;
    int64_t ahead[kAhead ? NR : 1], c_ahead = 0;
    auto fetch = [&](int i) {                   // edge i, f <= i <= e1 - 2
        if constexpr (kAhead) {
            const int64_t* Ri = R + (int64_t)i * KP * KP;
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int a = slice + r * SL < KP ? slice + r * SL : KP - 1;
                ahead[r] = __builtin_nontemporal_load(Ri + (int64_t)a * KP + b);
            }
            c_ahead = tid < KP ? c[(int64_t)(i + 1) * KP + b] : 0;
        }
    };
    if (f + 1 < e1) fetch(f);
    if (tid < KP) v[b] = sat(c[(int64_t)f * KP + b]);
    lds_barrier();
    for (int i = f; i + 1 < e1; ++i) {
        int64_t c_next;
        int64_t best = INT64_MAX;
        int besta = 0;
        if constexpr (kAhead) {
            int64_t rows[NR];
#pragma unroll
            for (int r = 0; r < NR; ++r) rows[r] = ahead[r];
            c_next = c_ahead;
            if (i + 2 < e1) fetch(i + 1);
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int a = slice + r * SL;
                const int64_t x = v[a < KP ? a : KP - 1] + rows[r];                          // both <= 2^52
                const bool lt = a < KP && x < best;
                best = lt ? x : best;
                besta = lt ? a : besta;
            }
        } else {
            const int64_t* Ri = R + (int64_t)i * KP * KP;
            c_next = tid < KP ? c[(int64_t)(i + 1) * KP + b] : 0;
#pragma unroll 4
            for (int a = slice; a < KP; a += SL) {
                const int64_t x = v[a] + __builtin_nontemporal_load(Ri + (int64_t)a * KP + b);   // both <= 2^52
                const bool lt = x < best;
                best = lt ? x : best;
                besta = lt ? a : besta;
            }
        }
        pv[slice][b] = best;
        pa[slice][b] = (uint16_t)besta;
        lds_barrier();                          // every read of v_i is done, the candidates are in LDS
        if (tid < KP) {
            int64_t m = pv[0][b];
            int ma = pa[0][b];
#pragma unroll
            for (int s = 1; s < SL; ++s) {
                const int64_t x = pv[s][b];
                const int xa = pa[s][b];
                const bool less = x < m || (x == m && xa < ma);
                m = less ? x : m;
                ma = less ? xa : ma;
            }
            const bool dead = m >= kInf;
            arg[(int64_t)i * KP + b] = (uint16_t)(dead ? 0 : ma);
            v[b] = sat(sat(c_next) + (dead ? kInf : m));
        }
        lds_barrier();
    }
    if (tid < 64) {                             // total and lowest best strategy of the stage's last operator
        unsigned long long key = ~0ull;
        for (int col = tid; col < KP; col += 64) {
            const unsigned long long k0 = ((unsigned long long)v[col] << 10) | (unsigned long long)col;
            key = k0 < key ? k0 : key;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const unsigned long long o = __shfl_xor(key, off, 64);
            key = o < key ? o : key;
        }
        if (tid == 0) {
            const int64_t tot = (int64_t)(key >> 10);
            stage_total[(int64_t)p * S + t] = tot;
            stage_last[(int64_t)p * S + t] = tot >= kInf ? 0 : (int32_t)(key & 1023u);
        }
    }
}

__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr int kSpWaves = 4;              // stages per workgroup
constexpr int kSpChunkBytes = 8192;      // of arg rows per wave in LDS
constexpr int kSpLoads = kSpChunkBytes / (64 * 16);

// plan[e1 - 1] = the stage's last strategy, plan[i] = arg_i[plan[i + 1]] down to the stage's first operator.
__global__ void __launch_bounds__(kSpWaves * 64)
stage_backtrack_kernel(int32_t L, int32_t S, int32_t Kp, int32_t lgKp, const int32_t* __restrict__ bounds,
                       const uint16_t* __restrict__ arg, const int32_t* __restrict__ stage_last,
                       int32_t* __restrict__ plan) {
    __shared__ int4v rows_all[kSpWaves][kSpChunkBytes / 16];
    __shared__ int32_t out_all[kSpWaves][kSpChunkBytes / 32];   // at most one plan entry per 32-byte row
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * kSpWaves + wave, p = blockIdx.y;
    if (t >= S) return;                         // no workgroup barrier below
    int f, e1;
    stage_range(bounds, S, L, p, t, &f, &e1);
    if (f < 0) return;
    int4v* rows = rows_all[wave];
    int32_t* out = out_all[wave];
    const uint16_t* rows16 = reinterpret_cast<const uint16_t*>(rows);
    int32_t* pl = plan + (int64_t)p * L;
    int32_t x = stage_last[(int64_t)p * S + t] & (Kp - 1);
    if (lane == 0) pl[e1 - 1] = x;
    const int n_rows = e1 - 1 - f;              // edges inside the stage: rows f .. e1 - 2 of arg
    if (n_rows == 0) return;
    const int cr = kSpChunkBytes >> (lgKp + 1);                 // rows per chunk
    const int n_chunks = (n_rows + cr - 1) / cr;
    const int words_per_row = Kp >> 3;                          // 16-byte words
    const int4v* base = reinterpret_cast<const int4v*>(arg + ((int64_t)p * (L - 1) + f) * Kp);
    int4v buf[kSpLoads];
    auto fetch = [&](int k) {
        const int hi = n_rows - k * cr;
        const int lo = hi - cr > 0 ? hi - cr : 0;
        const int n_words = (hi - lo) * words_per_row;
        const int4v* src = base + (int64_t)lo * words_per_row;
#pragma unroll
        for (int j = 0; j < kSpLoads; ++j) {
            const int w = lane + 64 * j;
            buf[j] = w < n_words ? src[w] : int4v{0, 0, 0, 0};
        }
    };
    fetch(0);
    for (int k = 0; k < n_chunks; ++k) {
        const int hi = n_rows - k * cr;
        const int lo = hi - cr > 0 ? hi - cr : 0;
#pragma unroll
        for (int j = 0; j < kSpLoads; ++j) rows[lane + 64 * j] = buf[j];
        if (k + 1 < n_chunks) fetch(k + 1);                     // in flight during the walk
        wave_sync();
        if (lane == 0) {
            for (int r = hi - lo - 1; r >= 0; --r) {
                x = rows16[(r << lgKp) + x] & (Kp - 1);         // Kp is a power of two: stay inside the row
                out[r] = x;
            }
        }
        wave_sync();
        x = __builtin_amdgcn_readfirstlane(x);
        for (int r = lane; r < hi - lo; r += 64) pl[f + lo + r] = out[r];
        wave_sync();                                            // out and rows are reused by the next chunk
    }
}

__global__ void __launch_bounds__(256)
stage_plans_clear_kernel(int64_t n, int32_t* __restrict__ plan) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) plan[i] = -1;
}

}  // namespace

hipError_t launch_stage_plans(int32_t B, int32_t L, int32_t Kp, int32_t S, const int32_t* bounds, const int64_t* c,
                              const int64_t* R, uint16_t* arg, int64_t* stage_total, int32_t* stage_last,
                              int32_t* plan, hipStream_t stream) {
    if (B == 0) return hipSuccess;
    const dim3 grid((unsigned)S, (unsigned)B);
#define RH_SP(KP)                                                                                                   \
    hipLaunchKernelGGL(stage_chains_kernel<KP>, grid, dim3(KP > kSpThreads ? KP : kSpThreads), 0, stream, L, S,     \
                       bounds, c, R, arg, stage_total, stage_last)
    switch (Kp) {
        case 16: RH_SP(16); break;
        case 32: RH_SP(32); break;
        case 64: RH_SP(64); break;
        case 128: RH_SP(128); break;
        case 256: RH_SP(256); break;
        case 512: RH_SP(512); break;
        case 1024: RH_SP(1024); break;
        default: return hipErrorInvalidValue;
    }
#undef RH_SP
    if (plan != nullptr) {
        const int64_t n = (int64_t)B * L;
        hipLaunchKernelGGL(stage_plans_clear_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, n, plan);
        int lg = 0;
        while ((1 << lg) < Kp) ++lg;
        hipLaunchKernelGGL(stage_backtrack_kernel, dim3((unsigned)((S + kSpWaves - 1) / kSpWaves), (unsigned)B),
                           dim3(kSpWaves * 64), 0, stream, L, S, Kp, lg, bounds, arg, stage_last, plan);
    }
    return hipGetLastError();
}

}  // namespace rh

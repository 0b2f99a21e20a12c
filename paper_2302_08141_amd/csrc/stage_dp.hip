// Balanced pipeline stages on a chain of L segments (Sec. 2.1, Sec. 5.1-5.2):
//     dp[1][j] = P(j);  dp[s][j] = min_{s-1<=i<j} max(dp[s-1][i], P(j)-P(i)),  lowest i on ties.
// Plain integer ALU work (about L^2/2 cells per stage count s, working set two L-vectors),
// one kernel launch per s because dp[s] needs all of dp[s-1].
//
// A workgroup owns 64 consecutive j (one per lane); its 16 waves split the i range into
// contiguous chunks.  i is uniform across a wave, so (dp[s-1][i], P(i)) -- stored interleaved
// in the workspace -- arrive through scalar loads and a cell is sub / max / min on the vector
// ALU with no cross-lane traffic.  The 16 partial minima per j are merged through LDS in
// chunk order, which keeps the lowest i on ties.
#include "kernels.h"

namespace rh {
namespace {

typedef long long ll2 __attribute__((ext_vector_type(2)));

constexpr int kJTile = 64;
constexpr int kWaves = 16;
constexpr int kScanThreads = 256;

// workspace per problem: two buffers of (dp, P) pairs, L+1 entries each
__host__ __device__ inline size_t pairs_per_problem(int32_t L) { return 2 * ((size_t)L + 1); }

// P and the s = 1 row.  One workgroup per problem; thread t sums a contiguous slice.
__global__ void __launch_bounds__(kScanThreads)
stage_init_kernel(int32_t L, int32_t S, const int64_t* __restrict__ cost, ll2* __restrict__ ws,
                  int64_t* __restrict__ bottleneck, int32_t* __restrict__ cut) {
    __shared__ int64_t part[kScanThreads];
    const int p = blockIdx.x, t = threadIdx.x;
    const int64_t* cs = cost + (int64_t)p * L;
    ll2* buf0 = ws + (size_t)p * pairs_per_problem(L);
    ll2* buf1 = buf0 + (L + 1);
    int32_t* ct = cut + (int64_t)p * S * (L + 1);
    const int per = (L + kScanThreads - 1) / kScanThreads;
    const int lo = t * per < L ? t * per : L;
    const int hi = lo + per < L ? lo + per : L;
    int64_t s = 0;
    for (int l = lo; l < hi; ++l) s += cs[l];
    part[t] = s;
    __syncthreads();
    if (t == 0) {
        int64_t run = 0;
        for (int k = 0; k < kScanThreads; ++k) {
            const int64_t x = part[k];
            part[k] = run;
            run += x;
        }
    }
    __syncthreads();
    int64_t run = part[t];
    if (t == 0) {
        ll2 z; z.x = 0; z.y = 0;
        buf0[0] = z; buf1[0] = z;
        ct[0] = -1;
    }
    for (int l = lo; l < hi; ++l) {
        run += cs[l];
        ll2 v; v.x = run; v.y = run;      // dp[1][j] = P(j)
        buf0[l + 1] = v;
        v.x = kInf;
        buf1[l + 1] = v;                  // P is kept in both buffers
        ct[l + 1] = 0;
        if (l + 1 == L) bottleneck[(int64_t)p * S] = run;
    }
}

__global__ void __launch_bounds__(kWaves * 64)
stage_step_kernel(int32_t L, int32_t S, int32_t s, ll2* __restrict__ ws,
                  int64_t* __restrict__ bottleneck, int32_t* __restrict__ cut) {
    __shared__ int64_t pv[kWaves][kJTile];
    __shared__ int32_t pi[kWaves][kJTile];

    const int p = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    ll2* base = ws + (size_t)p * pairs_per_problem(L);
    const ll2* __restrict__ prev = base + (size_t)(s & 1) * (L + 1);     // s-1 odd -> buffer 0
    ll2* cur = base + (size_t)((s & 1) ^ 1) * (L + 1);
    // s = 2 reads buffer 0 (written by init), writes buffer 1; s = 3 reads 1, writes 0; ...
    const int j0 = blockIdx.x * kJTile;          // first j of this tile
    const int j = j0 + lane;
    const int jhi = j0 + kJTile - 1 < L ? j0 + kJTile - 1 : L;   // largest j of the tile
    if (jhi < s) {
        // no j of this tile can be split into s non-empty stages
        if (threadIdx.x < kJTile && j <= L) {
            cut[((int64_t)p * S + (s - 1)) * (L + 1) + j] = -1;
            ll2 v = cur[j]; v.x = kInf; cur[j] = v;
        }
        return;
    }
    const int64_t Pj = j <= L ? prev[j].y : 0;

    // i in [s-1, jhi): 16 contiguous chunks
    const int lo = s - 1;
    const int span = jhi - lo;
    const int chunk = (span + kWaves - 1) / kWaves;
    const int ilo = lo + wave * chunk;
    int ihi = ilo + chunk;
    ihi = ihi < jhi ? ihi : jhi;

    int64_t best = INT64_MAX;
    int32_t besti = -1;
    // i < j0: valid for every lane of the tile
    const int imid = ihi < j0 ? ihi : j0;
    for (int i = ilo; i < imid; ++i) {
        const ll2 q = prev[i];                    // uniform address
        const int64_t tail = Pj - q.y;
        const int64_t m = q.x > tail ? q.x : tail;
        const bool lt = m < best;
        best = lt ? m : best;
        besti = lt ? i : besti;
    }
    // diagonal block: only lanes with i < j take part
    for (int i = ilo > j0 ? ilo : j0; i < ihi; ++i) {
        const ll2 q = prev[i];
        const int64_t tail = Pj - q.y;
        const int64_t m = q.x > tail ? q.x : tail;
        const bool lt = (m < best) && (i < j);
        best = lt ? m : best;
        besti = lt ? i : besti;
    }
    pv[wave][lane] = best;
    pi[wave][lane] = besti;
    __syncthreads();
    if (threadIdx.x < kJTile && j <= L) {
        int64_t b = INT64_MAX;
        int32_t bi = -1;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {        // ascending i: strict < keeps the lowest
            const int64_t x = pv[w][lane];
            const int32_t xi = pi[w][lane];
            const bool lt = x < b && xi >= 0;
            b = lt ? x : b;
            bi = lt ? xi : bi;
        }
        const bool ok = j >= s;                   // then i = s-1 < j exists, so bi >= 0
        ll2 v; v.x = ok ? b : kInf; v.y = Pj;
        cur[j] = v;
        cut[((int64_t)p * S + (s - 1)) * (L + 1) + j] = ok ? bi : -1;
        if (j == L) bottleneck[(int64_t)p * S + (s - 1)] = v.x;
    }
}

__global__ void __launch_bounds__(64)
stage_bounds_kernel(int32_t B, int32_t L, int32_t S, int32_t s_query,
                    const int32_t* __restrict__ cut, int32_t* __restrict__ bounds) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= B) return;
    const int32_t* ct = cut + (int64_t)p * S * (L + 1);
    int32_t* bd = bounds + (int64_t)p * (s_query + 1);
    int32_t x = L;
    bd[s_query] = x;
    for (int t = s_query; t >= 1; --t) {
        x = ct[(int64_t)(t - 1) * (L + 1) + x];
        x = x < 0 ? 0 : (x > L ? L : x);
        bd[t - 1] = x;
    }
}

}  // namespace

size_t stage_workspace_bytes(int32_t B, int32_t L, int32_t S) {
    (void)S;
    return (size_t)B * pairs_per_problem(L) * sizeof(ll2);
}

hipError_t launch_stage_dp(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost,
                           int64_t* bottleneck, int32_t* cut, int32_t s_query, int32_t* bounds,
                           void* workspace, hipStream_t stream) {
    if (B == 0) return hipSuccess;
    ll2* ws = static_cast<ll2*>(workspace);
    hipLaunchKernelGGL(stage_init_kernel, dim3(B), dim3(kScanThreads), 0, stream, L, S, seg_cost, ws,
                       bottleneck, cut);
    const dim3 grid((unsigned)((L + 1 + kJTile - 1) / kJTile), (unsigned)B);
    for (int s = 2; s <= S; ++s)
        hipLaunchKernelGGL(stage_step_kernel, grid, dim3(kWaves * 64), 0, stream, L, S, s, ws,
                           bottleneck, cut);
    if (s_query > 0 && bounds != nullptr)
        hipLaunchKernelGGL(stage_bounds_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, B, L, S,
                           s_query, cut, bounds);
    return hipGetLastError();
}

}  // namespace rh

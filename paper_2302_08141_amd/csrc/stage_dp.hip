// Balanced pipeline stages on a chain of L segments (Sec. 2.1, Sec. 5.1-5.2):
//     dp[1][j] = P(j);  dp[s][j] = min_{s-1<=i<j} max(dp[s-1][i], P(j)-P(i)),  lowest i on ties.
// Plain integer ALU work (about L^2/2 cells per stage count s, working set two L-vectors),
// one kernel launch per s because dp[s] needs all of dp[s-1].
//
// A workgroup owns 64 consecutive j (one per lane); its 16 waves split the i range into
// contiguous chunks.  i is uniform across a wave, so (dp[s-1][i], -P(i)) -- stored interleaved
// in the workspace -- arrive through scalar loads, eight i at a time, and a cell is add / max /
// min on the vector ALU with no cross-lane traffic.  The 16 partial minima per j are merged
// through LDS in chunk order, which keeps the lowest i on ties.  When there are few problems
// the i range of a tile is also split over several workgroups, so that the long tiles do not
// serialise on one CU, and a small second kernel merges the partial minima of each tile.
#include "kernels.h"

namespace rh {
namespace {

typedef long long ll2 __attribute__((ext_vector_type(2)));

constexpr int kJTile = 64;
constexpr int kWaves = 16;
constexpr int kScanThreads = 256;

// workspace: per problem two buffers of (dp, -P) pairs, L+1 entries each; then, if tiles are split,
// partial minima [B][tiles][splits][64] (value, index)
__host__ __device__ inline size_t pairs_per_problem(int32_t L) { return 2 * ((size_t)L + 1); }
inline int tiles_of(int32_t L) { return (L + 1 + kJTile - 1) / kJTile; }

// Workgroups along i per tile: enough to put about a thousand workgroups on the chip, never
// less than 256 i per workgroup.
inline int splits_of(int32_t B, int32_t L) {
    const int64_t wgs = (int64_t)B * tiles_of(L);
    int64_t want = wgs >= 1024 ? 1 : (1024 + wgs - 1) / wgs;
    const int64_t most = ((int64_t)L + 255) / 256;
    want = want < most ? want : most;
    want = want < 32 ? want : 32;
    return (int)(want < 1 ? 1 : want);
}

struct StageLayout {
    size_t pairs_bytes, pval_off, pidx_off, total;
    size_t pfull_off, win_off;   // windowed variant only: P(j) per problem, (first i, last j) per stage count
};
inline StageLayout layout_of(int32_t B, int32_t L, int32_t S_window = 0) {
    StageLayout o{};
    const size_t splits = (size_t)splits_of(B, L), tiles = (size_t)tiles_of(L);
    o.pairs_bytes = (size_t)B * pairs_per_problem(L) * 16;
    o.pval_off = (o.pairs_bytes + 255) & ~(size_t)255;
    const size_t parts = splits > 1 ? (size_t)B * tiles * splits * kJTile : 0;
    o.pidx_off = o.pval_off + parts * 8;
    o.total = o.pidx_off + parts * 4;
    if (S_window > 0) {
        o.pfull_off = (o.total + 255) & ~(size_t)255;
        o.win_off = o.pfull_off + (size_t)B * ((size_t)L + 1) * 8;
        o.total = o.win_off + (size_t)B * (size_t)S_window * 2 * 4;
    }
    return o;
}

// Exclusive prefix sum of one value per thread over the kScanThreads threads of a workgroup (inside a wave by
// shuffles, the four wave totals through LDS).
__device__ __forceinline__ int64_t scan_exclusive(int64_t mine, int64_t* wave_sum) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int64_t o = __shfl_up(incl, off, 64);
        incl += lane >= off ? o : 0;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int64_t base = 0;
    for (int w = 0; w < wave; ++w) base += wave_sum[w];
    return base + incl - mine;
}

// P and the s = 1 row.  One workgroup per problem; thread t sums a contiguous slice.
__global__ void __launch_bounds__(kScanThreads)
stage_init_kernel(int32_t L, int32_t S, const int64_t* __restrict__ cost, ll2* __restrict__ ws,
                  int64_t* __restrict__ bottleneck, int32_t* __restrict__ cut) {
    __shared__ int64_t part[kScanThreads / 64];
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
    int64_t run = scan_exclusive(s, part);
    if (t == 0) {
        ll2 z; z.x = 0; z.y = 0;
        buf0[0] = z; buf1[0] = z;
        ct[0] = -1;
    }
    for (int l = lo; l < hi; ++l) {
        run += cs[l];
        ll2 v; v.x = run; v.y = -run;     // dp[1][j] = P(j)
        buf0[l + 1] = v;
        v.x = kInf;
        buf1[l + 1] = v;                  // -P is kept in both buffers
        ct[l + 1] = 0;
        if (l + 1 == L) bottleneck[(int64_t)p * S] = run;
    }
}

// Variant with boundary transfers and bound tightening (Sec. 5.1, 5.2) for exactly S stages:
// stage [i, j) takes P(j) - P(i) + xfer[i]; segment l may sit in stage t only if
// floor(P(l)/tps - eps) <= t <= ceil(P(l)/tps + eps), tps = P(L)/S.  Both bounds grow with l, so
// for the stage count s they reduce to "i >= first_i[s]" and "j <= last_j[s]".
typedef __int128 i128;

// Segment l, whose earliest start is Pl = P(l), may sit in stage t only if lo(l) <= t <= hi(l) with
//     lo(l) = floor(Pl S / PL - eps) cut off to [0, S] (S = "none"),  hi(l) = ceil(Pl S / PL + eps) cut off to [0, S-1].
// The searches below only ask "hi(l) >= t" and "lo(l) <= t" for 0 <= t <= S-1; with x = Pl S den, e = num PL,
// d = PL den (all below 2^86) these are the division-free comparisons
//     hi(l) >= t  <=>  t = 0 or ceil((x + e) / d) >= t   <=>  t = 0 or x + e > (t - 1) d
//     lo(l) <= t  <=>  floor((x - e) / d) <= t           <=>  x - e < (t + 1) d
// (the cut-offs change neither: hi is cut to S-1 >= t, lo to 0 <= t or to S > t).  A negative eps or a chain
// without any work switches the bounds off.
__device__ inline bool hi_at_least(int64_t Pl, int64_t PL, int32_t S, int64_t num, int64_t den, int32_t t) {
    if (num < 0 || PL <= 0 || t <= 0) return true;
    const i128 x = (i128)Pl * S * den, e = (i128)num * PL, d = (i128)PL * den;
    return x + e > (i128)(t - 1) * d;
}
__device__ inline bool lo_at_most(int64_t Pl, int64_t PL, int32_t S, int64_t num, int64_t den, int32_t t) {
    if (num < 0 || PL <= 0) return true;
    const i128 x = (i128)Pl * S * den, e = (i128)num * PL, d = (i128)PL * den;
    return x - e < (i128)(t + 1) * d;
}

__global__ void __launch_bounds__(kScanThreads)
stage_window_init_kernel(int32_t L, int32_t S, const int64_t* __restrict__ cost, const int64_t* __restrict__ xfer,
                         int64_t eps_num, int64_t eps_den, ll2* __restrict__ ws, int64_t* __restrict__ pfull,
                         int32_t* __restrict__ win, int64_t* __restrict__ bottleneck, int32_t* __restrict__ cut) {
    __shared__ int64_t part[kScanThreads / 64];
    const int p = blockIdx.x, t = threadIdx.x;
    const int64_t* cs = cost + (int64_t)p * L;
    const int64_t* xf = xfer != nullptr ? xfer + (int64_t)p * (L + 1) : nullptr;
    ll2* buf0 = ws + (size_t)p * pairs_per_problem(L);
    ll2* buf1 = buf0 + (L + 1);
    int64_t* Pp = pfull + (size_t)p * (L + 1);
    int32_t* wp = win + (size_t)p * S * 2;
    int32_t* ct = cut + (int64_t)p * S * (L + 1);
    const int per = (L + kScanThreads - 1) / kScanThreads;
    const int lo = t * per < L ? t * per : L;
    const int hi = lo + per < L ? lo + per : L;
    int64_t sum = 0;
    for (int l = lo; l < hi; ++l) sum += cs[l];
    int64_t run = scan_exclusive(sum, part);
    if (t == 0) Pp[0] = 0;
    for (int l = lo; l < hi; ++l) {
        run += cs[l];
        Pp[l + 1] = run;
    }
    __syncthreads();   // P of this problem is complete (written and read by this workgroup only)
    const int64_t PL = Pp[L];
    // windows per stage count s = t+1: first_i = min{ i : hi(i) >= s-1 }, last_j = 1 + max{ l : lo(l) <= s-1 }
    for (int st = t; st < S; st += kScanThreads) {
        int a = 0, b = L;                       // first i in [0, L] with hi(i) >= st (hi grows with i)
        while (a < b) {
            const int m = (a + b) / 2;
            if (hi_at_least(Pp[m], PL, S, eps_num, eps_den, st)) b = m; else a = m + 1;
        }
        wp[2 * st] = a;
        int a2 = -1, b2 = L - 1;                // last l in [-1, L-1] with lo(l) <= st (lo grows with l)
        while (a2 < b2) {
            const int m = (a2 + b2 + 1) / 2;
            if (lo_at_most(Pp[m], PL, S, eps_num, eps_den, st)) a2 = m; else b2 = m - 1;
        }
        wp[2 * st + 1] = a2 + 1;
    }
    __syncthreads();
    const int last_j1 = wp[1];                  // stage count 1: j <= last_j
    for (int j = t; j <= L; j += kScanThreads) {
        const int64_t Pj = Pp[j];
        const bool ok = j >= 1 && j <= last_j1;
        ll2 v;
        v.x = ok ? Pj : kInf;                   // dp[1][j]
        v.y = (xf != nullptr && j >= 1 && j < L ? xf[j] : 0) - Pj;   // -(P(j) - xfer[j])
        buf0[j] = v;
        v.x = kInf;
        buf1[j] = v;
        ct[j] = ok ? 0 : -1;
        if (j == L && S == 1) bottleneck[p] = ok ? Pj : kInf;
    }
}

template <bool WIN>
__global__ void __launch_bounds__(kWaves * 64)
stage_step_kernel(int32_t L, int32_t S, int32_t s, int32_t splits, const ll2* __restrict__ prev_all,
                  ll2* __restrict__ cur_all, int64_t* __restrict__ pval, int32_t* __restrict__ pidx,
                  int64_t* __restrict__ bottleneck, int32_t* __restrict__ cut,
                  const int64_t* __restrict__ pfull, const int32_t* __restrict__ win) {
    __shared__ int64_t pv[kWaves][kJTile];
    __shared__ int32_t pi[kWaves][kJTile];

    const int p = blockIdx.y;
    const int tile = blockIdx.x / splits;
    const int split = blockIdx.x - tile * splits;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // prev_all / cur_all: the workspace buffers holding dp[s-1] (read only here) and dp[s]
    const ll2* __restrict__ prev = prev_all + (size_t)p * pairs_per_problem(L);
    ll2* __restrict__ cur = cur_all + (size_t)p * pairs_per_problem(L);
    const int j0 = tile * kJTile;                // first j of this tile
    const int j = j0 + lane;
    int lo = s - 1;                              // first i
    int jcap = L;                                // last j that may end stage s
    if constexpr (WIN) {
        const int first_i = win[((size_t)p * S + (s - 1)) * 2], last_j = win[((size_t)p * S + (s - 1)) * 2 + 1];
        lo = first_i > lo ? first_i : lo;
        jcap = last_j < jcap ? last_j : jcap;
    }
    const int jhi = j0 + kJTile - 1 < jcap ? j0 + kJTile - 1 : jcap;   // largest j of the tile that is allowed
    if (jhi < s || jhi <= lo || jhi < j0) {
        // no j of this tile can end stage s
        if (split == 0 && threadIdx.x < kJTile && j <= L) {
            cut[((int64_t)p * S + (s - 1)) * (L + 1) + j] = -1;
            ll2 v = cur[j]; v.x = kInf; cur[j] = v;
            if (WIN && j == L && s == S) bottleneck[p] = kInf;
        }
        return;
    }
    // i in [lo, jhi) goes to `used` workgroups in pieces of wg_chunk (a multiple of 16 * 8)
    const int span = jhi - lo;
    int wg_chunk = (span + splits - 1) / splits;
    wg_chunk = (wg_chunk + 127) & ~127;
    const int used = (span + wg_chunk - 1) / wg_chunk;
    if (split >= used) return;
    const int wlo = lo + split * wg_chunk;
    const int whi = wlo + wg_chunk < jhi ? wlo + wg_chunk : jhi;

    const int64_t negPj = j <= L ? prev[j].y : 0;      // second half of the pair, carried over to dp[s]
    int64_t Pj = -negPj;
    if constexpr (WIN) Pj = j <= L ? pfull[(size_t)p * (L + 1) + j] : 0;   // the pair holds xfer[j] - P(j) there
    asm volatile("" : "+v"(Pj));   // keep "Pj + (-P_i)" one 64-bit add instead of a two-part subtract

    // the workgroup's piece: 16 contiguous chunks, one per wave
    const int chunk = (whi - wlo + kWaves - 1) / kWaves;
    const int ilo = wlo + wave * chunk;
    int ihi = ilo + chunk;
    ihi = ihi < whi ? ihi : whi;

    int64_t best = INT64_MAX;
    int32_t besti = -1;
    constexpr int U = 8;   // pairs fetched per batch of scalar loads
    // i < j0: valid for every lane of the tile
    const int imid = ihi < j0 ? ihi : j0;
    int i = ilo;
    for (; i + U <= imid; i += U) {
        ll2 q[U];
#pragma unroll
        for (int u = 0; u < U; ++u) q[u] = prev[i + u];   // uniform addresses
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t tail = Pj + q[u].y;
            const int64_t m = q[u].x > tail ? q[u].x : tail;
            const bool lt = m < best;
            best = lt ? m : best;
            besti = lt ? i + u : besti;
        }
    }
    // the rest of the chunk, including the diagonal block where only lanes with i < j take part;
    // reads past ihi stay inside the buffer (index clamped) and are masked out
    for (; i < ihi; i += U) {
        ll2 q[U];
#pragma unroll
        for (int u = 0; u < U; ++u) q[u] = prev[i + u < L ? i + u : L];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t tail = Pj + q[u].y;
            const int64_t m = q[u].x > tail ? q[u].x : tail;
            const bool lt = (m < best) && (i + u < j) && (i + u < ihi);
            best = lt ? m : best;
            besti = lt ? i + u : besti;
        }
    }
    pv[wave][lane] = best;
    pi[wave][lane] = besti;
    __syncthreads();
    int64_t b = INT64_MAX;
    int32_t bi = -1;
    if (threadIdx.x < kJTile) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {        // ascending i: strict < keeps the lowest
            const int64_t x = pv[w][lane];
            const int32_t xi = pi[w][lane];
            const bool lt = x < b && xi >= 0;
            b = lt ? x : b;
            bi = lt ? xi : bi;
        }
    }
    if (used > 1) {
        // publish this workgroup's minima; stage_merge_kernel finishes the tile
        if (threadIdx.x < kJTile) {
            const size_t slot = (((size_t)p * gridDim.x + blockIdx.x) * kJTile) + lane;   // [p][tile][split][lane]
            pval[slot] = b;
            pidx[slot] = bi;
        }
        return;
    }
    if (threadIdx.x < kJTile && j <= L) {
        // plain: j >= s has i = s-1 < j, so bi >= 0 and b is finite; windowed: every allowed i may be infeasible
        const bool ok = WIN ? (j >= s && j <= jcap && bi >= 0 && b < kInf) : (j >= s);
        ll2 v; v.x = ok ? b : kInf; v.y = negPj;
        cur[j] = v;
        cut[((int64_t)p * S + (s - 1)) * (L + 1) + j] = ok ? bi : -1;
        if constexpr (WIN) {
            if (j == L && s == S) bottleneck[p] = v.x;
        } else {
            if (j == L) bottleneck[(int64_t)p * S + (s - 1)] = v.x;
        }
    }
}

// Tiles whose i range went to several workgroups: merge their minima (pieces ascend in i, so
// strict < keeps the lowest i) and finish dp[s][j], cut[s][j].  Same geometry as the step kernel.
template <bool WIN>
__global__ void __launch_bounds__(kJTile)
stage_merge_kernel(int32_t L, int32_t S, int32_t s, int32_t splits, ll2* __restrict__ cur_all,
                   const int64_t* __restrict__ pval, const int32_t* __restrict__ pidx,
                   int64_t* __restrict__ bottleneck, int32_t* __restrict__ cut, const int32_t* __restrict__ win) {
    const int p = blockIdx.y, tile = blockIdx.x, lane = threadIdx.x;
    const int j0 = tile * kJTile;
    const int j = j0 + lane;
    int lo = s - 1, jcap = L;
    if constexpr (WIN) {
        const int first_i = win[((size_t)p * S + (s - 1)) * 2], last_j = win[((size_t)p * S + (s - 1)) * 2 + 1];
        lo = first_i > lo ? first_i : lo;
        jcap = last_j < jcap ? last_j : jcap;
    }
    const int jhi = j0 + kJTile - 1 < jcap ? j0 + kJTile - 1 : jcap;
    if (jhi < s || jhi <= lo || jhi < j0) return;   // the step kernel wrote this tile off
    const int span = jhi - lo;
    int wg_chunk = (span + splits - 1) / splits;
    wg_chunk = (wg_chunk + 127) & ~127;
    const int used = (span + wg_chunk - 1) / wg_chunk;
    if (used <= 1 || j > L) return;             // the step kernel finished this tile itself
    ll2* cur = cur_all + (size_t)p * pairs_per_problem(L);
    const size_t first = (((size_t)p * gridDim.x + tile) * splits * kJTile) + lane;
    int64_t b = INT64_MAX;
    int32_t bi = -1;
    for (int k = 0; k < used; ++k) {
        const int64_t x = pval[first + (size_t)k * kJTile];
        const int32_t xi = pidx[first + (size_t)k * kJTile];
        const bool lt = x < b && xi >= 0;
        b = lt ? x : b;
        bi = lt ? xi : bi;
    }
    const bool ok = WIN ? (j >= s && j <= jcap && bi >= 0 && b < kInf) : (j >= s);
    ll2 v = cur[j];                             // keeps the second half of the pair
    v.x = ok ? b : kInf;
    cur[j] = v;
    cut[((int64_t)p * S + (s - 1)) * (L + 1) + j] = ok ? bi : -1;
    if constexpr (WIN) {
        if (j == L && s == S) bottleneck[p] = v.x;
    } else {
        if (j == L) bottleneck[(int64_t)p * S + (s - 1)] = v.x;
    }
}

// Boundaries for exactly S stages, or all -1 if the bounds allow no split.
__global__ void __launch_bounds__(64)
stage_window_bounds_kernel(int32_t B, int32_t L, int32_t S, const int64_t* __restrict__ bottleneck,
                           const int32_t* __restrict__ cut, int32_t* __restrict__ bounds) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= B) return;
    const int32_t* ct = cut + (int64_t)p * S * (L + 1);
    int32_t* bd = bounds + (int64_t)p * (S + 1);
    if (bottleneck[p] >= kInf) {
        for (int t = 0; t <= S; ++t) bd[t] = -1;
        return;
    }
    int32_t x = L;
    bd[S] = x;
    for (int t = S; t >= 1; --t) {
        x = ct[(int64_t)(t - 1) * (L + 1) + x];
        x = x < 0 ? 0 : (x > L ? L : x);
        bd[t - 1] = x;
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
    return layout_of(B, L).total;
}

hipError_t launch_stage_dp(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost,
                           int64_t* bottleneck, int32_t* cut, int32_t s_query, int32_t* bounds,
                           void* workspace, hipStream_t stream) {
    if (B == 0) return hipSuccess;
    const StageLayout lay = layout_of(B, L);
    const int splits = splits_of(B, L), tiles = tiles_of(L);
    char* wsb = static_cast<char*>(workspace);
    ll2* ws = reinterpret_cast<ll2*>(wsb);
    int64_t* pval = reinterpret_cast<int64_t*>(wsb + lay.pval_off);
    int32_t* pidx = reinterpret_cast<int32_t*>(wsb + lay.pidx_off);
    hipLaunchKernelGGL(stage_init_kernel, dim3(B), dim3(kScanThreads), 0, stream, L, S, seg_cost, ws,
                       bottleneck, cut);
    const dim3 grid((unsigned)(tiles * splits), (unsigned)B);
    const dim3 merge_grid((unsigned)tiles, (unsigned)B);
    for (int s = 2; s <= S; ++s) {
        // dp[s-1] lives in buffer (s-1) odd ? 0 : 1 of each problem: s = 2 reads buffer 0, which the
        // init kernel wrote, and writes buffer 1; s = 3 reads 1, writes 0; ...
        const ll2* prev_all = ws + (size_t)(s & 1) * (L + 1);
        ll2* cur_all = ws + (size_t)((s & 1) ^ 1) * (L + 1);
        hipLaunchKernelGGL(stage_step_kernel<false>, grid, dim3(kWaves * 64), 0, stream, L, S, s, splits, prev_all,
                           cur_all, pval, pidx, bottleneck, cut, nullptr, nullptr);
        if (splits > 1)
            hipLaunchKernelGGL(stage_merge_kernel<false>, merge_grid, dim3(kJTile), 0, stream, L, S, s, splits,
                               cur_all, pval, pidx, bottleneck, cut, nullptr);
    }
    if (s_query > 0 && bounds != nullptr)
        hipLaunchKernelGGL(stage_bounds_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, B, L, S,
                           s_query, cut, bounds);
    return hipGetLastError();
}

size_t stage_window_workspace_bytes(int32_t B, int32_t L, int32_t S) { return layout_of(B, L, S).total; }

hipError_t launch_stage_window(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost, const int64_t* xfer,
                               int64_t eps_num, int64_t eps_den, int64_t* bottleneck, int32_t* cut,
                               int32_t* bounds, void* workspace, hipStream_t stream) {
    if (B == 0) return hipSuccess;
    const StageLayout lay = layout_of(B, L, S);
    // A tile's rows: about (2 eps + 2) balanced stage lengths when the segments are of similar size.  Up to 1024 of
    // them a workgroup takes them all -- a second launch per stage count to merge parts would cost more than it
    // saves; wider windows (and bounds switched off) are split over workgroups as in the plain scan.  The choice
    // changes the time only: the kernels handle any window with any split.
    const double rows = eps_num < 0 ? (double)L : (2.0 * (double)eps_num / (double)eps_den + 2.0) * (double)L / (double)S;
    const int splits = rows <= 1024.0 ? 1 : splits_of(B, L), tiles = tiles_of(L);
    char* wsb = static_cast<char*>(workspace);
    ll2* ws = reinterpret_cast<ll2*>(wsb);
    int64_t* pval = reinterpret_cast<int64_t*>(wsb + lay.pval_off);
    int32_t* pidx = reinterpret_cast<int32_t*>(wsb + lay.pidx_off);
    int64_t* pfull = reinterpret_cast<int64_t*>(wsb + lay.pfull_off);
    int32_t* win = reinterpret_cast<int32_t*>(wsb + lay.win_off);
    hipLaunchKernelGGL(stage_window_init_kernel, dim3(B), dim3(kScanThreads), 0, stream, L, S, seg_cost, xfer,
                       eps_num, eps_den, ws, pfull, win, bottleneck, cut);
    const dim3 grid((unsigned)(tiles * splits), (unsigned)B);
    const dim3 merge_grid((unsigned)tiles, (unsigned)B);
    for (int s = 2; s <= S; ++s) {
        const ll2* prev_all = ws + (size_t)(s & 1) * (L + 1);
        ll2* cur_all = ws + (size_t)((s & 1) ^ 1) * (L + 1);
        hipLaunchKernelGGL(stage_step_kernel<true>, grid, dim3(kWaves * 64), 0, stream, L, S, s, splits, prev_all,
                           cur_all, pval, pidx, bottleneck, cut, pfull, win);
        if (splits > 1)
            hipLaunchKernelGGL(stage_merge_kernel<true>, merge_grid, dim3(kJTile), 0, stream, L, S, s, splits,
                               cur_all, pval, pidx, bottleneck, cut, win);
    }
    if (bounds != nullptr)
        hipLaunchKernelGGL(stage_window_bounds_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, B, L, S,
                           bottleneck, cut, bounds);
    return hipGetLastError();
}

}  // namespace rh

// Balanced pipeline stages when the time of stage [i, j) comes from a table (Sec. 3: every
// stage has its own plan, so its time is not a difference of prefix sums; Sec. 5.1 balances):
//     dp[1][j] = T[0][j],  dp[s][j] = min_{s-1 <= i < j} max(dp[s-1][i], T[i][j]),  lowest i on ties.
// Every stage count reads the upper triangle of T once, so the search is bound by the memory
// system (the table of one problem, L^2 * 8 bytes, is re-read S-1 times and mostly stays in the
// last-level cache): rows of T are read with coalesced 16-byte loads, two j per lane, eight rows
// in flight per lane; dp[s-1][i] is uniform over a wave and comes through scalar loads.
// A workgroup owns 128 consecutive j; its 8 waves take the rows i round-robin.  With few problems
// the i range is also split over several workgroups.  Their results meet without a launch of their
// own: per stage count and column one word (value << 6 | part) collects the parts' minima through an
// atomic minimum -- parts hold ascending rows, so the least word names the least value and the lowest
// part that reaches it -- each part keeps the row it found, and the next stage count's launch reads
// dp[s-1] straight from the words and turns them into cut entries on the side.
// When no stage may be longer than 1024 operators a column has few candidate rows and one launch
// per stage count does it all (si_band_kernel below).
#include "kernels.h"

namespace rh {
namespace {

typedef long long ll2 __attribute__((ext_vector_type(2)));

constexpr int kSiWaves = 8;
constexpr int kSiTile = 128;            // j per workgroup
constexpr int kSiUnroll = 8;

constexpr int kSiPartBits = 6;          // up to 32 parts; value <= 2^52, so a word stays below 2^59

struct SiLayout {
    size_t dp_off, key_off, pidx_off, total;
    int splits, tiles;
};

__host__ inline SiLayout si_layout(int32_t B, int32_t L, int32_t S) {
    SiLayout s;
    s.tiles = (L + 1 + kSiTile - 1) / kSiTile;
    int splits = 1;
    // aim at about a thousand workgroups per launch; a split should still hold 32 rows
    while (splits < 32 && (int64_t)B * s.tiles * splits < 1024 && (L / (splits * 2)) >= 32) splits *= 2;
    s.splits = splits;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t cols = (size_t)s.tiles * kSiTile;
    // dp: two buffers per problem (the route of limited stage length); keys: one row of words per stage count and
    // problem; pidx: the parts' rows, two sets that alternate with the stage count
    s.dp_off = 0;
    s.key_off = up((size_t)B * 2 * cols * sizeof(int64_t));
    s.pidx_off = s.key_off + up((size_t)B * (size_t)S * cols * sizeof(int64_t));
    s.total = s.pidx_off + up(2 * (size_t)B * splits * cols * sizeof(int32_t));
    return s;
}

typedef unsigned long long u64;

// dp value held by a word: words that no part has touched (all ones) and infeasible minima read as "infeasible"
__device__ __forceinline__ int64_t key_value(u64 k) {
    const u64 v = k >> kSiPartBits;
    return (int64_t)(v < (u64)kInf ? v : (u64)kInf);
}

__global__ void __launch_bounds__(256)
si_init_kernel(int32_t L, int32_t S, int32_t max_len, int64_t ldT, const int64_t* __restrict__ T, int64_t T_bs, int64_t cols,
               int64_t* __restrict__ dp, u64* __restrict__ keys, int64_t* __restrict__ bottleneck, int32_t* __restrict__ cut) {
    const int p = blockIdx.y;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= cols) return;
    if (keys != nullptr)                                   // no part has reported anything for s >= 2 yet
        for (int s = 2; s <= S; ++s) keys[((int64_t)p * S + (s - 1)) * cols + j] = ~0ull;
    if (j > L) return;
    const int64_t* row0 = T + (int64_t)p * T_bs;
    int64_t v = kInf;
    if (j >= 1 && j <= max_len) {                         // one stage of j operators
        v = row0[j];
        v = v < kInf ? v : kInf;
    }
    if (keys != nullptr) keys[(int64_t)p * S * cols + j] = (u64)v << kSiPartBits;      // dp[1]
    else dp[(int64_t)p * 2 * cols + j] = v;                 // buffer 0 = dp[1]
    cut[(int64_t)p * S * (L + 1) + j] = j >= 1 ? 0 : -1;
    if (j == L) bottleneck[(int64_t)p * S] = v;
}

// What the parts of stage count s left for column j, turned into dp[s][j]'s cut entry (and the bottleneck).
__device__ __forceinline__ void si_decode(int32_t L, int32_t S, int32_t s, int32_t splits, int64_t cols, int p, int j,
                                          const u64* __restrict__ keys, const int32_t* __restrict__ pidx,
                                          int64_t* __restrict__ bottleneck, int32_t* __restrict__ cut) {
    const u64 k = keys[((int64_t)p * S + (s - 1)) * cols + j];
    const int64_t v = key_value(k);
    int32_t bi = -1;
    if (v < kInf) {
        const int part = (int)(k & ((1u << kSiPartBits) - 1));
        bi = pidx[(((int64_t)(s & 1) * gridDim.y + p) * splits + part) * cols + j];
    } else {
        bi = j >= s ? s - 1 : -1;       // every candidate infeasible: the lowest i of the range holds that minimum
    }
    cut[((int64_t)p * S + (s - 1)) * (L + 1) + j] = bi;
    if (j == L) bottleneck[(int64_t)p * S + (s - 1)] = v;
}

// One stage count s for the tile blockIdx.x / splits of problem blockIdx.y, rows of split blockIdx.x % splits.
__global__ void __launch_bounds__(kSiWaves * 64)
si_step_kernel(int32_t L, int32_t S, int32_t s, int32_t splits, int32_t max_len, int64_t ldT, const int64_t* __restrict__ T,
               int64_t T_bs, int64_t cols, u64* __restrict__ keys, int32_t* __restrict__ pidx,
               int64_t* __restrict__ bottleneck, int32_t* __restrict__ cut) {
    __shared__ int64_t sval[kSiWaves][kSiTile];
    __shared__ int32_t sidx[kSiWaves][kSiTile];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int tile = blockIdx.x / splits, split = blockIdx.x % splits;
    const int p = blockIdx.y;
    const int64_t* Tp = T + (int64_t)p * T_bs;
    const u64* prev = keys + ((int64_t)p * S + (s - 2)) * cols;     // the words of stage count s - 1
    const int j0 = tile * kSiTile + 2 * lane;               // this lane's j0 and j0 + 1
    const bool in_range = j0 <= L;                          // then j0 + 1 < ldT (ldT is even and > L)

    // rows that can matter to this tile: s-1 <= i < min(L, last j of the tile), and where the caller says that no
    // stage is longer than max_len (such entries of T are infeasible) only i >= first j of the tile - max_len
    const int j_last = tile * kSiTile + kSiTile - 1 < L ? tile * kSiTile + kSiTile - 1 : L;
    const int i_band = tile * kSiTile - max_len;
    const int i_begin = s - 1 > i_band ? s - 1 : i_band, i_end = j_last;   // exclusive
    const int n_rows = i_end > i_begin ? i_end - i_begin : 0;
    const int per = (n_rows + splits - 1) / splits;
    const int lo = i_begin + split * per;
    const int hi = lo + per < i_end ? lo + per : i_end;

    int64_t best0 = INT64_MAX, best1 = INT64_MAX;
    int32_t idx0 = -1, idx1 = -1;
    auto relax = [&](int i, ll2 t, int64_t a) {
        // a = dp[s-1][i] (already <= 2^52); entries at or left of the diagonal do not take part
        int64_t t0 = t.x < kInf ? t.x : kInf, t1 = t.y < kInf ? t.y : kInf;
        int64_t m0 = a > t0 ? a : t0, m1 = a > t1 ? a : t1;
        // stages of more than max_len operators do not take part either, whatever the table holds for them
        const bool ok0 = i < j0 && j0 - i <= max_len && m0 < best0, ok1 = i < j0 + 1 && j0 + 1 - i <= max_len && m1 < best1;
        best0 = ok0 ? m0 : best0;
        idx0 = ok0 ? i : idx0;
        best1 = ok1 ? m1 : best1;
        idx1 = ok1 ? i : idx1;
    };
    if (in_range) {
        const int64_t* col = Tp + j0;
        int i = lo + wave;
        for (; i + (kSiUnroll - 1) * kSiWaves < hi; i += kSiUnroll * kSiWaves) {
            ll2 t[kSiUnroll];
            int64_t a[kSiUnroll];
#pragma unroll
            for (int u = 0; u < kSiUnroll; ++u) {
                const int r = i + u * kSiWaves;
                t[u] = *reinterpret_cast<const ll2*>(col + (int64_t)r * ldT);
                a[u] = key_value(prev[r]);
            }
#pragma unroll
            for (int u = 0; u < kSiUnroll; ++u) relax(i + u * kSiWaves, t[u], a[u]);
        }
        for (; i < hi; i += kSiWaves) relax(i, *reinterpret_cast<const ll2*>(col + (int64_t)i * ldT), key_value(prev[i]));
    }
    // the cut entries of stage count s - 1, whose parts all reported before this launch began
    if (split == 0 && s > 2 && splits > 1 && tid < kSiTile && tile * kSiTile + tid <= L)
        si_decode(L, S, s - 1, splits, cols, p, tile * kSiTile + tid, keys, pidx, bottleneck, cut);
    sval[wave][2 * lane] = best0;
    sval[wave][2 * lane + 1] = best1;
    sidx[wave][2 * lane] = idx0;
    sidx[wave][2 * lane + 1] = idx1;
    __syncthreads();
    if (tid < kSiTile) {
        // the waves hold interleaved rows: equal values are decided by the row index
        int64_t b = sval[0][tid];
        int32_t bi = sidx[0][tid];
#pragma unroll
        for (int w = 1; w < kSiWaves; ++w) {
            const int64_t v = sval[w][tid];
            const int32_t vi = sidx[w][tid];
            const bool take = vi >= 0 && (bi < 0 || v < b || (v == b && vi < bi));
            b = take ? v : b;
            bi = take ? vi : bi;
        }
        const int j = tile * kSiTile + tid;
        u64* mine = keys + ((int64_t)p * S + (s - 1)) * cols + j;
        if (splits > 1) {
            if (bi >= 0 && j <= L) {
                pidx[(((int64_t)(s & 1) * gridDim.y + p) * splits + split) * cols + j] = bi;
                atomicMin(mine, ((u64)b << kSiPartBits) | (u64)split);
            }
        } else if (j <= L) {
            const int64_t v = bi >= 0 ? b : kInf;
            // every candidate infeasible: the lowest i of the whole range s-1 <= i < j holds that minimum
            if (v >= kInf) bi = j >= s ? s - 1 : -1;
            *mine = (u64)v << kSiPartBits;
            cut[((int64_t)p * S + (s - 1)) * (L + 1) + j] = bi;
            if (j == L) bottleneck[(int64_t)p * S + (s - 1)] = v;
        }
    }
}

// The cut entries of the last stage count, then the boundaries of the requested one.
__global__ void __launch_bounds__(256)
si_finish_kernel(int32_t L, int32_t S, int32_t splits, int64_t cols, const u64* __restrict__ keys,
                 const int32_t* __restrict__ pidx, int64_t* __restrict__ bottleneck, int32_t* __restrict__ cut) {
    const int p = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j <= L) si_decode(L, S, S, splits, cols, p, j, keys, pidx, bottleneck, cut);
}

// The same stage count when no stage is longer than max_len <= kBandMaxLen operators: column j has at most max_len
// candidate rows, so a workgroup takes TJ neighbouring columns and all their rows and finishes them itself -- one
// launch per stage count, nothing to merge afterwards.  A wave instruction covers 64 / TJ rows of the tile's
// columns; the rows go round-robin over the waves.  A candidate travels as one word, (max(dp, T) << 11 | row
// relative to the tile's first row): the value is at most 2^52 and a tile has fewer than 2^11 rows, so the least
// word is the least value at its lowest row -- the merge inside a wave and across the waves is a plain minimum.
constexpr int kBandMaxLen = 1024;
constexpr int kBandRowBits = 11;

template <int TJ, int W, int U>
__global__ void __launch_bounds__(W * 64)
si_band_kernel(int32_t L, int32_t S, int32_t s, int32_t max_len, int64_t ldT, const int64_t* __restrict__ T, int64_t T_bs,
               int64_t cols, const int64_t* __restrict__ prev_all, int64_t* __restrict__ cur_all,
               int64_t* __restrict__ bottleneck, int32_t* __restrict__ cut) {
    constexpr int RPI = 64 / TJ;                 // rows per wave instruction; U rows in flight per lane
    static_assert(W % RPI == 0 && kBandMaxLen + TJ <= (1 << kBandRowBits), "tile does not fit the packed word");
    typedef unsigned long long u64;
    __shared__ u64 skey[W][TJ];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int col = lane % TJ, sub = lane / TJ;
    const int p = blockIdx.y;
    const int64_t* Tp = T + (int64_t)p * T_bs;
    const int64_t* prev = prev_all + (int64_t)p * 2 * cols;
    const int j0 = blockIdx.x * TJ;
    const int j = j0 + col;
    const int jc = j <= L ? j : L;               // a column inside the table for the lanes past its end

    // rows that can matter to this tile: max(s - 1, j0 - max_len) <= i < min(L, last column of the tile)
    const int j_last = j0 + TJ - 1 < L ? j0 + TJ - 1 : L;
    const int i_begin = s - 1 > j0 - max_len ? s - 1 : j0 - max_len;
    const int n_rows = j_last > i_begin ? j_last - i_begin : 0;
    const int n_rounds = (n_rows + W * RPI - 1) / (W * RPI);

    u64 best = ~0ull;
    for (int r0 = 0; r0 < n_rounds; r0 += U) {
        int64_t t[U], a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (r0 + u < n_rounds) {             // uniform over the workgroup
                const int rel = ((r0 + u) * W + wave) * RPI + sub;
                const int i = rel < n_rows ? i_begin + rel : i_begin + n_rows - 1;      // n_rows >= 1 here
                t[u] = Tp[(int64_t)i * ldT + jc];
                a[u] = prev[i];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (r0 + u < n_rounds) {
                const int rel = ((r0 + u) * W + wave) * RPI + sub;
                const int i = i_begin + rel;
                const int64_t tc = t[u] < kInf ? t[u] : kInf;
                const int64_t ac = a[u] < kInf ? a[u] : kInf;
                const int64_t m = ac > tc ? ac : tc;
                const u64 key = ((u64)m << kBandRowBits) | (u64)rel;
                // entries at or left of the diagonal and stages of more than max_len operators do not take part
                const bool ok = rel < n_rows && i < j && j - i <= max_len && j <= L && key < best;
                best = ok ? key : best;
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= TJ; off >>= 1) {
        const u64 o = __shfl_xor(best, off, 64);
        best = o < best ? o : best;
    }
    if (lane < TJ) skey[wave][col] = best;
    __syncthreads();
    if (wave == 0) {
        u64 k = ~0ull;
#pragma unroll
        for (int w = sub; w < W; w += RPI) {
            const u64 o = skey[w][col];
            k = o < k ? o : k;
        }
#pragma unroll
        for (int off = 32; off >= TJ; off >>= 1) {
            const u64 o = __shfl_xor(k, off, 64);
            k = o < k ? o : k;
        }
        if (lane < TJ && j <= L) {
            int64_t v = kInf;
            int32_t bi = -1;
            if (k != ~0ull) {
                v = (int64_t)(k >> kBandRowBits);
                bi = i_begin + (int32_t)(k & ((1u << kBandRowBits) - 1));
            }
            // every candidate infeasible: the lowest i of the whole range s-1 <= i < j holds that minimum
            if (v >= kInf) {
                v = kInf;
                bi = j >= s ? s - 1 : -1;
            }
            cur_all[(int64_t)p * 2 * cols + j] = v;
            cut[((int64_t)p * S + (s - 1)) * (L + 1) + j] = bi;
            if (j == L) bottleneck[(int64_t)p * S + (s - 1)] = v;
        }
    }
}

__global__ void __launch_bounds__(64)
si_bounds_kernel(int32_t B, int32_t L, int32_t S, int32_t s_query, const int32_t* __restrict__ cut,
                 int32_t* __restrict__ bounds) {
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

size_t stage_interval_workspace_bytes(int32_t B, int32_t L, int32_t S) { return si_layout(B, L, S).total; }

hipError_t launch_stage_interval(int32_t B, int32_t L, int32_t S, int32_t max_len, int64_t ldT, const int64_t* T, int64_t* bottleneck,
                                 int32_t* cut, int32_t s_query, int32_t* bounds, void* workspace,
                                 hipStream_t stream) {
    if (B == 0) return hipSuccess;
    const SiLayout lay = si_layout(B, L, S);
    if (max_len > L) max_len = L;
    const int64_t cols = (int64_t)lay.tiles * kSiTile;
    const int64_t T_bs = (int64_t)L * ldT;
    char* ws = static_cast<char*>(workspace);
    int64_t* dp = reinterpret_cast<int64_t*>(ws + lay.dp_off);
    u64* keys = reinterpret_cast<u64*>(ws + lay.key_off);
    int32_t* pidx = reinterpret_cast<int32_t*>(ws + lay.pidx_off);
    // 16 columns and 16 waves: 64 rows per round, five rounds for stages of at most 256 operators (narrower and
    // wider tiles from 8 x 8 waves to 64 x 16 waves were timed: this shape and its neighbours are the fastest)
    constexpr int kBandTile = 16, kBandWaves = 16, kBandInFlight = 8;
    const bool band = max_len <= kBandMaxLen;
    hipLaunchKernelGGL(si_init_kernel, dim3((unsigned)((cols + 255) / 256), B), dim3(256), 0, stream, L, S, max_len, ldT, T,
                       T_bs, cols, dp, band ? nullptr : keys, bottleneck, cut);
    const dim3 grid((unsigned)(lay.tiles * lay.splits), (unsigned)B);
    const dim3 band_grid((unsigned)((L + kBandTile) / kBandTile), (unsigned)B);
    for (int s = 2; s <= S; ++s) {
        if (band) {
            // dp[s-1] sits in buffer (s-1) odd ? 0 : 1 of each problem
            const int64_t* prev_all = dp + (size_t)(s & 1) * cols;
            int64_t* cur_all = dp + (size_t)((s & 1) ^ 1) * cols;
            hipLaunchKernelGGL((si_band_kernel<kBandTile, kBandWaves, kBandInFlight>), band_grid, dim3(kBandWaves * 64), 0,
                               stream, L, S, s, max_len, ldT, T, T_bs, cols, prev_all, cur_all, bottleneck, cut);
            continue;
        }
        hipLaunchKernelGGL(si_step_kernel, grid, dim3(kSiWaves * 64), 0, stream, L, S, s, lay.splits, max_len, ldT, T, T_bs,
                           cols, keys, pidx, bottleneck, cut);
    }
    if (!band && lay.splits > 1 && S >= 2)
        hipLaunchKernelGGL(si_finish_kernel, dim3((unsigned)((L + 256) / 256), (unsigned)B), dim3(256), 0, stream, L, S,
                           lay.splits, cols, keys, pidx, bottleneck, cut);
    if (s_query > 0 && bounds != nullptr)
        hipLaunchKernelGGL(si_bounds_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, B, L, S, s_query, cut, bounds);
    return hipGetLastError();
}

}  // namespace rh

// Dynamic program over an in-tree of operators: every operator feeds exactly one consumer (its parent) and may
// join several inputs; the root feeds nobody.  This is the cone of Sec. 4.3.2 (level 1: given the root's strategy
// the other nodes are optimised by dynamic programming) when inner nodes join several inputs too, with the
// objective of Sec. 4.2 on the tree's edges:
//     v_i[a] = c_i[a] + sum over the inputs j of i of w_j[a]
//     w_i[b] = min_a ( v_i[a] + R_i[a][b] ),  arg_i[b] = lowest such a      (R_i: edge from i to its parent)
// at the root table = v_root, total = its minimum at the lowest strategy; the plan follows arg from the root down.
//
// The tree is cut into runs on the host (plan_tree): a run is a stretch of consecutive nodes f..e in which every
// node but f has the node before it as its only input -- a chain, laid out in memory exactly like the operators of
// rh_minplus_chain.  A run's round is one more than the highest round among the runs that feed f.  One launch per
// round: a workgroup per (run, problem) first adds up what the finished runs hand to f, then walks the run edge
// by edge like the chain kernel and leaves w_e for the run of e's parent.  The backtrack goes through the rounds
// the other way: a run reads the strategy chosen for e's parent and walks down to f.
#include "kernels.h"

#include <vector>

namespace rh {
namespace {

constexpr int kTreeThreads = 512;

__device__ __forceinline__ int64_t sat(int64_t x) { return x < kInf ? x : kInf; }

// A barrier that orders LDS traffic only: loads of the next edge's rows and the stores of arg stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// One run of one problem.  Thread t: column b = t % KP, rows a = t / KP, t / KP + S, ... (S = threads / KP slices);
// the slices' (value, lowest a) candidates meet in LDS, lowest a first among equal values.
template <int KP>
__global__ void __launch_bounds__(KP > kTreeThreads ? KP : kTreeThreads)
tree_run_kernel(int32_t n, int32_t run0, const int32_t* __restrict__ run_first, const int32_t* __restrict__ run_last,
                const int32_t* __restrict__ child_start, const int32_t* __restrict__ child_list,
                const int64_t* __restrict__ c, int64_t c_bs, const int64_t* __restrict__ R, int64_t R_bs,
                uint16_t* __restrict__ arg, int64_t* __restrict__ w, int64_t* __restrict__ total,
                int32_t* __restrict__ root_choice) {
    constexpr int T = KP > kTreeThreads ? KP : kTreeThreads;
    constexpr int S = T / KP;                   // row slices
    __shared__ int64_t v[KP];
    __shared__ int64_t pv[S][KP];
    __shared__ uint16_t pa[S][KP];
    const int tid = threadIdx.x;
    const int b = tid % KP, slice = tid / KP;
    const int u = run0 + blockIdx.x, p = blockIdx.y;
    const int f = run_first[u], e = run_last[u];
    if (f < 0 || e < f || e >= n) return;       // a malformed run table must not lead outside the arrays
    c += (int64_t)p * c_bs;
    R += (int64_t)p * R_bs;
    arg += (int64_t)p * (n - 1) * KP;
    w += (int64_t)p * n * KP;

    // Narrow tables (at most 16 rows per thread): the rows of the next edge of the run wait in registers while this
    // edge is relaxed.
    constexpr int NR = KP >= S ? KP / S : 1;    // rows of an edge table per thread (slices beyond KP rows idle)
    constexpr bool kAhead = NR <= 16;
    int64_t ahead[kAhead ? NR : 1];
    auto fetch = [&](int i) {                   // edge i <= n - 2
        if constexpr (kAhead) {
            const int64_t* Ri = R + (int64_t)i * KP * KP;
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int a = slice + r * S < KP ? slice + r * S : KP - 1;
                ahead[r] = __builtin_nontemporal_load(Ri + (int64_t)a * KP + b);
            }
        }
    };
    if (f < n - 1) fetch(f);

    // v_f = c_f + what every input of f hands up (inputs in ascending order; saturating)
    if (tid < KP) {
        int64_t x = sat(c[(int64_t)f * KP + b]);
        int j0 = child_start[f], j1 = child_start[f + 1];
        j0 = j0 < 0 ? 0 : j0;
        j1 = j1 > n ? n : j1;
        for (int t = j0; t < j1; ++t) {
            const int j = child_list[t];
            if (j >= 0 && j < f) x = sat(x + sat(w[(int64_t)j * KP + b]));
        }
        v[b] = x;
    }
    lds_barrier();

    for (int i = f; i <= e; ++i) {
        if (i == n - 1) {                       // the root: its vector is the table
            if (tid < KP) w[(int64_t)i * KP + b] = v[b];
            if (tid < 64) {
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
                    total[p] = (int64_t)(key >> 10);
                    root_choice[p] = (int32_t)(key & 1023u);
                }
            }
            break;
        }
        // w_i[b] = min_a v_i[a] + R_i[a][b]: this thread's slice of the rows
        const int64_t* Ri = R + (int64_t)i * KP * KP;
        const int64_t c_next = (i < e && tid < KP) ? c[(int64_t)(i + 1) * KP + b] : 0;
        int64_t best = INT64_MAX;
        int besta = 0;
        if constexpr (kAhead) {
            int64_t rows[NR];
#pragma unroll
            for (int r = 0; r < NR; ++r) rows[r] = ahead[r];
            if (i < e && i + 1 < n - 1) fetch(i + 1);
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int a = slice + r * S;
                const int64_t x = v[a < KP ? a : KP - 1] + rows[r];                          // both <= 2^52
                const bool lt = a < KP && x < best;
                best = lt ? x : best;
                besta = lt ? a : besta;
            }
        } else {
#pragma unroll 4
            for (int a = slice; a < KP; a += S) {
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
            for (int s = 1; s < S; ++s) {
                const int64_t x = pv[s][b];
                const int xa = pa[s][b];
                const bool less = x < m || (x == m && xa < ma);
                m = less ? x : m;
                ma = less ? xa : ma;
            }
            const bool dead = m >= kInf;
            arg[(int64_t)i * KP + b] = (uint16_t)(dead ? 0 : ma);
            m = dead ? kInf : m;
            if (i < e) v[b] = sat(sat(c_next) + m);       // node i + 1 has node i as its only input
            else w[(int64_t)i * KP + b] = m;              // handed to the run of i's parent
        }
        lds_barrier();
    }
}

// Plan of the nodes of one run, from its last node down: the last node looks up its parent's strategy (chosen in
// an earlier launch, or the root's choice), every other node that of the node after it.
__global__ void __launch_bounds__(64)
tree_backtrack_kernel(int32_t n, int32_t Kp, int32_t run0, int32_t n_here, const int32_t* __restrict__ run_first,
                      const int32_t* __restrict__ run_last, const int32_t* __restrict__ parent,
                      const uint16_t* __restrict__ arg, const int32_t* __restrict__ root_choice,
                      int32_t* __restrict__ plan) {
    const int t = blockIdx.x * 64 + threadIdx.x;
    const int p = blockIdx.y;
    if (t >= n_here) return;
    const int u = run0 + t;
    const int f = run_first[u], e = run_last[u];
    if (f < 0 || e < f || e >= n) return;
    arg += (int64_t)p * (n - 1) * Kp;
    plan += (int64_t)p * n;
    int i = e, x;
    if (e == n - 1) {
        x = root_choice[p] & (Kp - 1);
        plan[e] = x;
        i = e - 1;
    } else {
        const int par = parent[e];
        x = (par > e && par < n) ? plan[par] & (Kp - 1) : 0;
    }
    for (; i >= f; --i) {
        x = arg[(int64_t)i * Kp + x] & (Kp - 1);         // Kp is a power of two: stay inside the row
        plan[i] = x;
    }
}

}  // namespace

// Runs, rounds and input lists of an in-tree (host arithmetic).  Returns the number of rounds, or -1 if parent is
// not an in-tree numbered inputs-first (parent[i] > i, parent[n-1] = -1).
int plan_tree(int32_t n, const int32_t* parent, int32_t* run_first, int32_t* run_last, int32_t* round_start,
              int32_t* child_start, int32_t* child_list, int32_t* n_runs_out) {
    if (n < 1 || parent[n - 1] != -1) return -1;
    for (int i = 0; i + 1 < n; ++i)
        if (parent[i] <= i || parent[i] >= n) return -1;
    // inputs of every node, ascending (counting sort by parent)
    for (int i = 0; i <= n; ++i) child_start[i] = 0;
    for (int i = 0; i + 1 < n; ++i) ++child_start[parent[i] + 1];
    for (int i = 0; i < n; ++i) child_start[i + 1] += child_start[i];
    std::vector<int32_t> fill(child_start, child_start + n);
    for (int i = 0; i + 1 < n; ++i) child_list[fill[parent[i]]++] = i;
    if (n > 1) child_list[n - 1] = -1;                   // (n - 1 edges; the last slot is unused)
    // a node continues the run of the node before it iff that node is its only input
    std::vector<int32_t> run_of(n), first, last, round;
    for (int i = 0; i < n; ++i) {
        const bool continues = i > 0 && child_start[i + 1] - child_start[i] == 1 && child_list[child_start[i]] == i - 1;
        if (continues) {
            run_of[i] = run_of[i - 1];
            last[run_of[i]] = i;
        } else {
            run_of[i] = (int32_t)first.size();
            first.push_back(i);
            last.push_back(i);
            // inputs come before their consumer, so their runs are complete and have their rounds
            int32_t r = 0;
            for (int t = child_start[i]; t < child_start[i + 1]; ++t) {
                const int32_t rc = round[run_of[child_list[t]]] + 1;
                r = rc > r ? rc : r;
            }
            round.push_back(r);
        }
    }
    const int n_runs = (int)first.size();
    int n_rounds = 0;
    for (int u = 0; u < n_runs; ++u) n_rounds = round[u] + 1 > n_rounds ? round[u] + 1 : n_rounds;
    // runs sorted by round, ascending first node within a round (counting sort)
    for (int t = 0; t <= n_rounds; ++t) round_start[t] = 0;
    for (int u = 0; u < n_runs; ++u) ++round_start[round[u] + 1];
    for (int t = 0; t < n_rounds; ++t) round_start[t + 1] += round_start[t];
    std::vector<int32_t> at(round_start, round_start + n_rounds);
    for (int u = 0; u < n_runs; ++u) {
        const int slot = at[round[u]]++;
        run_first[slot] = first[u];
        run_last[slot] = last[u];
    }
    *n_runs_out = n_runs;
    return n_rounds;
}

hipError_t launch_tree_dp(int32_t B, int32_t n, int32_t Kp, int32_t n_rounds, const int32_t* round_start,
                          const int32_t* run_first, const int32_t* run_last, const int32_t* parent,
                          const int32_t* child_start, const int32_t* child_list, const int64_t* c, int64_t c_bs,
                          const int64_t* R, int64_t R_bs, uint16_t* arg, int64_t* w, int64_t* total,
                          int32_t* root_choice, int32_t* plan, hipStream_t stream) {
    for (int t = 0; t < n_rounds; ++t) {
        const int n_here = round_start[t + 1] - round_start[t];
        if (n_here <= 0) continue;
        const dim3 grid((unsigned)n_here, (unsigned)B);
#define RH_TREE(KP)                                                                                                  \
    hipLaunchKernelGGL(tree_run_kernel<KP>, grid, dim3(KP > kTreeThreads ? KP : kTreeThreads), 0, stream, n,        \
                       round_start[t], run_first, run_last, child_start, child_list, c, c_bs, R, R_bs, arg, w, total, \
                       root_choice)
        switch (Kp) {
            case 16: RH_TREE(16); break;
            case 32: RH_TREE(32); break;
            case 64: RH_TREE(64); break;
            case 128: RH_TREE(128); break;
            case 256: RH_TREE(256); break;
            case 512: RH_TREE(512); break;
            case 1024: RH_TREE(1024); break;
            default: return hipErrorInvalidValue;
        }
#undef RH_TREE
    }
    if (plan != nullptr) {
        for (int t = n_rounds - 1; t >= 0; --t) {
            const int n_here = round_start[t + 1] - round_start[t];
            if (n_here <= 0) continue;
            hipLaunchKernelGGL(tree_backtrack_kernel, dim3((unsigned)((n_here + 63) / 64), (unsigned)B), dim3(64), 0,
                               stream, n, Kp, round_start[t], n_here, run_first, run_last, parent, arg, root_choice,
                               plan);
        }
    }
    return hipGetLastError();
}

}  // namespace rh

/*
 * CPU oracle for plan scoring (TEST INFRASTRUCTURE ONLY).
 *
 * This file is the slow, plain statement of what the GPU library must
 * compute.  It is linked into tests, the smoke check and the bench's CPU
 * baseline leg, and into nothing else; it shares no code, header, table or
 * constant generator with the HIP sources.  Everything is int64 nanoseconds.
 *
 * What follows the paper and where:
 *   - objective C = sum_i comp_i[x_i] + sum_(i,i+1) comm_i[x_i][x_{i+1}]
 *     (Sec. 4.2, "Problem Definition", the equation for C) on a path graph;
 *   - "stitched with dynamic programming" over the linear chain of segments
 *     (Sec. 4.3.2) -> oracle_chain / oracle_backtrack;
 *   - sharding spec (dim, stride), stride = consecutive units per block,
 *     maximum stride = extent / shards, plus "replicate" and "partial"
 *     (Sec. 4.1 and Sec. 4.3.3) -> oracle_owner, oracle_build_reshard;
 *   - sharding applied recursively per device-mesh dimension (Sec. 4);
 *   - resharding by All-Gather / Reduce-Scatter / All-Reduce / All-To-All
 *     when producer and consumer specs differ (Sec. 2.1);
 *   - balanced pipeline stages (Sec. 2.1, Sec. 5.1-5.2) on a chain:
 *     min over cut sets of the max stage sum -> oracle_stage_dp.
 *
 * The paper prints neither the chain recurrence, nor per-collective byte
 * volumes, nor a stage DP.  The readings taken here are:
 *   chain:   v_0 = c_0, v_{i+1}[b] = c_{i+1}[b] + min_a (v_i[a] + R_i[a][b]),
 *            ties -> lowest a, final tie -> lowest b, forward sweep;
 *            INF = 2^52 marks "infeasible", sums saturate at INF;
 *   reshard: per mesh axis, bytes a device must RECEIVE, found by counting
 *            tensor units it needs but does not own; axis 0 converted first,
 *            then axis 1; time = floor(bytes*1000 / bytes_per_us) + alpha;
 *   stages:  dp[1][j] = P(j); dp[s][j] = min_{s-1<=i<j} max(dp[s-1][i],
 *            P(j)-P(i)), ties -> lowest i, no empty stage;
 *   stage time from the intra-stage plan (Sec. 3: each stage's subgraph
 *            gets its own SPMD plan; Sec. 5.1 balances the stages):
 *            T[i][j] = min over plans of operators i..j-1 of the Sec. 4.2
 *            objective on those operators and the edges between them
 *            -> oracle_interval_costs (oracle_interval_costs_banded: no
 *            stage longer than a given number of operators, a limit in
 *            the spirit of the bound tightening of Sec. 5.2; longer
 *            intervals are INF); dp[1][j] = T[0][j], dp[s][j] =
 *            min_{s-1<=i<j} max(dp[s-1][i], T[i][j]), ties -> lowest i
 *            -> oracle_stage_interval.
 *
 * Parity pins (tests, CPU only): brute force over all K^N plans, layered
 * shortest path by a library routine, closed forms, invariances, hand-worked
 * collective volumes, element-level ownership on a tiny tensor, brute force
 * over all cut sets, binary search + greedy for the bottleneck.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_INF ((int64_t)1 << 52)

typedef unsigned __int128 u128;

/* ------------------------------------------------------------------ */
/* saturating non-negative add: anything that reaches INF stays INF    */
static int64_t sat_add(int64_t x, int64_t y)
{
    if (x >= ORC_INF || y >= ORC_INF) return ORC_INF;
    int64_t s = x + y;
    return s >= ORC_INF ? ORC_INF : s;
}

/* ------------------------------------------------------------------ */
/* Chain DP on a path of N operators with Kp (padded) candidates each.  */
/* c: [B][N][Kp] (batch stride c_bs elements), R: [B][N-1][Kp][Kp]      */
/* (batch stride R_bs elements, 0 = one R shared by every problem).     */
/* arg[B][N-1][Kp]: arg_i[b] = minimising a for column b of edge i.     */
static void chain_one(int N, int Kp, const int64_t *c, const int64_t *R,
                      uint16_t *arg, int64_t *vfinal, int64_t *total,
                      int32_t *last)
{
    int64_t *v = (int64_t *)malloc(sizeof(int64_t) * (size_t)Kp);
    int64_t *w = (int64_t *)malloc(sizeof(int64_t) * (size_t)Kp);
    for (int j = 0; j < Kp; ++j) v[j] = c[j] >= ORC_INF ? ORC_INF : c[j];
    for (int i = 0; i + 1 < N; ++i) {
        const int64_t *Ri = R + (size_t)i * Kp * Kp;
        const int64_t *cn = c + (size_t)(i + 1) * Kp;
        for (int b = 0; b < Kp; ++b) {
            int64_t best = sat_add(v[0], Ri[b]);
            int besta = 0;
            for (int a = 1; a < Kp; ++a) {
                int64_t t = sat_add(v[a], Ri[(size_t)a * Kp + b]);
                if (t < best) { best = t; besta = a; }
            }
            w[b] = sat_add(cn[b], best);
            arg[(size_t)i * Kp + b] = (uint16_t)besta;
        }
        int64_t *t = v; v = w; w = t;
    }
    int64_t best = v[0];
    int bestb = 0;
    for (int b = 1; b < Kp; ++b)
        if (v[b] < best) { best = v[b]; bestb = b; }
    if (vfinal) memcpy(vfinal, v, sizeof(int64_t) * (size_t)Kp);
    *total = best;
    *last = bestb;
    free(v);
    free(w);
}

int oracle_chain(int32_t B, int32_t N, int32_t Kp, const int64_t *c,
                 int64_t c_bs, const int64_t *R, int64_t R_bs, uint16_t *arg,
                 int64_t *vfinal, int64_t *total, int32_t *last,
                 int32_t nthreads)
{
    if (B < 0 || N < 1 || Kp < 1 || Kp > 65535) return -1;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int p = 0; p < B; ++p) {
        chain_one(N, Kp, c + (size_t)p * c_bs, R + (size_t)p * R_bs,
                  arg + (size_t)p * (N - 1) * Kp,
                  vfinal ? vfinal + (size_t)p * Kp : NULL, total + p,
                  last + p);
    }
    return 0;
}

/* plan[N-1] = last; plan[i] = arg_i[plan[i+1]]                         */
int oracle_backtrack(int32_t B, int32_t N, int32_t Kp, const uint16_t *arg,
                     const int32_t *last, int32_t *plan)
{
    if (B < 0 || N < 1 || Kp < 1) return -1;
    for (int p = 0; p < B; ++p) {
        const uint16_t *ap = arg + (size_t)p * (N - 1) * Kp;
        int32_t *pl = plan + (size_t)p * N;
        pl[N - 1] = last[p];
        for (int i = N - 2; i >= 0; --i)
            pl[i] = ap[(size_t)i * Kp + pl[i + 1]];
    }
    return 0;
}

/* The objective itself, for one given plan (Sec. 4.2, equation for C). */
int64_t oracle_plan_cost(int32_t N, int32_t Kp, const int64_t *c,
                         const int64_t *R, const int32_t *plan)
{
    int64_t s = 0;
    for (int i = 0; i < N; ++i) s = sat_add(s, c[(size_t)i * Kp + plan[i]]);
    for (int i = 0; i + 1 < N; ++i)
        s = sat_add(s, R[((size_t)i * Kp + plan[i]) * Kp + plan[i + 1]]);
    return s;
}

/* ------------------------------------------------------------------ */
/* Cone: one root operator with several inputs, every other node has   */
/* exactly one input (Sec. 4.3.2, level 1), i.e. n_br chains ("branches")*/
/* that end in the root.  For each root strategy r the best strategies  */
/* of all other nodes are found branch by branch:                       */
/*   table[r] = c_root[r] + sum_b min over plans of branch b of         */
/*              ( sum c + sum R along the branch + R_last->root[.][r] ) */
/* Branch b has len[b] >= 1 operators with tables cb[b] ([len][Kp]) and */
/* Rb[b] ([len][Kp][Kp], the last table is the edge into the root).     */
/* branch_plan[b][len[b]] is the plan of branch b for the best root     */
/* strategy (lowest index on ties, per branch the same tie rule as the  */
/* chain).                                                              */
int oracle_cone(int32_t n_br, int32_t Kp, const int32_t *len,
                const int64_t *const *cb, const int64_t *const *Rb,
                const int64_t *c_root, int64_t *table, int64_t *total,
                int32_t *root_choice, int32_t *const *branch_plan)
{
    if (n_br < 0 || Kp < 1) return -1;
    int64_t *w = (int64_t *)malloc(sizeof(int64_t) * (size_t)Kp);
    int64_t *v = (int64_t *)malloc(sizeof(int64_t) * (size_t)Kp);
    uint16_t **args = (uint16_t **)malloc(sizeof(uint16_t *) * (size_t)(n_br > 0 ? n_br : 1));
    for (int r = 0; r < Kp; ++r) table[r] = c_root[r] >= ORC_INF ? ORC_INF : c_root[r];
    for (int b = 0; b < n_br; ++b) {
        const int n = len[b];
        args[b] = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)n * Kp);
        for (int j = 0; j < Kp; ++j) v[j] = cb[b][j] >= ORC_INF ? ORC_INF : cb[b][j];
        for (int i = 0; i < n; ++i) {
            const int64_t *Ri = Rb[b] + (size_t)i * Kp * Kp;
            for (int x = 0; x < Kp; ++x) {
                int64_t best = sat_add(v[0], Ri[x]);
                int besta = 0;
                for (int a = 1; a < Kp; ++a) {
                    int64_t t = sat_add(v[a], Ri[(size_t)a * Kp + x]);
                    if (t < best) { best = t; besta = a; }
                }
                args[b][(size_t)i * Kp + x] = (uint16_t)besta;
                /* inside the branch the next operator's own cost is added; the */
                /* root's cost is added once, outside */
                w[x] = i + 1 < n ? sat_add(cb[b][(size_t)(i + 1) * Kp + x], best) : best;
            }
            memcpy(v, w, sizeof(int64_t) * (size_t)Kp);
        }
        for (int r = 0; r < Kp; ++r) table[r] = sat_add(table[r], v[r]);
    }
    int64_t best = table[0];
    int bestr = 0;
    for (int r = 1; r < Kp; ++r)
        if (table[r] < best) { best = table[r]; bestr = r; }
    *total = best;
    *root_choice = bestr;
    for (int b = 0; b < n_br; ++b) {
        int x = bestr;
        for (int i = len[b] - 1; i >= 0; --i) {
            x = args[b][(size_t)i * Kp + x];
            branch_plan[b][i] = x;
        }
        free(args[b]);
    }
    free(args); free(w); free(v);
    return 0;
}

/* ------------------------------------------------------------------ */
/* In-tree: every operator feeds exactly one consumer (its parent) and   */
/* may have several inputs; the root feeds nobody.  This is the shape of */
/* a cone whose inner nodes also join several inputs (Sec. 4.3.2, level  */
/* 1), and the objective is that of Sec. 4.2 with the tree's edges as E: */
/*   C = sum_i c_i[x_i] + sum_{i != root} R_i[x_i][x_parent(i)]          */
/* (R_i is the table of the edge from i to its parent: row = strategy of */
/* i, column = strategy of the parent).  By recursion over the parent    */
/* array, for a node i:                                                  */
/*   v_i[a] = c_i[a] + sum over the inputs j of i of w_j[a]              */
/*   w_i[b] = min_a ( v_i[a] + R_i[a][b] ),  arg_i[b] = lowest such a    */
/*            (0 if every candidate is infeasible)                       */
/* with saturating sums; at the root table = v_root, total = its minimum */
/* at the lowest r; the plan follows the args from the root down.  Nodes */
/* are numbered so that parent[i] > i (inputs before consumers), the     */
/* root is node n-1 and has parent -1; the inputs of a node are added in */
/* ascending order (saturating addition of non-negative costs does not   */
/* depend on the order).                                                 */
static void tree_node_vector(int32_t n, int32_t Kp, const int32_t *parent,
                             const int64_t *c, const int64_t *R, int i,
                             int64_t *v_all, uint16_t *arg_all)
{
    int64_t *v = v_all + (size_t)i * Kp;
    for (int a = 0; a < Kp; ++a) {
        const int64_t x = c[(size_t)i * Kp + a];
        v[a] = x >= ORC_INF ? ORC_INF : x;
    }
    for (int j = 0; j < n; ++j) {
        if (parent[j] != i) continue;
        /* the input's own vector first (recursion), then what it costs */
        /* this node per strategy b of this node                        */
        tree_node_vector(n, Kp, parent, c, R, j, v_all, arg_all);
        const int64_t *vj = v_all + (size_t)j * Kp;
        const int64_t *Rj = R + (size_t)j * Kp * Kp;
        for (int b = 0; b < Kp; ++b) {
            int64_t best = sat_add(vj[0], Rj[b]);
            int besta = 0;
            for (int a = 1; a < Kp; ++a) {
                const int64_t t = sat_add(vj[a], Rj[(size_t)a * Kp + b]);
                if (t < best) { best = t; besta = a; }
            }
            arg_all[(size_t)j * Kp + b] = (uint16_t)(best >= ORC_INF ? 0 : besta);
            v[b] = sat_add(v[b], best);
        }
    }
}

/* c[n][Kp], R[n-1][Kp][Kp] (entry i = edge from node i to parent[i]);   */
/* outputs: table[Kp], *total, *root_choice, plan[n], and optionally     */
/* arg[n-1][Kp] (may be NULL).  Returns -1 on a malformed parent array.  */
int oracle_tree(int32_t n, int32_t Kp, const int32_t *parent, const int64_t *c,
                const int64_t *R, int64_t *table, int64_t *total,
                int32_t *root_choice, int32_t *plan, uint16_t *arg)
{
    if (n < 1 || Kp < 1 || parent[n - 1] != -1) return -1;
    for (int i = 0; i + 1 < n; ++i)
        if (parent[i] <= i || parent[i] >= n) return -1;
    int64_t *v_all = (int64_t *)malloc(sizeof(int64_t) * (size_t)n * Kp);
    uint16_t *arg_all = (uint16_t *)calloc((size_t)n * Kp, sizeof(uint16_t));
    tree_node_vector(n, Kp, parent, c, R, n - 1, v_all, arg_all);
    const int64_t *vr = v_all + (size_t)(n - 1) * Kp;
    int64_t best = vr[0];
    int bestr = 0;
    for (int r = 0; r < Kp; ++r) {
        table[r] = vr[r];
        if (vr[r] < best) { best = vr[r]; bestr = r; }
    }
    *total = best;
    *root_choice = best >= ORC_INF ? 0 : bestr;
    plan[n - 1] = *root_choice;
    for (int i = n - 2; i >= 0; --i)   /* parent[i] > i: the parent's entry is there already */
        plan[i] = arg_all[(size_t)i * Kp + plan[parent[i]]];
    if (arg != NULL) memcpy(arg, arg_all, sizeof(uint16_t) * (size_t)(n - 1) * Kp);
    free(v_all); free(arg_all);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Memory-constrained search (Sec. 4.4).  Parameters are ranked by size, */
/* largest first (equal sizes: lower operator index first); for          */
/* k = k0 .. k0+n_k-1 the candidates that replicate one of the k largest */
/* parameters are removed (cost INF), the chain is solved, and the plan  */
/* is feasible if it exists and its parameter memory fits the limit.     */
/*   param_bytes[N]  size of operator i's parameter tensor (0: none)     */
/*   repl[N][Kp]     1 if candidate j of operator i replicates it        */
/*   mem[N][Kp]      bytes per device that candidate j keeps for it      */
/* Outputs per k: total[n_k], plan[n_k][N], plan_mem[n_k]; *first = the  */
/* smallest offset k-k0 whose plan is feasible, or -1.                   */
int oracle_memory_sweep(int32_t N, int32_t Kp, int32_t n_k, int32_t k0,
                        const int64_t *c, const int64_t *R,
                        const int64_t *param_bytes, const uint8_t *repl,
                        const int64_t *mem, int64_t limit, int64_t *total,
                        int32_t *plan, int64_t *plan_mem, int32_t *first)
{
    if (N < 1 || Kp < 1 || n_k < 0 || k0 < 0) return -1;
    int32_t *rank = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    for (int i = 0; i < N; ++i) {
        int r = 0;
        for (int l = 0; l < N; ++l)
            if (param_bytes[l] > param_bytes[i] || (param_bytes[l] == param_bytes[i] && l < i)) ++r;
        rank[i] = r;
    }
    int64_t *cm = (int64_t *)malloc(sizeof(int64_t) * (size_t)N * Kp);
    uint16_t *arg = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)(N > 1 ? N - 1 : 1) * Kp);
    *first = -1;
    for (int t = 0; t < n_k; ++t) {
        const int k = k0 + t;
        for (int i = 0; i < N; ++i)
            for (int j = 0; j < Kp; ++j) {
                const size_t x = (size_t)i * Kp + j;
                /* only operators that own a parameter can be marked */
                cm[x] = (rank[i] < k && param_bytes[i] > 0 && repl[x]) ? ORC_INF : c[x];
            }
        int32_t last;
        chain_one(N, Kp, cm, R, arg, NULL, total + t, &last);
        int32_t *pl = plan + (size_t)t * N;
        pl[N - 1] = last;
        for (int i = N - 2; i >= 0; --i) pl[i] = arg[(size_t)i * Kp + pl[i + 1]];
        int64_t m = 0;
        for (int i = 0; i < N; ++i) m += mem[(size_t)i * Kp + pl[i]];
        plan_mem[t] = m;
        if (*first < 0 && total[t] < ORC_INF && m <= limit) *first = t;
    }
    free(rank); free(cm); free(arg);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Pipeline stages on a chain of L segments.                            */
/* bottleneck[B][S]: entry s-1 = dp[s][L].  cut[B][S][L+1]: entry       */
/* [s-1][j] = minimising i (lowest on ties), 0 for s = 1, -1 where      */
/* j < s (no split of j segments into s non-empty stages exists).       */
/* bounds[B][s_query+1] (optional): stage t covers segments             */
/* [bounds[t-1], bounds[t]).                                            */
int oracle_stage_dp(int32_t B, int32_t L, int32_t S, const int64_t *cost,
                    int64_t *bottleneck, int32_t *cut, int32_t s_query,
                    int32_t *bounds, int32_t nthreads)
{
    if (B < 0 || L < 1 || S < 1 || S > L) return -1;
    if (s_query < 0 || s_query > S) return -1;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int p = 0; p < B; ++p) {
        const int64_t *cs = cost + (size_t)p * L;
        int32_t *ct = cut + (size_t)p * S * (L + 1);
        int64_t *P = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
        int64_t *prev = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
        int64_t *cur = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
        P[0] = 0;
        for (int l = 0; l < L; ++l) P[l + 1] = P[l] + cs[l];
        /* one stage: the stage is the whole prefix */
        for (int j = 0; j <= L; ++j) {
            prev[j] = P[j];
            ct[j] = j >= 1 ? 0 : -1;
        }
        bottleneck[(size_t)p * S] = prev[L];
        for (int s = 2; s <= S; ++s) {
            int32_t *cts = ct + (size_t)(s - 1) * (L + 1);
            for (int j = 0; j <= L; ++j) {
                if (j < s) { cur[j] = ORC_INF; cts[j] = -1; continue; }
                int64_t best = ORC_INF;
                int besti = -1;
                for (int i = s - 1; i < j; ++i) {
                    int64_t tail = P[j] - P[i];
                    int64_t m = prev[i] > tail ? prev[i] : tail;
                    if (besti < 0 || m < best) { best = m; besti = i; }
                }
                cur[j] = best;
                cts[j] = besti;
            }
            bottleneck[(size_t)p * S + (s - 1)] = cur[L];
            int64_t *t = prev; prev = cur; cur = t;
        }
        if (bounds && s_query > 0) {
            int32_t *bd = bounds + (size_t)p * (s_query + 1);
            bd[s_query] = L;
            for (int t = s_query; t >= 1; --t)
                bd[t - 1] = ct[(size_t)(t - 1) * (L + 1) + bd[t]];
        }
        free(P); free(prev); free(cur);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Stage time of every interval of one operator chain.                  */
/* c[L][Kp], R[L-1][Kp][Kp]; T[i*ldT + j] for 0 <= i < L, 0 <= j <= L:   */
/* the least objective over the plans of operators i..j-1 alone (their  */
/* node costs and the edges between them), INF where j <= i.            */
/* Written out start by start: a forward sweep from operator i, whose   */
/* running minimum after operator j-1 is T[i][j].                       */
static int interval_rows(int32_t L, int32_t Kp, int32_t max_len,
                         const int64_t *c, const int64_t *R, int64_t ldT,
                         int64_t *T, int32_t nthreads)
{
    if (L < 1 || Kp < 1 || max_len < 1 || ldT < (int64_t)L + 1) return -1;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int i = 0; i < L; ++i) {
        int64_t *row = T + (size_t)i * (size_t)ldT;
        int64_t *v = (int64_t *)malloc(sizeof(int64_t) * (size_t)Kp);
        int64_t *w = (int64_t *)malloc(sizeof(int64_t) * (size_t)Kp);
        for (int j = 0; j <= L; ++j) row[j] = ORC_INF;
        for (int b = 0; b < Kp; ++b) {
            int64_t x = c[(size_t)i * Kp + b];
            v[b] = x >= ORC_INF ? ORC_INF : x;
        }
        for (int l = i; l < L && l - i < max_len; ++l) {
            /* v = cost vector of the chain i..l by the strategy of operator l */
            int64_t best = v[0];
            for (int b = 1; b < Kp; ++b) if (v[b] < best) best = v[b];
            row[l + 1] = best;
            if (l + 1 == L) break;
            const int64_t *Rl = R + (size_t)l * Kp * Kp;
            const int64_t *cn = c + (size_t)(l + 1) * Kp;
            for (int b = 0; b < Kp; ++b) {
                int64_t m = sat_add(v[0], Rl[b]);
                for (int a = 1; a < Kp; ++a) {
                    int64_t t = sat_add(v[a], Rl[(size_t)a * Kp + b]);
                    if (t < m) m = t;
                }
                w[b] = sat_add(cn[b], m);
            }
            int64_t *t = v; v = w; w = t;
        }
        free(v); free(w);
    }
    return 0;
}

int oracle_interval_costs(int32_t L, int32_t Kp, const int64_t *c,
                          const int64_t *R, int64_t ldT, int64_t *T,
                          int32_t nthreads)
{
    return interval_rows(L, Kp, L, c, R, ldT, T, nthreads);
}

/* The same table when no stage may hold more than max_len operators    */
/* (Sec. 5.2 keeps every operator within a tolerance of the stage that   */
/* perfect balance gives it, so a stage cannot stretch over arbitrarily  */
/* many operators; here the caller states the limit): T[i][j] = INF for  */
/* j - i > max_len, the entries with j - i <= max_len as above.          */
int oracle_interval_costs_banded(int32_t L, int32_t Kp, int32_t max_len,
                                 const int64_t *c, const int64_t *R,
                                 int64_t ldT, int64_t *T, int32_t nthreads)
{
    return interval_rows(L, Kp, max_len, c, R, ldT, T, nthreads);
}

/* ------------------------------------------------------------------ */
/* Balanced stages when the time of stage [i, j) is a table entry        */
/* T[i*ldT + j] (any values in [0, INF], INF = the stage cannot run).   */
/* dp[1][j] = T[0][j]; dp[s][j] = min_{s-1<=i<j} max(dp[s-1][i], T[i][j]) */
/* with the lowest minimising i; dp = INF, cut = -1 for j < s.          */
/* T: [B][L][ldT]; outputs as oracle_stage_dp.                          */
int oracle_stage_interval(int32_t B, int32_t L, int32_t S, int64_t ldT,
                          const int64_t *T, int64_t *bottleneck, int32_t *cut,
                          int32_t s_query, int32_t *bounds, int32_t nthreads)
{
    if (B < 0 || L < 1 || S < 1 || S > L || ldT < (int64_t)L + 1) return -1;
    if (s_query < 0 || s_query > S) return -1;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int p = 0; p < B; ++p) {
        const int64_t *Tp = T + (size_t)p * (size_t)L * (size_t)ldT;
        int32_t *ct = cut + (size_t)p * S * (L + 1);
        int64_t *prev = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
        int64_t *cur = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
        prev[0] = ORC_INF;
        ct[0] = -1;
        for (int j = 1; j <= L; ++j) {
            prev[j] = Tp[j] >= ORC_INF ? ORC_INF : Tp[j];
            ct[j] = 0;
        }
        bottleneck[(size_t)p * S] = prev[L];
        for (int s = 2; s <= S; ++s) {
            int32_t *cts = ct + (size_t)(s - 1) * (L + 1);
            for (int j = 0; j <= L; ++j) {
                if (j < s) { cur[j] = ORC_INF; cts[j] = -1; continue; }
                int64_t best = 0;
                int besti = -1;
                for (int i = s - 1; i < j; ++i) {
                    int64_t t = Tp[(size_t)i * (size_t)ldT + j];
                    if (t > ORC_INF) t = ORC_INF;
                    int64_t m = prev[i] > t ? prev[i] : t;
                    if (besti < 0 || m < best) { best = m; besti = i; }
                }
                cur[j] = best;
                cts[j] = besti;
            }
            bottleneck[(size_t)p * S + (s - 1)] = cur[L];
            int64_t *t = prev; prev = cur; cur = t;
        }
        if (bounds && s_query > 0) {
            int32_t *bd = bounds + (size_t)p * (s_query + 1);
            bd[s_query] = L;
            for (int t = s_query; t >= 1; --t)
                bd[t - 1] = ct[(size_t)(t - 1) * (L + 1) + bd[t]];
        }
        free(prev); free(cur);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Pipeline stages with boundary transfers and bound tightening         */
/* (Sec. 5.1: a tensor that crosses a stage boundary is communicated;   */
/* Sec. 5.2: every operator must sit within a tolerance eps of the stage */
/* that perfect balance would give it).  On a chain of L segments split  */
/* into exactly d stages, with time_per_stage = P(L)/d:                  */
/*   stage t = segments [i, j) takes P(j) - P(i) + (i > 0 ? xfer[i] : 0) */
/*   segment l may sit in stage t only if                                */
/*       floor(P(l)/tps - eps) <= t <= ceil(P(l)/tps + eps)              */
/*   (the accumulated time of the segments before l is both its earliest */
/*   and, on a chain, its latest start), eps = eps_num/eps_den >= 0;     */
/*   eps_num < 0 switches the bounds off.                                */
/* dp[1][j] = P(j); dp[s][j] = min over allowed i of                     */
/*   max(dp[s-1][i], P(j) - P(i) + xfer[i]), lowest i on ties.           */
/* bottleneck[p] = dp[d][L] (INF if the bounds allow no split);          */
/* cut[p][s-1][j] = minimising i or -1; bounds[p][0..d] or all -1.       */
static int64_t floor_div128(__int128 a, __int128 b) { /* b > 0 */
    __int128 q = a / b;
    if ((a % b != 0) && (a < 0)) --q;
    return (int64_t)q;
}

int oracle_stage_window(int32_t B, int32_t L, int32_t d, const int64_t *cost,
                        const int64_t *xfer, int64_t eps_num, int64_t eps_den,
                        int64_t *bottleneck, int32_t *cut, int32_t *bounds)
{
    if (B < 0 || L < 1 || d < 1 || d > L || eps_den < 1) return -1;
    for (int p = 0; p < B; ++p) {
        const int64_t *cs = cost + (size_t)p * L;
        const int64_t *xf = xfer ? xfer + (size_t)p * (L + 1) : NULL;
        int32_t *ct = cut + (size_t)p * d * (L + 1);
        int64_t *P = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
        int32_t *lo = (int32_t *)malloc(sizeof(int32_t) * (size_t)L);
        int32_t *hi = (int32_t *)malloc(sizeof(int32_t) * (size_t)L);
        int64_t *prev = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
        int64_t *cur = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
        P[0] = 0;
        for (int l = 0; l < L; ++l) P[l + 1] = P[l] + cs[l];
        for (int l = 0; l < L; ++l) {
            lo[l] = 0; hi[l] = d - 1;
            if (eps_num >= 0 && P[L] > 0) {
                /* P(l)/tps -+ eps = (P(l)*d*den -+ num*P(L)) / (P(L)*den) */
                __int128 x = (__int128)P[l] * d * eps_den, e = (__int128)eps_num * P[L];
                __int128 den = (__int128)P[L] * eps_den;
                int64_t f = floor_div128(x - e, den);
                int64_t c = -floor_div128(-(x + e), den);
                lo[l] = (int32_t)(f < 0 ? 0 : (f > d - 1 ? d - 1 : f));
                hi[l] = (int32_t)(c > d - 1 ? d - 1 : (c < 0 ? 0 : c));
                if (f > d - 1) lo[l] = d;          /* no stage is late enough: never allowed */
            }
        }
        for (int j = 0; j <= L; ++j) {
            /* one stage so far (stage 0 = segments [0, j)) */
            int ok = j >= 1 && lo[j - 1] <= 0;
            prev[j] = ok ? P[j] : ORC_INF;
            ct[j] = ok ? 0 : -1;
        }
        for (int s = 2; s <= d; ++s) {
            int32_t *cts = ct + (size_t)(s - 1) * (L + 1);
            for (int j = 0; j <= L; ++j) {
                int64_t best = ORC_INF;
                int besti = -1;
                if (j >= s && lo[j - 1] <= s - 1) {
                    for (int i = s - 1; i < j; ++i) {
                        if (hi[i] < s - 1 || prev[i] >= ORC_INF) continue;
                        int64_t t = P[j] - P[i] + (xf ? xf[i] : 0);
                        int64_t m = prev[i] > t ? prev[i] : t;
                        if (m < best) { best = m; besti = i; }
                    }
                }
                cur[j] = besti < 0 ? ORC_INF : best;
                cts[j] = besti;
            }
            int64_t *t = prev; prev = cur; cur = t;
        }
        bottleneck[p] = prev[L];
        if (bounds) {
            int32_t *bd = bounds + (size_t)p * (d + 1);
            if (prev[L] >= ORC_INF) {
                for (int t = 0; t <= d; ++t) bd[t] = -1;
            } else {
                bd[d] = L;
                for (int t = d; t >= 1; --t) bd[t - 1] = ct[(size_t)(t - 1) * (L + 1) + bd[t]];
            }
        }
        free(P); free(lo); free(hi); free(prev); free(cur);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Sharding specs.  One byte per mesh axis inside a 32-bit word         */
/* (axis 0 = bits 0..7, axis 1 = bits 8..15):                           */
/*   bits 0..1 state: 0 replicate, 1 split, 2 partial (3 = invalid)     */
/*   bits 2..4 dim   (tensor dimension that is split, 0..3)             */
/*   bits 5..7 lgdiv (stride = (extent / m) >> lgdiv)                   */
/* 0xFFFFFFFF marks an empty (padding) slot.                            */
enum { ST_R = 0, ST_S = 1, ST_P = 2 };

typedef struct {
    int valid;
    int state[2];
    int dim[2];
    int64_t stride[2];
} spec_t;

/* unit u of a dimension split with the given stride over m shards      */
/* belongs to shard (u div stride) mod m  (Sec. 4.1: stride = number of */
/* consecutive units per block)                                         */
int64_t oracle_owner(int64_t u, int64_t stride, int64_t m)
{
    return (u / stride) % m;
}

static spec_t decode_spec(uint32_t w, const int64_t *dims, const int32_t *m,
                          int naxes)
{
    spec_t s;
    memset(&s, 0, sizeof s);
    s.valid = 1;
    if (w == 0xFFFFFFFFu) { s.valid = 0; return s; }
    for (int x = 0; x < 2; ++x) {
        unsigned byte = (w >> (8 * x)) & 0xFFu;
        int st = byte & 3, d = (byte >> 2) & 7, lg = (byte >> 5) & 7;
        s.state[x] = ST_R; s.dim[x] = 0; s.stride[x] = 0;
        if (x >= naxes) continue;          /* axis not present: ignored */
        if (st == 3) { s.valid = 0; return s; }
        s.state[x] = st;
        if (st == ST_S) {
            if (d > 3) { s.valid = 0; return s; }
            int64_t n = dims[d];
            int64_t blocks = (int64_t)m[x] << lg;
            if (n % blocks != 0) { s.valid = 0; return s; }
            s.dim[x] = d;
            s.stride[x] = n / blocks;      /* (n / m) >> lg, exact */
        }
    }
    if (naxes == 2 && s.state[0] == ST_S && s.state[1] == ST_S &&
        s.dim[0] == s.dim[1])
        s.valid = 0;                       /* one dim on both axes: not a candidate */
    return s;
}

static int64_t shards_of(const spec_t *s, int x, const int32_t *m)
{
    return s->state[x] == ST_S ? m[x] : 1;
}

/* Bytes one device receives on one mesh axis of size m when its local  */
/* tensor of T bytes goes from state p to state q.  Returns -1 if the   */
/* transition cannot be done.  Found by counting units.                 */
static int64_t axis_bytes(int ps, int pd, int64_t pst, int qs, int qd,
                          int64_t qst, const int64_t *dims, int64_t m,
                          int64_t T)
{
    if (ps == qs && (ps != ST_S || (pd == qd && pst == qst))) return 0;
    if (qs == ST_P) return -1;             /* nothing turns into "partial" */
    if (ps == ST_R) return 0;              /* replicate -> split: local slice */
    if (ps == ST_S && qs == ST_R) {
        /* all-gather: device 0 needs every unit, owns some */
        int64_t n = dims[pd], missing = 0;
        for (int64_t u = 0; u < n; ++u)
            if (oracle_owner(u, pst, m) != 0) ++missing;
        return (int64_t)((u128)T * (u128)missing / (u128)n);
    }
    if (ps == ST_S && qs == ST_S && pd == qd) {
        /* same dim, other stride: a unit stays iff both layouts put it  */
        /* on the same device; per-device average of the moved units     */
        int64_t n = dims[pd], keep = 0;
        for (int64_t u = 0; u < n; ++u)
            if (oracle_owner(u, pst, m) == oracle_owner(u, qst, m)) ++keep;
        return (int64_t)((u128)T * (u128)(n - keep) / ((u128)n * (u128)m));
    }
    if (ps == ST_S && qs == ST_S) {
        /* other dim: device 0 needs its slab of dim qd and already owns */
        /* the part of it that lies in its slab of dim pd                */
        int64_t n1 = dims[pd], n2 = dims[qd], need = 0, foreign = 0;
        for (int64_t u = 0; u < n2; ++u)
            if (oracle_owner(u, qst, m) == 0) ++need;
        for (int64_t u = 0; u < n1; ++u)
            if (oracle_owner(u, pst, m) != 0) ++foreign;
        return (int64_t)((u128)T * (u128)need * (u128)foreign /
                         ((u128)n1 * (u128)n2));
    }
    if (ps == ST_P && qs == ST_S) {
        /* reduce-scatter: every needed unit takes m-1 remote partials   */
        int64_t n = dims[qd], need = 0;
        for (int64_t u = 0; u < n; ++u)
            if (oracle_owner(u, qst, m) == 0) ++need;
        return (int64_t)((u128)T * (u128)need * (u128)(m - 1) / (u128)n);
    }
    /* partial -> replicate: all-reduce = reduce-scatter + all-gather,  */
    /* each moving (m-1)/m of the local bytes                            */
    int64_t half = (int64_t)((u128)T * (u128)(m - 1) / (u128)m);
    return half + half;
}

/* mesh given as plain arrays: m[2], bw_bytes_per_us[2], alpha_ns[2]    */
/* K[n_edges+1]: real candidate counts; slots >= K[i] are padding.      */
/* dims[n_edges][4], elem_bytes[n_edges] describe the tensor on edge i, */
/* produced by operator i (out_spec[i][a]) and consumed by operator     */
/* i+1 (in_spec[i+1][b]).  R[n_edges][Kp][Kp].                          */
int oracle_build_reshard(int32_t naxes, const int32_t *m,
                         const int64_t *bw_bytes_per_us,
                         const int64_t *alpha_ns, int32_t n_edges, int32_t Kp,
                         const int32_t *K, const uint32_t *out_spec,
                         const uint32_t *in_spec, const int64_t *dims,
                         const int32_t *elem_bytes, int64_t *R)
{
    if (naxes < 1 || naxes > 2 || n_edges < 0 || Kp < 1) return -1;
    const size_t memo_n = 2u * 256u * 256u * 2u;
    int32_t *memo_edge = (int32_t *)calloc(memo_n, sizeof(int32_t));
    int64_t *memo_T = (int64_t *)calloc(memo_n, sizeof(int64_t));
    int64_t *memo_V = (int64_t *)calloc(memo_n, sizeof(int64_t));
    for (int e = 0; e < n_edges; ++e) {
        const int64_t *dm = dims + (size_t)e * 4;
        int64_t total = elem_bytes[e];
        for (int d = 0; d < 4; ++d) total *= dm[d];
        spec_t *ps = (spec_t *)malloc(sizeof(spec_t) * (size_t)Kp);
        spec_t *qs = (spec_t *)malloc(sizeof(spec_t) * (size_t)Kp);
        for (int j = 0; j < Kp; ++j) {
            ps[j] = decode_spec(out_spec[(size_t)e * Kp + j], dm, m, naxes);
            qs[j] = decode_spec(in_spec[(size_t)(e + 1) * Kp + j], dm, m, naxes);
            if (j >= K[e]) ps[j].valid = 0;
            if (j >= K[e + 1]) qs[j].valid = 0;
        }
        for (int a = 0; a < Kp; ++a)
            for (int b = 0; b < Kp; ++b) {
                int64_t *out = R + ((size_t)e * Kp + a) * Kp + b;
                if (!ps[a].valid || !qs[b].valid) { *out = ORC_INF; continue; }
                int64_t t = 0;
                for (int x = 0; x < naxes && t < ORC_INF; ++x) {
                    /* axes before x already hold q, axes after x still p */
                    int64_t sh = 1;
                    for (int y = 0; y < x; ++y) sh *= shards_of(&qs[b], y, m);
                    for (int y = x + 1; y < naxes; ++y) sh *= shards_of(&ps[a], y, m);
                    int64_t T = total / sh;
                    /* identical arguments recur K^2 times per edge: keep  */
                    /* the counted result per (axis, p byte, q byte, T)    */
                    unsigned pb = (out_spec[(size_t)e * Kp + a] >> (8 * x)) & 0xFFu;
                    unsigned qb = (in_spec[(size_t)(e + 1) * Kp + b] >> (8 * x)) & 0xFFu;
                    size_t slot = (((size_t)x * 256 + pb) * 256 + qb) * 2 + (sh > 1);
                    int64_t V;
                    if (memo_edge[slot] == e + 1 && memo_T[slot] == T) {
                        V = memo_V[slot];
                    } else {
                        V = axis_bytes(ps[a].state[x], ps[a].dim[x],
                                       ps[a].stride[x], qs[b].state[x],
                                       qs[b].dim[x], qs[b].stride[x], dm,
                                       m[x], T);
                        memo_edge[slot] = e + 1; memo_T[slot] = T; memo_V[slot] = V;
                    }
                    if (V < 0) { t = ORC_INF; break; }
                    if (V > 0) {
                        int64_t ns = (int64_t)((u128)V * 1000u /
                                               (u128)bw_bytes_per_us[x]) +
                                     alpha_ns[x];
                        t = sat_add(t, ns);
                    }
                }
                *out = t;
            }
        free(ps); free(qs);
    }
    free(memo_edge); free(memo_T); free(memo_V);
    return 0;
}

/* received bytes only (no time), one axis, for hand-worked volume pins */
int64_t oracle_axis_bytes(uint32_t p_byte, uint32_t q_byte,
                          const int64_t *dims, int32_t m, int64_t T)
{
    int32_t mm[2] = { m, 1 };
    spec_t p = decode_spec(p_byte & 0xFFu, dims, mm, 1);
    spec_t q = decode_spec(q_byte & 0xFFu, dims, mm, 1);
    if (!p.valid || !q.valid) return -2;
    return axis_bytes(p.state[0], p.dim[0], p.stride[0], q.state[0], q.dim[0],
                      q.stride[0], dims, m, T);
}

int32_t oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * rhino.h -- plan scoring for automatic parallelization, C ABI.
 *
 * The library scores candidate parallel execution plans of a linearised
 * operator graph, as the strategy search of "Auto-Parallelizing Large Models
 * with Rhino" (arXiv 2302.08141) needs it:
 *
 *   operators i = 0..N-1, operator i has K_i candidate sharding strategies;
 *   comp cost c_i[j] per (operator, strategy) and comm cost R_i[a][b] per
 *   (edge i -> i+1, strategy pair)          -- Sec. 4.2, "Problem Definition";
 *   the plan minimising C = sum c_i[x_i] + sum R_i[x_i][x_{i+1}] on the
 *   chain is found by dynamic programming   -- Sec. 4.3.2 (cones, and the
 *   linear chain of segments between critical nodes).
 *
 * All costs are int64 nanoseconds.  All pointers are DEVICE pointers unless a
 * parameter says "host".  The caller owns every buffer; the library allocates
 * nothing and keeps no state between calls (one entry point,
 * rh_stage_dp_window_static, works on a static device array of its own
 * instead of a workspace: see there).  Every call only enqueues kernels on `stream`
 * (a hipStream_t passed as void*, NULL = the default stream) and returns; the
 * caller synchronises.  Calls on different streams may run concurrently.
 * Return value: RH_OK or a negative RH_ERR_* code; argument errors are found
 * on the host before anything is launched, so a failing call writes nothing.
 *
 * Entry points, in the order of a search:
 *   rh_build_reshard                      edge tables from sharding specs
 *   rh_minplus_chain, rh_backtrack        chain DP and its plan (tables in memory)
 *   rh_minplus_chain_specs                chain DP straight from the specs
 *   rh_cone_merge, rh_tree_plan/_dp       cones and in-trees
 *   rh_mask_replicated, rh_plan_memory    search under a memory limit
 *   rh_stage_dp, rh_stage_dp_window       pipeline stages from segment costs
 *   rh_interval_costs, rh_stage_dp_interval (and _banded), rh_stage_plans
 *                                         stages timed by their own plans
 *   rh_workspace_size, rh_check_costs, rh_gang_workgroups, rh_strerror, rh_version
 *
 * Cost contract: a finite cost lies in [0, 2^36) ns; RH_INF (2^52) means
 * "infeasible"; any sum that reaches RH_INF is RH_INF.  N <= 2^14 keeps every
 * finite total below 2^51.
 */
#ifndef RHINO_H
#define RHINO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RH_INF ((int64_t)1 << 52)
#define RH_KMIN 16   /* padded candidate count: a power of two in [16, 1024] */
#define RH_KMAX 1024
#define RH_NMAX 16384

#define RH_OK 0
#define RH_ERR_NULL (-1)      /* a required pointer is NULL */
#define RH_ERR_SHAPE (-2)     /* a size is out of range or inconsistent */
#define RH_ERR_K_RANGE (-3)   /* Kp is not a power of two in [RH_KMIN, RH_KMAX] */
#define RH_ERR_WORKSPACE (-4) /* workspace missing or too small */
#define RH_ERR_OVERFLOW (-5)  /* a cost violates the cost contract (rh_check_costs) */
#define RH_ERR_HIP (-6)       /* the HIP runtime refused a launch */
#define RH_ERR_STATIC_SCRATCH (-7) /* sizes beyond the static scratch of rh_stage_dp_window_static */

/* Logical device mesh the plans are searched for (Sec. 4: devices form a
 * mesh and sharding is applied per mesh axis).  A search input: no device
 * of the mesh is ever touched.  Host struct, read during the call. */
typedef struct rh_mesh_t {
    int32_t naxes;              /* 1 or 2 */
    int32_t m[2];               /* axis sizes, powers of two, <= 1024 */
    int64_t bw_bytes_per_us[2]; /* link bandwidth along each axis, > 0 */
    int64_t alpha_ns[2];        /* latency added when an axis moves > 0 bytes */
} rh_mesh_t;

/*
 * Sharding spec word (Sec. 4.1: a spec is (dim, stride), stride = number of
 * consecutive units per block, maximum stride = extent / shards; Sec. 4.3.3:
 * plus "replicate" and "partial").  One byte per mesh axis, axis 0 in bits
 * 0..7, axis 1 in bits 8..15:
 *     bits 0..1 state  0 replicate, 1 split, 2 partial
 *     bits 2..4 dim    split tensor dimension, 0..3
 *     bits 5..7 lgdiv  stride = (extent[dim] / m[axis]) >> lgdiv
 * 0xFFFFFFFF = empty slot.  A word is an invalid candidate (all its costs are
 * RH_INF) if its state is 3, if m[axis] << lgdiv does not divide the extent,
 * or if both axes split the same dimension.
 */
#define RH_SPEC_EMPTY 0xFFFFFFFFu

/*
 * rh_build_reshard -- comm cost tables from sharding specs.
 *
 * R[e][a][b] = time to bring the tensor on edge e from the layout operator e
 * produces under its strategy a (out_spec[e][a]) to the layout operator e+1
 * consumes under its strategy b (in_spec[e+1][b]); the collectives of Sec. 2.1
 * (All-Gather, Reduce-Scatter, All-Reduce, All-To-All) costed by the bytes
 * one device receives.  Mesh axis 0 is converted first, then axis 1; while
 * axis x is converted the local tensor is the whole tensor divided by the
 * shard counts of the other axes (already-converted axes in the consumer's
 * state).  With local bytes T and axis size m:
 *     same state (same dim and stride if split)   0
 *     replicate -> split                          0
 *     split -> replicate     (all-gather)         T*(m-1)/m
 *     split -> split, other dim or other stride
 *                            (all-to-all)         T*(m-1)/m^2
 *     partial -> split       (reduce-scatter)     T*(m-1)/m
 *     partial -> replicate   (all-reduce)         2*(T*(m-1)/m)
 *     anything else -> partial                    infeasible
 * (divisions round down); time = bytes*1000 / bw_bytes_per_us (round down)
 * + alpha_ns if bytes > 0; R = sum over axes, RH_INF if infeasible or if
 * either slot is empty, invalid or >= its operator's K.
 *
 *   mesh        host
 *   n_edges     >= 0 (0: nothing is written)
 *   Kp          row length of every table, power of two in [RH_KMIN, RH_KMAX]
 *   K           [n_edges+1] real candidate counts, 0 <= K[i] <= Kp
 *   out_spec    [n_edges+1][Kp] (row n_edges unused)
 *   in_spec     [n_edges+1][Kp] (row 0 unused)
 *   dims        [n_edges][4] extents of the tensor on edge e, unused dims = 1
 *   elem_bytes  [n_edges]
 *   R           [n_edges][Kp][Kp] out, row a (producer), column b contiguous
 * Whole-tensor bytes must stay below 2^50.
 */
int rh_build_reshard(const rh_mesh_t* mesh, int32_t n_edges, int32_t Kp,
                     const int32_t* K, const uint32_t* out_spec,
                     const uint32_t* in_spec, const int64_t* dims,
                     const int32_t* elem_bytes, int64_t* R, void* stream);

/*
 * rh_minplus_chain -- the chain dynamic program, B independent problems
 * (e.g. one per candidate device-mesh shape, Sec. 3 / Sec. 4: mesh
 * configurations are searched in parallel).
 *
 *     v_0 = c_0
 *     v_{i+1}[b] = c_{i+1}[b] + min_a ( v_i[a] + R_i[a][b] )
 *     arg_i[b]   = the minimising a, lowest a on ties (0 if column b is infeasible)
 *     total      = min_b v_{N-1}[b],  last = lowest such b
 * which minimises the objective C of Sec. 4.2 on a path graph.
 *
 *   B >= 0, 1 <= N <= RH_NMAX, Kp power of two in [RH_KMIN, RH_KMAX]
 *   c       [B][N][Kp], problem p starts at c + p*c_batch_stride (elements);
 *           empty slots hold RH_INF
 *   R       [B][N-1][Kp][Kp], problem p starts at R + p*R_batch_stride;
 *           R_batch_stride = 0 shares one R among all problems; rows/columns
 *           of empty slots hold RH_INF.  May be NULL if N == 1.
 *   arg     [B][N-1][Kp] out (dense)
 *   vfinal  [B][Kp] out, v_{N-1}; may be NULL
 *   total   [B] out;  last [B] out
 *   workspace  optional; rh_workspace_size(RH_WS_MINPLUS_CHAIN, B, N, Kp) says how many bytes
 *           help for these sizes (0 = none).  Given that many bytes (256-byte aligned, contents
 *           undefined before and after; calls that share a workspace must not overlap):
 *           - one or two long chains (B <= 2, N >= 128, Kp 64, 128 or 256) are cut into
 *             segments: the min-plus matrix of every segment (all at once), the vectors at
 *             the segment boundaries, then the plain sweep inside all segments at once.
 *             Same outputs bit for bit; 8192 operators x 256 take a quarter of the time when
 *             every strategy is feasible and a fortieth on tables from sharding specs, where a
 *             third of the slots are valid layouts (infeasible strategies are skipped);
 *           - otherwise a few long (N >= 64) chains of wide tables (Kp 128 or 256) are spread
 *             over eight workgroups each, or four each, whichever lets every workgroup of the
 *             launch have a compute unit of the current device to itself (rh_gang_workgroups;
 *             B <= 32 resp. B <= 64 on 256 compute units); the workgroups of a problem meet once
 *             per edge through the workspace.  This route needs the device otherwise idle: the
 *             meeting is a bounded wait, and if the workgroups of a problem are not resident
 *             together (other kernels hold compute units) a workgroup gives up after 2^22 polls
 *             and the problem returns total = -1 with undefined arg, vfinal and last, under
 *             RH_OK.  A caller that overlaps this call with other work on the device checks
 *             total >= 0 before rh_backtrack (rh_plan_memory never takes such a problem as
 *             feasible) or passes no workspace;
 *           - given EXACTLY rh_workspace_size(RH_WS_MINPLUS_CHAIN_SEGMENTED, B, N, Kp) bytes
 *             (3 <= B <= 32, N >= 128, Kp 64, 128 or 256; more bytes than the above), all problems
 *             take the segmented route (their matrices one problem after the other).  Worth
 *             it when most strategies are infeasible: then a problem takes a fifteenth of what the eight
 *             workgroups need for up to 32 problems together; with every strategy feasible
 *             a problem takes two thirds of that.  Any other size of at least the
 *             RH_WS_MINPLUS_CHAIN bytes takes the route above, so a caller that passes one large
 *             pool to every call never lands here by accident.
 *           With NULL, 0 the call needs no workspace.
 * Base pointers and batch strides must keep every row 16-byte aligned.
 */
int rh_minplus_chain(int32_t B, int32_t N, int32_t Kp, const int64_t* c,
                     int64_t c_batch_stride, const int64_t* R,
                     int64_t R_batch_stride, uint16_t* arg, int64_t* vfinal,
                     int64_t* total, int32_t* last, void* workspace,
                     size_t workspace_bytes, void* stream);

/*
 * rh_minplus_chain_specs -- the same dynamic program with the resharding times computed from
 * the spec words per cell instead of read from tables: R_i[a][b] is exactly what
 * rh_build_reshard would write for (out_spec[i][a], in_spec[i+1][b]) on problem p's mesh.  One
 * operator graph, several logical meshes (mesh shapes are searched in parallel, Sec. 3 /
 * Sec. 4): problem p is searched on meshes[p mod n_meshes].  Nothing of size Kp x Kp is ever
 * stored, so it serves batches whose tables would not fit in memory.  Bound by the vector
 * ALU, not by HBM.  Without a workspace a workgroup walks each problem edge by edge; with
 * rh_workspace_size(RH_WS_MINPLUS_CHAIN_SPECS, B, N, Kp) bytes (B <= 32, N >= 128; 0 = does not
 * apply) the chains are cut into segments as in rh_minplus_chain -- the min-plus matrix of
 * every segment (the per-segment strategy tables of Sec. 4.3.2), the vectors at the segment
 * boundaries, then the sweep inside all segments at once -- with every table entry computed
 * from the spec words: one 8192-operator chain of 256 strategies takes a twentieth of the time,
 * and less than building the tables and running rh_minplus_chain on them.  Same outputs bit
 * for bit on either route.
 *
 *   B >= 0, 1 <= N <= RH_NMAX, Kp 64, 128 or 256, 1 <= n_meshes <= 64
 *   meshes   host, [n_meshes], read during the call
 *   c        [B][N][Kp] node costs per problem (they depend on the mesh), batch stride in elements
 *   K, out_spec, in_spec, dims, elem_bytes   as for rh_build_reshard with n_edges = N-1, shared by
 *            all problems
 *   arg [B][N-1][Kp], vfinal [B][Kp] (may be NULL), total [B], last [B]   as for rh_minplus_chain
 *   workspace  NULL, 0 or the bytes above (256-byte aligned, contents undefined before and after;
 *            calls that share a workspace must not overlap)
 */
int rh_minplus_chain_specs(int32_t B, int32_t N, int32_t Kp, int32_t n_meshes,
                           const rh_mesh_t* meshes,
                           const int64_t* c, int64_t c_batch_stride, const int32_t* K,
                           const uint32_t* out_spec, const uint32_t* in_spec,
                           const int64_t* dims, const int32_t* elem_bytes, uint16_t* arg,
                           int64_t* vfinal, int64_t* total, int32_t* last, void* workspace,
                           size_t workspace_bytes, void* stream);

/*
 * rh_backtrack -- the plan X of Sec. 4.2 in index form:
 *     plan[N-1] = last;  plan[i] = arg_i[plan[i+1]],  i = N-2 .. 0.
 *   arg [B][N-1][Kp] (16-byte aligned), last [B] (values in [0,Kp)), plan [B][N] out.
 */
int rh_backtrack(int32_t B, int32_t N, int32_t Kp, const uint16_t* arg,
                 const int32_t* last, int32_t* plan, void* stream);

/*
 * rh_cone_merge -- join the branches of cones at their roots (Sec. 4.3.2, level 1:
 * a cone is one root operator with several inputs whose other nodes have one
 * input each; given the root's strategy the other nodes are optimised by dynamic
 * programming, and every root strategy is kept for the next level).
 *
 * The branches of a cone are chains that end in its root.  Run all branches of all
 * cones as one rh_minplus_chain batch, each with the root appended as its last
 * operator with cost 0 (shorter branches padded in front with zero-cost operators
 * and identity tables: 0 on the diagonal, RH_INF elsewhere); then w = vfinal holds,
 * per branch b and root strategy r, the branch's best cost given r, and
 *     table[q][r]    = c_root[q][r] + sum over the branches b of cone q of w[b][r]
 *     total[q]       = min_r table[q][r],  root_choice[q] = lowest such r
 *     branch_last[b] = root_choice of b's cone  (the `last` input of rh_backtrack
 *                      on the branch batch, which then yields every node's strategy)
 * with sums saturating at RH_INF.
 *
 *   n_cones >= 0, n_branches >= 0
 *   branch_start  [n_cones+1] ascending offsets into the branch batch; the branches
 *                 of cone q are branch_start[q] .. branch_start[q+1]-1 (offsets
 *                 outside [0, n_branches] are clamped)
 *   w             [n_branches][Kp]
 *   c_root        [n_cones][Kp]
 *   table         [n_cones][Kp] out, may be NULL
 *   total         [n_cones] out;  root_choice [n_cones] out
 *   branch_last   [n_branches] out, may be NULL
 */
int rh_cone_merge(int32_t n_cones, int32_t n_branches, int32_t Kp,
                  const int32_t* branch_start, const int64_t* w,
                  const int64_t* c_root, int64_t* table, int64_t* total,
                  int32_t* root_choice, int32_t* branch_last, void* stream);

/*
 * rh_tree_plan, rh_tree_dp -- the dynamic program over an in-tree of operators: every operator
 * feeds exactly one consumer (its parent) and may join several inputs; the root feeds nobody.
 * This is the cone of Sec. 4.3.2 (level 1: given the root's strategy the other nodes are
 * optimised by dynamic programming, and every root strategy is kept for the next level) when
 * nodes below the root join several inputs too, with the objective of Sec. 4.2 on the tree's
 * edges.  With R_i the table of the edge from node i to its parent (row = strategy of i):
 *     v_i[a] = c_i[a] + sum over the inputs j of i of w_j[a]
 *     w_i[b] = min_a ( v_i[a] + R_i[a][b] ),  arg_i[b] = the lowest such a (0 if none is feasible)
 *     table  = v_root,  total = min_r table[r],  root_choice = the lowest such r
 *     plan[root] = root_choice,  plan[i] = arg_i[ plan[parent(i)] ]
 * with saturating sums (rh_minplus_chain is the case of a path, rh_cone_merge that of a root
 * whose inputs are paths).  Nodes are numbered inputs-first: parent[i] > i, node n-1 is the root
 * and has parent -1.  B problems share the tree (one operator graph searched on several logical
 * meshes, Sec. 3 / Sec. 4) and differ in their costs.
 *
 * rh_tree_plan is host arithmetic (all its pointers are HOST pointers; nothing touches a device).
 * It cuts the tree into runs -- stretches of consecutive nodes in which every node but the first
 * has the node before it as its only input, i.e. chains laid out like the operators of
 * rh_minplus_chain -- and gives every run a round: one more than the highest round among the
 * runs that feed its first node, 0 if that node has no input.  rh_tree_dp then takes one launch
 * per round (a workgroup per run and problem) and as many for the plan.
 *   n             1 <= n <= RH_NMAX
 *   parent        [n]
 *   run_first, run_last   [n] out, entries 0 .. *n_runs - 1 used: run u = nodes run_first[u] ..
 *                 run_last[u]; sorted by round, by first node within a round
 *   round_start   [n + 1] out: the runs of round t are round_start[t] .. round_start[t+1] - 1
 *   child_start   [n + 1] out, child_list [n] out: the inputs of node i are
 *                 child_list[child_start[i] .. child_start[i+1] - 1], ascending
 *   returns the number of rounds (>= 1), or RH_ERR_SHAPE if parent is not such a tree
 *
 * rh_tree_dp: round_start is the HOST array above (read during the call); run_first, run_last,
 * parent, child_start, child_list are DEVICE copies of the arrays above.
 *   0 <= B <= 65535
 *   c       [B][n][Kp], problem p at c + p*c_batch_stride; empty slots hold RH_INF
 *   R       [B][n-1][Kp][Kp], problem p at R + p*R_batch_stride (0 = one R for all problems);
 *           may be NULL if n == 1
 *   arg     [B][n-1][Kp] out
 *   w       [B][n][Kp] out: w_i for the last node of every run (the other rows are not written),
 *           row n-1 = table
 *   total   [B] out;  root_choice [B] out
 *   plan    [B][n] out, may be NULL (then no plan is made)
 */
int rh_tree_plan(int32_t n, const int32_t* parent, int32_t* run_first, int32_t* run_last,
                 int32_t* round_start, int32_t* child_start, int32_t* child_list,
                 int32_t* n_runs);
int rh_tree_dp(int32_t B, int32_t n, int32_t Kp, int32_t n_runs, int32_t n_rounds,
               const int32_t* round_start, const int32_t* run_first, const int32_t* run_last,
               const int32_t* parent, const int32_t* child_start, const int32_t* child_list,
               const int64_t* c, int64_t c_batch_stride, const int64_t* R,
               int64_t R_batch_stride, uint16_t* arg, int64_t* w, int64_t* total,
               int32_t* root_choice, int32_t* plan, void* stream);

/*
 * rh_mask_replicated, rh_plan_memory -- the memory-constrained search of Sec. 4.4:
 * sort the parameters by size, mark the k largest, remove the candidates that
 * replicate a marked parameter, search again, and take the smallest k whose plan
 * fits the device memory.  The sweep over k is ONE rh_minplus_chain batch: problem t
 * uses the node costs masked for k = k0 + t and all problems share the edge tables
 * (R_batch_stride = 0).
 *
 * rh_mask_replicated writes those node-cost tables:
 *     rank(i) = number of operators l with param_bytes[l] > param_bytes[i], or equal and l < i
 *     c_out[t][i][j] = RH_INF  if param_bytes[i] > 0, repl[i][j] != 0 and rank(i) < k0 + t
 *                    = c[i][j] otherwise
 *   1 <= N <= RH_NMAX, n_k >= 0, k0 >= 0
 *   c [N][Kp]; param_bytes [N] (0 = the operator has no parameter); repl [N][Kp] bytes;
 *   c_out [n_k][N][Kp] out
 *
 * rh_plan_memory adds up what the plans keep per device and picks the first feasible one:
 *     plan_mem[b] = sum_i mem[i][plan[b][i]]
 *     *first = smallest b with total[b] < RH_INF and plan_mem[b] <= limit, or -1
 *   plan [B][N] (from rh_backtrack); mem [N][Kp]; total [B] (from rh_minplus_chain);
 *   plan_mem [B] out; first [1] out, may be NULL (then total may be NULL too)
 */
int rh_mask_replicated(int32_t N, int32_t Kp, int32_t n_k, int32_t k0,
                       const int64_t* c, const int64_t* param_bytes,
                       const uint8_t* repl, int64_t* c_out, void* stream);
int rh_plan_memory(int32_t B, int32_t N, int32_t Kp, const int32_t* plan,
                   const int64_t* mem, const int64_t* total, int64_t limit,
                   int64_t* plan_mem, int32_t* first, void* stream);

/*
 * rh_stage_dp -- balanced pipeline stages on a chain of L segments (Sec. 2.1:
 * stages should balance computation time; Sec. 5.1: stage ids never decrease
 * along an edge; Sec. 5.2: time_per_stage = total / stages is the ideal).
 * With P(j) = cost[0] + .. + cost[j-1]:
 *     dp[1][j] = P(j)
 *     dp[s][j] = min_{s-1 <= i < j} max( dp[s-1][i], P(j) - P(i) ),  j >= s
 *     cut[s][j] = the minimising i, lowest on ties
 * for every s = 1..S in one call.
 *
 *   0 <= B <= 65535, 1 <= S <= L <= 65536, S <= 1024; cost[l] in [0, 2^36)
 *   seg_cost    [B][L]
 *   bottleneck  [B][S] out, entry s-1 = dp[s][L]
 *   cut         [B][S][L+1] out, entry [s-1][j]; 0 for s = 1, -1 where j < s
 *   s_query     0 (no bounds wanted) or 1..S
 *   bounds      [B][s_query+1] out: stage t = segments [bounds[t-1], bounds[t]);
 *               may be NULL if s_query == 0
 *   workspace   rh_workspace_size(RH_WS_STAGE_DP, B, L, S) bytes, 256-byte
 *               aligned; contents undefined before and after the call
 */
int rh_stage_dp(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost,
                int64_t* bottleneck, int32_t* cut, int32_t s_query,
                int32_t* bounds, void* workspace, size_t workspace_bytes,
                void* stream);

/*
 * rh_stage_dp_window -- the same partition for exactly S stages, with the transfer at a
 * stage boundary and the bound tightening of Sec. 5.2.  Sec. 5.1: a tensor that crosses a
 * stage boundary is communicated; Sec. 5.2: with time_per_stage = total / S an operator may
 * only sit in a stage within a tolerance eps of the one perfect balance gives it.  On a chain
 * the accumulated time of the segments before l is both its earliest and its latest start, so
 *     stage [i, j) takes P(j) - P(i) + (i > 0 ? xfer[i] : 0)
 *     segment l may sit in stage t only if
 *         floor(P(l)/tps - eps) <= t <= ceil(P(l)/tps + eps),   tps = P(L)/S, eps = eps_num/eps_den
 *     dp[1][j] = P(j);  dp[s][j] = min over allowed i of max(dp[s-1][i], P(j) - P(i) + xfer[i])
 * lowest i on ties.  The bounds prune the search to a band around the balanced cuts.
 *
 *   0 <= B <= 65535, 1 <= S <= L <= 65536, S <= 1024; cost[l], xfer[i] in [0, 2^36)
 *   seg_cost    [B][L]
 *   xfer        [B][L+1] time to pass the tensor that crosses a boundary placed before
 *               segment i (entries 0 and L unused); NULL = no transfer time
 *   eps_num, eps_den   tolerance as a fraction, 1 <= eps_den <= 2^20; eps_num < 0 = no bounds
 *   bottleneck  [B] out, dp[S][L], RH_INF if the bounds allow no split into S stages
 *   cut         [B][S][L+1] out, minimising i per (s, j), -1 where none
 *   bounds      [B][S+1] out (stage t = segments [bounds[t-1], bounds[t])), all -1 if there
 *               is no split; may be NULL
 *   workspace   rh_workspace_size(RH_WS_STAGE_DP_WINDOW, B, L, S) bytes, 256-byte aligned
 */
int rh_stage_dp_window(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost,
                       const int64_t* xfer, int64_t eps_num, int64_t eps_den,
                       int64_t* bottleneck, int32_t* cut, int32_t* bounds,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * rh_stage_dp_window_static -- rh_stage_dp_window for callers that cannot allocate device
 * memory and have no workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments (without the workspace), same kernels, same
 * results bit for bit; the scratch is a static array in device memory, rh_static_scratch_bytes()
 * = 8 MiB per GPU, which every GPU the library runs on holds until the process ends.  The call
 * allocates and frees nothing.
 *   - Sizes whose rh_workspace_size(RH_WS_STAGE_DP_WINDOW, B, L, S) exceeds that maximum return
 *     RH_ERR_STATIC_SCRATCH and launch nothing (e.g. one problem with L = 4096, S = 64 needs
 *     0.9 MiB and with L = 65536 2.5 MiB; eight problems with L = 65536 do not fit).
 *   - The scratch used is the copy of the device that is current at the call; `stream` must
 *     belong to that device.
 *   - All calls on one GPU share the one array: two calls that overlap on a GPU (different
 *     streams, different host threads) race and return garbage.  Calls in stream order are safe;
 *     nothing needs clearing between them.
 */
int rh_stage_dp_window_static(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost,
                              const int64_t* xfer, int64_t eps_num, int64_t eps_den,
                              int64_t* bottleneck, int32_t* cut, int32_t* bounds,
                              void* stream);
size_t rh_static_scratch_bytes(void);

/*
 * rh_interval_costs -- the time of every candidate pipeline stage of an operator chain.
 * Sec. 3: each stage's subgraph gets its own SPMD plan; Sec. 5.1 balances the stages.  On a
 * chain, stage [i, j) holds the operators i..j-1 and its time is the least value of Sec. 4.2's
 * objective over the plans of these operators alone (their node costs and the edges between
 * them; an edge that crosses a stage boundary belongs to neither stage):
 *     T[i][j] = min over x_i..x_{j-1} of  sum_l c_l[x_l] + sum_{i <= l < j-1} R_l[x_l][x_{l+1}]
 * with the saturation rule of rh_minplus_chain (anything >= RH_INF is RH_INF).
 *
 *   0 <= B <= 65535, 1 <= L <= RH_NMAX, Kp in {16, 32, 64, 128, 256}
 *   c    [B][L][Kp], R [B][L-1][Kp][Kp] (dense; R may be NULL if L == 1); slots beyond an
 *        operator's candidates carry RH_INF in c
 *   ldT  row stride of T in elements, even, >= L + 1
 *   T    [B][L][ldT] out: entry [i][j] for i < j <= L; RH_INF for j <= i; columns beyond L
 *        are not written
 *   workspace  optional.  Row i of the table is a sweep from operator i to the end of the chain, so the
 *        whole table costs L^2/2 sweep steps.  Given rh_workspace_size(RH_WS_INTERVAL_COSTS, B, L, Kp)
 *        bytes (Kp = 64 and L >= 512; 0 = does not apply; 256-byte aligned, contents undefined before
 *        and after), the same table is put together from blocks of 128 operators instead: sweeps
 *        inside the blocks, the min-plus matrices of the blocks (the per-segment strategy tables of
 *        Sec. 4.3.2) multiplied along the chain, and one small min-plus product per pair of blocks.
 *        A tenth of the arithmetic at L = 4096, no chain of dependent steps longer than a block,
 *        the same entries bit for bit.  With NULL, 0 the call needs no workspace.
 * c, R and T must be 16-byte aligned.  The plan of a chosen stage is what rh_minplus_chain and
 * rh_backtrack return for the sub-chain (pass c + i*Kp, R + i*Kp*Kp and N = j - i).
 */
int rh_interval_costs(int32_t B, int32_t L, int32_t Kp, const int64_t* c,
                      const int64_t* R, int64_t ldT, int64_t* T, void* workspace,
                      size_t workspace_bytes, void* stream);

/*
 * rh_stage_dp_interval -- balanced pipeline stages (Sec. 2.1, Sec. 5.1-5.2) when the time of
 * stage [i, j) is a table entry, as rh_interval_costs produces (any table with entries in
 * [0, RH_INF] will do; RH_INF = the stage cannot run):
 *     dp[1][j] = T[0][j]
 *     dp[s][j] = min_{s-1 <= i < j} max( dp[s-1][i], T[i][j] ),  j >= s
 *     cut[s][j] = the minimising i, lowest on ties (also when every candidate is RH_INF)
 * for every s = 1..S in one call.
 *
 *   0 <= B <= 65535, 1 <= S <= L <= RH_NMAX, S <= 1024; ldT even, >= L + 1
 *   T           [B][L][ldT], 16-byte aligned
 *   bottleneck  [B][S] out, entry s-1 = dp[s][L]
 *   cut         [B][S][L+1] out, entry [s-1][j]; 0 for s = 1, -1 where j < s
 *   s_query     0 (no bounds wanted) or 1..S
 *   bounds      [B][s_query+1] out: stage t = operators [bounds[t-1], bounds[t]); may be
 *               NULL if s_query == 0
 *   workspace   rh_workspace_size(RH_WS_STAGE_DP_INTERVAL, B, L, S) bytes, 256-byte aligned;
 *               contents undefined before and after the call
 */
int rh_stage_dp_interval(int32_t B, int32_t L, int32_t S, int64_t ldT,
                         const int64_t* T, int64_t* bottleneck, int32_t* cut,
                         int32_t s_query, int32_t* bounds, void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * rh_interval_costs_banded, rh_stage_dp_interval_banded -- the same two calls when no stage may
 * hold more than max_len operators.  Sec. 5.2 keeps every operator within a tolerance of the stage
 * that perfect balance gives it, so useful stages are short compared with the chain; the caller
 * states the limit.  The sweep that starts at operator i then stops after max_len operators, and
 * the search looks at the max_len rows above the diagonal only:
 *     T[i][j]  as rh_interval_costs for 0 < j - i <= max_len, RH_INF for j - i > max_len
 *     dp[s][j] = min over max(s-1, j - max_len) <= i < j of max( dp[s-1][i], T[i][j] ),
 *     cut as rh_stage_dp_interval: where no candidate is feasible, dp = RH_INF and cut = s-1
 * i.e. exactly what the unlimited calls return on a table whose entries with j - i > max_len are
 * RH_INF (the search ignores whatever T holds there).  max_len >= 1; max_len >= L is no limit.
 * With max_len <= L/2 the table costs about (max_len + 15) / (L/2) of the full one row by row.
 * The optional workspace of rh_interval_costs serves here too (same size, same conditions, and
 * max_len > 128): the table is then put together from blocks, and only pairs of blocks that an
 * interval of max_len operators can span are multiplied.
 * All other arguments as rh_interval_costs / rh_stage_dp_interval.
 */
int rh_interval_costs_banded(int32_t B, int32_t L, int32_t Kp, int32_t max_len,
                             const int64_t* c, const int64_t* R, int64_t ldT,
                             int64_t* T, void* workspace, size_t workspace_bytes,
                             void* stream);
int rh_stage_dp_interval_banded(int32_t B, int32_t L, int32_t S, int32_t max_len,
                                int64_t ldT, const int64_t* T, int64_t* bottleneck,
                                int32_t* cut, int32_t s_query, int32_t* bounds,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * rh_stage_plans -- the plans of the chosen stages, all at once.  Sec. 3 plans every stage's
 * subgraph on its own: once rh_stage_dp_interval (or any of the stage searches) has fixed the
 * boundaries, stage t of a chain holds the operators bounds[t] .. bounds[t+1]-1 and its plan is
 * what rh_minplus_chain and rh_backtrack return for that sub-chain (the edges between its
 * operators only; an edge that crosses a stage boundary belongs to no stage):
 *     stage_total[t] = T[bounds[t]][bounds[t+1]] of rh_interval_costs,
 *     stage_last[t]  = the lowest best strategy of the stage's last operator,
 *     plan[i]        = strategy of operator i, the chain DP's tie rule inside every stage.
 * One launch for the sweeps of all stages of all chains (a ragged batch), one for the walks back.
 *
 *   0 <= B <= 65535, 1 <= S <= L <= RH_NMAX, S <= 1024, Kp a power of two in [16, 1024]
 *   bounds      [B][S+1] device, as the stage searches write them.  A pair that describes no
 *               stage (negative, not increasing, beyond L: what a search without a feasible
 *               split leaves) gives stage_total = RH_INF, stage_last = 0 and no plan entries.
 *   c [B][L][Kp], R [B][L-1][Kp][Kp] (dense; R may be NULL if L == 1), as rh_interval_costs
 *   arg         [B][L-1][Kp] out: rows of the edges inside stages as rh_minplus_chain writes
 *               them; rows of edges between stages are not written.  May be NULL if L == 1.
 *   stage_total [B][S] out, stage_last [B][S] out
 *   plan        [B][L] out; operators that no stage holds get -1.  May be NULL: totals only.
 * c, R and arg must be 16-byte aligned.  A stage without a feasible plan returns RH_INF, last 0
 * and a plan of zeros, as rh_minplus_chain does.
 */
int rh_stage_plans(int32_t B, int32_t L, int32_t Kp, int32_t S, const int32_t* bounds,
                   const int64_t* c, const int64_t* R, uint16_t* arg, int64_t* stage_total,
                   int32_t* stage_last, int32_t* plan, void* stream);

#define RH_WS_MINPLUS_CHAIN 0
#define RH_WS_STAGE_DP 1
#define RH_WS_STAGE_DP_WINDOW 2
#define RH_WS_STAGE_DP_INTERVAL 3
#define RH_WS_MINPLUS_CHAIN_SEGMENTED 4
#define RH_WS_MINPLUS_CHAIN_SPECS 5
#define RH_WS_INTERVAL_COSTS 6
/* Bytes of workspace the call `which` needs for these sizes (0 if none or
 * if the sizes are invalid). */
size_t rh_workspace_size(int32_t which, int32_t B, int32_t N_or_L,
                         int32_t Kp_or_S);

/* Workgroups per problem that rh_minplus_chain's several-workgroups route uses for B
 * problems on a device with `compute_units` compute units: 8 or 4, the largest that gives
 * every workgroup of the launch a compute unit of its own, or 0 if not even 4 fit (the call
 * then runs one workgroup per problem and RH_WS_MINPLUS_CHAIN asks for no bytes).  Pure host
 * arithmetic; the library itself asks the current device for its count. */
int rh_gang_workgroups(int32_t B, int32_t compute_units);

/*
 * rh_check_costs -- optional guard for the cost contract.  Counts the entries
 * of x[0..n) that are neither in [0, 2^36) nor equal to RH_INF and adds the
 * count to *violations (device, caller-zeroed).  Never part of a timed path.
 */
int rh_check_costs(const int64_t* x, int64_t n, int64_t* violations,
                   void* stream);

const char* rh_strerror(int code);
int rh_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RHINO_H */

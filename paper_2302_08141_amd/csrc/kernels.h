// Internal launch interface between the C-ABI layer and the gfx950 kernels.
// Every launcher only enqueues work on `stream`; arguments are already validated.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rh {

constexpr int64_t kInf = (int64_t)1 << 52;

struct Mesh {
    int32_t naxes;
    int32_t lgm[2];             // log2 of the axis sizes
    int64_t bw_bytes_per_us[2];
    int64_t alpha_ns[2];
};

hipError_t launch_chain(int32_t B, int32_t N, int32_t Kp, const int64_t* c, int64_t c_bs,
                        const int64_t* R, int64_t R_bs, uint16_t* arg, int64_t* vfinal,
                        int64_t* total, int32_t* last, hipStream_t stream);

// Few long chains of wide tables: eight workgroups per problem (needs a workspace).
int gang_workgroups(int32_t B, int32_t compute_units);            // workgroups per problem, 0 = route not taken
size_t gang_workspace_bytes(int32_t B, int32_t N, int32_t Kp);   // 0 = not applicable to these sizes or this device
hipError_t launch_chain_gang(int32_t B, int32_t N, int32_t Kp, const int64_t* c, int64_t c_bs,
                             const int64_t* R, int64_t R_bs, uint16_t* arg, int64_t* vfinal,
                             int64_t* total, int32_t* last, void* workspace, hipStream_t stream);

// One or two long chains, parallel along the chain: segment matrices, boundary vectors, then the plain sweep
// inside all segments as one batch (needs a workspace).
size_t scan_workspace_bytes(int32_t B, int32_t N, int32_t Kp);   // 0 = not applicable to these sizes
hipError_t launch_chain_scan(int32_t B, int32_t N, int32_t Kp, const int64_t* c, int64_t c_bs, const int64_t* R,
                             int64_t R_bs, uint16_t* arg, int64_t* vfinal, int64_t* total, int32_t* last,
                             void* workspace, hipStream_t stream);

// Chain DP with the resharding times computed from the spec words per cell; problem p uses mesh p % n_meshes
// (n_meshes <= 64).
hipError_t launch_chain_fused(int32_t B, int32_t N, int32_t Kp, int32_t n_meshes, const Mesh* meshes,
                              const int64_t* c, int64_t c_bs,
                              const int32_t* K, const uint32_t* out_spec, const uint32_t* in_spec,
                              const int64_t* dims, const int32_t* elem_bytes, uint16_t* arg, int64_t* vfinal,
                              int64_t* total, int32_t* last, hipStream_t stream);

// The same kernel sweeping parts of chains: part q of problem p (part_len edges from operator q * part_len; part
// n_full takes the rest of the chain and alone writes vfinal, total, last) starts from the vector at
// v_start + p * v_bs + q * v_stride.
hipError_t launch_chain_fused_parts(int32_t B, int32_t N, int32_t Kp, int32_t n_meshes, const Mesh* meshes,
                                    const int64_t* c, int64_t c_bs, const int32_t* K, const uint32_t* out_spec,
                                    const uint32_t* in_spec, const int64_t* dims, const int32_t* elem_bytes,
                                    int32_t part_len, int32_t n_full, const int64_t* v_start, int64_t v_stride,
                                    int64_t v_bs, uint16_t* arg, int64_t* vfinal, int64_t* total, int32_t* last,
                                    hipStream_t stream);

// Long chains from specs, parallel along the chain (needs a workspace): the segmented route with every table
// entry computed from the spec words.
size_t scan_specs_workspace_bytes(int32_t B, int32_t N, int32_t Kp);   // 0 = not applicable to these sizes
hipError_t launch_chain_scan_specs(int32_t B, int32_t N, int32_t Kp, int32_t n_meshes, const Mesh* meshes,
                                   const int64_t* c, int64_t c_bs, const int32_t* K, const uint32_t* out_spec,
                                   const uint32_t* in_spec, const int64_t* dims, const int32_t* elem_bytes,
                                   uint16_t* arg, int64_t* vfinal, int64_t* total, int32_t* last, void* workspace,
                                   hipStream_t stream);

hipError_t launch_backtrack(int32_t B, int32_t N, int32_t Kp, const uint16_t* arg,
                            const int32_t* last, int32_t* plan, hipStream_t stream);

hipError_t launch_reshard(const Mesh& mesh, int32_t n_edges, int32_t Kp, const int32_t* K,
                          const uint32_t* out_spec, const uint32_t* in_spec, const int64_t* dims,
                          const int32_t* elem_bytes, int64_t* R, hipStream_t stream);

hipError_t launch_cone_merge(int32_t n_cones, int32_t n_branches, int32_t Kp, const int32_t* branch_start,
                             const int64_t* w, const int64_t* c_root, int64_t* table, int64_t* total,
                             int32_t* root_choice, int32_t* branch_last, hipStream_t stream);

// In-tree of operators: runs, rounds and input lists on the host, then one launch per round and the backtrack.
int plan_tree(int32_t n, const int32_t* parent, int32_t* run_first, int32_t* run_last, int32_t* round_start,
              int32_t* child_start, int32_t* child_list, int32_t* n_runs_out);
hipError_t launch_tree_dp(int32_t B, int32_t n, int32_t Kp, int32_t n_rounds, const int32_t* round_start,
                          const int32_t* run_first, const int32_t* run_last, const int32_t* parent,
                          const int32_t* child_start, const int32_t* child_list, const int64_t* c, int64_t c_bs,
                          const int64_t* R, int64_t R_bs, uint16_t* arg, int64_t* w, int64_t* total,
                          int32_t* root_choice, int32_t* plan, hipStream_t stream);

hipError_t launch_mask_replicated(int32_t N, int32_t Kp, int32_t n_k, int32_t k0, const int64_t* c,
                                  const int64_t* param_bytes, const uint8_t* repl, int64_t* c_out,
                                  hipStream_t stream);
hipError_t launch_plan_memory(int32_t B, int32_t N, int32_t Kp, const int32_t* plan, const int64_t* mem,
                              const int64_t* total, int64_t limit, int64_t* plan_mem, int32_t* first,
                              hipStream_t stream);

size_t stage_workspace_bytes(int32_t B, int32_t L, int32_t S);
hipError_t launch_stage_dp(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost,
                           int64_t* bottleneck, int32_t* cut, int32_t s_query, int32_t* bounds,
                           void* workspace, hipStream_t stream);

// Exact search by bisection for chains short enough to live in LDS (one workgroup per problem).
bool stage_fast_applies(int32_t L);
hipError_t launch_stage_fast(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost, int64_t* bottleneck,
                             int32_t* cut, int32_t s_query, int32_t* bounds, hipStream_t stream);

size_t stage_window_workspace_bytes(int32_t B, int32_t L, int32_t S);
hipError_t launch_stage_window(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost, const int64_t* xfer,
                               int64_t eps_num, int64_t eps_den, int64_t* bottleneck, int32_t* cut,
                               int32_t* bounds, void* workspace, hipStream_t stream);

// Stage times of all intervals of B operator chains: T[p][i][j] for 0 <= i < L, 0 <= j <= L (row stride ldT).
// With `parts`, every chain is parts->n sub-chains of L operators each: sub-chain t of problem p reads
// c + p*c_bs + t*c_stride, R + p*R_bs + t*R_stride and writes T + p*T_bs + t*T_stride; only its first n_rows rows
// are made; a part never reaches past the end of the chain: part t has min(L, ops_total - t * ops_stride)
// operators (ops_stride = operators between the starts of neighbouring parts, ops_total = operators from the
// start of part 0 to the chain's end).  v_end, if given, receives every row's vector at the last operator of every
// part of full length ([problem][part][row][Kp] at strides v_bs, v_stride).  unit_rows (Kp = 64): the rows are
// not start operators but the Kp strategies of operator 0, each fixed there at no cost.
struct IntervalParts {
    int32_t n;
    int64_t c_stride, R_stride, T_stride;
    int32_t n_rows;
    int64_t* v_end;
    int64_t v_stride, v_bs;
    int32_t ops_stride, ops_total;
};
hipError_t launch_interval_costs(int32_t B, int32_t L, int32_t Kp, int32_t max_len, const int64_t* c, int64_t c_bs, const int64_t* R,
                                 int64_t R_bs, int64_t ldT, int64_t* T, int64_t T_bs, hipStream_t stream,
                                 const IntervalParts* parts = nullptr, bool unit_rows = false);

// The same table put together from blocks of 128 operators (Kp = 64, at least four blocks; needs a workspace).
size_t interval_blocks_workspace_bytes(int32_t B, int32_t L, int32_t Kp);   // 0 = not applicable to these sizes
hipError_t launch_interval_costs_blocked(int32_t B, int32_t L, int32_t max_len, const int64_t* c, const int64_t* R,
                                         int64_t ldT, int64_t* T, void* workspace, hipStream_t stream);

// Stage search over a table of interval times.
size_t stage_interval_workspace_bytes(int32_t B, int32_t L, int32_t S);
hipError_t launch_stage_interval(int32_t B, int32_t L, int32_t S, int32_t max_len, int64_t ldT, const int64_t* T, int64_t* bottleneck,
                                 int32_t* cut, int32_t s_query, int32_t* bounds, void* workspace,
                                 hipStream_t stream);

// The plans of S stages of every chain at once (a ragged batch of sub-chains; stage_plans.hip).
hipError_t launch_stage_plans(int32_t B, int32_t L, int32_t Kp, int32_t S, const int32_t* bounds, const int64_t* c,
                              const int64_t* R, uint16_t* arg, int64_t* stage_total, int32_t* stage_last,
                              int32_t* plan, hipStream_t stream);

hipError_t launch_check_costs(const int64_t* x, int64_t n, int64_t* violations, hipStream_t stream);

}  // namespace rh

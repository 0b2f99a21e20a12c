// C-ABI layer: argument validation on the host, then kernel launches on the caller's stream.
// Nothing is allocated, nothing is synchronised, no state is kept.
#include "../../include/rhino.h"

#include "kernels.h"

#include <mutex>

// Scratch memory of rh_stage_dp_window_static: one copy per GPU, held until the process ends.  In host code the
// name below is only a handle for hipGetSymbolAddress; the device address is looked up once per device.
#define RH_STATIC_SCRATCH_BYTES ((size_t)8 << 20)
static __device__ __align__(256) unsigned char scratch[RH_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, nullptr until first asked for

// Address of the current device's copy of `scratch`.
int scratch_of_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RH_ERR_HIP;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return RH_ERR_HIP;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return RH_OK;
}

bool valid_kp(int32_t Kp) { return Kp >= RH_KMIN && Kp <= RH_KMAX && (Kp & (Kp - 1)) == 0; }

int lg2_exact(int64_t x) {   // log2 of a power of two, -1 otherwise
    if (x <= 0 || (x & (x - 1)) != 0) return -1;
    int l = 0;
    while (((int64_t)1 << l) < x) ++l;
    return l;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int from_hip(hipError_t e) { return e == hipSuccess ? RH_OK : RH_ERR_HIP; }

// Validates a caller's mesh and converts it to the kernels' form.
int convert_mesh(const rh_mesh_t* mesh, rh::Mesh* out) {
    if (mesh->naxes < 1 || mesh->naxes > 2) return RH_ERR_SHAPE;
    rh::Mesh m{};
    m.naxes = mesh->naxes;
    for (int x = 0; x < 2; ++x) {
        m.lgm[x] = 0;
        m.bw_bytes_per_us[x] = 1;
        m.alpha_ns[x] = 0;
        if (x >= mesh->naxes) continue;
        const int lg = lg2_exact(mesh->m[x]);
        if (lg < 0 || lg > 10) return RH_ERR_SHAPE;
        if (mesh->bw_bytes_per_us[x] <= 0 || mesh->alpha_ns[x] < 0) return RH_ERR_SHAPE;
        m.lgm[x] = lg;
        m.bw_bytes_per_us[x] = mesh->bw_bytes_per_us[x];
        m.alpha_ns[x] = mesh->alpha_ns[x];
    }
    *out = m;
    return RH_OK;
}

}  // namespace

extern "C" {

int rh_build_reshard(const rh_mesh_t* mesh, int32_t n_edges, int32_t Kp, const int32_t* K,
                     const uint32_t* out_spec, const uint32_t* in_spec, const int64_t* dims,
                     const int32_t* elem_bytes, int64_t* R, void* stream) {
    if (mesh == nullptr) return RH_ERR_NULL;
    if (n_edges < 0) return RH_ERR_SHAPE;
    if (!valid_kp(Kp)) return RH_ERR_K_RANGE;
    rh::Mesh m{};
    if (const int rc = convert_mesh(mesh, &m)) return rc;
    if (n_edges == 0) return RH_OK;
    if (!K || !out_spec || !in_spec || !dims || !elem_bytes || !R) return RH_ERR_NULL;
    if (!aligned16(R) || (reinterpret_cast<uintptr_t>(in_spec) & 7u) != 0) return RH_ERR_SHAPE;
    return from_hip(rh::launch_reshard(m, n_edges, Kp, K, out_spec, in_spec, dims, elem_bytes, R,
                                       static_cast<hipStream_t>(stream)));
}

int rh_minplus_chain(int32_t B, int32_t N, int32_t Kp, const int64_t* c, int64_t c_batch_stride,
                     const int64_t* R, int64_t R_batch_stride, uint16_t* arg, int64_t* vfinal,
                     int64_t* total, int32_t* last, void* workspace, size_t workspace_bytes,
                     void* stream) {
    if (B < 0 || N < 1 || N > RH_NMAX) return RH_ERR_SHAPE;
    if (!valid_kp(Kp)) return RH_ERR_K_RANGE;
    if (B == 0) return RH_OK;
    if (!c || !total || !last) return RH_ERR_NULL;
    if (N > 1 && (!R || !arg)) return RH_ERR_NULL;
    if (c_batch_stride < 0 || R_batch_stride < 0) return RH_ERR_SHAPE;
    if (B > 1 && c_batch_stride < (int64_t)N * Kp) return RH_ERR_SHAPE;
    if (B > 1 && R_batch_stride != 0 && R_batch_stride < (int64_t)(N - 1) * Kp * Kp) return RH_ERR_SHAPE;
    // 16-byte loads and stores: rows start on 16-byte boundaries
    if (!aligned16(c) || (c_batch_stride & 1) || (R && (!aligned16(R) || (R_batch_stride & 1))))
        return RH_ERR_SHAPE;
    if ((arg && (reinterpret_cast<uintptr_t>(arg) & 3u)) || (vfinal && !aligned16(vfinal)))
        return RH_ERR_SHAPE;
    if (workspace != nullptr && (!aligned16(workspace) || (reinterpret_cast<uintptr_t>(workspace) & 255u)))
        return RH_ERR_WORKSPACE;
    // One or two long chains are cut into segments; three and more take the segmented route only when the caller
    // states the size of that route's workspace exactly, which says that the tables are sparse enough for it to
    // pay (a caller that hands over one large pool for every call must not land on it by accident).
    const size_t scan = rh::scan_workspace_bytes(B, N, Kp);
    const size_t gang = rh::gang_workspace_bytes(B, N, Kp);
    if (scan != 0 && workspace != nullptr && (B <= 2 ? workspace_bytes >= scan : workspace_bytes == scan))
        return from_hip(rh::launch_chain_scan(B, N, Kp, c, c_batch_stride, R, R_batch_stride, arg, vfinal, total,
                                              last, workspace, static_cast<hipStream_t>(stream)));
    if (gang != 0 && workspace != nullptr && workspace_bytes >= gang)
        return from_hip(rh::launch_chain_gang(B, N, Kp, c, c_batch_stride, R, R_batch_stride, arg, vfinal,
                                              total, last, workspace, static_cast<hipStream_t>(stream)));
    return from_hip(rh::launch_chain(B, N, Kp, c, c_batch_stride, R, R_batch_stride, arg, vfinal, total,
                                     last, static_cast<hipStream_t>(stream)));
}

int rh_minplus_chain_specs(int32_t B, int32_t N, int32_t Kp, int32_t n_meshes, const rh_mesh_t* meshes, const int64_t* c,
                           int64_t c_batch_stride, const int32_t* K, const uint32_t* out_spec,
                           const uint32_t* in_spec, const int64_t* dims, const int32_t* elem_bytes,
                           uint16_t* arg, int64_t* vfinal, int64_t* total, int32_t* last, void* workspace,
                           size_t workspace_bytes, void* stream) {
    if (B < 0 || N < 1 || N > RH_NMAX || n_meshes < 1 || n_meshes > 64) return RH_ERR_SHAPE;
    if (Kp != 64 && Kp != 128 && Kp != 256) return RH_ERR_K_RANGE;
    if (B == 0) return RH_OK;
    if (!meshes || !c || !total || !last) return RH_ERR_NULL;
    if (N > 1 && (!K || !out_spec || !in_spec || !dims || !elem_bytes || !arg)) return RH_ERR_NULL;
    if (c_batch_stride < 0 || (B > 1 && c_batch_stride < (int64_t)N * Kp)) return RH_ERR_SHAPE;
    rh::Mesh ms[64];
    for (int p = 0; p < n_meshes; ++p)
        if (const int rc = convert_mesh(meshes + p, ms + p)) return rc;
    if (N == 1)   // no edge, nothing to compute from specs (their pointers may be NULL): v_0 = c_0 by the plain kernel
        return from_hip(rh::launch_chain(B, 1, Kp, c, c_batch_stride, nullptr, 0, nullptr, vfinal, total, last,
                                         static_cast<hipStream_t>(stream)));
    if (workspace != nullptr && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return RH_ERR_WORKSPACE;
    // with its workspace a few long chains are cut into segments, as in rh_minplus_chain
    const size_t scan = rh::scan_specs_workspace_bytes(B, N, Kp);
    if (scan != 0 && workspace != nullptr && workspace_bytes >= scan)
        return from_hip(rh::launch_chain_scan_specs(B, N, Kp, n_meshes, ms, c, c_batch_stride, K, out_spec, in_spec,
                                                    dims, elem_bytes, arg, vfinal, total, last, workspace,
                                                    static_cast<hipStream_t>(stream)));
    return from_hip(rh::launch_chain_fused(B, N, Kp, n_meshes, ms, c, c_batch_stride, K, out_spec, in_spec, dims,
                                           elem_bytes, arg, vfinal, total, last,
                                           static_cast<hipStream_t>(stream)));
}

int rh_backtrack(int32_t B, int32_t N, int32_t Kp, const uint16_t* arg, const int32_t* last,
                 int32_t* plan, void* stream) {
    if (B < 0 || N < 1 || N > RH_NMAX) return RH_ERR_SHAPE;
    if (!valid_kp(Kp)) return RH_ERR_K_RANGE;
    if (B == 0) return RH_OK;
    if (!last || !plan || (N > 1 && !arg)) return RH_ERR_NULL;
    if (arg && !aligned16(arg)) return RH_ERR_SHAPE;   // rows are fetched as 16-byte words
    return from_hip(rh::launch_backtrack(B, N, Kp, arg, last, plan, static_cast<hipStream_t>(stream)));
}

int rh_cone_merge(int32_t n_cones, int32_t n_branches, int32_t Kp, const int32_t* branch_start,
                  const int64_t* w, const int64_t* c_root, int64_t* table, int64_t* total,
                  int32_t* root_choice, int32_t* branch_last, void* stream) {
    if (n_cones < 0 || n_branches < 0) return RH_ERR_SHAPE;
    if (!valid_kp(Kp)) return RH_ERR_K_RANGE;
    if (n_cones == 0) return RH_OK;
    if (!branch_start || !c_root || !total || !root_choice || (n_branches > 0 && !w)) return RH_ERR_NULL;
    return from_hip(rh::launch_cone_merge(n_cones, n_branches, Kp, branch_start, w, c_root, table, total,
                                          root_choice, branch_last, static_cast<hipStream_t>(stream)));
}

int rh_tree_plan(int32_t n, const int32_t* parent, int32_t* run_first, int32_t* run_last, int32_t* round_start,
                 int32_t* child_start, int32_t* child_list, int32_t* n_runs) {
    if (n < 1 || n > RH_NMAX) return RH_ERR_SHAPE;
    if (!parent || !run_first || !run_last || !round_start || !child_start || !child_list || !n_runs) return RH_ERR_NULL;
    const int rounds = rh::plan_tree(n, parent, run_first, run_last, round_start, child_start, child_list, n_runs);
    return rounds < 0 ? RH_ERR_SHAPE : rounds;
}

int rh_tree_dp(int32_t B, int32_t n, int32_t Kp, int32_t n_runs, int32_t n_rounds, const int32_t* round_start,
               const int32_t* run_first, const int32_t* run_last, const int32_t* parent, const int32_t* child_start,
               const int32_t* child_list, const int64_t* c, int64_t c_batch_stride, const int64_t* R,
               int64_t R_batch_stride, uint16_t* arg, int64_t* w, int64_t* total, int32_t* root_choice,
               int32_t* plan, void* stream) {
    if (B < 0 || B > 65535 || n < 1 || n > RH_NMAX || n_runs < 1 || n_runs > n || n_rounds < 1 || n_rounds > n_runs)
        return RH_ERR_SHAPE;
    if (!valid_kp(Kp)) return RH_ERR_K_RANGE;
    if (!round_start) return RH_ERR_NULL;
    if (round_start[0] != 0 || round_start[n_rounds] != n_runs) return RH_ERR_SHAPE;
    for (int t = 0; t < n_rounds; ++t)
        if (round_start[t + 1] < round_start[t]) return RH_ERR_SHAPE;
    if (B == 0) return RH_OK;
    if (!run_first || !run_last || !parent || !child_start || !child_list || !c || !w || !total || !root_choice)
        return RH_ERR_NULL;
    if (n > 1 && (!R || !arg)) return RH_ERR_NULL;
    if (c_batch_stride < 0 || R_batch_stride < 0) return RH_ERR_SHAPE;
    if (B > 1 && c_batch_stride < (int64_t)n * Kp) return RH_ERR_SHAPE;
    if (B > 1 && R_batch_stride != 0 && R_batch_stride < (int64_t)(n - 1) * Kp * Kp) return RH_ERR_SHAPE;
    return from_hip(rh::launch_tree_dp(B, n, Kp, n_rounds, round_start, run_first, run_last, parent, child_start,
                                       child_list, c, c_batch_stride, R, R_batch_stride, arg, w, total, root_choice,
                                       plan, static_cast<hipStream_t>(stream)));
}

int rh_mask_replicated(int32_t N, int32_t Kp, int32_t n_k, int32_t k0, const int64_t* c,
                       const int64_t* param_bytes, const uint8_t* repl, int64_t* c_out, void* stream) {
    if (N < 1 || N > RH_NMAX || n_k < 0 || k0 < 0) return RH_ERR_SHAPE;
    if (!valid_kp(Kp)) return RH_ERR_K_RANGE;
    if (n_k == 0) return RH_OK;
    if (!c || !param_bytes || !repl || !c_out) return RH_ERR_NULL;
    return from_hip(rh::launch_mask_replicated(N, Kp, n_k, k0, c, param_bytes, repl, c_out,
                                               static_cast<hipStream_t>(stream)));
}

int rh_plan_memory(int32_t B, int32_t N, int32_t Kp, const int32_t* plan, const int64_t* mem,
                   const int64_t* total, int64_t limit, int64_t* plan_mem, int32_t* first, void* stream) {
    if (B < 0 || N < 1 || N > RH_NMAX) return RH_ERR_SHAPE;
    if (!valid_kp(Kp)) return RH_ERR_K_RANGE;
    if (B > 0 && (!plan || !mem || !plan_mem)) return RH_ERR_NULL;
    if (first != nullptr && B > 0 && !total) return RH_ERR_NULL;
    if (B == 0 && first == nullptr) return RH_OK;
    return from_hip(rh::launch_plan_memory(B, N, Kp, plan, mem, total, limit, plan_mem, first,
                                           static_cast<hipStream_t>(stream)));
}

int rh_stage_dp(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost, int64_t* bottleneck,
                int32_t* cut, int32_t s_query, int32_t* bounds, void* workspace,
                size_t workspace_bytes, void* stream) {
    if (B < 0 || B > 65535 || L < 1 || L > 65536 || S < 1 || S > L || S > 1024) return RH_ERR_SHAPE;
    if (s_query < 0 || s_query > S) return RH_ERR_SHAPE;
    if (B == 0) return RH_OK;
    if (!seg_cost || !bottleneck || !cut) return RH_ERR_NULL;
    if (s_query > 0 && !bounds) return RH_ERR_NULL;
    if (!workspace) return RH_ERR_WORKSPACE;
    if (workspace_bytes < rh::stage_workspace_bytes(B, L, S)) return RH_ERR_WORKSPACE;
    if (!aligned16(workspace)) return RH_ERR_WORKSPACE;
    if (rh::stage_fast_applies(L))
        return from_hip(rh::launch_stage_fast(B, L, S, seg_cost, bottleneck, cut, s_query, bounds,
                                              static_cast<hipStream_t>(stream)));
    return from_hip(rh::launch_stage_dp(B, L, S, seg_cost, bottleneck, cut, s_query, bounds, workspace,
                                        static_cast<hipStream_t>(stream)));
}

int rh_stage_dp_window(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost, const int64_t* xfer,
                       int64_t eps_num, int64_t eps_den, int64_t* bottleneck, int32_t* cut, int32_t* bounds,
                       void* workspace, size_t workspace_bytes, void* stream) {
    if (B < 0 || B > 65535 || L < 1 || L > 65536 || S < 1 || S > L || S > 1024) return RH_ERR_SHAPE;
    if (eps_den < 1 || eps_den > (1 << 20) || eps_num > ((int64_t)1 << 30)) return RH_ERR_SHAPE;
    if (B == 0) return RH_OK;
    if (!seg_cost || !bottleneck || !cut) return RH_ERR_NULL;
    if (!workspace || !aligned16(workspace)) return RH_ERR_WORKSPACE;
    if (workspace_bytes < rh::stage_window_workspace_bytes(B, L, S)) return RH_ERR_WORKSPACE;
    return from_hip(rh::launch_stage_window(B, L, S, seg_cost, xfer, eps_num, eps_den, bottleneck, cut, bounds,
                                            workspace, static_cast<hipStream_t>(stream)));
}

int rh_stage_dp_window_static(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost, const int64_t* xfer,
                              int64_t eps_num, int64_t eps_den, int64_t* bottleneck, int32_t* cut, int32_t* bounds,
                              void* stream) {
    if (B < 0 || B > 65535 || L < 1 || L > 65536 || S < 1 || S > L || S > 1024) return RH_ERR_SHAPE;
    if (eps_den < 1 || eps_den > (1 << 20) || eps_num > ((int64_t)1 << 30)) return RH_ERR_SHAPE;
    if (B == 0) return RH_OK;
    if (!seg_cost || !bottleneck || !cut) return RH_ERR_NULL;
    if (rh::stage_window_workspace_bytes(B, L, S) > RH_STATIC_SCRATCH_BYTES) return RH_ERR_STATIC_SCRATCH;
    void* ws = nullptr;
    if (const int rc = scratch_of_current_device(&ws)) return rc;
    // the kernels write every word of the scratch they read (as with a caller's workspace of undefined contents),
    // so nothing has to be cleared between calls
    return from_hip(rh::launch_stage_window(B, L, S, seg_cost, xfer, eps_num, eps_den, bottleneck, cut, bounds, ws,
                                            static_cast<hipStream_t>(stream)));
}

size_t rh_static_scratch_bytes(void) { return RH_STATIC_SCRATCH_BYTES; }

int rh_interval_costs_banded(int32_t B, int32_t L, int32_t Kp, int32_t max_len, const int64_t* c, const int64_t* R,
                             int64_t ldT, int64_t* T, void* workspace, size_t workspace_bytes, void* stream) {
    if (B < 0 || B > 65535 || L < 1 || L > RH_NMAX || max_len < 1) return RH_ERR_SHAPE;
    if (Kp != 16 && Kp != 32 && Kp != 64 && Kp != 128 && Kp != 256) return RH_ERR_K_RANGE;
    if (ldT < (int64_t)L + 1 || (ldT & 1)) return RH_ERR_SHAPE;
    if (workspace != nullptr && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return RH_ERR_WORKSPACE;
    if (B == 0) return RH_OK;
    if (!c || !T || (L > 1 && !R)) return RH_ERR_NULL;
    if (!aligned16(c) || !aligned16(T) || (R && !aligned16(R))) return RH_ERR_SHAPE;
    if (max_len > L) max_len = L;
    // from blocks of 128 operators where that applies: the caller brought the workspace, and an interval may be
    // longer than a block
    const size_t need = workspace != nullptr ? rh::interval_blocks_workspace_bytes(B, L, Kp) : 0;
    if (need > 0 && workspace_bytes >= need && max_len > 128)
        return from_hip(rh::launch_interval_costs_blocked(B, L, max_len, c, R, ldT, T, workspace,
                                                          static_cast<hipStream_t>(stream)));
    return from_hip(rh::launch_interval_costs(B, L, Kp, max_len, c, (int64_t)L * Kp, R, (int64_t)(L - 1) * Kp * Kp,
                                              ldT, T, (int64_t)L * ldT, static_cast<hipStream_t>(stream)));
}

int rh_interval_costs(int32_t B, int32_t L, int32_t Kp, const int64_t* c, const int64_t* R, int64_t ldT, int64_t* T,
                      void* workspace, size_t workspace_bytes, void* stream) {
    return rh_interval_costs_banded(B, L, Kp, L > 0 ? L : 1, c, R, ldT, T, workspace, workspace_bytes, stream);
}

int rh_stage_dp_interval_banded(int32_t B, int32_t L, int32_t S, int32_t max_len, int64_t ldT, const int64_t* T,
                                int64_t* bottleneck, int32_t* cut, int32_t s_query, int32_t* bounds, void* workspace,
                                size_t workspace_bytes, void* stream) {
    if (B < 0 || B > 65535 || L < 1 || L > RH_NMAX || S < 1 || S > L || S > 1024 || max_len < 1) return RH_ERR_SHAPE;
    if (ldT < (int64_t)L + 1 || (ldT & 1)) return RH_ERR_SHAPE;
    if (s_query < 0 || s_query > S) return RH_ERR_SHAPE;
    if (B == 0) return RH_OK;
    if (!T || !bottleneck || !cut) return RH_ERR_NULL;
    if (s_query > 0 && !bounds) return RH_ERR_NULL;
    if (!aligned16(T)) return RH_ERR_SHAPE;
    if (!workspace || !aligned16(workspace)) return RH_ERR_WORKSPACE;
    if (workspace_bytes < rh::stage_interval_workspace_bytes(B, L, S)) return RH_ERR_WORKSPACE;
    return from_hip(rh::launch_stage_interval(B, L, S, max_len, ldT, T, bottleneck, cut, s_query, bounds, workspace,
                                              static_cast<hipStream_t>(stream)));
}

int rh_stage_plans(int32_t B, int32_t L, int32_t Kp, int32_t S, const int32_t* bounds, const int64_t* c,
                   const int64_t* R, uint16_t* arg, int64_t* stage_total, int32_t* stage_last, int32_t* plan,
                   void* stream) {
    if (B < 0 || B > 65535 || L < 1 || L > RH_NMAX || S < 1 || S > L || S > 1024) return RH_ERR_SHAPE;
    if (!valid_kp(Kp)) return RH_ERR_K_RANGE;
    if (B == 0) return RH_OK;
    if (!bounds || !c || !stage_total || !stage_last) return RH_ERR_NULL;
    if (L > 1 && (!R || !arg)) return RH_ERR_NULL;
    if (!aligned16(c) || (R && !aligned16(R)) || (arg && !aligned16(arg))) return RH_ERR_SHAPE;
    return from_hip(rh::launch_stage_plans(B, L, Kp, S, bounds, c, R, arg, stage_total, stage_last, plan,
                                           static_cast<hipStream_t>(stream)));
}

int rh_stage_dp_interval(int32_t B, int32_t L, int32_t S, int64_t ldT, const int64_t* T, int64_t* bottleneck,
                         int32_t* cut, int32_t s_query, int32_t* bounds, void* workspace, size_t workspace_bytes,
                         void* stream) {
    return rh_stage_dp_interval_banded(B, L, S, L > 0 ? L : 1, ldT, T, bottleneck, cut, s_query, bounds, workspace,
                                       workspace_bytes, stream);
}

size_t rh_workspace_size(int32_t which, int32_t B, int32_t N_or_L, int32_t Kp_or_S) {
    if (B < 1) return 0;                          // no problem, no workspace (and nothing below divides by B)
    if (which == RH_WS_MINPLUS_CHAIN) {
        const size_t scan = B <= 2 ? rh::scan_workspace_bytes(B, N_or_L, Kp_or_S) : 0;
        return scan != 0 ? scan : rh::gang_workspace_bytes(B, N_or_L, Kp_or_S);
    }
    if (which == RH_WS_MINPLUS_CHAIN_SEGMENTED) return rh::scan_workspace_bytes(B, N_or_L, Kp_or_S);
    if (which == RH_WS_MINPLUS_CHAIN_SPECS) return rh::scan_specs_workspace_bytes(B, N_or_L, Kp_or_S);
    if (which == RH_WS_INTERVAL_COSTS) return rh::interval_blocks_workspace_bytes(B, N_or_L, Kp_or_S);
    if (which == RH_WS_STAGE_DP) {
        if (B > 65535 || N_or_L < 1 || N_or_L > 65536 || Kp_or_S < 1 || Kp_or_S > N_or_L) return 0;
        return rh::stage_workspace_bytes(B, N_or_L, Kp_or_S);
    }
    if (which == RH_WS_STAGE_DP_WINDOW) {
        if (B > 65535 || N_or_L < 1 || N_or_L > 65536 || Kp_or_S < 1 || Kp_or_S > N_or_L) return 0;
        return rh::stage_window_workspace_bytes(B, N_or_L, Kp_or_S);
    }
    if (which == RH_WS_STAGE_DP_INTERVAL) {
        if (B > 65535 || N_or_L < 1 || N_or_L > RH_NMAX || Kp_or_S < 1 || Kp_or_S > N_or_L) return 0;
        return rh::stage_interval_workspace_bytes(B, N_or_L, Kp_or_S);
    }
    return 0;
}

int rh_check_costs(const int64_t* x, int64_t n, int64_t* violations, void* stream) {
    if (n < 0) return RH_ERR_SHAPE;
    if (n == 0) return RH_OK;
    if (!x || !violations) return RH_ERR_NULL;
    return from_hip(rh::launch_check_costs(x, n, violations, static_cast<hipStream_t>(stream)));
}

const char* rh_strerror(int code) {
    switch (code) {
        case RH_OK: return "ok";
        case RH_ERR_NULL: return "a required pointer is NULL";
        case RH_ERR_SHAPE: return "a size, stride or alignment is out of range or inconsistent";
        case RH_ERR_K_RANGE: return "Kp must be a power of two in [16, 1024]";
        case RH_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case RH_ERR_OVERFLOW: return "a cost violates the cost contract";
        case RH_ERR_HIP: return "the HIP runtime refused a launch";
        case RH_ERR_STATIC_SCRATCH:
            return "these sizes need more scratch than the library's static 8 MiB (use rh_stage_dp_window with a workspace)";
        default: return "unknown error code";
    }
}

int rh_gang_workgroups(int32_t B, int32_t compute_units) { return rh::gang_workgroups(B, compute_units); }

int rh_version(void) { return 106; }

}  // extern "C"

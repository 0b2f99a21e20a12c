// Device helpers shared by the kernels that turn sharding-spec words into resharding times
// (the standalone table builder and the chain DP that computes the tables on the fly).
#pragma once
#include "kernels.h"

namespace rh {

enum : uint32_t { kNone = 0, kGather = 1, kAllToAll = 2, kAllReduce = 3, kImpossible = 4 };

// Canonical form of a spec word for one edge: per axis the state and, for a split, dim and
// lgdiv; bit 31 set = not a usable candidate.
__device__ __forceinline__ uint32_t canonical(uint32_t w, int slot, int k_real, const int64_t* dm,
                                              const Mesh& mesh) {
    uint32_t out = 0;
    bool ok = slot < k_real;
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        if (x >= mesh.naxes) break;
        const uint32_t byte = (w >> (8 * x)) & 0xFFu;
        const uint32_t st = byte & 3u, d = (byte >> 2) & 7u, lg = (byte >> 5) & 7u;
        if (st == 3u) ok = false;
        if (st == 1u) {
            if (d > 3u) {
                ok = false;
            } else {
                const int64_t blocks = (int64_t)1 << (mesh.lgm[x] + (int)lg);
                if ((dm[d] & (blocks - 1)) != 0) ok = false;
            }
            out |= byte << (8 * x);
        } else {
            out |= st << (8 * x);
        }
    }
    if (mesh.naxes == 2 && (out & 3u) == 1u && ((out >> 8) & 3u) == 1u &&
        ((out >> 2) & 7u) == ((out >> 10) & 7u))
        ok = false;   // one dim on both axes
    return ok ? out : (out | 0x80000000u);
}

// Row of the state matrix for a producer state, one nibble per consumer state (0 replicate, 1 split, 2 partial):
// replicate -> {none, none (local slice), impossible}; split -> {gather, all-to-all, impossible};
// partial -> {all-reduce, reduce-scatter = gather volume, none}.  Two equal canonical bytes cost nothing whatever
// the row says (same dim and stride).
__device__ __forceinline__ uint32_t kind_row(uint32_t ps) {
    return ps == 0u ? 0x400u : (ps == 1u ? 0x421u : 0x013u);
}

// Time of one mesh axis x for one kind of byte volume, when the other axis splits the tensor
// (o = 1) or not: the local tensor is the whole tensor over the other axis' shard count, and
// the bytes a device receives are T(m-1)/m (all-gather, reduce-scatter), T(m-1)/m^2
// (all-to-all) or twice T(m-1)/m (all-reduce); time = bytes * 1000 / bandwidth + latency.
__device__ inline int64_t axis_time(int x, int o, uint32_t kind, const Mesh& mesh, const int64_t* dm,
                                    int32_t elem_bytes) {
    if (kind == kNone || x >= mesh.naxes) return 0;
    if (kind >= kImpossible) return kInf;
    const uint64_t whole = (uint64_t)elem_bytes * (uint64_t)dm[0] * (uint64_t)dm[1] * (uint64_t)dm[2] *
                           (uint64_t)dm[3];
    const int lgo = (o && mesh.naxes == 2) ? mesh.lgm[1 - x] : 0;
    const uint64_t T = whole >> lgo;
    const int lg = mesh.lgm[x];
    const uint64_t moved = T * (((uint64_t)1 << lg) - 1);
    uint64_t V = kind == kAllToAll ? (moved >> (2 * lg)) : (moved >> lg);
    if (kind == kAllReduce) V += V;
    if (V == 0) return 0;
    const uint64_t t = V * 1000u / (uint64_t)mesh.bw_bytes_per_us[x] + (uint64_t)mesh.alpha_ns[x];
    return t < (uint64_t)kInf ? (int64_t)t : kInf;
}

}  // namespace rh

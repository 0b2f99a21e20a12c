// Chain DP that computes the resharding times from the spec words on the fly instead of
// streaming materialised tables: v_{i+1}[b] = c_{i+1}[b] + min_a (v_i[a] + R_i[a][b]) with
// R_i[a][b] evaluated per cell exactly as the table builder does (same helpers).  One graph,
// many logical meshes (Sec. 3 / Sec. 4: mesh shapes are searched in parallel): problem p is
// searched on mesh p mod n_meshes with its own node costs and shares operators, specs and
// tensor shapes with the others.
// No table ever touches HBM, so the kernel is bound by the vector ALU (about 17 operations
// per cell against 6 plus 8 streamed bytes): worth it when the tables of all problems would
// not fit in memory, and faster than streaming once many problems fill the chip.
//
// One workgroup per problem.  Per edge: 16 threads compute the 20-entry time table
// ([axis][other axis splits][none | gather | all-to-all | all-reduce | impossible]), Kp threads
// the canonical producer words; a lane owns Kp/64 consumer columns, the waves take the rows
// round-robin; a cell is two byte compares, two nibble extractions from the producer's row of
// the 3x3 state matrix, two LDS table reads and the min update.  Per-wave minima meet in LDS.
#include "kernels.h"
#include "reshard_common.h"

namespace rh {

struct MeshBatch {
    static constexpr int kMax = 64;
    int8_t naxes[kMax];
    int8_t lgm[kMax][2];
    int64_t bw_bytes_per_us[kMax][2];
    int64_t alpha_ns[kMax][2];
};

namespace {

typedef unsigned long long u64;

__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// row of the state matrix for a producer state, one nibble per consumer state (0 R, 1 S, 2 P)
__device__ __forceinline__ uint32_t kind_row(uint32_t ps) {
    // R -> {R none, S none (local slice), P impossible}; S -> {R gather, S all-to-all, P impossible};
    // P -> {R all-reduce, S reduce-scatter = gather volume, P none}
    return ps == 0u ? 0x400u : (ps == 1u ? 0x421u : 0x013u);
}

template <int KP, int W>
__global__ void __launch_bounds__(W * 64)
chain_fused_kernel(int32_t N, int32_t n_meshes, MeshBatch meshes, const int64_t* __restrict__ c, int64_t c_bs,
                   const int32_t* __restrict__ K, const uint32_t* __restrict__ out_spec,
                   const uint32_t* __restrict__ in_spec, const int64_t* __restrict__ dims,
                   const int32_t* __restrict__ elem_bytes, uint16_t* __restrict__ arg,
                   int64_t* __restrict__ vfinal, int64_t* __restrict__ total, int32_t* __restrict__ last) {
    constexpr int CPL = KP / 64;                // columns per lane: lane + 64*k
    constexpr int kThreads = W * 64;
    constexpr int MP = (KP + kThreads - 1) / kThreads;   // columns finished per thread
    __shared__ int64_t vs[KP];
    __shared__ uint32_t prow[KP];
    __shared__ int64_t tab[2][2][8];            // kinds 0..4 used
    __shared__ u64 pkey[W][KP];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int p = blockIdx.x;
    const int mi = p % n_meshes;                // problem p is searched on mesh p mod n_meshes
    Mesh mesh;
    mesh.naxes = meshes.naxes[mi];
    for (int x = 0; x < 2; ++x) {
        mesh.lgm[x] = meshes.lgm[mi][x];
        mesh.bw_bytes_per_us[x] = meshes.bw_bytes_per_us[mi][x];
        mesh.alpha_ns[x] = meshes.alpha_ns[mi][x];
    }
    const int64_t* cp = c + (int64_t)p * c_bs;

#pragma unroll
    for (int m = 0; m < MP; ++m) {
        const int col = tid + m * kThreads;
        if (col < KP) {
            const int64_t x = cp[col];
            vs[col] = x < kInf ? x : kInf;
        }
    }
    lds_barrier();

    for (int i = 0; i < N - 1; ++i) {
        const int64_t* dm = dims + (int64_t)i * 4;
        // per-edge tables
        if (tid < 20) {
            const int x = tid / 10, o = (tid / 5) & 1, kind = tid % 5;
            tab[x][o][kind] = axis_time(x, o, (uint32_t)kind, mesh, dm, elem_bytes[i]);
        }
        for (int a = tid; a < KP; a += kThreads)
            prow[a] = canonical(out_spec[(int64_t)i * KP + a], a, K[i], dm, mesh);
        // this lane's consumer columns
        uint32_t q0b[CPL], q1b[CPL], sh0[CPL], sh1[CPL], base1[CPL];
        bool qbad[CPL];
        const int k_next = K[i + 1];
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const int col = lane + 64 * k;
            const uint32_t q = canonical(in_spec[(int64_t)(i + 1) * KP + col], col, k_next, dm, mesh);
            qbad[k] = (q & 0x80000000u) != 0;
            q0b[k] = q & 0xFFu;
            q1b[k] = (q >> 8) & 0xFFu;
            sh0[k] = 4u * (q0b[k] & 3u);
            sh1[k] = 4u * (q1b[k] & 3u);
            base1[k] = ((q0b[k] & 3u) == 1u) ? 8u : 0u;   // axis 1 moves after axis 0 has the consumer's state
        }
        int64_t cn[MP];
#pragma unroll
        for (int m = 0; m < MP; ++m) {
            const int col = tid + m * kThreads;
            cn[m] = col < KP ? cp[(int64_t)(i + 1) * KP + col] : 0;
        }
        int64_t best[CPL];
        int32_t bidx[CPL];
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            best[k] = INT64_MAX;
            bidx[k] = 0;
        }
        lds_barrier();   // tab and prow are ready

        const int64_t* tab0 = &tab[0][0][0];
        const int64_t* tab1 = &tab[1][0][0];
        auto relax_row = [&](int a, uint32_t pw, int64_t va) {
            if (pw & 0x80000000u) return;     // not a candidate: the whole row is infeasible
            const uint32_t p0b = pw & 0xFFu, p1b = (pw >> 8) & 0xFFu;
            const uint32_t row0 = kind_row(p0b & 3u), row1 = kind_row(p1b & 3u);
            const uint32_t base0 = ((p1b & 3u) == 1u) ? 8u : 0u;   // axis 0 moves while axis 1 has the producer's state
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
                const uint32_t k0 = q0b[k] == p0b ? 0u : ((row0 >> sh0[k]) & 7u);
                const uint32_t k1 = q1b[k] == p1b ? 0u : ((row1 >> sh1[k]) & 7u);
                const int64_t t = tab0[base0 + k0] + tab1[base1[k] + k1];
                const int64_t key = va + t;          // <= 3 * 2^52: anything that reaches 2^52 counts as infeasible
                const bool lt = key < best[k];
                best[k] = lt ? key : best[k];
                bidx[k] = lt ? a : bidx[k];
            }
        };
        // two rows per trip so that the second row's words are already on their way
        static_assert((KP / W) % 2 == 0, "rows per wave must be even");
        for (int a = wave; a < KP; a += 2 * W) {
            const uint32_t pa = prow[a], pb = prow[a + W];
            const int64_t va = vs[a], vb = vs[a + W];
            relax_row(a, __builtin_amdgcn_readfirstlane(pa), va);
            relax_row(a + W, __builtin_amdgcn_readfirstlane(pb), vb);
        }
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const int64_t v = (qbad[k] || best[k] >= kInf) ? kInf : best[k];
            pkey[wave][lane + 64 * k] = ((u64)v << 10) | (u64)(v >= kInf ? 0 : bidx[k]);
        }
        lds_barrier();   // the waves' minima are in LDS; every read of v_i, tab, prow is done
#pragma unroll
        for (int m = 0; m < MP; ++m) {
            const int col = tid + m * kThreads;
            if (col < KP) {
                u64 mk = pkey[0][col];
#pragma unroll
                for (int w = 1; w < W; ++w) {
                    const u64 o = pkey[w][col];
                    mk = o < mk ? o : mk;
                }
                const int64_t b = (int64_t)(mk >> 10);
                const bool dead = b >= kInf;
                int64_t nv = cn[m] + (dead ? kInf : b);
                nv = nv < kInf ? nv : kInf;
                vs[col] = nv;
                arg[((int64_t)p * (N - 1) + i) * KP + col] = dead ? (uint16_t)0 : (uint16_t)(mk & 1023u);
            }
        }
        lds_barrier();   // v_{i+1} visible
    }

#pragma unroll
    for (int m = 0; m < MP; ++m) {
        const int col = tid + m * kThreads;
        if (col < KP && vfinal != nullptr) vfinal[(int64_t)p * KP + col] = vs[col];
    }
    if (wave == 0) {
        u64 key = ~0ull;
        for (int col = lane; col < KP; col += 64) {
            const u64 k0 = ((u64)vs[col] << 10) | (u64)col;
            key = k0 < key ? k0 : key;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const u64 o = __shfl_xor(key, off, 64);
            key = o < key ? o : key;
        }
        if (lane == 0) {
            total[p] = (int64_t)(key >> 10);
            last[p] = (int32_t)(key & 1023u);
        }
    }
}

}  // namespace

hipError_t launch_chain_fused(int32_t B, int32_t N, int32_t Kp, int32_t n_meshes, const Mesh* meshes,
                              const int64_t* c, int64_t c_bs,
                              const int32_t* K, const uint32_t* out_spec, const uint32_t* in_spec,
                              const int64_t* dims, const int32_t* elem_bytes, uint16_t* arg, int64_t* vfinal,
                              int64_t* total, int32_t* last, hipStream_t stream) {
    if (B == 0) return hipSuccess;
    MeshBatch mb{};
    for (int p = 0; p < n_meshes; ++p) {
        mb.naxes[p] = (int8_t)meshes[p].naxes;
        for (int x = 0; x < 2; ++x) {
            mb.lgm[p][x] = (int8_t)meshes[p].lgm[x];
            mb.bw_bytes_per_us[p][x] = meshes[p].bw_bytes_per_us[x];
            mb.alpha_ns[p][x] = meshes[p].alpha_ns[x];
        }
    }
#define RH_FUSED(KP, W)                                                                                         \
    hipLaunchKernelGGL((chain_fused_kernel<KP, W>), dim3(B), dim3(W * 64), 0, stream, N, n_meshes, mb, c, c_bs, K, \
                       out_spec, in_spec, dims, elem_bytes, arg, vfinal, total, last)
    switch (Kp) {
        case 64: RH_FUSED(64, 8); break;
        case 128: RH_FUSED(128, 16); break;
        case 256: RH_FUSED(256, 16); break;
        default: return hipErrorInvalidValue;
    }
#undef RH_FUSED
    return hipGetLastError();
}

}  // namespace rh

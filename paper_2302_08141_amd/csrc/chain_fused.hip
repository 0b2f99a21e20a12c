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
// One workgroup per problem.  Per edge: 20 threads compute the time table
// ([axis][other axis splits][none | gather | all-to-all | all-reduce | impossible]), Kp threads
// the canonical producer and consumer words; the usable producer strategies (valid spec, feasible
// v_i) and the valid consumer strategies are listed, a lane owns up to Kp/64 of the listed
// consumer columns, the waves take the listed rows round-robin; a cell is two byte compares,
// two nibble extractions from the producer's row of the 3x3 state matrix, two LDS table reads
// and the min update.  Per-wave minima meet in LDS.
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
    constexpr int CPL = KP / 64;                // consumer columns per lane: ranks lane + 64*k of the valid ones
    constexpr int kThreads = W * 64;
    static_assert(KP <= kThreads, "one thread per strategy slot");
    __shared__ int64_t vs[KP];
    __shared__ uint32_t prow[KP], qrow[KP];     // canonical producer / consumer words of the edge
    __shared__ uint16_t lrows[KP], lcols[KP];   // usable producer strategies / valid consumer strategies, ascending
    __shared__ int64_t cnx[KP];                 // node costs of the consumer operator
    __shared__ int64_t dml[2][4];
    __shared__ int32_t cnt[2][CPL];
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

    if (tid < KP) {
        const int64_t x = cp[tid];
        vs[tid] = x < kInf ? x : kInf;
    }
    lds_barrier();

    // What edge i needs from memory is asked for during edge i-1: the spec words and node costs of slot tid, the
    // tensor shape, element size and candidate counts.
    struct EdgeIn {
        uint32_t osp, isp;
        int64_t cnext, dim;                          // dim: extent tid of the edge's tensor (threads 0..3)
        int32_t k_out, k_in, eb;
    };
    auto load_edge = [&](int i) {
        EdgeIn e;
        i = i < N - 1 ? i : N - 2;                   // a load past the last edge repeats it
        const int slot = tid < KP ? tid : 0;
        e.osp = out_spec[(int64_t)i * KP + slot];
        e.isp = in_spec[(int64_t)(i + 1) * KP + slot];
        e.cnext = cp[(int64_t)(i + 1) * KP + slot];
        e.dim = dims[(int64_t)i * 4 + (tid & 3)];
        e.k_out = K[i];
        e.k_in = K[i + 1];
        e.eb = elem_bytes[i];
        return e;
    };
    // the tensor shape is indexed by the spec's dim field, so it lives in LDS (two edges, alternating)
    EdgeIn cur = load_edge(0);
    if (tid < 4) dml[0][tid] = cur.dim;
    lds_barrier();
    for (int i = 0; i < N - 1; ++i) {
        const EdgeIn nxt = load_edge(i + 1);
        const int64_t* dm = dml[i & 1];
        // per-edge tables
        if (tid < 20) {
            const int x = tid / 10, o = (tid / 5) & 1, kind = tid % 5;
            tab[x][o][kind] = axis_time(x, o, (uint32_t)kind, mesh, dm, cur.eb);
        }
        // Thread t owns strategy slot t of both operators of the edge.  A producer strategy is worth a row only if
        // its spec is a valid layout and v_i is feasible there; a consumer strategy is worth a column only if its
        // spec is valid.  Both sets are listed in ascending order and only they are visited (on graphs built from
        // specs about a third of the slots are valid, so this is a ninth of the cells).
        bool row_ok = false, col_ok = false;
        if (tid < KP) {
            const uint32_t pw = canonical(cur.osp, tid, cur.k_out, dm, mesh);
            const uint32_t qw = canonical(cur.isp, tid, cur.k_in, dm, mesh);
            prow[tid] = pw;
            qrow[tid] = qw;
            cnx[tid] = cur.cnext;
            row_ok = !(pw & 0x80000000u) && vs[tid] < kInf;
            col_ok = !(qw & 0x80000000u);
        }
        const u64 row_mask = __ballot(row_ok), col_mask = __ballot(col_ok);
        if (tid < KP && lane == 0) {
            cnt[0][wave] = __popcll(row_mask);
            cnt[1][wave] = __popcll(col_mask);
        }
        lds_barrier();
        int n_rows = 0, n_cols = 0, rows_before = 0, cols_before = 0;
#pragma unroll
        for (int w = 0; w < CPL; ++w) {
            rows_before += w < wave ? cnt[0][w] : 0;
            cols_before += w < wave ? cnt[1][w] : 0;
            n_rows += cnt[0][w];
            n_cols += cnt[1][w];
        }
        const u64 below = ((u64)1 << lane) - 1;
        if (row_ok) lrows[rows_before + __popcll(row_mask & below)] = (uint16_t)tid;
        if (col_ok) lcols[cols_before + __popcll(col_mask & below)] = (uint16_t)tid;
        lds_barrier();   // tab, prow, qrow and the two lists are ready

        // this lane's consumer columns: ranks lane + 64 k of the valid ones
        const int cplc = (n_cols + 63) >> 6;           // groups of 64 columns in use (wave-uniform)
        uint32_t q0b[CPL], q1b[CPL], sh0[CPL], sh1[CPL], base1[CPL];
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const int rank = lane + 64 * k;
            const uint32_t q = qrow[rank < n_cols ? lcols[rank] : 0];
            q0b[k] = q & 0xFFu;
            q1b[k] = (q >> 8) & 0xFFu;
            sh0[k] = 4u * (q0b[k] & 3u);
            sh1[k] = 4u * (q1b[k] & 3u);
            base1[k] = ((q0b[k] & 3u) == 1u) ? 8u : 0u;   // axis 1 moves after axis 0 has the consumer's state
        }
        // thread t finishes the column of rank t
        const int my_col = tid < n_cols ? lcols[tid] : 0;
        const int64_t cn = cnx[my_col];
        int64_t best[CPL];
        int32_t bidx[CPL];
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            best[k] = INT64_MAX;
            bidx[k] = 0;
        }

        const int64_t* tab0 = &tab[0][0][0];
        const int64_t* tab1 = &tab[1][0][0];
        auto relax_row = [&](int a, uint32_t pw, int64_t va) {
            const uint32_t p0b = pw & 0xFFu, p1b = (pw >> 8) & 0xFFu;
            const uint32_t row0 = kind_row(p0b & 3u), row1 = kind_row(p1b & 3u);
            const uint32_t base0 = ((p1b & 3u) == 1u) ? 8u : 0u;   // axis 0 moves while axis 1 has the producer's state
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
                if (k < cplc) {
                    const uint32_t k0 = q0b[k] == p0b ? 0u : ((row0 >> sh0[k]) & 7u);
                    const uint32_t k1 = q1b[k] == p1b ? 0u : ((row1 >> sh1[k]) & 7u);
                    const int64_t t = tab0[base0 + k0] + tab1[base1[k] + k1];
                    const int64_t key = va + t;          // <= 3 * 2^52: anything that reaches 2^52 counts as infeasible
                    const bool lt = key < best[k];
                    best[k] = lt ? key : best[k];
                    bidx[k] = lt ? a : bidx[k];
                }
            }
        };
        // The waves take the usable rows round-robin, in ascending order within a wave (so that a lane's first
        // minimum is its lowest row); two rows per trip so that the second row's words are already on their way.
        for (int r = wave; r < n_rows; r += 2 * W) {
            const int a = __builtin_amdgcn_readfirstlane((int)lrows[r]);
            const bool two = r + W < n_rows;
            const int b = __builtin_amdgcn_readfirstlane((int)lrows[two ? r + W : r]);
            const uint32_t pa = prow[a], pb = prow[b];
            const int64_t va = vs[a], vb = vs[b];
            relax_row(a, __builtin_amdgcn_readfirstlane(pa), va);
            if (two) relax_row(b, __builtin_amdgcn_readfirstlane(pb), vb);
        }
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const int64_t v = best[k] >= kInf ? kInf : best[k];
            pkey[wave][lane + 64 * k] = ((u64)v << 10) | (u64)(v >= kInf ? 0 : bidx[k]);
        }
        lds_barrier();   // the waves' minima are in LDS; every read of v_i, tab, prow is done
        if (tid < n_cols) {
            u64 mk = pkey[0][tid];
#pragma unroll
            for (int w = 1; w < W; ++w) {
                const u64 o = pkey[w][tid];
                mk = o < mk ? o : mk;
            }
            const int64_t b = (int64_t)(mk >> 10);
            const bool dead = b >= kInf;
            int64_t nv = cn + (dead ? kInf : b);
            nv = nv < kInf ? nv : kInf;
            vs[my_col] = nv;
            arg[((int64_t)p * (N - 1) + i) * KP + my_col] = dead ? (uint16_t)0 : (uint16_t)(mk & 1023u);
        }
        if (tid < KP && !col_ok) {                     // a strategy without a valid consumer spec
            vs[tid] = kInf;
            arg[((int64_t)p * (N - 1) + i) * KP + tid] = 0;
        }
        if (tid < 4) dml[(i + 1) & 1][tid] = nxt.dim;
        lds_barrier();   // v_{i+1} visible
        cur = nxt;
    }

    constexpr int MP = 1;
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

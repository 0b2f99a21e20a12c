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
// ([axis][other axis splits][none | gather | all-to-all | all-reduce | impossible]), 2 Kp threads
// the canonical producer and consumer words; the valid producer and consumer strategies are
// listed, a lane owns up to Kp/64 of the listed consumer columns, the waves take the listed rows
// round-robin (a row whose v_i is infeasible is passed over); a cell is two byte compares, two
// nibble extractions from the producer's row of the 3x3 state matrix, two LDS table reads and the
// min update.  Per-wave minima meet in LDS.  None of the tables and lists of an edge depends on
// the vector, so those of edge i + 1 are made (in a second set of buffers) while edge i is
// relaxed: two workgroup barriers per edge, and the table's 64-bit divisions off the critical path.
#include "kernels.h"
#include "reshard_common.h"

namespace rh {

// Sweeping parts of chains instead of whole chains (the segmented route): see the kernel.
struct FusedParts {
    int32_t len;                 // edges per part; 0 = whole chains
    int32_t n_full;              // parts of that length per problem; one more part takes the rest of the chain
    const int64_t* v_start;      // start vector of part q of problem p at v_start + p * v_bs + q * v_stride
    int64_t v_stride, v_bs;
};

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

template <int KP, int W>
__global__ void __launch_bounds__(W * 64)
chain_fused_kernel(int32_t N_chain, int32_t n_meshes, MeshBatch meshes, const int64_t* __restrict__ c, int64_t c_bs,
                   const int32_t* __restrict__ K, const uint32_t* __restrict__ out_spec,
                   const uint32_t* __restrict__ in_spec, const int64_t* __restrict__ dims,
                   const int32_t* __restrict__ elem_bytes, uint16_t* __restrict__ arg,
                   int64_t* __restrict__ vfinal, int64_t* __restrict__ total, int32_t* __restrict__ last,
                   FusedParts parts) {
    constexpr int CPL = KP / 64;                // consumer columns per lane: ranks lane + 64*k of the valid ones
    constexpr int kThreads = W * 64;
    static_assert(2 * KP <= kThreads, "a thread per strategy slot and side of the edge");
    __shared__ int64_t vs[KP];
    // per-edge tables, two sets: while edge i is relaxed out of set i & 1, set (i + 1) & 1 is made ready for the next
    __shared__ uint32_t prow[2][KP], qrow[2][KP];   // canonical producer / consumer words of the edge
    __shared__ uint16_t lrows[2][KP], lcols[2][KP]; // valid producer / consumer strategies, ascending
    __shared__ int64_t cnx[2][KP];                  // node costs of the consumer operator
    __shared__ int64_t dml[2][4];                   // extents of the edge's tensor (indexed by the spec's dim field)
    __shared__ int32_t cnt[2][2][CPL];              // [set][producer | consumer][wave]: valid strategies per 64 slots
    __shared__ int64_t tab[2][2][2][8];             // [set][axis][other axis splits][kind], kinds 0..4 used
    __shared__ u64 pkey[W][KP];
    __shared__ uint16_t argl[KP];                   // arg of the edge just finished, by strategy slot

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    // Whole chains: workgroup = problem.  Parts of chains (parts.len > 0): workgroup (q, p) sweeps part q of problem
    // p from the start vector it is handed: parts.len edges from operator q * parts.len, the last workgroup of a
    // problem (q = parts.n_full) the rest of the chain, and only that one writes vfinal, total and last.
    const int p = parts.len > 0 ? blockIdx.y : blockIdx.x;
    const int q = parts.len > 0 ? blockIdx.x : 0;
    const int o_first = q * parts.len;
    const int N = parts.len > 0 ? (q < parts.n_full ? parts.len : N_chain - 1 - o_first) + 1 : N_chain;
    const bool writes_final = parts.len == 0 || q == parts.n_full;
    K += o_first;
    out_spec += (int64_t)o_first * KP;
    in_spec += (int64_t)o_first * KP;
    dims += (int64_t)o_first * 4;
    elem_bytes += o_first;
    uint16_t* argp = arg + ((int64_t)p * (N_chain - 1) + o_first) * KP;
    const int mi = p % n_meshes;                // problem p is searched on mesh p mod n_meshes
    // The mesh is indexed by axis numbers computed at run time: in LDS that is an address, in registers it would
    // send the struct to scratch memory (and every wait for a scratch access drains the loads that run ahead).
    __shared__ Mesh mesh;
    if (tid == 0) {
        mesh.naxes = meshes.naxes[mi];
        for (int x = 0; x < 2; ++x) {
            mesh.lgm[x] = meshes.lgm[mi][x];
            mesh.bw_bytes_per_us[x] = meshes.bw_bytes_per_us[mi][x];
            mesh.alpha_ns[x] = meshes.alpha_ns[mi][x];
        }
    }
    const int64_t* cp = c + (int64_t)p * c_bs + (int64_t)o_first * KP;

    if (tid < KP) {
        const int64_t x = parts.len > 0 ? parts.v_start[(int64_t)p * parts.v_bs + (int64_t)q * parts.v_stride + tid]
                                        : cp[tid];
        vs[tid] = x < kInf ? x : kInf;
        argl[tid] = 0;
    }

    // What edge i needs from memory is asked for two edges ahead: the spec words and node costs of slot tid, the
    // tensor shape, element size and candidate counts.
    struct EdgeIn {
        uint32_t osp, isp;
        int64_t cnext, dim;                          // dim: extent tid of the edge's tensor (threads 0..3)
        int32_t k_out, k_in, eb;
    };
    auto load_edge = [&](int i) {
        EdgeIn e;
        i = i < N - 1 ? i : N - 2;                   // a load past the last edge repeats it
        i = i > 0 ? i : 0;
        const int slot = tid & (KP - 1);
        e.osp = out_spec[(int64_t)i * KP + slot];
        e.isp = in_spec[(int64_t)(i + 1) * KP + slot];
        e.cnext = cp[(int64_t)(i + 1) * KP + slot];
        e.dim = dims[(int64_t)i * 4 + (tid & 3)];
        e.k_out = K[i];
        e.k_in = K[i + 1];
        e.eb = elem_bytes[i];
        return e;
    };
    // Everything about an edge that does not depend on the vector: the time table (one wave's 20 lanes; it holds
    // the only 64-bit divisions), the canonical words of slot tid, which slots are valid layouts, how many per
    // 64 slots.  Thread t owns strategy slot t of both operators of the edge; the masks stay in registers until
    // the counts of all waves are visible and the ascending lists can be written (list_edge).
    struct Prepared {
        bool row_ok, col_ok;
        u64 row_mask, col_mask;
    };
    auto prepare_edge = [&](const EdgeIn& e, int set) {
        const int64_t* dm = dml[set];
        if (wave == W - 1 && lane < 20) {
            const int x = lane / 10, o = (lane / 5) & 1, kind = lane % 5;
            tab[set][x][o][kind] = axis_time(x, o, (uint32_t)kind, mesh, dm, e.eb);
        }
        // the producer words by the first Kp threads, the consumer words (and node costs) by the next Kp
        Prepared pr{false, false, 0, 0};
        if (tid < KP) {
            const uint32_t pw = canonical(e.osp, tid, e.k_out, dm, mesh);
            prow[set][tid] = pw;
            pr.row_ok = !(pw & 0x80000000u);
        } else if (tid < 2 * KP) {
            const uint32_t qw = canonical(e.isp, tid - KP, e.k_in, dm, mesh);
            qrow[set][tid - KP] = qw;
            cnx[set][tid - KP] = e.cnext;
            pr.col_ok = !(qw & 0x80000000u);
        }
        pr.row_mask = __ballot(pr.row_ok);
        pr.col_mask = __ballot(pr.col_ok);
        if (lane == 0) {
            if (tid < KP) cnt[set][0][wave] = __popcll(pr.row_mask);
            else if (tid < 2 * KP) cnt[set][1][wave - CPL] = __popcll(pr.col_mask);
        }
        return pr;
    };
    auto list_edge = [&](const Prepared& pr, int set) {
        const int which = tid < KP ? 0 : 1, w0 = tid < KP ? wave : wave - CPL;   // which list, which 64 slots of it
        if (tid < 2 * KP) {
            int before = 0;
#pragma unroll
            for (int w = 0; w < CPL; ++w) before += w < w0 ? cnt[set][which][w] : 0;
            const u64 below = ((u64)1 << lane) - 1;
            if (pr.row_ok) lrows[set][before + __popcll(pr.row_mask & below)] = (uint16_t)tid;
            if (pr.col_ok) lcols[set][before + __popcll(pr.col_mask & below)] = (uint16_t)(tid - KP);
        }
    };

    EdgeIn e1 = load_edge(0);
    if (tid < 4) dml[0][tid] = e1.dim;
    lds_barrier();
    Prepared ready = prepare_edge(e1, 0);
    e1 = load_edge(1);
    if (tid < 4) dml[1][tid] = e1.dim;
    lds_barrier();
    list_edge(ready, 0);
    lds_barrier();
    for (int i = 0; i < N - 1; ++i) {
        const int cs = i & 1, ns = cs ^ 1;           // this edge's set of tables, the next edge's
        const EdgeIn e2 = load_edge(i + 2);
        // arg of edge i - 1 leaves now, one store per thread whatever the thread (a store under a condition would
        // keep the waits below from counting the loads that run ahead; threads beyond Kp repeat a slot).  At i = 0
        // the store puts a placeholder into edge 0's row.  Every thread that writes a slot writes the same slot of
        // the same row again one edge later (or after the loop) with the final value, and a thread's own stores to
        // one address keep their order, so whichever thread's store lands last, it is a final one.
        argp[(int64_t)(i > 0 ? i - 1 : 0) * KP + (tid & (KP - 1))] = argl[tid & (KP - 1)];
        // ---- first half: relax edge i; on the side, the tables of edge i + 1 ----
        ready = prepare_edge(e1, ns);
        int n_rows = 0, n_cols = 0;
#pragma unroll
        for (int w = 0; w < CPL; ++w) {
            n_rows += cnt[cs][0][w];
            n_cols += cnt[cs][1][w];
        }
        // A producer strategy is worth a row only if its spec is a valid layout (listed) and v_i is feasible there
        // (checked when its turn comes); a consumer strategy is worth a column only if its spec is valid.  On
        // graphs built from specs about a third of the slots are valid, so this is a ninth of the cells.
        // This lane's consumer columns: ranks lane + 64 k of the valid ones.
        const int cplc = (n_cols + 63) >> 6;           // groups of 64 columns in use (wave-uniform)
        uint32_t q0b[CPL], q1b[CPL], sh0[CPL], sh1[CPL], base1[CPL];
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const int rank = lane + 64 * k;
            const uint32_t q = qrow[cs][rank < n_cols ? lcols[cs][rank] : 0];
            q0b[k] = q & 0xFFu;
            q1b[k] = (q >> 8) & 0xFFu;
            sh0[k] = 4u * (q0b[k] & 3u);
            sh1[k] = 4u * (q1b[k] & 3u);
            base1[k] = ((q0b[k] & 3u) == 1u) ? 8u : 0u;   // axis 1 moves after axis 0 has the consumer's state
        }
        // thread t finishes the column of rank t
        const int my_col = tid < n_cols ? lcols[cs][tid] : 0;
        const int64_t cn = cnx[cs][my_col];
        int64_t best[CPL];
        int32_t bidx[CPL];
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            best[k] = INT64_MAX;
            bidx[k] = 0;
        }

        const int64_t* tab0 = &tab[cs][0][0][0];
        const int64_t* tab1 = &tab[cs][1][0][0];
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
        // The waves take the listed rows round-robin, in ascending order within a wave (so that a lane's first
        // minimum is its lowest row); two rows per trip so that the second row's words are already on their way.
        for (int r = wave; r < n_rows; r += 2 * W) {
            const int a = __builtin_amdgcn_readfirstlane((int)lrows[cs][r]);
            const bool two = r + W < n_rows;
            const int b = __builtin_amdgcn_readfirstlane((int)lrows[cs][two ? r + W : r]);
            const uint32_t pa = prow[cs][a], pb = prow[cs][b];
            const int64_t va = vs[a], vb = vs[b];
            if (va < kInf) relax_row(a, __builtin_amdgcn_readfirstlane(pa), va);
            if (two && vb < kInf) relax_row(b, __builtin_amdgcn_readfirstlane(pb), vb);
        }
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const int64_t v = best[k] >= kInf ? kInf : best[k];
            pkey[wave][lane + 64 * k] = ((u64)v << 10) | (u64)(v >= kInf ? 0 : bidx[k]);
        }
        lds_barrier();   // the waves' minima and the next edge's counts are in LDS; every read of v_i is done
        // ---- second half: v_{i+1} and arg; the lists of edge i + 1 ----
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
            argl[my_col] = dead ? (uint16_t)0 : (uint16_t)(mk & 1023u);
        }
        if (tid < KP && (qrow[cs][tid] & 0x80000000u)) {   // a strategy without a valid consumer spec
            vs[tid] = kInf;
            argl[tid] = 0;
        }
        list_edge(ready, ns);
        if (tid < 4) dml[cs][tid] = e2.dim;            // set cs serves edge i + 2 next
        lds_barrier();   // v_{i+1} and the lists of edge i + 1 visible
        e1 = e2;
    }
    if (N > 1) argp[(int64_t)(N - 2) * KP + (tid & (KP - 1))] = argl[tid & (KP - 1)];
    if (!writes_final) return;

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

static hipError_t launch_fused(int32_t B, int32_t N, int32_t Kp, int32_t n_meshes, const Mesh* meshes,
                               const int64_t* c, int64_t c_bs,
                               const int32_t* K, const uint32_t* out_spec, const uint32_t* in_spec,
                               const int64_t* dims, const int32_t* elem_bytes, uint16_t* arg, int64_t* vfinal,
                               int64_t* total, int32_t* last, const FusedParts& parts, hipStream_t stream) {
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
    const dim3 grid = parts.len > 0 ? dim3((unsigned)(parts.n_full + 1), (unsigned)B) : dim3((unsigned)B);
#define RH_FUSED(KP, W)                                                                                         \
    hipLaunchKernelGGL((chain_fused_kernel<KP, W>), grid, dim3(W * 64), 0, stream, N, n_meshes, mb, c, c_bs, K, \
                       out_spec, in_spec, dims, elem_bytes, arg, vfinal, total, last, parts)
    switch (Kp) {
        case 64: RH_FUSED(64, 8); break;
        case 128: RH_FUSED(128, 16); break;
        case 256: RH_FUSED(256, 16); break;
        default: return hipErrorInvalidValue;
    }
#undef RH_FUSED
    return hipGetLastError();
}

hipError_t launch_chain_fused(int32_t B, int32_t N, int32_t Kp, int32_t n_meshes, const Mesh* meshes,
                              const int64_t* c, int64_t c_bs,
                              const int32_t* K, const uint32_t* out_spec, const uint32_t* in_spec,
                              const int64_t* dims, const int32_t* elem_bytes, uint16_t* arg, int64_t* vfinal,
                              int64_t* total, int32_t* last, hipStream_t stream) {
    return launch_fused(B, N, Kp, n_meshes, meshes, c, c_bs, K, out_spec, in_spec, dims, elem_bytes, arg, vfinal, total,
                        last, FusedParts{0, 0, nullptr, 0, 0}, stream);
}

hipError_t launch_chain_fused_parts(int32_t B, int32_t N, int32_t Kp, int32_t n_meshes, const Mesh* meshes,
                                    const int64_t* c, int64_t c_bs, const int32_t* K, const uint32_t* out_spec,
                                    const uint32_t* in_spec, const int64_t* dims, const int32_t* elem_bytes,
                                    int32_t part_len, int32_t n_full, const int64_t* v_start, int64_t v_stride,
                                    int64_t v_bs, uint16_t* arg, int64_t* vfinal, int64_t* total, int32_t* last,
                                    hipStream_t stream) {
    return launch_fused(B, N, Kp, n_meshes, meshes, c, c_bs, K, out_spec, in_spec, dims, elem_bytes, arg, vfinal, total,
                        last, FusedParts{part_len, n_full, v_start, v_stride, v_bs}, stream);
}

}  // namespace rh

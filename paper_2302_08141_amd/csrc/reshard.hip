// Resharding-cost tables from sharding specs on gfx950.
//
// R[e][a][b] = time to move the tensor on edge e from the producer's layout a to the
// consumer's layout b.  Layouts are (dim, stride) splits, replicate or partial per mesh
// axis (Sec. 4.1, Sec. 4.3.3), the mesh axes are handled one after the other (Sec. 4),
// and a mismatch costs one of the collectives of Sec. 2.1.  With power-of-two axis sizes
// a stride change on the same dim moves exactly the bytes of a dim change, so per axis
// only four byte volumes exist -- none, T(m-1)/m, T(m-1)/m^2, 2T(m-1)/m -- for two
// possible local sizes T.  Each workgroup turns those into a 16-entry time table once
// (the only 64-bit divisions), and a cell is two classifications and two table reads.
// The kernel is bound by the 8 bytes it writes per cell; rows are written as coalesced
// 16-byte stores.
#include "kernels.h"
#include "reshard_common.h"

namespace rh {
namespace {

typedef long long ll2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kPanelRows = 16;   // rows of one edge table per workgroup

__device__ __forceinline__ uint32_t transition(uint32_t pb, uint32_t qb) {
    const uint32_t ps = pb & 3u, qs = qb & 3u;
    if (pb == qb) return kNone;
    if (qs == 2u) return kImpossible;        // nothing becomes partial
    if (ps == 0u) return kNone;              // replicate -> split: local slice
    if (ps == 1u) return qs == 0u ? kGather : kAllToAll;
    return qs == 1u ? kGather : kAllReduce;  // partial -> split moves the all-gather volume
}

__device__ __forceinline__ int64_t cell(uint32_t p, uint32_t q, const int64_t (*tab)[2][4]) {
    if ((p | q) & 0x80000000u) return kInf;
    const uint32_t k0 = transition(p & 0xFFu, q & 0xFFu);
    const uint32_t k1 = transition((p >> 8) & 0xFFu, (q >> 8) & 0xFFu);
    if ((k0 | k1) & 4u) return kInf;
    // axis 0 moves while axis 1 still has the producer's state; axis 1 moves after axis 0
    // already has the consumer's state
    const uint32_t o0 = ((p >> 8) & 3u) == 1u;
    const uint32_t o1 = (q & 3u) == 1u;
    const int64_t t = tab[0][o0][k0] + tab[1][o1][k1];
    return t < kInf ? t : kInf;
}

__global__ void __launch_bounds__(kThreads)
reshard_kernel(Mesh mesh, int32_t Kp, int32_t lgKp, const int32_t* __restrict__ K,
               const uint32_t* __restrict__ out_spec, const uint32_t* __restrict__ in_spec,
               const int64_t* __restrict__ dims, const int32_t* __restrict__ elem_bytes,
               int64_t* __restrict__ R) {
    __shared__ int64_t tab[2][2][4];          // [axis][other axis splits][volume kind] -> ns
    __shared__ uint32_t prow[kPanelRows];

    const int e = blockIdx.x;
    const int row0 = blockIdx.y * kPanelRows;
    const int tid = threadIdx.x;
    const int64_t* dm = dims + (int64_t)e * 4;

    if (tid < 16) {
        const int x = tid >> 3, o = (tid >> 2) & 1, kind = tid & 3;
        tab[x][o][kind] = axis_time(x, o, kind, mesh, dm, elem_bytes[e]);
    }
    if (tid >= 64 && tid < 64 + kPanelRows) {
        const int a = row0 + (tid - 64);
        prow[tid - 64] = a < Kp ? canonical(out_spec[(int64_t)e * Kp + a], a, K[e], dm, mesh)
                                : 0x80000000u;
    }
    __syncthreads();

    const int pairs = Kp >> 1;                         // 16-byte column pairs per row
    const int tc = pairs < kThreads ? pairs : kThreads; // threads along a row
    const int tr = kThreads / tc;                       // rows handled at once
    const int my_c = tid % tc, my_r = tid / tc;
    const int k_next = K[e + 1];
    int64_t* Re = R + ((int64_t)e << (2 * lgKp));
    for (int cpair = my_c; cpair < pairs; cpair += tc) {
        const int b = 2 * cpair;
        const uint2 qw = *reinterpret_cast<const uint2*>(in_spec + (int64_t)(e + 1) * Kp + b);
        const uint32_t q0 = canonical(qw.x, b, k_next, dm, mesh);
        const uint32_t q1 = canonical(qw.y, b + 1, k_next, dm, mesh);
        for (int r = my_r; r < kPanelRows && row0 + r < Kp; r += tr) {
            const uint32_t p = prow[r];
            ll2 out;
            out.x = cell(p, q0, tab);
            out.y = cell(p, q1, tab);
            __builtin_nontemporal_store(out, reinterpret_cast<ll2*>(Re + ((int64_t)(row0 + r) << lgKp) + b));
        }
    }
}

}  // namespace

hipError_t launch_reshard(const Mesh& mesh, int32_t n_edges, int32_t Kp, const int32_t* K,
                          const uint32_t* out_spec, const uint32_t* in_spec, const int64_t* dims,
                          const int32_t* elem_bytes, int64_t* R, hipStream_t stream) {
    if (n_edges == 0) return hipSuccess;
    int lgKp = 0;
    while ((1 << lgKp) < Kp) ++lgKp;
    // grid.x carries the edges (up to 2^31-1), grid.y the row panels
    dim3 grid((unsigned)n_edges, (unsigned)((Kp + kPanelRows - 1) / kPanelRows));
    hipLaunchKernelGGL(reshard_kernel, grid, dim3(kThreads), 0, stream, mesh, Kp, lgKp, K, out_spec,
                       in_spec, dims, elem_bytes, R);
    return hipGetLastError();
}

}  // namespace rh

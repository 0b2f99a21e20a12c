// The table of all interval stage times (see interval_costs.hip) by blocks instead of row by row.
//
// Row i of the table is a forward sweep from operator i to the end of the chain: L^2/2 sweep steps of Kp^2 cells.
// Min-plus products are associative, so an interval that crosses block boundaries can be put together from three
// pieces.  Cut the chain into blocks of kBlk operators; write B(p) for the first operator of block p.  For i in
// block p and B(q+1) < j <= B(q+2) (the interval ends in block q+1, q >= p):
//     T[i][j] = min_{x,z}  A_i[x]  +  P_pq[x][z]  +  Z_{q+1}[z][j - B(q+1)]
//   A_i[x]      least cost of operators i .. B(p+1) with strategy x at B(p+1), its node cost included
//               (the sweep of row i, stopped one operator into the next block)
//   P_pq[x][z]  least cost from B(p+1) with x (node cost left out) to B(q+1) with z (included): the product of
//               the blocks' own matrices M_{p+1} (x) .. (x) M_q; the identity for q = p
//   Z_b[z][t]   least cost of the first t operators of block b given strategy z at its first operator, that node
//               cost left out: sweeps with the Kp strategies of B(b) as rows; the last of them is M_b
// Intervals inside a block (and one operator beyond) come from the row sweeps directly.  Every value is a minimum
// of the same saturating sums as in the plain sweep, regrouped; saturation at "infeasible" is monotone, so it
// commutes with the regrouping and the table is the same bit for bit.
// Work: sweeps inside blocks (2 L kBlk Kp^2 cells), L/kBlk - 2 chains of Kp^3 products, and per pair of blocks
// kBlk Kp^2 + kBlk^2 Kp cells -- about a tenth of L^2/2 Kp^2 at L = 4096, Kp = 64 -- and no chain of dependent
// steps longer than a block.
// Kp = 64 only; fp64 arithmetic as in interval_costs.hip (exact for these integers).
#include "kernels.h"
#include "minplus_rows.h"

namespace rh {
namespace {

constexpr int kBlk = 128;                    // operators per block
constexpr int kK = 64;                       // Kp
constexpr int kLdz = kBlk + 2;               // row stride of a block's Z table (entries t = 0 .. kBlk + 1)
constexpr int kTile = 64;
constexpr int kLds = kTile + 2;              // row stride of a staged tile in LDS (16-byte aligned rows, fewer bank clashes)

// C[i][n] = min_x A[i][x] + Bm[x][n] (saturated) for i < m, n < nn (both <= 64), x < 64.  256 threads; thread
// (tx, ty) keeps a 4 x 4 corner of the tile.  As (transposed, [x][i]) and Bs ([x][n]) are LDS tiles of kK * kLds
// doubles.  With a limit on the interval length (the tiles of T only) entries beyond it are stored as infeasible.
__device__ __forceinline__ void mm_tile(const int64_t* __restrict__ A, int64_t lda, int m, const int64_t* __restrict__ Bm,
                                        int64_t ldb, int nn, int64_t* __restrict__ C, int64_t ldc, double* As,
                                        double* Bs, int len0 = 0, int max_len = INT32_MAX) {
    const int tid = threadIdx.x;
    const int lx = tid & 63, l4 = tid >> 6;
#pragma unroll 4
    for (int r = 0; r < 16; ++r) {
        const int i = l4 + 4 * r;
        As[lx * kLds + i] = i < m ? to_f64(A[(int64_t)i * lda + lx]) : kInfD;
    }
#pragma unroll 4
    for (int r = 0; r < 16; ++r) {
        const int x = l4 + 4 * r;
        Bs[x * kLds + lx] = lx < nn ? to_f64(Bm[(int64_t)x * ldb + lx]) : kInfD;
    }
    __syncthreads();
    const int tx = tid & 15, ty = tid >> 4;
    double acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[r][k] = kInfD;
#pragma unroll 8
    for (int x = 0; x < kK; ++x) {
        double a[4], b[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) a[r] = As[x * kLds + 4 * ty + r];
#pragma unroll
        for (int k = 0; k < 4; ++k) b[k] = Bs[x * kLds + 4 * tx + k];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[r][k] = __builtin_fmin(acc[r][k], a[r] + b[k]);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = 4 * ty + r;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int n = 4 * tx + k;
            const double v = __builtin_fmin(acc[r][k], kInfD);
            // entry (i, n) stands for an interval of len0 + n - i operators: longer than max_len counts as infeasible
            if (i < m && n < nn) C[(int64_t)i * ldc + n] = len0 + n - i > max_len ? kInf : to_i64(v);
        }
    }
}

// T[i][j] = infeasible for the columns left of row i's own block (the row sweeps write the rest of the columns at
// and left of the diagonal themselves) and, when intervals are limited in length, for the columns right of the
// last block that the row's pairs of blocks reach (dq = how many blocks lie between the two of a pair at most).
__global__ void __launch_bounds__(256)
ib_fill_kernel(int32_t L, int32_t dq, int64_t ldT, int64_t* __restrict__ T, int64_t T_bs) {
    const int i = blockIdx.x;
    const int pb = i / kBlk;
    const int n = pb * kBlk;
    int64_t* row = T + (int64_t)blockIdx.y * T_bs + (int64_t)i * ldT;
    for (int j = threadIdx.x; j < n; j += 256) row[j] = kInf;
    const int64_t reach = ((int64_t)pb + dq + 2) * kBlk;          // the pairs (pb, pb .. pb + dq) end at this column
    for (int64_t j = reach + 1 + threadIdx.x; j <= L; j += 256) row[j] = kInf;
}

// Chain p: P[p][q] = P[p][q-1] (x) M[q] for q = p + 2 .. nb - 2, with P[p][p+1] = M[p+1].  The rows of a product only
// depend on the same rows of the product before, so a chain is shared out over kPrefixSplit workgroups of 8 waves;
// a wave keeps its rows of the running product in registers (lane = column), M[q] is staged in LDS (the next one
// is fetched while this one is used), and a step is the row relaxation of the interval kernel.
constexpr int kPrefixWaves = 8;
constexpr int kPrefixSplit = 4;
__global__ void __launch_bounds__(kPrefixWaves * 64)
ib_prefix_kernel(int32_t nb, int32_t dq, const int64_t* __restrict__ M, int64_t* __restrict__ P, int64_t ws_bs) {
    constexpr int kThreads = kPrefixWaves * 64, kPairs = kK / kPrefixSplit / kPrefixWaves / 2, kEpt = kK * kK / kThreads;
    static_assert(kPairs >= 1, "two rows per wave at least");
    extern __shared__ double tiles[];             // two tables of Kp x Kp
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int p = blockIdx.x / kPrefixSplit, part = blockIdx.x % kPrefixSplit;
    M += (int64_t)blockIdx.y * ws_bs;
    P += (int64_t)blockIdx.y * ws_bs;
    const int64_t mat = (int64_t)kK * kK;
    const int q0 = p + 2, q1 = p + dq < nb - 2 ? p + dq : nb - 2;   // products beyond p + dq serve no pair
    if (q0 > q1) return;
    const int row0 = (part * kPrefixWaves + wave) * 2 * kPairs;   // this wave's rows: row0 .. row0 + 2 kPairs - 1
    double V[kPairs][2][1];
#pragma unroll
    for (int h = 0; h < kPairs; ++h)
#pragma unroll
        for (int s = 0; s < 2; ++s) V[h][s][0] = to_f64(M[(int64_t)(p + 1) * mat + (row0 + 2 * h + s) * kK + lane]);
    int64_t pre[kEpt];
    auto fetch = [&](int q) {
        q = q <= q1 ? q : q1;
#pragma unroll
        for (int e = 0; e < kEpt; ++e) pre[e] = M[(int64_t)q * mat + e * kThreads + tid];
    };
    auto stash = [&](int q) {
        double* dst = tiles + ((q - q0) & 1) * (kK * kK);
#pragma unroll
        for (int e = 0; e < kEpt; ++e) dst[e * kThreads + tid] = to_f64(pre[e]);
    };
    fetch(q0);
    stash(q0);
    fetch(q0 + 1);
    lds_barrier();
    for (int q = q0; q <= q1; ++q) {
        const double* table = tiles + ((q - q0) & 1) * (kK * kK);
#pragma unroll
        for (int h = 0; h < kPairs; ++h) {
            double acc[2][1] = {{kInfD}, {kInfD}};
            relax_rows64<2, 2>(table, lane, V[h], acc);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                V[h][s][0] = __builtin_fmin(acc[s][0], kInfD);
                P[((int64_t)p * nb + q) * mat + (row0 + 2 * h + s) * kK + lane] = to_i64(V[h][s][0]);
            }
            __builtin_amdgcn_sched_barrier(0);    // one pair of rows after the other: their registers are reused
        }
        if (q < q1) stash(q + 1);
        fetch(q + 2);
        lds_barrier();                            // the next table is in LDS; this one has been read for the last time
    }
}

// U[p][q] = A[p] (x) P_pq for p < q <= nb - 2 (kBlk x Kp each; P_pq = M[p+1] for q = p + 1).  blockIdx.x = half of
// the rows, blockIdx.y = pair index, blockIdx.z = problem.
__global__ void __launch_bounds__(256)
ib_left_kernel(int32_t nb, const int32_t* __restrict__ pair_p, const int32_t* __restrict__ pair_q,
               const int64_t* __restrict__ A, const int64_t* __restrict__ M, const int64_t* __restrict__ P,
               int64_t* __restrict__ U, int64_t ws_bs) {
    extern __shared__ double tiles[];
    const int p = pair_p[blockIdx.y], q = pair_q[blockIdx.y];
    if (q <= p) return;                           // the pair (p, p) needs no product
    const int64_t off = (int64_t)blockIdx.z * ws_bs, mat = (int64_t)kK * kK;
    const int64_t* Ap = A + off + ((int64_t)p * kBlk + blockIdx.x * kTile) * kK;
    const int64_t* Pq = q == p + 1 ? M + off + (int64_t)q * mat : P + off + ((int64_t)p * nb + q) * mat;
    int64_t* Uq = U + off + (((int64_t)p * nb + q) * kBlk + blockIdx.x * kTile) * kK;
    mm_tile(Ap, kK, kTile, Pq, kK, kK, Uq, kK, tiles, tiles + kK * kLds);
}

// The entries of T for rows in block p and columns B(q+1) + 1 .. B(q+1) + n_t: U_pq (x) Z_{q+1}.  blockIdx.x = tile
// of 64 x 64 entries (2 x 2 per pair), blockIdx.y = pair, blockIdx.z = problem.
__global__ void __launch_bounds__(256)
ib_tiles_kernel(int32_t L, int32_t nb, const int32_t* __restrict__ pair_p, const int32_t* __restrict__ pair_q,
                const int64_t* __restrict__ A, const int64_t* __restrict__ U, const int64_t* __restrict__ Z,
                int64_t ws_bs, int64_t ldT, int64_t* __restrict__ T, int64_t T_bs, int32_t max_len) {
    extern __shared__ double tiles[];
    const int p = pair_p[blockIdx.y], q = pair_q[blockIdx.y];
    if (p < 0 || q < p) return;                   // an unused slot of the pair list
    const int ti = blockIdx.x >> 1, tj = blockIdx.x & 1;
    const int col0 = (q + 1) * kBlk;              // B(q+1)
    const int n_t = L - col0 < kBlk ? L - col0 : kBlk;        // columns col0 + 1 .. col0 + n_t
    const int nn = n_t - tj * kTile < kTile ? n_t - tj * kTile : kTile;
    if (nn <= 0) return;
    const int64_t off = (int64_t)blockIdx.z * ws_bs;
    const int64_t* Up = q == p ? A + off + ((int64_t)p * kBlk + ti * kTile) * kK
                               : U + off + (((int64_t)p * nb + q) * kBlk + ti * kTile) * kK;
    const int64_t* Zq = Z + off + (int64_t)(q + 1) * kK * kLdz + 1 + tj * kTile;   // entry t = 1 + n of every row z
    int64_t* Tt = T + (int64_t)blockIdx.z * T_bs + ((int64_t)p * kBlk + ti * kTile) * ldT + col0 + 1 + tj * kTile;
    mm_tile(Up, kK, kTile, Zq, kLdz, nn, Tt, ldT, tiles, tiles + kK * kLds,
            col0 + 1 + tj * kTile - (p * kBlk + ti * kTile), max_len);
}

struct IbLayout {
    int nb, n_pairs;
    size_t a_off, z_off, m_off, p_off, u_off, pair_off, total;   // bytes; a..u per problem, the pair lists shared
    size_t per_problem;
};

IbLayout ib_layout(int32_t B, int32_t L) {
    IbLayout o{};
    o.nb = (L + kBlk - 1) / kBlk;
    o.n_pairs = (o.nb - 1) * o.nb / 2;            // 0 <= p <= q <= nb - 2: the longest list
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t nb = (size_t)o.nb, mat = (size_t)kK * kK * 8;
    o.a_off = 0;
    o.z_off = o.a_off + up(nb * kBlk * kK * 8);
    o.m_off = o.z_off + up(nb * kK * kLdz * 8);
    o.p_off = o.m_off + up(nb * mat);
    o.u_off = o.p_off + up(nb * nb * mat);
    o.per_problem = o.u_off + up(nb * nb * kBlk * kK * 8);
    o.pair_off = (size_t)B * o.per_problem;
    o.total = o.pair_off + up(2 * (size_t)(o.n_pairs > 0 ? o.n_pairs : 1) * sizeof(int32_t));
    return o;
}

// the pair lists (p, q), 0 <= p <= q <= min(p + dq, nb - 2), in the order p = 0: q = 0 .. ; p = 1: q = 1 .. ; ...,
// written by the device itself: nothing is copied from the host
__global__ void __launch_bounds__(256)
ib_pairs_kernel(int32_t nb, int32_t dq, int32_t n_pairs, int32_t* __restrict__ pair_p, int32_t* __restrict__ pair_q) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= n_pairs) return;
    int p = 0, first = 0;
    for (; p < nb - 2; ++p) {
        const int len = (dq < nb - 2 - p ? dq : nb - 2 - p) + 1;
        if (t < first + len) break;
        first += len;
    }
    pair_p[t] = p;
    pair_q[t] = p + (t - first);
}

}  // namespace

// Chains of at least four blocks of Kp = 64 strategies; 0 = the route does not apply.
size_t interval_blocks_workspace_bytes(int32_t B, int32_t L, int32_t Kp) {
    if (B < 1 || Kp != kK || L < 4 * kBlk || L > 16384) return 0;
    return ib_layout(B, L).total;
}

hipError_t launch_interval_costs_blocked(int32_t B, int32_t L, int32_t max_len, const int64_t* c, const int64_t* R,
                                         int64_t ldT, int64_t* T, void* workspace, hipStream_t stream) {
    if (B == 0) return hipSuccess;
    if (max_len < kBlk + 1) return hipErrorInvalidValue;      // the sweeps inside a block run to its end
    const IbLayout lay = ib_layout(B, L);
    const int nb = lay.nb;
    // Rows of block p and columns of block q + 1 are at least (q - p) kBlk + 2 operators apart: pairs further
    // apart hold no interval within the limit.
    int dq = (int)(((int64_t)max_len - 2) / kBlk);
    dq = dq < nb - 2 ? dq : nb - 2;
    int n_pairs = 0;                              // pairs (p, q), p <= q <= min(p + dq, nb - 2)
    for (int p = 0; p <= nb - 2; ++p) n_pairs += (dq < nb - 2 - p ? dq : nb - 2 - p) + 1;
    char* ws = static_cast<char*>(workspace);
    int64_t* A = reinterpret_cast<int64_t*>(ws + lay.a_off);
    int64_t* Z = reinterpret_cast<int64_t*>(ws + lay.z_off);
    int64_t* M = reinterpret_cast<int64_t*>(ws + lay.m_off);
    int64_t* P = reinterpret_cast<int64_t*>(ws + lay.p_off);
    int64_t* U = reinterpret_cast<int64_t*>(ws + lay.u_off);
    int32_t* pair_p = reinterpret_cast<int32_t*>(ws + lay.pair_off);
    int32_t* pair_q = pair_p + lay.n_pairs;       // (room for the largest list)
    const int64_t ws_bs = (int64_t)(lay.per_problem / 8);
    const int64_t c_bs = (int64_t)L * kK, R_bs = (int64_t)(L - 1) * kK * kK, T_bs = (int64_t)L * ldT;
    const int64_t c_st = (int64_t)kBlk * kK, R_st = (int64_t)kBlk * kK * kK;
    hipError_t e;

    hipLaunchKernelGGL(ib_pairs_kernel, dim3((unsigned)((n_pairs + 255) / 256)), dim3(256), 0, stream, nb, dq, n_pairs,
                       pair_p, pair_q);
    hipLaunchKernelGGL(ib_fill_kernel, dim3((unsigned)L, (unsigned)B), dim3(256), 0, stream, L, dq, ldT, T, T_bs);
    // row sweeps inside the blocks, one operator into the next block: the table's entries there, and A (the last
    // block stops at the chain's end and leaves no A)
    IntervalParts rows{nb, c_st, R_st, (int64_t)kBlk * (ldT + 1), kBlk, A, (int64_t)kBlk * kK, ws_bs, kBlk, L};
    e = launch_interval_costs(B, kBlk + 1, kK, kBlk + 1, c, c_bs, R, R_bs, ldT, T, T_bs, stream, &rows, false);
    if (e != hipSuccess) return e;
    // strategy sweeps of the blocks 1 .. nb - 1: Z, and M for all but the last
    IntervalParts strat{nb - 1, c_st, R_st, (int64_t)kK * kLdz, kK, M + (int64_t)kK * kK, (int64_t)kK * kK, ws_bs,
                        kBlk, L - kBlk};
    e = launch_interval_costs(B, kBlk + 1, kK, kBlk + 1, c + c_st, c_bs, R + R_st, R_bs, kLdz, Z + (int64_t)kK * kLdz,
                              ws_bs, stream, &strat, true);
    if (e != hipSuccess) return e;

    const size_t lds = 2 * (size_t)kK * kLds * sizeof(double);
    const size_t lds_prefix = 2 * (size_t)kK * kK * sizeof(double);
    for (const void* k : {reinterpret_cast<const void*>(ib_prefix_kernel), reinterpret_cast<const void*>(ib_left_kernel),
                          reinterpret_cast<const void*>(ib_tiles_kernel)}) {
        e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(lds > lds_prefix ? lds : lds_prefix));
        if (e != hipSuccess) return e;
    }
    if (nb > 3 && dq >= 2)
        hipLaunchKernelGGL(ib_prefix_kernel, dim3((unsigned)((nb - 3) * kPrefixSplit), (unsigned)B), dim3(kPrefixWaves * 64), lds_prefix,
                           stream, nb, dq, M, P, ws_bs);
    if (dq >= 1)
        hipLaunchKernelGGL(ib_left_kernel, dim3(kBlk / kTile, (unsigned)n_pairs, (unsigned)B), dim3(256), lds, stream, nb,
                           pair_p, pair_q, A, M, P, U, ws_bs);
    hipLaunchKernelGGL(ib_tiles_kernel, dim3(4, (unsigned)n_pairs, (unsigned)B), dim3(256), lds, stream, L, nb, pair_p,
                       pair_q, A, U, Z, ws_bs, ldT, T, T_bs, max_len);
    return hipGetLastError();
}

}  // namespace rh

// Min-plus chain DP of ONE long chain, parallel along the chain.
//
// The forward sweep v_{i+1}[b] = c_{i+1}[b] + min_a (v_i[a] + R_i[a][b]) (Sec. 4.2 objective on the
// linear chain of Sec. 4.3.2) is a chain of N-1 dependent steps; a single workgroup needs about
// 10 us per step at Kp = 256, eight cooperating workgroups about 6 us, however fast the memory is.
// Min-plus products are associative, so the chain is cut into segments of SL edges:
//   1. for every segment but the last, all at once: the matrix M_g[a][b] = cost of the best way
//      through the segment that enters with strategy a and leaves with strategy b (one forward
//      sweep per entering strategy, Kp sweeps sharing the segment's edge tables; strategies whose
//      node cost is infeasible are skipped, as entering strategies and as rows of every edge table);
//   2. the vectors at the segment boundaries, v_{g+1} = v_g (x) M_g, a short sequential pass;
//   3. the ordinary vector sweep inside every third of a segment (step 1 runs as one launch per
//      third and keeps the matrices that reach one and two thirds of a segment, so those start
//      vectors cost one product each), all at once as one batch: it writes arg exactly as the sequential sweep would,
//      because the boundary vectors are the sequential sweep's own values (saturation at
//      "infeasible" is monotone, so it commutes with the regrouping).
// Step 1 does Kp times the arithmetic of the plain sweep, in fp64 (exact for these integers, see
// interval_costs.hip) at two lane-operations per cell, in exchange for removing the dependent chain.
#include "kernels.h"

namespace rh {
namespace {

typedef long long ll2 __attribute__((ext_vector_type(2)));

constexpr int kScWaves = 16;                 // waves per workgroup of the matrix kernel
constexpr int kScRows = 2;                   // entering strategies (rows of M_g) per wave: R values are read once for both
constexpr int kScThreads = kScWaves * 64;
constexpr int kScBlock = kScWaves * kScRows; // rows of M_g per workgroup
constexpr int kScSub = 3;                    // the final sweep starts at every kScSub-th part of a segment
constexpr int kBdThreads = 1024;             // the boundary kernels
constexpr int kBdWaves = 16;
constexpr int kScPiece = 4096;               // elements of R per LDS buffer
constexpr int kMaxSegLen = 255;              // edges per segment (the planner stays below)
constexpr double kInfD = 4503599627370495.0; // 2^52 - 1 stands for "infeasible" inside the kernel

__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// exact for 0 <= x < 2^52 - 1; anything larger (RH_INF included) becomes the kernel's infeasible value
__device__ __forceinline__ double to_f64(int64_t x) {
    uint32_t lo = (uint32_t)x, hi = (uint32_t)((uint64_t)x >> 32);
    const bool big = hi >= 0x100000u;
    lo = big ? 0xFFFFFFFFu : lo;
    hi = big ? 0xFFFFFu : hi;
    return __hiloint2double((int)(hi | 0x43300000u), (int)lo) - 4503599627370496.0;
}

__device__ __forceinline__ int64_t to_i64(double m) { return m >= kInfD ? kInf : (int64_t)m; }

__device__ __forceinline__ double bcast(double x, int lane) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), lane);
    return __hiloint2double(hi, lo);
}

template <int KP>
struct Shape {
    static constexpr int CPT = KP / 64;                       // columns per lane: lane + 64 k
    static constexpr int CH = kScPiece / KP;                  // rows a of R_l per piece
    static constexpr int NCH = KP / CH;                       // pieces per edge
    static constexpr int EPT = kScPiece / kScThreads;         // elements per thread per piece
};

// acc[q][k] = min(acc[q][k], V[q][a] + R[a][lane + 64 k]) over the rows a of one piece whose strategy is feasible
// (bit a of amask; an infeasible a has V[q][a] = infeasible and cannot win), NR rows of M_g at once.
template <int KP, int NR>
__device__ __forceinline__ void relax_piece(const double* __restrict__ piece, int lane, int ch,
                                            const uint64_t (&amask)[Shape<KP>::CPT],
                                            const double (&V)[kScRows][Shape<KP>::CPT],
                                            double (&acc)[kScRows][Shape<KP>::CPT]) {
    using G = Shape<KP>;
    const int a0 = ch * G::CH;
    const int k_src = a0 >> 6, lane0 = a0 & 63;   // V[q][a] sits in register k_src, lane a mod 64
    // The selects below must stay selects: folded into an indexed read of V they would move V to scratch memory
    // (the empty asm statements keep the compiler from doing that).
    double src[NR];
    uint64_t word = amask[0];
#pragma unroll
    for (int k = 1; k < G::CPT; ++k) {
        word = k_src == k ? amask[k] : word;
        asm volatile("" : "+s"(word));
    }
#pragma unroll
    for (int q = 0; q < NR; ++q) {
        src[q] = V[q][0];
#pragma unroll
        for (int k = 1; k < G::CPT; ++k) {
            src[q] = k_src == k ? V[q][k] : src[q];
            asm volatile("" : "+v"(src[q]));
        }
    }
    uint64_t bits = word >> lane0;
    if (G::CH < 64) bits &= (1ull << G::CH) - 1;
    while (bits != 0) {
        const int u = __builtin_ctzll(bits);
        bits &= bits - 1;
        double r[G::CPT];
#pragma unroll
        for (int k = 0; k < G::CPT; ++k) r[k] = piece[u * KP + lane + 64 * k];
#pragma unroll
        for (int q = 0; q < NR; ++q) {
            const double sv = bcast(src[q], lane0 + u);
#pragma unroll
            for (int k = 0; k < G::CPT; ++k) acc[q][k] = __builtin_fmin(acc[q][k], r[k] + sv);
        }
    }
}

// the instance of relax_piece for the number of rows this wave holds
template <int KP, int NR>
__device__ __forceinline__ void relax_rows(int n_rows, const double* __restrict__ piece, int lane, int ch,
                                           const uint64_t (&amask)[Shape<KP>::CPT],
                                           const double (&V)[kScRows][Shape<KP>::CPT],
                                           double (&acc)[kScRows][Shape<KP>::CPT]) {
    if (n_rows == NR) relax_piece<KP, NR>(piece, lane, ch, amask, V, acc);
    if constexpr (NR > 1) {
        if (n_rows < NR) relax_rows<KP, NR - 1>(n_rows, piece, lane, ch, amask, V, acc);
    }
}

// ---- step 1: segment matrices -------------------------------------------------------------------
// Workgroup (rb, g): up to kScBlock feasible entering strategies of segment g, kScRows per wave.  blockIdx.x = rb *
// nseg_pad + g with nseg_pad a multiple of 8, so the workgroups of one segment, which read the same tables at
// the same time, share an XCD and its L2.
template <int KP>
__global__ void __launch_bounds__(kScThreads)
scan_matrix_kernel(int32_t SL, int32_t SLq, int32_t part, int32_t nseg, int32_t nseg_pad,
                   const int64_t* __restrict__ c, const int64_t* __restrict__ R, const int64_t* __restrict__ Vin,
                   int64_t in_stride, int64_t* __restrict__ Vout, int64_t out_stride, int32_t fill_dead) {
    using G = Shape<KP>;
    extern __shared__ double lds[];               // two pieces of kScPiece doubles
    __shared__ int32_t live_rows[KP];
    __shared__ int32_t wave_cnt[KP / 64];
    __shared__ uint64_t opmask[kMaxSegLen + 1][G::CPT];   // feasible strategies of every operator of the segment
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int g = blockIdx.x % nseg_pad, rb = blockIdx.x / nseg_pad;
    if (g >= nseg) return;
    // One launch per part of the segments: this one takes the rows from the segment's first operator + part * SLq
    // (unit vectors for part 0, else what the launch before left in Vin) over SLq edges and leaves them in Vout.
    const int64_t* cseg = c + (int64_t)g * SL * KP;           // node costs of the segment's first operator
    const int l0 = g * SL + part * SLq;                       // first operator and first edge of this part
    const int64_t* c0 = c + (int64_t)l0 * KP;
    int64_t* Mg = Vout + (int64_t)g * out_stride;

    // entering strategies (of the segment) with a feasible node cost, in ascending order
    bool live = false;
    if (tid < KP) live = cseg[tid] < kInf;
    const uint64_t mask = __ballot(live);
    if (tid < KP && lane == 0) wave_cnt[wave] = __popcll(mask);
    __syncthreads();
    int n_live = 0, before = 0;
#pragma unroll
    for (int w = 0; w < KP / 64; ++w) {
        const int n = wave_cnt[w];
        before += w < wave ? n : 0;
        n_live += n;
    }
    if (live) live_rows[before + __popcll(mask & ((1ull << lane) - 1))] = tid;
    __syncthreads();

    // rows of M_g that nobody computes are infeasible: every workgroup fills its share of them
    for (int a = kScBlock * rb + wave; fill_dead && a < KP && a < kScBlock * (rb + 1); a += kScWaves) {
        if (cseg[a] >= kInf) {
#pragma unroll
            for (int k = 0; k < G::CPT; ++k) Mg[(int64_t)a * KP + lane + 64 * k] = kInf;
        }
    }
    if (kScBlock * rb >= n_live) return;          // whole workgroup, after its last __syncthreads
    // slot q of this wave takes the feasible strategy of rank kScBlock rb + q kScWaves + wave: ranks fill slot 0 of
    // every wave before any slot 1
    int a_row[kScRows];
    int n_rows = 0;                               // wave-uniform
#pragma unroll
    for (int q = 0; q < kScRows; ++q) {
        const int rank = kScBlock * rb + q * kScWaves + wave;
        a_row[q] = rank < n_live ? live_rows[rank] : -1;
        n_rows += rank < n_live ? 1 : 0;
    }

    // bit j of opmask[o][k]: strategy 64 k + j of operator l0 + o is feasible.  An infeasible strategy a makes
    // row a of the edge table that leaves from its operator irrelevant (v[a] is infeasible): such rows are neither
    // fetched nor used.
    for (int o = wave; o <= SLq; o += kScWaves) {
#pragma unroll
        for (int k = 0; k < G::CPT; ++k) {
            const uint64_t m = __ballot(c0[(int64_t)o * KP + lane + 64 * k] < kInf);
            if (lane == 0) opmask[o][k] = m;
        }
    }
    lds_barrier();
    auto row_live = [&](int o, int a) -> bool { return (opmask[o][a >> 6] >> (a & 63)) & 1; };

    // Pieces travel global memory -> registers -> LDS.  A piece is fetched two pieces before it is used (raw0 holds
    // the even pieces, raw1 the odd ones), converted and stored to LDS while its predecessor is being used.
    // Piece p = rows a in [CH (p % NCH), CH (p % NCH + 1)) of the table of edge p / NCH.
    const int n_pieces = SLq * G::NCH;
    int64_t raw0[G::EPT], raw1[G::EPT];
    // Every load of the main loop is unconditional and every piece issues the same number of them, so that the
    // waits can count outstanding loads instead of draining them all (a fetch past the end repeats the last piece).
    auto fetch = [&](int p, int64_t (&raw)[G::EPT]) {
        p = p < n_pieces ? p : n_pieces - 1;
        const int64_t* src = R + ((int64_t)l0 * KP * KP + (int64_t)p * kScPiece);
#pragma unroll
        for (int e = 0; e < G::EPT / 2; ++e) {
            const ll2 v = *reinterpret_cast<const ll2*>(src + 2 * (e * kScThreads + tid));
            raw[2 * e] = v.x;
            raw[2 * e + 1] = v.y;
        }
    };
    auto stash = [&](int p, const int64_t (&raw)[G::EPT]) {
        double* dst = lds + (p & 1) * kScPiece;
        const int o = p / G::NCH, a0 = (p & (G::NCH - 1)) * G::CH;
#pragma unroll
        for (int e = 0; e < G::EPT / 2; ++e) {
            const int at = 2 * (e * kScThreads + tid);
            if (row_live(o, a0 + at / KP)) {
                dst[at] = to_f64(raw[2 * e]);
                dst[at + 1] = to_f64(raw[2 * e + 1]);
            }
        }
    };
    fetch(0, raw0);
    fetch(1, raw1);
    stash(0, raw0);
    lds_barrier();

    // node costs of the operator the current edge arrives at, in this lane's columns
    double cB[G::CPT];
#pragma unroll
    for (int k = 0; k < G::CPT; ++k) cB[k] = to_f64(c0[KP + lane + 64 * k]);   // operator l0 + 1 exists: SL >= 1

    // feasible strategies of the operator the current edge leaves from (wave-uniform copies of the table's words)
    uint64_t amask[G::CPT];
    auto load_amask = [&](int o) {
#pragma unroll
        for (int k = 0; k < G::CPT; ++k) {
            const uint64_t m = opmask[o][k];
            amask[k] = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(m >> 32)) << 32) |
                       (uint32_t)__builtin_amdgcn_readfirstlane((int)m);
        }
    };
    load_amask(0);

    // entering with strategy a_row costs nothing extra: v = 0 at a_row, infeasible elsewhere
    double V[kScRows][G::CPT], acc[kScRows][G::CPT];
#pragma unroll
    for (int q = 0; q < kScRows; ++q)
#pragma unroll
        for (int k = 0; k < G::CPT; ++k) {
            V[q][k] = (lane + 64 * k == a_row[q]) ? 0.0 : kInfD;
            if (Vin != nullptr && q < n_rows)
                V[q][k] = to_f64(Vin[(int64_t)g * in_stride + (int64_t)a_row[q] * KP + lane + 64 * k]);
        }

    // piece p = rows a of piece p % NCH of edge p / NCH
    auto one_piece = [&](int p, int64_t (&mine)[G::EPT], const int64_t (&next)[G::EPT]) {
        const int ch = p & (G::NCH - 1);
        if (ch == 0) {
#pragma unroll
            for (int q = 0; q < kScRows; ++q)
#pragma unroll
                for (int k = 0; k < G::CPT; ++k) acc[q][k] = kInfD;
        }
        // node costs for the edge after this one (read again by every piece of an edge: a load that only the last
        // piece issued would be a conditional one)
        const int e = p / G::NCH;
        const int o_next = e + 2 <= SLq ? e + 2 : SLq;
        int64_t cC[G::CPT];
#pragma unroll
        for (int k = 0; k < G::CPT; ++k)
            cC[k] = c0[(int64_t)o_next * KP + lane + 64 * k];
        fetch(p + 2, mine);                               // the registers of piece p are free: it is in LDS
        const double* piece = lds + (p & 1) * kScPiece;
        relax_rows<KP, kScRows>(n_rows, piece, lane, ch, amask, V, acc);
        if (p + 1 < n_pieces) stash(p + 1, next);
        lds_barrier();                                    // piece p+1 is in LDS; piece p has been read for the last time
#pragma unroll
        for (int k = 0; k < G::CPT; ++k) asm volatile("" ::"v"(cC[k]));   // keeps the load in every piece
        if (ch == G::NCH - 1) {
#pragma unroll
            for (int k = 0; k < G::CPT; ++k) {
#pragma unroll
                for (int q = 0; q < kScRows; ++q)
                    V[q][k] = __builtin_fmin(cB[k] + __builtin_fmin(acc[q][k], kInfD), kInfD);
                cB[k] = to_f64(cC[k]);
            }
            load_amask(e + 1);                            // the operator just reached is where the next edge leaves from
        }
    };
    for (int p = 0; p < n_pieces; p += 4) {               // n_pieces is a multiple of 4 (the planner sees to it)
        one_piece(p, raw0, raw1);
        one_piece(p + 1, raw1, raw0);
        one_piece(p + 2, raw0, raw1);
        one_piece(p + 3, raw1, raw0);
    }
#pragma unroll
    for (int q = 0; q < kScRows; ++q) {
        if (q < n_rows) {
#pragma unroll
            for (int k = 0; k < G::CPT; ++k) Mg[(int64_t)a_row[q] * KP + lane + 64 * k] = to_i64(V[q][k]);
        }
    }
}

// ---- step 2: boundary vectors ---------------------------------------------------------------------
// vs[b] <- min_a (vs[a] + Mg[a][b]), saturated; the whole workgroup (kBdThreads) takes part.  Rows whose vs[a] is
// infeasible are not read (rows of entering strategies nobody computed hold nothing).
template <int KP>
__device__ __forceinline__ void vector_times_matrix(int64_t (&vs)[KP], int64_t (&part)[kBdWaves][KP],
                                                    const int64_t* __restrict__ Mg, int tid, int wave, int lane) {
    constexpr int LPG = KP / 128 > 0 ? KP / 128 : 1;      // 16-byte loads per lane per row
    constexpr int ROW_LANES = KP / 2 < 64 ? KP / 2 : 64;  // lanes that hold a row (KP = 64: half a wave)
    int64_t best[2 * LPG];
#pragma unroll
    for (int j = 0; j < 2 * LPG; ++j) best[j] = kInf;
    for (int a = wave; a < KP; a += kBdWaves) {
        const int64_t va = vs[a];
        if (va >= kInf) continue;                 // wave-uniform
        if (lane < ROW_LANES) {
#pragma unroll
            for (int k = 0; k < LPG; ++k) {
                const ll2 m = *reinterpret_cast<const ll2*>(Mg + (int64_t)a * KP + 2 * lane + 128 * k);
                const int64_t x0 = va + m.x, x1 = va + m.y;
                best[2 * k] = x0 < best[2 * k] ? x0 : best[2 * k];
                best[2 * k + 1] = x1 < best[2 * k + 1] ? x1 : best[2 * k + 1];
            }
        }
    }
    if (lane < ROW_LANES) {
#pragma unroll
        for (int k = 0; k < LPG; ++k) {
            part[wave][2 * lane + 128 * k] = best[2 * k];
            part[wave][2 * lane + 128 * k + 1] = best[2 * k + 1];
        }
    }
    __syncthreads();
    if (tid < KP) {
        int64_t m = part[0][tid];
#pragma unroll
        for (int w = 1; w < kBdWaves; ++w) m = part[w][tid] < m ? part[w][tid] : m;
        vs[tid] = m < kInf ? m : kInf;
    }
    __syncthreads();
}

// One workgroup: v_0 = c_0 (saturated), v_{g+1} = v_g (x) M_g.  The final sweep runs on problems of SLq = SL / kScSub
// edges; problem q's node costs are c_seg[q][SLq + 1][KP] with the start vector as row 0: v_g is row 0 of problem
// kScSub * g.
template <int KP>
__global__ void __launch_bounds__(kBdThreads)
scan_boundary_kernel(int32_t SLq, int32_t nseg, const int64_t* __restrict__ c, const int64_t* __restrict__ M,
                     int64_t* __restrict__ c_seg) {
    __shared__ int64_t vs[KP];
    __shared__ int64_t part[kBdWaves][KP];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int64_t seg_stride = (int64_t)kScSub * (SLq + 1) * KP;
    if (tid < KP) {
        int64_t x = c[tid];
        x = x < kInf ? x : kInf;
        vs[tid] = x;
        c_seg[tid] = x;
    }
    __syncthreads();
    for (int g = 0; g < nseg; ++g) {
        vector_times_matrix<KP>(vs, part, M + (int64_t)g * KP * KP, tid, wave, lane);
        if (tid < KP) c_seg[(int64_t)(g + 1) * seg_stride + tid] = vs[tid];
    }
}

// Workgroup (j, g): start vector of part j + 1 of segment g = v_g (x) Msub[g][j], row 0 of problem kScSub * g + j + 1.
template <int KP>
__global__ void __launch_bounds__(kBdThreads)
scan_part_vectors_kernel(int32_t SLq, const int64_t* __restrict__ Msub, int64_t* __restrict__ c_seg) {
    __shared__ int64_t vs[KP];
    __shared__ int64_t part[kBdWaves][KP];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int j = blockIdx.x, g = blockIdx.y;
    const int64_t prob_stride = (int64_t)(SLq + 1) * KP;
    if (tid < KP) vs[tid] = c_seg[(int64_t)kScSub * g * prob_stride + tid];
    __syncthreads();
    vector_times_matrix<KP>(vs, part, Msub + ((int64_t)g * (kScSub - 1) + j) * KP * KP, tid, wave, lane);
    if (tid < KP) c_seg[((int64_t)kScSub * g + j + 1) * prob_stride + tid] = vs[tid];
}

// rows 1.. of every segment's node costs: c_seg[g][r][:] = c[g * SL + r][:], r >= 1, while g * SL + r < N
__global__ void __launch_bounds__(256)
scan_copy_c_kernel(int32_t N, int32_t SL, int32_t Kp, int32_t n_seg_total, const int64_t* __restrict__ c,
                   int64_t* __restrict__ c_seg) {
    const int64_t per_seg = (int64_t)SL * Kp;     // elements of rows 1..SL
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)n_seg_total * per_seg) return;
    const int g = (int)(t / per_seg);
    const int64_t off = t - (int64_t)g * per_seg;             // (r - 1) * Kp + column
    const int64_t src = ((int64_t)g * SL + 1) * Kp + off;
    if (src < (int64_t)N * Kp) c_seg[(int64_t)g * (SL + 1) * Kp + Kp + off] = c[src];
}

struct ScanPlan {
    int32_t SL, G, r;                             // G segments: G-1 of SL edges and a last one of r edges, 1 <= r <= SL
    size_t m_off, msub_off, cseg_off, tot_off, last_off, total;
};

// Segment length: near sqrt(edges) (the boundary pass costs per segment, the final sweep per edge of a part),
// but long enough that the matrix kernel's workgroups are resident all at once.  Its registers allow one
// workgroup per compute unit, and a segment whose operators have up to 96 feasible strategies takes three
// workgroups of 32 rows, so at most 256 / 3 segments get a matrix.  SL is a multiple of kScSub, and the pieces of
// a part a multiple of 4 (Kp = 64 has one piece per edge).  Among the next few such lengths the one that leaves
// the shortest last segment wins (that segment is swept after the batch).
constexpr int kMaxMatrixSegments = 85;

__host__ ScanPlan plan_scan(int32_t N, int32_t Kp) {
    ScanPlan p{};
    const int E = N - 1;
    int s0 = 16;
    while ((int64_t)(s0 + 1) * (s0 + 1) <= E) ++s0;
    while ((E - 1) / s0 > kMaxMatrixSegments) ++s0;
    const int step = Kp == 64 ? 4 * kScSub : kScSub;
    s0 = (s0 + step - 1) / step * step;
    int best_sl = s0, best_r = E;
    const int candidates = Kp == 64 ? 5 : 16;
    for (int sl = s0; sl < s0 + candidates * step; sl += step) {
        const int r = (E - 1) % sl + 1;           // 1..sl
        if (r < best_r) {
            best_r = r;
            best_sl = sl;
        }
    }
    p.SL = best_sl;
    p.r = best_r;
    p.G = (E - best_r) / best_sl + 1;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t nseg = (size_t)p.G - 1, mat = (size_t)Kp * Kp * sizeof(int64_t);
    const size_t n_prob = nseg * kScSub + 1;      // parts of the full segments, then the last segment
    p.m_off = 0;
    p.msub_off = up(nseg * mat);
    p.cseg_off = p.msub_off + up(nseg * (kScSub - 1) * mat);
    p.tot_off = p.cseg_off + up((nseg * kScSub * (p.SL / kScSub + 1) + (size_t)p.SL + 1) * Kp * sizeof(int64_t));
    p.last_off = p.tot_off + up(n_prob * sizeof(int64_t));
    p.total = p.last_off + up(n_prob * sizeof(int32_t));
    return p;
}

}  // namespace

size_t scan_workspace_bytes(int32_t B, int32_t N, int32_t Kp) {
    // worth it for one or two long chains; more problems fill the chip better with a workgroup (or eight) each
    if (B < 1 || B > 2 || N < 128 || (Kp != 64 && Kp != 128 && Kp != 256)) return 0;
    const ScanPlan pl = plan_scan(N, Kp);
    if (pl.SL > kMaxSegLen) return 0;
    return (size_t)B * pl.total;
}

hipError_t launch_chain_scan(int32_t B, int32_t N, int32_t Kp, const int64_t* c, int64_t c_bs, const int64_t* R,
                             int64_t R_bs, uint16_t* arg, int64_t* vfinal, int64_t* total, int32_t* last,
                             void* workspace, hipStream_t stream) {
    const ScanPlan pl = plan_scan(N, Kp);
    const int nseg = pl.G - 1;                    // segments that need a matrix: all but the last
    const int nseg_pad = (nseg + 7) & ~7;
    const size_t lds = 2 * kScPiece * sizeof(double);
    for (int p = 0; p < B; ++p) {
        char* ws = static_cast<char*>(workspace) + (size_t)p * pl.total;
        int64_t* M = reinterpret_cast<int64_t*>(ws + pl.m_off);
        int64_t* Msub = reinterpret_cast<int64_t*>(ws + pl.msub_off);
        int64_t* c_seg = reinterpret_cast<int64_t*>(ws + pl.cseg_off);
        int64_t* seg_total = reinterpret_cast<int64_t*>(ws + pl.tot_off);
        int32_t* seg_last = reinterpret_cast<int32_t*>(ws + pl.last_off);
        const int64_t* cp = c + (int64_t)p * c_bs;
        const int64_t* Rp = R + (int64_t)p * R_bs;
        uint16_t* argp = arg + (int64_t)p * (N - 1) * Kp;
        const int SLq = pl.SL / kScSub, n_part = nseg * kScSub;
        const int64_t prob_c = (int64_t)(SLq + 1) * Kp, prob_R = (int64_t)SLq * Kp * Kp;
        int64_t* c_last = c_seg + (int64_t)n_part * prob_c;   // node costs of the last segment: r + 1 rows
        const int l_last = nseg * pl.SL;                      // its first operator

        const dim3 grid((unsigned)(((Kp + kScBlock - 1) / kScBlock) * nseg_pad));
        // rows 1.. of the node costs of every part and of the last segment
        const int64_t n_copy = (int64_t)n_part * SLq * Kp, n_copy_last = (int64_t)pl.r * Kp;
        hipLaunchKernelGGL(scan_copy_c_kernel, dim3((unsigned)((n_copy + 255) / 256)), dim3(256), 0, stream, N, SLq, Kp,
                           n_part, cp, c_seg);
        hipLaunchKernelGGL(scan_copy_c_kernel, dim3((unsigned)((n_copy_last + 255) / 256)), dim3(256), 0, stream,
                           N - l_last, pl.r, Kp, 1, cp + (int64_t)l_last * Kp, c_last);
#define RH_SCAN(KP)                                                                                                 \
    do {                                                                                                            \
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(scan_matrix_kernel<KP>),                   \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                   \
        if (e != hipSuccess) return e;                                                                              \
        for (int j = 0; j < kScSub; ++j) {                                                                          \
            const int64_t mat = (int64_t)KP * KP, sub = (kScSub - 1) * mat;                                         \
            const bool fin = j + 1 == kScSub;                                                                       \
            hipLaunchKernelGGL((scan_matrix_kernel<KP>), grid, dim3(kScThreads), lds, stream, pl.SL, SLq, j, nseg,  \
                               nseg_pad, cp, Rp, j ? Msub + (j - 1) * mat : nullptr, sub, fin ? M : Msub + j * mat, \
                               fin ? mat : sub, fin ? 1 : 0);                                                       \
        }                                                                                                           \
        hipLaunchKernelGGL((scan_boundary_kernel<KP>), dim3(1), dim3(kBdThreads), 0, stream, SLq, nseg, cp, M,      \
                           c_seg);                                                                                  \
        hipLaunchKernelGGL((scan_part_vectors_kernel<KP>), dim3(kScSub - 1, nseg), dim3(kBdThreads), 0, stream,     \
                           SLq, Msub, c_seg);                                                                       \
    } while (0)
        switch (Kp) {
            case 64: RH_SCAN(64); break;
            case 128: RH_SCAN(128); break;
            case 256: RH_SCAN(256); break;
            default: return hipErrorInvalidValue;
        }
#undef RH_SCAN
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        // step 3: the sweep inside every part as one batch (their totals are scratch), then the last segment,
        // whose final vector, total and last are the chain's.
        e = launch_chain(n_part, SLq + 1, Kp, c_seg, prob_c, Rp, prob_R, argp, nullptr, seg_total, seg_last, stream);
        if (e != hipSuccess) return e;
        e = launch_chain(1, pl.r + 1, Kp, c_last, 0, Rp + (int64_t)n_part * prob_R, 0,
                         argp + (int64_t)l_last * Kp, vfinal ? vfinal + (int64_t)p * Kp : nullptr, total + p, last + p,
                         stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rh

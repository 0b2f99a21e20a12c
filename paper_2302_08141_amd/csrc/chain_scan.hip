// Min-plus chain DP of a long chain, parallel along the chain.
//
// The forward sweep v_{i+1}[b] = c_{i+1}[b] + min_a (v_i[a] + R_i[a][b]) (Sec. 4.2 objective on the
// linear chain of Sec. 4.3.2) is a chain of N-1 dependent steps; a single workgroup needs about
// 10 us per step at Kp = 256, eight cooperating workgroups about 3.4 us, however fast the memory is.
// Min-plus products are associative, so the chain is cut into segments of SL edges:
//   1. for every segment but the last, all at once: the matrix M_g[a][b] = cost of the best way
//      through the segment that enters with strategy a and leaves with strategy b (one forward
//      sweep per entering strategy, all sharing the segment's edge tables);
//   2. the vectors at the segment boundaries, v_{g+1} = v_g (x) M_g, a short sequential pass;
//   3. the ordinary vector sweep inside every third of a segment, all thirds at once (step 1
//      runs as one launch per third and keeps the matrices that reach one and two thirds of a
//      segment, so those start vectors cost one product each): it writes arg exactly as the
//      sequential sweep would, because the start vectors are the sequential sweep's own values
//      (saturation at "infeasible" is monotone, so it commutes with the regrouping).
// A strategy whose node cost is infeasible can neither be entered nor passed through: all
// three steps work on the feasible strategies of every operator only, in rank order (rows of M_g,
// rows and columns of the edge tables, rows of the sweep) -- on tables built from sharding specs
// about a third of the slots are valid layouts.
// Step 1 does (feasible strategies) times the arithmetic of the plain sweep, in fp64 (exact for
// these integers, see interval_costs.hip) at two lane-operations per cell, in exchange for
// removing the dependent chain.
#include "kernels.h"
#include "reshard_common.h"

namespace rh {
namespace {

typedef long long ll2 __attribute__((ext_vector_type(2)));

// What the matrix kernel needs to compute an edge table's entries from sharding specs instead of reading them
// (rh_minplus_chain_specs with a workspace): the arrays of rh_build_reshard and the problem's mesh.
struct SpecSource {
    const int32_t* K;
    const uint32_t* out_spec;
    const uint32_t* in_spec;
    const int64_t* dims;
    const int32_t* elem_bytes;
    Mesh mesh;
};

constexpr int kScWaves = 16;                 // waves per workgroup of the matrix kernel
constexpr int kScRows = 2;                   // entering strategies (rows of M_g) per wave: R values are read once for both
constexpr int kScThreads = kScWaves * 64;
constexpr int kScBlock = kScWaves * kScRows; // rows of M_g per workgroup
constexpr int kScSub = 3;                    // parts per segment: the sweep of step 3 starts at every part
constexpr int kBdThreads = 1024;             // the boundary kernels
constexpr int kBdWaves = 16;
constexpr int kScPiece = 4096;               // elements of R per LDS buffer
constexpr int kMaxSegLen = 255;              // edges per segment (the planner stays below)
constexpr int kMaxPartLen = kMaxSegLen / kScSub;   // edges per part of a segment
constexpr int kSpecPartLen = 48;             // the same when the tables are computed from specs: the canonical words and
                                             // time tables of a whole part live in LDS next to the staged pieces
constexpr int kSpecTab = 20;                 // [axis][other axis splits][none | gather | all-to-all | all-reduce | impossible]
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
    static constexpr int CPT = KP / 64;                       // columns per lane: rank lane + 64 k
    static constexpr int EPT = kScPiece / kScThreads;         // elements per thread per piece
    static_assert(EPT == 4, "a thread stages four neighbouring columns of one row");
};

// Layout of the table of one edge in LDS.  Only the rows of strategies that are feasible where the edge leaves
// from (na of them) and the columns of strategies feasible where it arrives (nb) are staged, in rank order: a
// row of a piece has 64 << lgc columns (the power of two that holds nb), a piece 64 >> lgc rows.
struct EdgeShape {
    int na, nb, lgc, np;                          // np = pieces of the edge, at least one
};

__device__ __forceinline__ EdgeShape edge_shape(int na, int nb) {
    EdgeShape s;
    s.na = na;
    s.nb = nb;
    s.lgc = nb <= 64 ? 0 : nb <= 128 ? 1 : 2;
    const int np = (na + (64 >> s.lgc) - 1) >> (6 - s.lgc);
    s.np = np > 0 ? np : 1;
    return s;
}

// acc[q][k] = min(acc[q][k], V[q][rank0 + r] + piece[r][lane + 64 k]) over the rows r < nr of one piece (nr a
// multiple of 8: the piece's rows past the last feasible strategy hold "infeasible", and so does V there), NR
// rows of M_g at once, CC groups of 64 columns.
template <int KP, int NR, int CC>
__device__ __forceinline__ void relax_piece(const double* __restrict__ piece, int lane, int nr, int rank0,
                                            const double (&V)[kScRows][Shape<KP>::CPT],
                                            double (&acc)[kScRows][Shape<KP>::CPT]) {
    using G = Shape<KP>;
    constexpr int W = 64 * CC;
    const int k_src = rank0 >> 6, lane0 = rank0 & 63;   // V[q][rank] sits in register rank / 64, lane rank mod 64
    // The selects below must stay selects: folded into an indexed read of V they would move V to scratch memory
    // (the empty asm statements keep the compiler from doing that).
    double src[NR];
#pragma unroll
    for (int q = 0; q < NR; ++q) {
        src[q] = V[q][0];
#pragma unroll
        for (int k = 1; k < G::CPT; ++k) {
            src[q] = k_src == k ? V[q][k] : src[q];
            asm volatile("" : "+v"(src[q]));
        }
    }
    // The rows of the piece go with lanes lane0, lane0 + 1, ... of src; turned round so that they go with lanes
    // 0, 1, ..., every broadcast below names its lane by a constant (a lane number computed at run time makes
    // the broadcast markedly slower).
    const int from = ((lane + lane0) & 63) << 2;
#pragma unroll
    for (int q = 0; q < NR; ++q) {
        const int lo = __builtin_amdgcn_ds_bpermute(from, __double2loint(src[q]));
        const int hi = __builtin_amdgcn_ds_bpermute(from, __double2hiint(src[q]));
        src[q] = __hiloint2double(hi, lo);
    }
    // Four LDS values per lane and trip; the next trip's values are asked for before this trip's arithmetic.
    constexpr int UR = 4 / CC;                    // rows per trip
    constexpr int ROWS = kScPiece / W;            // rows a piece has room for
    double ra[UR][CC], rb[UR][CC];
    auto load = [&](double (&rv)[UR][CC], int r) {
        r = r < ROWS - UR ? r : ROWS - UR;
#pragma unroll
        for (int u = 0; u < UR; ++u)
#pragma unroll
            for (int k = 0; k < CC; ++k) rv[u][k] = piece[(r + u) * W + lane + 64 * k];
    };
    auto relax = [&](const double (&rv)[UR][CC], int r) {
#pragma unroll
        for (int u = 0; u < UR; ++u)
#pragma unroll
            for (int q = 0; q < NR; ++q) {
                const double sv = bcast(src[q], r + u);
#pragma unroll
                for (int k = 0; k < CC; ++k) acc[q][k] = __builtin_fmin(acc[q][k], rv[u][k] + sv);
            }
    };
    load(ra, 0);
#pragma unroll
    for (int r = 0; r < ROWS; r += 2 * UR) {
        if ((r & 7) == 0 && r >= nr) break;       // nr is a multiple of 8
        load(rb, r + UR);
        relax(ra, r);
        load(ra, r + 2 * UR);
        relax(rb, r + UR);
    }
}

// the instance of relax_piece for the number of rows this wave holds and the width of the piece
template <int KP, int NR>
__device__ __forceinline__ void relax_width(int lgc, const double* __restrict__ piece, int lane, int nr, int rank0,
                                            const double (&V)[kScRows][Shape<KP>::CPT],
                                            double (&acc)[kScRows][Shape<KP>::CPT]) {
    if (lgc == 0) relax_piece<KP, NR, 1>(piece, lane, nr, rank0, V, acc);
    if constexpr (KP >= 128) {
        if (lgc == 1) relax_piece<KP, NR, 2>(piece, lane, nr, rank0, V, acc);
    }
    if constexpr (KP >= 256) {
        if (lgc == 2) relax_piece<KP, NR, 4>(piece, lane, nr, rank0, V, acc);
    }
}

// lidx[o][rank] = the rank-th feasible strategy (finite node cost) of operator o, o < n_ops, ascending; ranks past
// the last one repeat it (strategy 0 if there is none), so that a lookup always names a strategy; nl[o] = how many
// there are.  c0 = node costs of operator 0.  The waves of the workgroup share the operators out.
template <int KP>
__device__ __forceinline__ void rank_operators(const int64_t* __restrict__ c0, int n_ops, uint8_t (*lidx)[KP],
                                               int32_t* nl, int wave, int lane) {
    for (int o = wave; o < n_ops; o += kScWaves) {
        int64_t x[KP / 64];                       // all loads of the operator first: one trip to memory, not KP / 64
#pragma unroll
        for (int k = 0; k < KP / 64; ++k) x[k] = c0[(int64_t)o * KP + lane + 64 * k];
        int base = 0, last_live = 0;
#pragma unroll
        for (int k = 0; k < KP / 64; ++k) {
            const bool ok = x[k] < kInf;
            const uint64_t m = __ballot(ok);
            if (ok) lidx[o][base + __popcll(m & ((1ull << lane) - 1))] = (uint8_t)(lane + 64 * k);
            if (m != 0) last_live = 64 * k + 63 - __builtin_clzll(m);
            base += __popcll(m);
        }
#pragma unroll
        for (int k = 0; k < KP / 64; ++k) {
            if (lane + 64 * k >= base) lidx[o][lane + 64 * k] = (uint8_t)last_live;
        }
        if (lane == 0) nl[o] = base;
    }
}

// ---- step 1: segment matrices -------------------------------------------------------------------
// Workgroup (rb, g): up to kScBlock feasible entering strategies of segment g, kScRows per wave.  blockIdx.x = rb *
// nseg_pad + g with nseg_pad a multiple of 8, so the workgroups of one segment, which read the same tables at
// the same time, share an XCD and its L2.
template <int KP, bool SPECS>
__global__ void __launch_bounds__(kScThreads)
scan_matrix_kernel(int32_t SL, int32_t SLq, int32_t part, int32_t nseg, int32_t nseg_pad,
                   const int64_t* __restrict__ c, const int64_t* __restrict__ R, const int64_t* __restrict__ Vin,
                   int64_t in_stride, int64_t* __restrict__ Vout, int64_t out_stride, SpecSource sp) {
    using G = Shape<KP>;
    constexpr int PL = SPECS ? kSpecPartLen : kMaxPartLen;    // edges of a part at most
    extern __shared__ double lds[];               // two pieces of kScPiece doubles
    __shared__ int32_t live_rows[KP];
    __shared__ int32_t wave_cnt[KP / 64];
    // lidx[o][rank] = the rank-th feasible strategy of operator l0 + o (ranks past the last repeat it, so that a
    // lookup is always a valid strategy); nl[o] = how many there are
    __shared__ __align__(4) uint8_t lidx[PL + 1][KP];
    __shared__ int32_t nl[PL + 1];
    __shared__ double c_arrive[2][KP];            // node costs (rank order) of the operator each staged piece's edge arrives at
    // SPECS: per edge of the part the canonical producer and consumer words of every strategy slot (two bytes each,
    // 0xFFFF = not a usable layout) and the edge's table of per-axis times; an entry of the edge table is then two
    // classifications and two table reads (exactly what rh_build_reshard stores)
    __shared__ uint16_t pwords[SPECS ? PL : 1][KP], qwords[SPECS ? PL : 1][KP];
    __shared__ int64_t tabs[SPECS ? PL : 1][kSpecTab];
    __shared__ Mesh mesh_s;                        // in LDS: indexed by axis numbers computed at run time
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
    if (SPECS && tid == 0) mesh_s = sp.mesh;
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

    if (kScBlock * rb >= n_live) return;          // whole workgroup, after its last __syncthreads
    // slot q of this wave takes the feasible strategy of rank kScBlock rb + q kScWaves + wave: ranks fill slot 0 of
    // every wave before any slot 1
    int a_row[kScRows], a_rank[kScRows];
    int n_rows = 0;                               // wave-uniform
#pragma unroll
    for (int q = 0; q < kScRows; ++q) {
        a_rank[q] = kScBlock * rb + q * kScWaves + wave;
        a_row[q] = a_rank[q] < n_live ? live_rows[a_rank[q]] : -1;
        n_rows += a_rank[q] < n_live ? 1 : 0;
    }

    // The feasible strategies of every operator of the part, ranked.  An infeasible strategy makes its row of the
    // edge table that leaves from its operator and its column of the table that arrives there irrelevant (the
    // vector is infeasible there whatever the table says): such rows and columns are neither fetched nor used.
    rank_operators<KP>(c0, SLq + 1, lidx, nl, wave, lane);
    if constexpr (SPECS) {
        for (int idx = tid; idx < SLq * KP; idx += kScThreads) {
            const int e = idx / KP, slot = idx & (KP - 1);
            const int64_t* dm = sp.dims + (int64_t)(l0 + e) * 4;
            const uint32_t pw = canonical(sp.out_spec[(int64_t)(l0 + e) * KP + slot], slot, sp.K[l0 + e], dm, mesh_s);
            const uint32_t qw = canonical(sp.in_spec[(int64_t)(l0 + e + 1) * KP + slot], slot, sp.K[l0 + e + 1], dm, mesh_s);
            pwords[e][slot] = (pw & 0x80000000u) ? (uint16_t)0xFFFFu : (uint16_t)pw;
            qwords[e][slot] = (qw & 0x80000000u) ? (uint16_t)0xFFFFu : (uint16_t)qw;
        }
        for (int idx = tid; idx < SLq * kSpecTab; idx += kScThreads) {
            const int e = idx / kSpecTab, r = idx - e * kSpecTab;
            const int x = r / 10, o = (r / 5) & 1, kind = r % 5;
            tabs[e][r] = axis_time(x, o, (uint32_t)kind, mesh_s, sp.dims + (int64_t)(l0 + e) * 4, sp.elem_bytes[l0 + e]);
        }
    }
    lds_barrier();
    auto count_at = [&](int o) -> int { return __builtin_amdgcn_readfirstlane(nl[o]); };

    // Pieces travel global memory -> registers -> LDS.  A piece is fetched two pieces before it is used (raw0 holds
    // the even pieces, raw1 the odd ones), converted and stored to LDS while its predecessor is being used.  The
    // pieces of an edge follow each other, then the next edge's; a cursor names one.
    struct Cursor {
        int e, j;                                 // edge of the part, piece of the edge
        EdgeShape s;
        bool past;                                // ran off the end: stands on the last piece
    };
    auto cursor_at = [&](int e) -> Cursor { return Cursor{e, 0, edge_shape(count_at(e), count_at(e + 1)), false}; };
    auto advance = [&](Cursor cur) -> Cursor {
        if (cur.j + 1 < cur.s.np) {
            ++cur.j;
            return cur;
        }
        if (cur.e + 1 < SLq) return cursor_at(cur.e + 1);
        cur.past = true;
        return cur;
    };
    // A wave stages 64 neighbouring columns (in rank order) of one row at a time: thread tid takes the elements
    // tid, tid + 1024, ... of the piece, and one node cost of the operator the piece's edge arrives at (that row
    // travels with every piece of the edge, so that all pieces issue the same loads).
    // Every load of the main loop is unconditional and every piece issues the same number of them, so that the
    // waits can count outstanding loads instead of draining them all (a fetch past the end repeats the last piece,
    // ranks past the last feasible strategy repeat that strategy).
    struct Raw {
        int64_t r[G::EPT], c;
    };
    Raw raw0, raw1;
    auto fetch = [&](const Cursor& cur, Raw& raw) {
        if constexpr (!SPECS) {
            const int lgw = 6 + cur.s.lgc;
            const int row = tid >> lgw, col = tid & ((1 << lgw) - 1);
            const int b = lidx[cur.e + 1][col];
            const int64_t* src = R + (int64_t)(l0 + cur.e) * KP * KP + b;
#pragma unroll
            for (int i = 0; i < G::EPT; ++i) {
                const int a = lidx[cur.e][(cur.j << (12 - lgw)) + (i << (10 - lgw)) + row];
                raw.r[i] = src[a * KP];
            }
        }
        raw.c = c0[(int64_t)(cur.e + 1) * KP + lidx[cur.e + 1][tid & (KP - 1)]];
    };
    auto stash = [&](const Cursor& cur, const Raw& raw, int parity) {
        double* dst = lds + parity * kScPiece;
        const int lgw = 6 + cur.s.lgc;
        const int row = tid >> lgw, col = tid & ((1 << lgw) - 1);
        const bool col_ok = col < cur.s.nb;
        if constexpr (SPECS) {
            // the entries of this thread's column, rows (cur.j ...) of the edge's table in rank order
            const uint32_t qw = qwords[cur.e][lidx[cur.e + 1][col]];
            const uint32_t q0 = qw & 0xFFu, q1 = qw >> 8;
            const uint32_t sh0 = 4u * (q0 & 3u), sh1 = 4u * (q1 & 3u);
            const int64_t* t0 = &tabs[cur.e][0];
            const int64_t* t1 = &tabs[cur.e][10 + ((q0 & 3u) == 1u ? 5 : 0)];   // axis 1 moves after axis 0 has the consumer's state
#pragma unroll
            for (int i = 0; i < G::EPT; ++i) {
                const int rank = (cur.j << (12 - lgw)) + (i << (10 - lgw)) + row;
                const uint32_t pw = pwords[cur.e][lidx[cur.e][rank]];
                const uint32_t p0 = pw & 0xFFu, p1 = pw >> 8;
                const uint32_t k0 = q0 == p0 ? 0u : ((kind_row(p0 & 3u) >> sh0) & 7u);
                const uint32_t k1 = q1 == p1 ? 0u : ((kind_row(p1 & 3u) >> sh1) & 7u);
                // axis 0 moves while axis 1 still has the producer's state
                const int64_t t = t0[((p1 & 3u) == 1u ? 5u : 0u) + k0] + t1[k1];
                const bool ok = rank < cur.s.na && col_ok && pw != 0xFFFFu && qw != 0xFFFFu;
                dst[i * kScThreads + tid] = ok ? to_f64(t) : kInfD;
            }
        } else {
#pragma unroll
            for (int i = 0; i < G::EPT; ++i) {
                const bool row_ok = (cur.j << (12 - lgw)) + (i << (10 - lgw)) + row < cur.s.na;
                dst[i * kScThreads + tid] = (row_ok && col_ok) ? to_f64(raw.r[i]) : kInfD;
            }
        }
        if (tid < KP) c_arrive[parity][tid] = to_f64(raw.c);
    };
    Cursor cc = cursor_at(0);                     // the piece being used, the one after it, the one after that
    Cursor cs = advance(cc);
    Cursor cf = advance(cs);
    fetch(cc, raw0);
    fetch(cs, raw1);
    stash(cc, raw0, 0);
    lds_barrier();

    // entering with strategy a_row costs nothing extra: v = 0 at a_row, infeasible elsewhere
    double V[kScRows][G::CPT], acc[kScRows][G::CPT];
    const int n0 = count_at(0);
#pragma unroll
    for (int q = 0; q < kScRows; ++q)
#pragma unroll
        for (int k = 0; k < G::CPT; ++k) {
            const int b = lidx[0][lane + 64 * k];
            const bool ranked = lane + 64 * k < n0;
            V[q][k] = (ranked && b == a_row[q]) ? 0.0 : kInfD;
            if (Vin != nullptr && q < n_rows) {
                const double x = to_f64(Vin[(int64_t)g * in_stride + (int64_t)a_rank[q] * KP + lane + 64 * k]);
                V[q][k] = ranked ? x : kInfD;
            }
        }

    // one piece: parity = which LDS buffer and which registers hold it
    auto one_piece = [&](int parity, Raw& mine, const Raw& next) {
        if (cc.j == 0) {
#pragma unroll
            for (int q = 0; q < kScRows; ++q)
#pragma unroll
                for (int k = 0; k < G::CPT; ++k) acc[q][k] = kInfD;
        }
        fetch(cf, mine);                                  // the registers of this piece are free: it is in LDS
        const double* piece = lds + parity * kScPiece;
        const int rows_pp = 64 >> cc.s.lgc, rank0 = cc.j * rows_pp;
        int nr = cc.s.na - rank0;
        nr = nr < rows_pp ? nr : rows_pp;
        nr = (nr + 7) & ~7;                               // a piece has a multiple of 8 rows
        if (n_rows == 1) relax_width<KP, 1>(cc.s.lgc, piece, lane, nr, rank0, V, acc);
        if constexpr (kScRows == 2) {
            if (n_rows == 2) relax_width<KP, 2>(cc.s.lgc, piece, lane, nr, rank0, V, acc);
        }
        if (cc.j == cc.s.np - 1) {                        // the edge is done: on to the operator it arrives at
#pragma unroll
            for (int k = 0; k < G::CPT; ++k) {
                const double cb = c_arrive[parity][lane + 64 * k];
#pragma unroll
                for (int q = 0; q < kScRows; ++q)
                    V[q][k] = __builtin_fmin(cb + __builtin_fmin(acc[q][k], kInfD), kInfD);
            }
        }
        if (!cs.past) stash(cs, next, parity ^ 1);
        lds_barrier();                                    // the next piece is in LDS; this one has been read for the last time
        cc = cs;
        cs = cf;
        cf = advance(cf);
    };
    static_assert(kScRows <= 2, "one case per number of rows");
    while (true) {
        one_piece(0, raw0, raw1);
        if (cc.past) break;
        one_piece(1, raw1, raw0);
        if (cc.past) break;
    }

    // row a_rank of the matrix, columns in rank order of the part's last operator (infeasible past the last rank)
#pragma unroll
    for (int q = 0; q < kScRows; ++q) {
        if (q < n_rows) {
#pragma unroll
            for (int k = 0; k < G::CPT; ++k) Mg[(int64_t)a_rank[q] * KP + lane + 64 * k] = to_i64(V[q][k]);
        }
    }
}

// ---- step 2: boundary vectors ---------------------------------------------------------------------
// The matrices are in rank order (row = rank of the entering strategy among the feasible ones of the segment's
// first operator, column = rank at the operator the matrix reaches), and so are the vectors these kernels
// multiply; the node-cost rows they hand to the final sweep are in strategy order again.

// Ranks the feasible strategies of one operator (node costs c_op[0..KP), already in x for thread tid < KP):
// returns how many there are; live/rank describe strategy tid.  The whole workgroup calls it.
template <int KP>
__device__ __forceinline__ int rank_feasible(int64_t x, int tid, int wave, int lane, int32_t (&wave_cnt)[KP / 64],
                                             bool& live, int& rank) {
    live = tid < KP && x < kInf;
    const uint64_t mask = __ballot(live);
    __syncthreads();                              // the counts of the call before have been read
    if (tid < KP && lane == 0) wave_cnt[wave] = __popcll(mask);
    __syncthreads();
    int n = 0, before = 0;
#pragma unroll
    for (int w = 0; w < KP / 64; ++w) {
        const int cnt = wave_cnt[w];
        before += w < wave ? cnt : 0;
        n += cnt;
    }
    rank = before + __popcll(mask & ((1ull << lane) - 1));
    return n;
}

// vout[b] <- min_a (vs[a] + Mg[a][b]) for a < n_a, b < n_b, saturated; the whole workgroup (kBdThreads) takes part.
// A wave takes the rows a = wave, wave + 16, ..., eight at a time with all their loads in flight together.
template <int KP>
__device__ __forceinline__ void vector_times_matrix(const int64_t* __restrict__ vs, int n_a, int n_b,
                                                    int64_t (&part)[kBdWaves][KP], const int64_t* __restrict__ Mg,
                                                    int64_t* __restrict__ vout, int tid, int wave, int lane) {
    constexpr int LPG = KP / 128 > 0 ? KP / 128 : 1;      // 16-byte loads per lane per row
    constexpr int U = 8;
    int64_t best[2 * LPG];
#pragma unroll
    for (int j = 0; j < 2 * LPG; ++j) best[j] = kInf;
    for (int r0 = wave; r0 < n_a; r0 += kBdWaves * U) {
        ll2 m[U][LPG];
        int64_t va[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = r0 + kBdWaves * u;
            const int rr = row < n_a ? row : n_a - 1;     // a row past the end repeats the last one and cannot win
            va[u] = row < n_a ? vs[rr] : kInf;
#pragma unroll
            for (int k = 0; k < LPG; ++k) {
                const int col = (2 * lane + 128 * k) & (KP - 1);
                m[u][k] = ll2{0, 0};
                if (col < n_b) m[u][k] = *reinterpret_cast<const ll2*>(Mg + (int64_t)rr * KP + col);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int k = 0; k < LPG; ++k) {
                const int64_t x0 = va[u] + m[u][k].x, x1 = va[u] + m[u][k].y;
                best[2 * k] = x0 < best[2 * k] ? x0 : best[2 * k];
                best[2 * k + 1] = x1 < best[2 * k + 1] ? x1 : best[2 * k + 1];
            }
    }
    if (2 * lane < KP) {
#pragma unroll
        for (int k = 0; k < LPG; ++k) {
            part[wave][2 * lane + 128 * k] = best[2 * k];
            part[wave][2 * lane + 128 * k + 1] = best[2 * k + 1];
        }
    }
    __syncthreads();
    if (tid < KP) {
        int64_t x = part[0][tid];
#pragma unroll
        for (int w = 1; w < kBdWaves; ++w) x = part[w][tid] < x ? part[w][tid] : x;
        vout[tid] = (tid < n_b && x < kInf) ? x : kInf;
    }
    __syncthreads();
}

// One workgroup per problem: v_0 = c_0 (saturated), v_{g+1} = v_g (x) M_g.  The final sweep runs on problems of SLq = SL / kScSub
// edges; problem q's node costs are c_seg[q][SLq + 1][KP] with the start vector as row 0: v_g is row 0 of problem
// kScSub * g.
template <int KP>
__global__ void __launch_bounds__(kBdThreads)
scan_boundary_kernel(int32_t SL, int32_t SLq, int32_t nseg, const int64_t* __restrict__ c, int64_t c_bs,
                     const int64_t* __restrict__ M, int64_t* __restrict__ c_seg, int64_t ws_elems) {
    c += (int64_t)blockIdx.x * c_bs;              // one workgroup per problem; a problem's workspace is ws_elems long
    M += (int64_t)blockIdx.x * ws_elems;
    c_seg += (int64_t)blockIdx.x * ws_elems;
    __shared__ int64_t vs[2][KP];
    __shared__ int64_t part[kBdWaves][KP];
    __shared__ int32_t wave_cnt[KP / 64];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int64_t seg_stride = (int64_t)kScSub * (SLq + 1) * KP;
    bool live;
    int rank;
    int64_t x = tid < KP ? c[tid] : kInf;
    int n_a = rank_feasible<KP>(x, tid, wave, lane, wave_cnt, live, rank);
    if (tid < KP) c_seg[tid] = x < kInf ? x : kInf;
    if (live) vs[0][rank] = x;
    // node costs of the operator the next matrix reaches: asked for one product ahead
    int64_t c_reach = (tid < KP && nseg > 0) ? c[(int64_t)SL * KP + tid] : kInf;
    __syncthreads();
    for (int g = 0; g < nseg; ++g) {
        const int64_t c_now = c_reach;
        const int g_ahead = g + 2 <= nseg ? g + 2 : nseg;     // operator g_ahead * SL exists: the last segment follows
        c_reach = tid < KP ? c[(int64_t)g_ahead * SL * KP + tid] : kInf;
        const int n_b = rank_feasible<KP>(c_now, tid, wave, lane, wave_cnt, live, rank);
        int64_t* vnew = vs[(g + 1) & 1];
        vector_times_matrix<KP>(vs[g & 1], n_a, n_b, part, M + (int64_t)g * KP * KP, vnew, tid, wave, lane);
        if (tid < KP) c_seg[(int64_t)(g + 1) * seg_stride + tid] = live ? vnew[rank] : kInf;
        n_a = n_b;
    }
}

// Workgroup (j, g, problem): start vector of part j + 1 of segment g = v_g (x) Msub[g][j], row 0 of problem kScSub * g + j + 1.
template <int KP>
__global__ void __launch_bounds__(kBdThreads)
scan_part_vectors_kernel(int32_t SL, int32_t SLq, const int64_t* __restrict__ c, int64_t c_bs,
                         const int64_t* __restrict__ Msub, int64_t* __restrict__ c_seg, int64_t ws_elems) {
    c += (int64_t)blockIdx.z * c_bs;              // blockIdx.z = problem
    Msub += (int64_t)blockIdx.z * ws_elems;
    c_seg += (int64_t)blockIdx.z * ws_elems;
    __shared__ int64_t vs[2][KP];
    __shared__ int64_t part[kBdWaves][KP];
    __shared__ int32_t wave_cnt[KP / 64];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int j = blockIdx.x, g = blockIdx.y;
    const int64_t prob_stride = (int64_t)(SLq + 1) * KP;
    const int op_a = g * SL, op_b = op_a + (j + 1) * SLq;   // where the matrix starts and what it reaches
    bool live;
    int rank;
    const int64_t ca = tid < KP ? c[(int64_t)op_a * KP + tid] : kInf;
    const int64_t cb = tid < KP ? c[(int64_t)op_b * KP + tid] : kInf;
    const int64_t v = tid < KP ? c_seg[(int64_t)kScSub * g * prob_stride + tid] : kInf;
    const int n_a = rank_feasible<KP>(ca, tid, wave, lane, wave_cnt, live, rank);
    if (live) vs[0][rank] = v;
    const int n_b = rank_feasible<KP>(cb, tid, wave, lane, wave_cnt, live, rank);   // its barriers publish vs[0]
    vector_times_matrix<KP>(vs[0], n_a, n_b, part, Msub + ((int64_t)g * (kScSub - 1) + j) * KP * KP, vs[1], tid,
                            wave, lane);
    if (tid < KP) c_seg[((int64_t)kScSub * g + j + 1) * prob_stride + tid] = live ? vs[1][rank] : kInf;
}

// ---- step 3: the sweep inside every part --------------------------------------------------------
// One workgroup per part (and problem): the plain forward sweep from the part's start vector (row 0 of its problem in c_seg)
// over its SLq edges, writing arg.  Rows of an edge table whose strategy has an infeasible node cost cannot
// hold a minimum (their vector entry is infeasible) and are not read; the others are dealt to the 16 waves in
// rank order, D rows per wave in flight (D * trips covers the fullest edge): a slot is refilled with the same wave's row of the next edge as soon as
// it has been used, so the loads run ahead of the dependent chain of edges.
template <int KP, int D>
__device__ __forceinline__ void sweep_part(int SLq, int trips, const int64_t* __restrict__ c0,
                                           const int64_t* __restrict__ R0, uint16_t* __restrict__ arg0,
                                           int64_t* vs, const uint8_t (*lidx)[KP], const int32_t* nl,
                                           int64_t (*part_v)[KP], uint16_t (*part_a)[KP], int tid, int wave,
                                           int lane) {
    constexpr int LPG = KP / 128;                 // 16-byte loads per lane per row
    ll2 buf[D][LPG];                              // a wave takes D * trips rows of every edge
    auto row_of = [&](int e, int t, bool& ok) -> int {
        const int n = __builtin_amdgcn_readfirstlane(nl[e]);
        const int rank = wave + kScWaves * t;
        ok = rank < n;
        return lidx[e][ok ? rank : (n > 0 ? n - 1 : 0)];
    };
    auto fetch = [&](int e, int t, ll2 (&dst)[LPG]) {
        bool ok;
        const int a = __builtin_amdgcn_readfirstlane(row_of(e, t, ok));
        const int64_t* src = R0 + ((int64_t)e * KP + a) * KP + 2 * lane;
#pragma unroll
        for (int k = 0; k < LPG; ++k) dst[k] = __builtin_nontemporal_load(reinterpret_cast<const ll2*>(src + 128 * k));
    };
#pragma unroll
    for (int d = 0; d < D; ++d) fetch(0, d, buf[d]);
    int64_t c_next = tid < KP ? c0[KP + tid] : kInf;         // node costs of the operator edge 0 arrives at
    for (int e = 0; e < SLq; ++e) {
        const int64_t c_here = c_next;
        const int o_ahead = e + 2 <= SLq ? e + 2 : SLq;
        c_next = tid < KP ? c0[(int64_t)o_ahead * KP + tid] : kInf;
        int64_t best[2 * LPG];
        int32_t bidx[2 * LPG];
#pragma unroll
        for (int j = 0; j < 2 * LPG; ++j) {
            best[j] = INT64_MAX;
            bidx[j] = 0;
        }
        const int e_ahead = e + 1 < SLq ? e + 1 : SLq - 1;   // past the end the last edge is read again
#pragma unroll 1
        for (int tb = 0; tb < trips; ++tb) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const int t = tb * D + d;
                bool ok;
                const int a = __builtin_amdgcn_readfirstlane(row_of(e, t, ok));
                const int64_t va = ok ? vs[a] : kInf;        // a row past the last rank cannot win
#pragma unroll
                for (int k = 0; k < LPG; ++k) {
                    const int64_t x0 = va + buf[d][k].x, x1 = va + buf[d][k].y;
                    const bool l0 = x0 < best[2 * k], l1 = x1 < best[2 * k + 1];   // a ascends within a wave
                    best[2 * k] = l0 ? x0 : best[2 * k];
                    bidx[2 * k] = l0 ? a : bidx[2 * k];
                    best[2 * k + 1] = l1 ? x1 : best[2 * k + 1];
                    bidx[2 * k + 1] = l1 ? a : bidx[2 * k + 1];
                }
                // the same slot of the next trip, or of the next edge's first trip
                const bool wraps = tb + 1 == trips;
                fetch(wraps ? e_ahead : e, wraps ? d : t + D, buf[d]);
                __builtin_amdgcn_sched_barrier(0);   // use slot d, then refill slot d
            }
        }
#pragma unroll
        for (int k = 0; k < LPG; ++k) {
            *reinterpret_cast<ll2*>(&part_v[wave][2 * lane + 128 * k]) = ll2{best[2 * k], best[2 * k + 1]};
            part_a[wave][2 * lane + 128 * k] = (uint16_t)bidx[2 * k];
            part_a[wave][2 * lane + 128 * k + 1] = (uint16_t)bidx[2 * k + 1];
        }
        __syncthreads();
        if (tid < KP) {
            // the waves hold interleaved ranks: among equal values the lowest strategy wins
            int64_t m = part_v[0][tid];
            int32_t ma = part_a[0][tid];
#pragma unroll 4
            for (int w = 1; w < kScWaves; ++w) {   // (a few at a time: the rows in flight hold most registers)
                const int64_t x = part_v[w][tid];
                const int32_t xa = part_a[w][tid];
                const bool less = x < m || (x == m && xa < ma);
                m = less ? x : m;
                ma = less ? xa : ma;
            }
            const bool dead = m >= kInf;          // no feasible way into this strategy: (infeasible, 0)
            arg0[(int64_t)e * KP + tid] = (uint16_t)(dead ? 0 : ma);
            const int64_t v = m + c_here;
            vs[tid] = (dead || v >= kInf) ? kInf : v;
        }
        __syncthreads();
    }
}

template <int KP>
__global__ void __launch_bounds__(kScThreads)
scan_sweep_kernel(int32_t SLq, const int64_t* __restrict__ c, int64_t c_bs, const int64_t* __restrict__ R,
                  int64_t R_bs, const int64_t* __restrict__ c_seg, int64_t ws_elems, uint16_t* __restrict__ arg,
                  int64_t arg_bs) {
    c += (int64_t)blockIdx.y * c_bs;              // blockIdx.y = problem
    R += (int64_t)blockIdx.y * R_bs;
    c_seg += (int64_t)blockIdx.y * ws_elems;
    arg += (int64_t)blockIdx.y * arg_bs;
    __shared__ __align__(16) int64_t part_v[kScWaves][KP];
    __shared__ uint16_t part_a[kScWaves][KP];
    __shared__ int64_t vs[KP];
    __shared__ __align__(4) uint8_t lidx[kMaxPartLen + 1][KP];
    __shared__ int32_t nl[kMaxPartLen + 1];
    __shared__ int32_t n_max;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int q = blockIdx.x;                     // part q starts at operator q * SLq
    const int64_t* c0 = c + (int64_t)q * SLq * KP;
    if (tid == 0) n_max = 0;
    if (tid < KP) vs[tid] = c_seg[(int64_t)q * (SLq + 1) * KP + tid];
    __syncthreads();
    rank_operators<KP>(c0, SLq, lidx, nl, wave, lane);        // the operators edges leave from
    lds_barrier();
    if (tid < SLq) atomicMax(&n_max, nl[tid]);
    __syncthreads();
    const int t_max = (n_max + kScWaves - 1) / kScWaves;      // rows per wave of the fullest edge
    const int64_t* R0 = R + (int64_t)q * SLq * KP * KP;
    uint16_t* arg0 = arg + (int64_t)q * SLq * KP;
    // (four rows in flight per wave are 128 KiB per compute unit at Kp = 256: enough to keep the memory busy)
    if (t_max <= 2)
        sweep_part<KP, 2>(SLq, 1, c0, R0, arg0, vs, lidx, nl, part_v, part_a, tid, wave, lane);
    else
        sweep_part<KP, 4>(SLq, (t_max + 3) / 4, c0, R0, arg0, vs, lidx, nl, part_v, part_a, tid, wave, lane);
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

__host__ ScanPlan plan_scan(int32_t N, int32_t Kp, int32_t max_sl = kMaxSegLen) {
    ScanPlan p{};
    const int E = N - 1;
    const int step = Kp == 64 ? 4 * kScSub : kScSub;
    const int top = max_sl / step * step;        // longest segment allowed
    int s0 = 16;
    while ((int64_t)(s0 + 1) * (s0 + 1) <= E) ++s0;
    while ((E - 1) / s0 > kMaxMatrixSegments && s0 < top) ++s0;   // (beyond `top` the matrix launches take more rounds)
    s0 = (s0 + step - 1) / step * step;
    s0 = s0 < top ? s0 : top;
    int best_sl = s0, best_r = E;
    const int candidates = Kp == 64 ? 5 : 16;
    for (int sl = s0; sl < s0 + candidates * step && sl <= top; sl += step) {
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
    if (B < 1 || B > 32 || N < 128 || (Kp != 64 && Kp != 128 && Kp != 256)) return 0;
    const ScanPlan pl = plan_scan(N, Kp);
    if (pl.SL > kMaxSegLen) return 0;
    return (size_t)B * pl.total;
}

namespace {

// The segment matrices problem by problem (each fills the chip); then the boundary vectors, the part vectors and
// the sweep inside the parts for all problems together (the boundary pass is one workgroup per problem); the last
// segments one by one.
template <int KP>
hipError_t run_scan(const ScanPlan& pl, int32_t B, int32_t N, const int64_t* c, int64_t c_bs, const int64_t* R,
                    int64_t R_bs, uint16_t* arg, int64_t* vfinal, int64_t* total, int32_t* last, void* workspace,
                    hipStream_t stream) {
    const int nseg = pl.G - 1;                    // segments that need a matrix: all but the last
    const int nseg_pad = (nseg + 7) & ~7;
    const size_t lds = 2 * kScPiece * sizeof(double);
    const int SLq = pl.SL / kScSub, n_part = nseg * kScSub;
    const int64_t prob_c = (int64_t)(SLq + 1) * KP, prob_R = (int64_t)SLq * KP * KP;
    const int64_t mat = (int64_t)KP * KP, sub = (kScSub - 1) * mat;
    const int64_t ws_elems = (int64_t)(pl.total / sizeof(int64_t));
    const int64_t arg_bs = (int64_t)(N - 1) * KP;
    const int l_last = nseg * pl.SL;              // first operator of the last segment
    constexpr bool own_sweep = KP >= 128;         // step 3 by scan_sweep_kernel, which reads the node costs in place
    char* ws0 = static_cast<char*>(workspace);
    int64_t* M0 = reinterpret_cast<int64_t*>(ws0 + pl.m_off);
    int64_t* Msub0 = reinterpret_cast<int64_t*>(ws0 + pl.msub_off);
    int64_t* c_seg0 = reinterpret_cast<int64_t*>(ws0 + pl.cseg_off);

    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(scan_matrix_kernel<KP, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)(((KP + kScBlock - 1) / kScBlock) * nseg_pad));
    for (int p = 0; p < B; ++p) {
        int64_t* M = M0 + p * ws_elems;
        int64_t* Msub = Msub0 + p * ws_elems;
        int64_t* c_seg = c_seg0 + p * ws_elems;
        const int64_t* cp = c + (int64_t)p * c_bs;
        const int64_t* Rp = R + (int64_t)p * R_bs;
        // rows 1.. of the node costs of the last segment (and of every part, where chain_coop_kernel sweeps them)
        const int64_t n_copy = (int64_t)n_part * SLq * KP, n_copy_last = (int64_t)pl.r * KP;
        if (!own_sweep)
            hipLaunchKernelGGL(scan_copy_c_kernel, dim3((unsigned)((n_copy + 255) / 256)), dim3(256), 0, stream, N, SLq,
                               KP, n_part, cp, c_seg);
        hipLaunchKernelGGL(scan_copy_c_kernel, dim3((unsigned)((n_copy_last + 255) / 256)), dim3(256), 0, stream,
                           N - l_last, pl.r, KP, 1, cp + (int64_t)l_last * KP, c_seg + (int64_t)n_part * prob_c);
        for (int j = 0; j < kScSub; ++j) {
            const bool fin = j + 1 == kScSub;
            hipLaunchKernelGGL((scan_matrix_kernel<KP, false>), grid, dim3(kScThreads), lds, stream, pl.SL, SLq, j, nseg,
                               nseg_pad, cp, Rp, j ? Msub + (j - 1) * mat : nullptr, sub, fin ? M : Msub + j * mat,
                               fin ? mat : sub, SpecSource{});
        }
    }
    hipLaunchKernelGGL((scan_boundary_kernel<KP>), dim3((unsigned)B), dim3(kBdThreads), 0, stream, pl.SL, SLq, nseg, c,
                       c_bs, M0, c_seg0, ws_elems);
    hipLaunchKernelGGL((scan_part_vectors_kernel<KP>), dim3(kScSub - 1, nseg, (unsigned)B), dim3(kBdThreads), 0, stream,
                       pl.SL, SLq, c, c_bs, Msub0, c_seg0, ws_elems);
    if constexpr (own_sweep)
        hipLaunchKernelGGL((scan_sweep_kernel<KP>), dim3((unsigned)n_part, (unsigned)B), dim3(kScThreads), 0, stream, SLq,
                           c, c_bs, R, R_bs, c_seg0, ws_elems, arg, arg_bs);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    for (int p = 0; p < B; ++p) {
        int64_t* c_seg = c_seg0 + p * ws_elems;
        const int64_t* Rp = R + (int64_t)p * R_bs;
        uint16_t* argp = arg + p * arg_bs;
        if constexpr (!own_sweep) {
            // the parts as one batch (their totals are scratch)
            int64_t* seg_total = reinterpret_cast<int64_t*>(ws0 + pl.tot_off) + p * ws_elems;
            int32_t* seg_last = reinterpret_cast<int32_t*>(ws0 + pl.last_off) + 2 * p * ws_elems;
            e = launch_chain(n_part, SLq + 1, KP, c_seg, prob_c, Rp, prob_R, argp, nullptr, seg_total, seg_last, stream);
            if (e != hipSuccess) return e;
        }
        // the last segment, whose final vector, total and last are the chain's
        e = launch_chain(1, pl.r + 1, KP, c_seg + (int64_t)n_part * prob_c, 0, Rp + (int64_t)n_part * prob_R, 0,
                         argp + (int64_t)l_last * KP, vfinal ? vfinal + (int64_t)p * KP : nullptr, total + p, last + p,
                         stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

namespace {

// The same route with every table entry computed from the sharding specs: the matrices problem by problem on the
// problem's own mesh, the boundary and part vectors as above, then all parts and last segments of all problems in
// one launch of the kernel that relaxes edges from spec words (it starts every part from its vector and writes arg).
template <int KP>
hipError_t run_scan_specs(const ScanPlan& pl, int32_t B, int32_t N, int32_t n_meshes, const Mesh* meshes,
                          const int64_t* c, int64_t c_bs, const int32_t* K, const uint32_t* out_spec,
                          const uint32_t* in_spec, const int64_t* dims, const int32_t* elem_bytes, uint16_t* arg,
                          int64_t* vfinal, int64_t* total, int32_t* last, void* workspace, hipStream_t stream) {
    const int nseg = pl.G - 1;
    const int nseg_pad = (nseg + 7) & ~7;
    const size_t lds = 2 * kScPiece * sizeof(double);
    const int SLq = pl.SL / kScSub, n_part = nseg * kScSub;
    const int64_t prob_c = (int64_t)(SLq + 1) * KP;
    const int64_t mat = (int64_t)KP * KP, sub = (kScSub - 1) * mat;
    const int64_t ws_elems = (int64_t)(pl.total / sizeof(int64_t));
    char* ws0 = static_cast<char*>(workspace);
    int64_t* M0 = reinterpret_cast<int64_t*>(ws0 + pl.m_off);
    int64_t* Msub0 = reinterpret_cast<int64_t*>(ws0 + pl.msub_off);
    int64_t* c_seg0 = reinterpret_cast<int64_t*>(ws0 + pl.cseg_off);

    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(scan_matrix_kernel<KP, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)(((KP + kScBlock - 1) / kScBlock) * nseg_pad));
    for (int p = 0; p < B; ++p) {
        int64_t* M = M0 + p * ws_elems;
        int64_t* Msub = Msub0 + p * ws_elems;
        const int64_t* cp = c + (int64_t)p * c_bs;
        const SpecSource sp{K, out_spec, in_spec, dims, elem_bytes, meshes[p % n_meshes]};
        for (int j = 0; j < kScSub; ++j) {
            const bool fin = j + 1 == kScSub;
            hipLaunchKernelGGL((scan_matrix_kernel<KP, true>), grid, dim3(kScThreads), lds, stream, pl.SL, SLq, j, nseg,
                               nseg_pad, cp, static_cast<const int64_t*>(nullptr), j ? Msub + (j - 1) * mat : nullptr,
                               sub, fin ? M : Msub + j * mat, fin ? mat : sub, sp);
        }
    }
    hipLaunchKernelGGL((scan_boundary_kernel<KP>), dim3((unsigned)B), dim3(kBdThreads), 0, stream, pl.SL, SLq, nseg, c,
                       c_bs, M0, c_seg0, ws_elems);
    hipLaunchKernelGGL((scan_part_vectors_kernel<KP>), dim3(kScSub - 1, nseg, (unsigned)B), dim3(kBdThreads), 0, stream,
                       pl.SL, SLq, c, c_bs, Msub0, c_seg0, ws_elems);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_chain_fused_parts(B, N, KP, n_meshes, meshes, c, c_bs, K, out_spec, in_spec, dims, elem_bytes, SLq,
                                    n_part, c_seg0, prob_c, ws_elems, arg, vfinal, total, last, stream);
}

}  // namespace

size_t scan_specs_workspace_bytes(int32_t B, int32_t N, int32_t Kp) {
    if (B < 1 || B > 32 || N < 128 || (Kp != 64 && Kp != 128 && Kp != 256)) return 0;
    const ScanPlan pl = plan_scan(N, Kp, kSpecPartLen * kScSub);
    return (size_t)B * pl.total;
}

hipError_t launch_chain_scan_specs(int32_t B, int32_t N, int32_t Kp, int32_t n_meshes, const Mesh* meshes,
                                   const int64_t* c, int64_t c_bs, const int32_t* K, const uint32_t* out_spec,
                                   const uint32_t* in_spec, const int64_t* dims, const int32_t* elem_bytes,
                                   uint16_t* arg, int64_t* vfinal, int64_t* total, int32_t* last, void* workspace,
                                   hipStream_t stream) {
    const ScanPlan pl = plan_scan(N, Kp, kSpecPartLen * kScSub);
    switch (Kp) {
        case 64:
            return run_scan_specs<64>(pl, B, N, n_meshes, meshes, c, c_bs, K, out_spec, in_spec, dims, elem_bytes, arg,
                                      vfinal, total, last, workspace, stream);
        case 128:
            return run_scan_specs<128>(pl, B, N, n_meshes, meshes, c, c_bs, K, out_spec, in_spec, dims, elem_bytes, arg,
                                       vfinal, total, last, workspace, stream);
        case 256:
            return run_scan_specs<256>(pl, B, N, n_meshes, meshes, c, c_bs, K, out_spec, in_spec, dims, elem_bytes, arg,
                                       vfinal, total, last, workspace, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_chain_scan(int32_t B, int32_t N, int32_t Kp, const int64_t* c, int64_t c_bs, const int64_t* R,
                             int64_t R_bs, uint16_t* arg, int64_t* vfinal, int64_t* total, int32_t* last,
                             void* workspace, hipStream_t stream) {
    const ScanPlan pl = plan_scan(N, Kp);
    switch (Kp) {
        case 64: return run_scan<64>(pl, B, N, c, c_bs, R, R_bs, arg, vfinal, total, last, workspace, stream);
        case 128: return run_scan<128>(pl, B, N, c, c_bs, R, R_bs, arg, vfinal, total, last, workspace, stream);
        case 256: return run_scan<256>(pl, B, N, c, c_bs, R, R_bs, arg, vfinal, total, last, workspace, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace rh

// Stage times of all intervals of an operator chain: T[i][j] = least value of the Sec. 4.2
// objective over the plans of operators i..j-1 alone (Sec. 3 plans every pipeline stage on its
// own; Sec. 5.1 balances the stages, so the search needs the time of every candidate stage).
// For a fixed start i this is the running minimum of a forward chain sweep that begins at
// operator i; all L starts share the edge tables, so one step of all sweeps is a min-plus
// product of the matrix of live cost vectors (one row per start) with R_l.
//
// Arithmetic: values are integers in [0, 2^52] and every intermediate sum stays < 2^53, so the
// sweep runs in fp64 (exactly) -- a cell is v_add_f64 + v_min_f64 instead of five 64-bit
// integer operations.  Sums are clamped to "infeasible" after the minimum, which gives the same
// result as clamping every term because the clamp is monotone.  Inside the kernel infeasible
// is 2^52 - 1 (so that the conversion from int64 is an OR and a subtraction); feasible sums stay
// below 2^51 (at most 2^15 terms below 2^36), so the two thresholds cut at the same place.
//
// Mapping for Kp other than 64: a lane owns Kp/64 columns b; a wave keeps one row (start) in registers and
// broadcasts V[row][a] with two v_readlane per a, so the broadcast operand travels in scalar registers.
// Mapping at Kp = 64: the four rows of 16 lanes of a wave take different a at the same time (a = 4 n + r in step n
// for lanes 16 r .. 16 r + 15): one v_mov_b64_dpp row_newbcast per row and step hands V[row][a] to the 16
// lanes, each of which then relaxes four columns (j, j + 16, j + 32, j + 48); the four partial minima per
// column meet once per edge through two lane exchanges.  Per 256 cells that is 9 vector instructions instead of
// 16.  A wave keeps one row when every row walks its own number of edges (so that eight waves share a table),
// two neighbouring rows when the rows are of limited length.
// A workgroup stages R_l through LDS in 32 KiB pieces, converted to fp64 on the way in, double buffered, each
// piece asked for two pieces ahead.  At Kp = 64 four further waves do nothing but stage, so that fetching and
// converting run beside the arithmetic of the row waves instead of in turn with it.
// A workgroup takes a block of neighbouring rows and walks the
// edges they need, so that all its waves are busy together.  With a limit of at most half the chain
// (no stage longer than max_len operators: the sweep of row i stops after max_len operators and the
// rest of the row is infeasible) every block of 16 rows walks max_len + 15 edges: equal work, one
// block per workgroup.  Without such a limit the block that starts at operator i walks
// L - i edges, a triangle: then blocks have 8 rows, a workgroup takes block b and
// afterwards block (last - b), and every workgroup walks L + 8 edges.
#include "kernels.h"
#include "minplus_rows.h"

namespace rh {
namespace {

constexpr int kPiece = 4096;                 // elements of R per LDS buffer
// x of the lane that the DPP pattern CTRL pairs this lane with (patterns that stay inside a row of 16 lanes)
template <int CTRL>
__device__ __forceinline__ double dpp_peer(double x) {
    const int lo = __builtin_amdgcn_update_dpp(__double2loint(x), __double2loint(x), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(__double2hiint(x), __double2hiint(x), CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

// minimum over the wave, the same value in every lane: quads, half rows and rows through DPP
// (lane^1, lane^2, 7-lane within a half row, 15-lane within a row), the four rows through scalar registers
__device__ __forceinline__ double wave_min(double m) {
    m = __builtin_fmin(m, dpp_peer<0xB1>(m));    // quad_perm [1,0,3,2]
    m = __builtin_fmin(m, dpp_peer<0x4E>(m));    // quad_perm [2,3,0,1]
    m = __builtin_fmin(m, dpp_peer<0x141>(m));   // row_half_mirror
    m = __builtin_fmin(m, dpp_peer<0x140>(m));   // row_mirror
    return __builtin_fmin(__builtin_fmin(bcast(m, 0), bcast(m, 16)), __builtin_fmin(bcast(m, 32), bcast(m, 48)));
}

template <int KP>
struct Shape {
    static constexpr int CPT = KP >= 64 ? KP / 64 : 1;                  // columns per lane
    static constexpr int CH = KP >= 64 ? kPiece / KP : KP;              // rows a of R_l per piece
    static constexpr int NCH = KP / CH;                                 // pieces per edge
    static constexpr int ELEMS = CH * KP;                               // elements per piece
};

// acc[q][k] = min(acc[q][k], V[q][a] + R[a][col + 64 k]) for the CH rows a of one piece
template <int KP, int NA, int SLOTS>
__device__ __forceinline__ void relax_piece(const double* __restrict__ piece, int col, int ch,
                                            const double (&V)[SLOTS][Shape<KP>::CPT],
                                            double (&acc)[SLOTS][Shape<KP>::CPT]) {
    using G = Shape<KP>;
    const int a0 = ch * G::CH;
    const int k_src = a0 >> 6, lane0 = a0 & 63;    // V[q][a] sits in register k_src, lane a mod 64
    double src[NA];
#pragma unroll
    for (int q = 0; q < NA; ++q) {
        src[q] = V[q][0];
#pragma unroll
        for (int k = 1; k < G::CPT; ++k) {
            // must stay a select: folded into an indexed read of V it would move V to scratch memory
            src[q] = k_src == k ? V[q][k] : src[q];
            asm volatile("" : "+v"(src[q]));
        }
    }
    // The rows of the piece go with lanes lane0, lane0 + 1, ... of src.  With several pieces per edge lane0 is
    // only known at run time, and a broadcast from a lane numbered at run time is markedly slower than one
    // from a constant lane: turn src round so that the rows go with lanes 0, 1, ...
    int first = lane0;
    if constexpr (G::NCH > 1) {
        const int from = ((col + lane0) & 63) << 2;
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const int lo = __builtin_amdgcn_ds_bpermute(from, __double2loint(src[q]));
            const int hi = __builtin_amdgcn_ds_bpermute(from, __double2hiint(src[q]));
            src[q] = __hiloint2double(hi, lo);
        }
        first = 0;
    }
    // eight rows a at a time: their R values are fetched while the eight before them are worked on
    constexpr int AB = G::CPT >= 4 ? 2 : 8;
    static_assert(G::CH % AB == 0, "piece height");
    double r[2][AB][G::CPT];
#pragma unroll
    for (int u = 0; u < AB; ++u)
#pragma unroll
        for (int k = 0; k < G::CPT; ++k) r[0][u][k] = piece[u * KP + col + 64 * k];
#pragma unroll
    for (int blk = 0; blk < G::CH / AB; ++blk) {
        if (blk + 1 < G::CH / AB) {
#pragma unroll
            for (int u = 0; u < AB; ++u)
#pragma unroll
                for (int k = 0; k < G::CPT; ++k)
                    r[(blk + 1) & 1][u][k] = piece[((blk + 1) * AB + u) * KP + col + 64 * k];
        }
#pragma unroll
        for (int u = 0; u < AB; ++u) {
            double sv[NA], t[NA][G::CPT];
#pragma unroll
            for (int q = 0; q < NA; ++q) sv[q] = bcast(src[q], first + blk * AB + u);
#pragma unroll
            for (int q = 0; q < NA; ++q)
#pragma unroll
                for (int k = 0; k < G::CPT; ++k) t[q][k] = r[blk & 1][u][k] + sv[q];
#pragma unroll
            for (int q = 0; q < NA; ++q)
#pragma unroll
                for (int k = 0; k < G::CPT; ++k) acc[q][k] = __builtin_fmin(acc[q][k], t[q][k]);
        }
    }
}

// WAVES waves of SLOTS rows each = WAVES * SLOTS rows per block (wave w keeps rows SLOTS w .. SLOTS w + SLOTS - 1 of
// the block); the workgroup takes block blockIdx.x and, if PASSES == 2, block n_blocks - 1 - blockIdx.x after it.
// STAGERS = 0: every wave takes part in staging the tables.  STAGERS > 0: that many further waves do nothing but
// stage (fetch, convert, store to LDS) while the WAVES row waves do nothing but relax, so that the memory side and
// the arithmetic of an edge run side by side instead of one after the other in every wave.
// UNIT = false: row r is the sweep that starts at operator r with that operator's node costs (the table's row r).
// UNIT = true: all rows start at operator 0, row r with strategy r fixed there at no cost (a unit vector): row r of
// the output is then the least cost of the operators 0..j-1 given operator 0's strategy, its node cost left out.
// blockIdx.y = problem * sub.n + part: the parts of a problem are sub-chains at fixed strides; sub.v_end, if
// given, receives every row's vector at the last operator.
template <int KP, int WAVES, int PASSES, int SLOTS, int STAGERS, bool UNIT>
__global__ void __launch_bounds__((WAVES + STAGERS) * 64)
interval_costs_kernel(int32_t L_full, int32_t max_len, int32_t n_blocks,
                      const int64_t* __restrict__ c, int64_t c_bs, const int64_t* __restrict__ R, int64_t R_bs,
                      int64_t ldT, int64_t* __restrict__ T, int64_t T_bs, IntervalParts sub) {
    using G = Shape<KP>;
    constexpr int kThreads = (STAGERS > 0 ? STAGERS : WAVES) * 64;         // threads that stage
    constexpr int EPT = G::ELEMS / kThreads > 0 ? G::ELEMS / kThreads : 1;   // elements of a piece per thread
    extern __shared__ double lds[];               // two pieces of kPiece doubles
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const bool stages = STAGERS == 0 || wave >= WAVES;                      // wave-uniform
    const bool has_rows = wave < WAVES;
    const int tid = STAGERS > 0 ? (int)threadIdx.x - WAVES * 64 : (int)threadIdx.x;   // index among the staging threads
    const int prob = (int)blockIdx.y / sub.n, part = (int)blockIdx.y - prob * sub.n;
    c += (int64_t)prob * c_bs + (int64_t)part * sub.c_stride;
    R += (int64_t)prob * R_bs + (int64_t)part * sub.R_stride;
    T += (int64_t)prob * T_bs + (int64_t)part * sub.T_stride;
    // operators of this part: a part stops at the end of the chain (workgroup-uniform)
    const int left = sub.ops_total - part * sub.ops_stride;
    const int L = left < L_full ? left : L_full;
    if (L < 1) return;
    int64_t* v_end = (sub.v_end != nullptr && L == L_full)
                         ? sub.v_end + (int64_t)prob * sub.v_bs + (int64_t)part * sub.v_stride : nullptr;
    const int n_rows = UNIT ? KP : (sub.n_rows < L ? sub.n_rows : L);     // rows there are (a later one never starts)
    const bool live_lane = lane < KP;             // KP < 64: the upper lanes carry infeasible columns
    const int col = live_lane ? lane : 0;

#pragma unroll 1
  for (int pass = 0; pass < PASSES; ++pass) {
    const int block = pass == 0 ? (int)blockIdx.x : n_blocks - 1 - (int)blockIdx.x;
    if (pass > 0 && block <= (int)blockIdx.x) break;      // an odd number of blocks: the middle one has no partner
    lds_barrier();                                // the pass before has read its last piece

    // rows of this wave: slot q holds row block * WAVES * SLOTS + wave * SLOTS + q of the output (trow); it starts
    // at operator `row` (the same number, or operator 0 for every row when UNIT); L: never starts
    int row[SLOTS], trow[SLOTS];
#pragma unroll
    for (int q = 0; q < SLOTS; ++q) {
        trow[q] = (block * WAVES + wave) * SLOTS + q;
        row[q] = (has_rows && trow[q] < n_rows) ? (UNIT ? 0 : trow[q]) : L;
    }

    // entries at and left of the diagonal, and those of stages longer than max_len operators
#pragma unroll
    for (int q = 0; q < SLOTS; ++q) {
        if (row[q] < L)
            for (int j = lane; j <= L; j += 64)
                if (j <= row[q] || j - row[q] > max_len) T[(int64_t)trow[q] * ldT + j] = kInf;
    }

    constexpr int kRows = WAVES * SLOTS;          // rows of a block
    const int l0 = UNIT ? 0 : block * kRows;      // the first row of this block starts at operator l0
    // the last operator any row of this block reaches: its highest row, max_len operators on, or the chain's end
    const int row_hi = l0 + (UNIT ? 0 : kRows - 1) < L - 1 ? l0 + (UNIT ? 0 : kRows - 1) : L - 1;
    const int l_last = row_hi + max_len - 1 < L - 1 ? row_hi + max_len - 1 : L - 1;
    const int n_edges = l_last - l0;              // edges l0 .. l_last - 1
    const int n_pieces = n_edges * G::NCH;

    // piece g = (edge l0 + g / NCH, rows a of piece g % NCH); the pieces of one edge are contiguous in R.
    // A piece is asked for two pieces before it is used and waits in registers (two sets, taken in turn) until
    // its predecessor is being used, when it is converted and stored to LDS: one trip to memory takes about as
    // long as two edges.  Every load is unconditional (a piece past the end repeats the last one) so that the waits
    // count the loads still under way instead of draining them.
    struct Raw {
        int64_t r[EPT];
    };
    Raw preA, preB;
    auto fetch = [&](int g, Raw& pre) {
        g = g < n_pieces ? g : n_pieces - 1;
        const int64_t* src = R + ((int64_t)l0 * KP * KP + (int64_t)g * G::ELEMS);
        if constexpr (EPT >= 2) {
            typedef long long ll2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int e = 0; e < EPT / 2; ++e) {
                const ll2 v = *reinterpret_cast<const ll2*>(src + 2 * (e * kThreads + tid));
                pre.r[2 * e] = v.x;
                pre.r[2 * e + 1] = v.y;
            }
        } else {
            pre.r[0] = src[tid < G::ELEMS ? tid : 0];
        }
    };
    auto stash = [&](int g, const Raw& pre) {
        double* dst = lds + (g & 1) * kPiece;
        if constexpr (EPT >= 2) {
#pragma unroll
            for (int e = 0; e < EPT / 2; ++e) {
                const int at = 2 * (e * kThreads + tid);
                dst[at] = to_f64(pre.r[2 * e]);
                dst[at + 1] = to_f64(pre.r[2 * e + 1]);
            }
        } else {
            if (tid < G::ELEMS) dst[tid] = to_f64(pre.r[0]);
        }
    };
    if (n_pieces > 0 && stages) {
        fetch(0, preA);
        fetch(1, preB);
        stash(0, preA);
    }
    lds_barrier();

    // node costs of operators l and l+1 in this lane's columns; operators l+2 and l+3 on their way
    double cA[G::CPT], cB[G::CPT];
    int64_t cC[G::CPT], cD[G::CPT];
    auto load_c = [&](int l, int k) -> int64_t {
        const int64_t x = c[(int64_t)(l < L ? l : L - 1) * KP + col + 64 * k];
        return (l < L && live_lane) ? x : kInf;
    };
#pragma unroll
    for (int k = 0; k < G::CPT; ++k) {
        cA[k] = to_f64(load_c(l0, k));
        cB[k] = to_f64(load_c(l0 + 1, k));
        cC[k] = load_c(l0 + 2, k);
        cD[k] = kInf;
    }

    double V[SLOTS][G::CPT], acc[SLOTS][G::CPT];
#pragma unroll
    for (int q = 0; q < SLOTS; ++q)
#pragma unroll
        for (int k = 0; k < G::CPT; ++k) {
            V[q][k] = kInfD;
            acc[q][k] = kInfD;
        }

    double tcol[SLOTS];                           // finished columns of T waiting for their store
    bool running[SLOTS];                          // rows under way: started, not yet max_len operators long
#pragma unroll
    for (int q = 0; q < SLOTS; ++q) {
        tcol[q] = kInfD;
        running[q] = false;
    }

    // What happens when the sweeps arrive at operator l: rows that start here take its node costs; every row
    // under way gets its entry T[row][l+1] = cheapest strategy of operator l for the chain row..l.  Lane j mod 64
    // keeps column j; a full block of 64 columns (or the last, partial one) leaves as one coalesced store.
    auto arrive = [&](int l) {
#pragma unroll
        for (int q = 0; q < SLOTS; ++q) {
            if (row[q] == l) {
#pragma unroll
                for (int k = 0; k < G::CPT; ++k)
                    V[q][k] = UNIT ? ((live_lane && col + 64 * k == trow[q]) ? 0.0 : kInfD) : cA[k];
            }
            // (the rows of a wave start one after the other and stop one after the other, so with two slots the
            // cases are: 0 alone, both, 1 alone)
            running[q] = row[q] <= l && l - row[q] < max_len;     // wave-uniform
        }
        const int j = l + 1;
#pragma unroll
        for (int q = 0; q < SLOTS; ++q) {
            if (running[q]) {
                double m = V[q][0];
#pragma unroll
                for (int k = 1; k < G::CPT; ++k) m = __builtin_fmin(m, V[q][k]);
                m = wave_min(m);
                tcol[q] = lane == (j & 63) ? m : tcol[q];
                if ((j & 63) == 63 || j == L || j - row[q] == max_len) {
                    // columns of this block at or left of the diagonal still hold 2^52, which is their value
                    if (lane <= (j & 63)) T[(int64_t)trow[q] * ldT + (j & ~63) + lane] = to_i64(tcol[q]);
                }
            }
        }
    };
    // one piece: `mine` held piece g (it is in LDS by now) and takes piece g + 2, `next` holds piece g + 1
    auto one_piece = [&](int g, Raw& mine, const Raw& next) {
        const int e = g / G::NCH, ch = g - e * G::NCH;
        const int l = l0 + e;
        if (ch == 0 && has_rows) {
            arrive(l);
            // node costs three operators ahead: asked for now, so that the arithmetic below covers the trip
#pragma unroll
            for (int k = 0; k < G::CPT; ++k) cD[k] = load_c(l + 3, k);
#pragma unroll
            for (int q = 0; q < SLOTS; ++q)
#pragma unroll
                for (int k = 0; k < G::CPT; ++k) acc[q][k] = kInfD;
        }
        if (stages) fetch(g + 2, mine);
        const double* piece = lds + (g & 1) * kPiece;
        if constexpr (KP == 64) {
            if constexpr (SLOTS == 2) {
                // (slot 1 alone: slot 0 has stopped and is relaxed along with it, its results are not used)
                if (running[1]) relax_rows64<2, SLOTS>(piece, lane, V, acc);
                else if (running[0]) relax_rows64<1, SLOTS>(piece, lane, V, acc);
            } else {
                if (running[0]) relax_rows64<1, SLOTS>(piece, lane, V, acc);
            }
        } else {
            static_assert(SLOTS == 1 || KP == 64, "two rows per wave only in the Kp = 64 layout");
            if (running[0]) relax_piece<KP, 1, SLOTS>(piece, col, ch, V, acc);
        }
        if (stages && g + 1 < n_pieces) stash(g + 1, next);
        lds_barrier();                            // piece g+1 is in LDS; piece g has been read for the last time
        if (ch == G::NCH - 1 && has_rows) {                   // the edge is done: on to the operator it arrives at
#pragma unroll
            for (int q = 0; q < SLOTS; ++q) {
                if (running[q]) {
#pragma unroll
                    for (int k = 0; k < G::CPT; ++k) {
                        const double m = __builtin_fmin(acc[q][k], kInfD);
                        V[q][k] = __builtin_fmin(cB[k] + m, kInfD);
                    }
                }
            }
#pragma unroll
            for (int k = 0; k < G::CPT; ++k) {
                cA[k] = cB[k];
                cB[k] = to_f64(cC[k]);
                cC[k] = cD[k];
            }
        }
    };
    for (int g = 0; g < n_pieces; g += 2) {
        one_piece(g, preA, preB);
        if (g + 1 < n_pieces) one_piece(g + 1, preB, preA);
    }
    if (has_rows) arrive(l_last);                 // the entries of the last operator
    if (v_end != nullptr) {                       // every row's vector there
#pragma unroll
        for (int q = 0; q < SLOTS; ++q) {
            if (running[q] && live_lane) {
#pragma unroll
                for (int k = 0; k < G::CPT; ++k) v_end[(int64_t)trow[q] * KP + col + 64 * k] = to_i64(V[q][k]);
            }
        }
    }
  }
}

}  // namespace

// parts == nullptr: the table of B chains.  Otherwise every chain is n sub-chains at fixed strides (see kernels.h).
hipError_t launch_interval_costs(int32_t B, int32_t L, int32_t Kp, int32_t max_len, const int64_t* c, int64_t c_bs,
                                 const int64_t* R, int64_t R_bs, int64_t ldT, int64_t* T, int64_t T_bs,
                                 hipStream_t stream, const IntervalParts* parts, bool unit_rows) {
    if (B == 0) return hipSuccess;
    if (max_len > L) max_len = L;
    IntervalParts sub{1, 0, 0, 0, L, nullptr, 0, 0, 0, L};
    if (parts != nullptr) sub = *parts;
    if (sub.n < 1) return hipSuccess;
    if (unit_rows && Kp != 64) return hipErrorInvalidValue;
    const int rows_total = unit_rows ? Kp : (sub.n_rows < L ? sub.n_rows : L);
    // short stages only: blocks of 16 rows, equal work, one per workgroup; else blocks of 8 rows, a long one and a
    // short one per workgroup.  At Kp = 64: 8 waves of two rows, or 8 waves of one row, and four staging waves.
    const bool equal_blocks = max_len <= L / 2;
    const size_t lds = 2 * kPiece * sizeof(double);
#define RH_IC(KP, WAVES, PASSES, SLOTS, STAGERS, UNIT)                                                             \
    do {                                                                                                           \
        const int n_blocks = (rows_total + (WAVES) * (SLOTS)-1) / ((WAVES) * (SLOTS));                             \
        const dim3 grid((unsigned)((n_blocks + (PASSES)-1) / (PASSES)), (unsigned)(B * sub.n));                    \
        auto kern = interval_costs_kernel<KP, WAVES, PASSES, SLOTS, STAGERS, UNIT>;                                \
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                    \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                  \
        if (e != hipSuccess) return e;                                                                             \
        hipLaunchKernelGGL(kern, grid, dim3(((WAVES) + (STAGERS)) * 64), lds, stream, L, max_len, n_blocks, c,     \
                           c_bs, R, R_bs, ldT, T, T_bs, sub);                                                      \
    } while (0)
#define RH_IC_KP(KP)                                                                                               \
    do {                                                                                                           \
        if (equal_blocks)                                                                                          \
            RH_IC(KP, 16, 1, 1, 0, false);                                                                         \
        else                                                                                                       \
            RH_IC(KP, 8, 2, 1, 0, false);                                                                          \
    } while (0)
    switch (Kp) {
        case 16: RH_IC_KP(16); break;
        case 32: RH_IC_KP(32); break;
        case 64:
            if (unit_rows)
                RH_IC(64, 8, 1, 1, 4, true);
            else if (equal_blocks)
                RH_IC(64, 8, 1, 2, 4, false);
            else
                RH_IC(64, 8, 2, 1, 4, false);
            break;
        case 128: RH_IC_KP(128); break;
        case 256: RH_IC_KP(256); break;
        default: return hipErrorInvalidValue;
    }
#undef RH_IC_KP
#undef RH_IC
    return hipGetLastError();
}

}  // namespace rh

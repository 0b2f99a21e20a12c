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
// Mapping: a lane owns Kp/64 columns b; a wave keeps one row (start) in registers and
// broadcasts V[row][a] with two v_readlane per a, so the broadcast operand travels in scalar
// registers.  A workgroup (16 waves, 16 rows) stages R_l through LDS in 32 KiB pieces, converted
// to fp64 on the way in, double buffered.  A workgroup takes a block of neighbouring rows and walks the
// edges they need, so that all its waves are busy together.  With a limit of at most half the chain
// (no stage longer than max_len operators: the sweep of row i stops after max_len operators and the
// rest of the row is infeasible) every block of 16 rows walks max_len + 15 edges: equal work, one
// block per workgroup of 16 waves.  Without such a limit the block that starts at operator i walks
// L - i edges, a triangle: then blocks have 8 rows, a workgroup of 8 waves takes block b and
// afterwards block (last - b), and every workgroup walks L + 8 edges.
#include "kernels.h"

namespace rh {
namespace {

constexpr int kIcSlots = 1;                  // rows per wave
constexpr int kPiece = 4096;                 // elements of R per LDS buffer
constexpr double kInfD = 4503599627370495.0; // 2^52 - 1 stands for "infeasible" inside the kernel

__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Exact for 0 <= x < 2^52 - 1 (two full-rate instructions: the integer becomes the mantissa of 2^52 + x);
// anything from 2^52 - 1 up, which includes RH_INF, becomes the kernel's infeasible value.
__device__ __forceinline__ double to_f64(int64_t x) {
    uint32_t lo = (uint32_t)x, hi = (uint32_t)((uint64_t)x >> 32);
    const bool big = hi >= 0x100000u;
    lo = big ? 0xFFFFFFFFu : lo;
    hi = big ? 0xFFFFFu : hi;
    return __hiloint2double((int)(hi | 0x43300000u), (int)lo) - 4503599627370496.0;
}

// back to the interface's integers: infeasible is 2^52
__device__ __forceinline__ int64_t to_i64(double m) { return m >= kInfD ? kInf : (int64_t)m; }

__device__ __forceinline__ double bcast(double x, int lane) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), lane);
    return __hiloint2double(hi, lo);
}

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
template <int KP, int NA>
__device__ __forceinline__ void relax_piece(const double* __restrict__ piece, int col, int ch,
                                            const double (&V)[kIcSlots][Shape<KP>::CPT],
                                            double (&acc)[kIcSlots][Shape<KP>::CPT]) {
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
    constexpr int AB = G::CPT >= 4 ? 4 : 8;
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

// WAVES waves = WAVES rows per block; the workgroup takes block blockIdx.x and, if PASSES == 2, block
// n_blocks - 1 - blockIdx.x after it.
template <int KP, int WAVES, int PASSES>
__global__ void __launch_bounds__(WAVES * 64)
interval_costs_kernel(int32_t L, int32_t max_len, int32_t n_blocks,
                      const int64_t* __restrict__ c, int64_t c_bs, const int64_t* __restrict__ R, int64_t R_bs,
                      int64_t ldT, int64_t* __restrict__ T, int64_t T_bs) {
    using G = Shape<KP>;
    constexpr int kThreads = WAVES * 64;
    constexpr int EPT = G::ELEMS / kThreads > 0 ? G::ELEMS / kThreads : 1;   // elements of a piece per thread
    extern __shared__ double lds[];               // two pieces of kPiece doubles
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    c += (int64_t)blockIdx.y * c_bs;
    R += (int64_t)blockIdx.y * R_bs;
    T += (int64_t)blockIdx.y * T_bs;
    const bool live_lane = lane < KP;             // KP < 64: the upper lanes carry infeasible columns
    const int col = live_lane ? lane : 0;

#pragma unroll 1
  for (int pass = 0; pass < PASSES; ++pass) {
    const int block = pass == 0 ? (int)blockIdx.x : n_blocks - 1 - (int)blockIdx.x;
    if (pass > 0 && block <= (int)blockIdx.x) break;      // an odd number of blocks: the middle one has no partner
    lds_barrier();                                // the pass before has read its last piece

    // rows of this wave: slot q holds start block * WAVES + wave (kIcSlots is 1)
    int row[kIcSlots];
#pragma unroll
    for (int q = 0; q < kIcSlots; ++q) row[q] = block * WAVES + wave;

    // entries at and left of the diagonal, and those of stages longer than max_len operators
#pragma unroll
    for (int q = 0; q < kIcSlots; ++q) {
        if (row[q] < L)
            for (int j = lane; j <= L; j += 64)
                if (j <= row[q] || j - row[q] > max_len) T[(int64_t)row[q] * ldT + j] = kInf;
    }

    const int l0 = block * WAVES;                 // the first row of this block starts at operator l0
    // the last operator any row of this block reaches: its highest row, max_len operators on, or the chain's end
    const int row_hi = l0 + WAVES - 1 < L - 1 ? l0 + WAVES - 1 : L - 1;
    const int l_last = row_hi + max_len - 1 < L - 1 ? row_hi + max_len - 1 : L - 1;
    const int n_edges = l_last - l0;              // edges l0 .. l_last - 1
    const int n_pieces = n_edges * G::NCH;

    // piece g = (edge l0 + g / NCH, rows a of piece g % NCH); the pieces of one edge are contiguous in R
    int64_t pre[EPT];
    auto fetch = [&](int g) {
        const int64_t* src = R + ((int64_t)l0 * KP * KP + (int64_t)g * G::ELEMS);
        if constexpr (EPT >= 2) {
            typedef long long ll2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int e = 0; e < EPT / 2; ++e) {
                const ll2 v = *reinterpret_cast<const ll2*>(src + 2 * (e * kThreads + tid));
                pre[2 * e] = v.x;
                pre[2 * e + 1] = v.y;
            }
        } else {
            pre[0] = tid < G::ELEMS ? src[tid] : 0;
        }
    };
    auto stash = [&](int g) {
        double* dst = lds + (g & 1) * kPiece;
        if constexpr (EPT >= 2) {
#pragma unroll
            for (int e = 0; e < EPT / 2; ++e) {
                const int at = 2 * (e * kThreads + tid);
                dst[at] = to_f64(pre[2 * e]);
                dst[at + 1] = to_f64(pre[2 * e + 1]);
            }
        } else {
            if (tid < G::ELEMS) dst[tid] = to_f64(pre[0]);
        }
    };
    if (n_pieces > 0) {
        fetch(0);
        stash(0);
    }
    lds_barrier();

    // node costs of operators l and l+1 in this lane's columns; operator l+2 on its way
    double cA[G::CPT], cB[G::CPT];
    int64_t cC[G::CPT];
    auto load_c = [&](int l, int k) -> int64_t {
        return (l < L && live_lane) ? c[(int64_t)l * KP + col + 64 * k] : kInf;
    };
#pragma unroll
    for (int k = 0; k < G::CPT; ++k) {
        cA[k] = to_f64(load_c(l0, k));
        cB[k] = to_f64(load_c(l0 + 1, k));
        cC[k] = load_c(l0 + 2, k);
    }

    double V[kIcSlots][G::CPT];
#pragma unroll
    for (int q = 0; q < kIcSlots; ++q)
#pragma unroll
        for (int k = 0; k < G::CPT; ++k) V[q][k] = kInfD;

    double tcol[kIcSlots];                        // finished columns of T waiting for their store
#pragma unroll
    for (int q = 0; q < kIcSlots; ++q) tcol[q] = kInfD;

    int g = 0;
    for (int l = l0; l <= l_last; ++l) {
        int n_act = 0;                            // rows under way: started (they start in slot order), not yet max_len long
        static_assert(kIcSlots == 1, "a finished row in slot 0 beside a running one in slot 1 has no case below");
#pragma unroll
        for (int q = 0; q < kIcSlots; ++q) {
            if (row[q] == l) {
#pragma unroll
                for (int k = 0; k < G::CPT; ++k) V[q][k] = cA[k];
            }
            n_act += (row[q] <= l && l - row[q] < max_len) ? 1 : 0;
        }
        // T[row][l+1] = cheapest strategy of operator l for the chain row..l.  Lane j mod 64 keeps column
        // j; a full block of 64 columns (or the last, partial one) leaves as one coalesced store.
        const int j = l + 1;
#pragma unroll
        for (int q = 0; q < kIcSlots; ++q) {
            if (q < n_act) {
                double m = V[q][0];
#pragma unroll
                for (int k = 1; k < G::CPT; ++k) m = __builtin_fmin(m, V[q][k]);
                m = wave_min(m);
                tcol[q] = lane == (j & 63) ? m : tcol[q];
                if ((j & 63) == 63 || j == L || j - row[q] == max_len) {
                    // columns of this block at or left of the diagonal still hold 2^52, which is their value
                    if (lane <= (j & 63)) T[(int64_t)row[q] * ldT + (j & ~63) + lane] = to_i64(tcol[q]);
                }
            }
        }
        if (l == l_last) break;

        // node costs three operators ahead: asked for now, so that the arithmetic below covers the trip
        int64_t cD[G::CPT];
#pragma unroll
        for (int k = 0; k < G::CPT; ++k) cD[k] = load_c(l + 3, k);

        double acc[kIcSlots][G::CPT];
#pragma unroll
        for (int q = 0; q < kIcSlots; ++q)
#pragma unroll
            for (int k = 0; k < G::CPT; ++k) acc[q][k] = kInfD;
        for (int ch = 0; ch < G::NCH; ++ch, ++g) {
            const bool more = g + 1 < n_pieces;
            if (more) fetch(g + 1);               // in flight during the arithmetic
            const double* piece = lds + (g & 1) * kPiece;
            static_assert(kIcSlots <= 2, "one case per number of live rows");
            if (n_act == 1) relax_piece<KP, 1>(piece, col, ch, V, acc);
            if constexpr (kIcSlots == 2) {
                if (n_act == 2) relax_piece<KP, 2>(piece, col, ch, V, acc);
            }
            if (more) stash(g + 1);
            lds_barrier();                        // piece g+1 is in LDS; piece g has been read for the last time
        }
#pragma unroll
        for (int q = 0; q < kIcSlots; ++q) {
            if (q < n_act) {
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
  }
}

}  // namespace

hipError_t launch_interval_costs(int32_t B, int32_t L, int32_t Kp, int32_t max_len, const int64_t* c, int64_t c_bs,
                                 const int64_t* R, int64_t R_bs, int64_t ldT, int64_t* T, int64_t T_bs,
                                 hipStream_t stream) {
    if (B == 0) return hipSuccess;
    if (max_len > L) max_len = L;
    // short stages only: blocks of 16 rows, equal work, one per workgroup; else blocks of 8 rows, a long one and a
    // short one per workgroup
    const bool equal_blocks = max_len <= L / 2;
    const size_t lds = 2 * kPiece * sizeof(double);
#define RH_IC(KP, WAVES, PASSES)                                                                                   \
    do {                                                                                                           \
        const int n_blocks = (L + (WAVES)-1) / (WAVES);                                                            \
        const dim3 grid((unsigned)((n_blocks + (PASSES)-1) / (PASSES)), (unsigned)B);                              \
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(interval_costs_kernel<KP, WAVES, PASSES>),        \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                  \
        if (e != hipSuccess) return e;                                                                             \
        hipLaunchKernelGGL((interval_costs_kernel<KP, WAVES, PASSES>), grid, dim3((WAVES)*64), lds, stream, L, max_len,    \
                           n_blocks, c, c_bs, R, R_bs, ldT, T, T_bs);                                              \
    } while (0)
#define RH_IC_KP(KP)                                                                                               \
    do {                                                                                                           \
        if (equal_blocks)                                                                                          \
            RH_IC(KP, 16, 1);                                                                                      \
        else                                                                                                       \
            RH_IC(KP, 8, 2);                                                                                       \
    } while (0)
    switch (Kp) {
        case 16: RH_IC_KP(16); break;
        case 32: RH_IC_KP(32); break;
        case 64: RH_IC_KP(64); break;
        case 128: RH_IC_KP(128); break;
        case 256: RH_IC_KP(256); break;
        default: return hipErrorInvalidValue;
    }
#undef RH_IC_KP
#undef RH_IC
    return hipGetLastError();
}

}  // namespace rh

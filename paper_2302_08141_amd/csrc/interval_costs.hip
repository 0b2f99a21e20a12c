// Stage times of all intervals of an operator chain: T[i][j] = least value of the Sec. 4.2
// objective over the plans of operators i..j-1 alone (Sec. 3 plans every pipeline stage on its
// own; Sec. 5.1 balances the stages, so the search needs the time of every candidate stage).
// For a fixed start i this is the running minimum of a forward chain sweep that begins at
// operator i; all L starts share the edge tables, so one step of all sweeps is a min-plus
// product of the matrix of live cost vectors (one row per start) with R_l.
//
// Arithmetic: values are integers in [0, 2^52] and every intermediate sum stays <= 2^53, so the
// sweep runs in fp64 (exactly) -- a cell is v_add_f64 + v_min_f64 instead of five 64-bit
// integer operations.  Sums are clamped to 2^52 (infeasible) after the minimum, which gives the
// same result as clamping every term because the clamp is monotone.
//
// Mapping: a lane owns Kp/64 columns b; a wave keeps up to four rows (starts) in registers and
// broadcasts V[row][a] with two v_readlane per (row, a), so the broadcast operand travels in
// scalar registers and R_l[a][b] is read once from LDS for all four rows.  A workgroup (4 waves,
// 16 rows) stages R_l through LDS in 32 KiB pieces, converted to fp64 on the way in, double
// buffered.  Rows are dealt to workgroups round-robin (row i to workgroup i mod NW): every
// workgroup has rows of all ages, so the triangular work is balanced and all workgroups walk
// the edges in the same order, which lets one trip to HBM serve the chip.
#include "kernels.h"

namespace rh {
namespace {

constexpr int kIcThreads = 256;
constexpr int kIcWaves = 4;
constexpr int kIcSlots = 4;                  // rows per wave
constexpr int kIcRows = kIcWaves * kIcSlots; // rows per workgroup
constexpr int kPiece = 4096;                 // elements of R per LDS buffer
constexpr double kInfD = 4503599627370496.0; // 2^52

__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ double to_f64(int64_t x) { return (double)(x < kInf ? x : kInf); }

__device__ __forceinline__ double bcast(double x, int lane) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), lane);
    return __hiloint2double(hi, lo);
}

template <int KP>
struct Shape {
    static constexpr int CPT = KP >= 64 ? KP / 64 : 1;                  // columns per lane
    static constexpr int CH = KP >= 64 ? kPiece / KP : KP;              // rows a of R_l per piece
    static constexpr int NCH = KP / CH;                                 // pieces per edge
    static constexpr int ELEMS = CH * KP;                               // elements per piece
    static constexpr int EPT = ELEMS / kIcThreads > 0 ? ELEMS / kIcThreads : 1;   // per thread
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
        for (int k = 1; k < G::CPT; ++k) src[q] = k_src == k ? V[q][k] : src[q];
    }
#pragma unroll
    for (int a = 0; a < G::CH; ++a) {
        double r[G::CPT];
#pragma unroll
        for (int k = 0; k < G::CPT; ++k) r[k] = piece[a * KP + col + 64 * k];
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const double s = bcast(src[q], lane0 + a);
#pragma unroll
            for (int k = 0; k < G::CPT; ++k) acc[q][k] = __builtin_fmin(acc[q][k], r[k] + s);
        }
    }
}

template <int KP>
__global__ void __launch_bounds__(kIcThreads)
interval_costs_kernel(int32_t L, int32_t NW, const int64_t* __restrict__ c, int64_t c_bs,
                      const int64_t* __restrict__ R, int64_t R_bs, int64_t ldT, int64_t* __restrict__ T,
                      int64_t T_bs) {
    using G = Shape<KP>;
    extern __shared__ double lds[];               // two pieces of kPiece doubles
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int w = blockIdx.x;
    c += (int64_t)blockIdx.y * c_bs;
    R += (int64_t)blockIdx.y * R_bs;
    T += (int64_t)blockIdx.y * T_bs;
    const bool live_lane = lane < KP;             // KP < 64: the upper lanes carry infeasible columns
    const int col = live_lane ? lane : 0;

    // rows of this wave, ascending: slot q holds start w + NW * (4 q + wave)
    int row[kIcSlots];
#pragma unroll
    for (int q = 0; q < kIcSlots; ++q) row[q] = w + NW * (kIcWaves * q + wave);

    // entries at and left of the diagonal
#pragma unroll
    for (int q = 0; q < kIcSlots; ++q) {
        if (row[q] < L)
            for (int j = lane; j <= row[q]; j += 64) T[(int64_t)row[q] * ldT + j] = kInf;
    }

    const int l0 = w;                             // the first row of this workgroup starts at operator w
    const int n_edges = L - 1 - l0;               // edges l0 .. L-2
    const int n_pieces = n_edges * G::NCH;

    // piece g = (edge l0 + g / NCH, rows a of piece g % NCH); the pieces of one edge are contiguous in R
    int64_t pre[G::EPT];
    auto fetch = [&](int g) {
        const int64_t* src = R + ((int64_t)l0 * KP * KP + (int64_t)g * G::ELEMS);
        if constexpr (G::EPT >= 2) {
            typedef long long ll2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int e = 0; e < G::EPT / 2; ++e) {
                const ll2 v = *reinterpret_cast<const ll2*>(src + 2 * (e * kIcThreads + tid));
                pre[2 * e] = v.x;
                pre[2 * e + 1] = v.y;
            }
        } else {
            pre[0] = tid < G::ELEMS ? src[tid] : 0;
        }
    };
    auto stash = [&](int g) {
        double* dst = lds + (g & 1) * kPiece;
        if constexpr (G::EPT >= 2) {
#pragma unroll
            for (int e = 0; e < G::EPT / 2; ++e) {
                const int at = 2 * (e * kIcThreads + tid);
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

    int g = 0;
    for (int l = l0; l < L; ++l) {
        int n_act = 0;                            // rows started so far; they start in slot order
#pragma unroll
        for (int q = 0; q < kIcSlots; ++q) {
            if (row[q] == l) {
#pragma unroll
                for (int k = 0; k < G::CPT; ++k) V[q][k] = cA[k];
            }
            n_act += row[q] <= l ? 1 : 0;
        }
        // T[row][l+1] = cheapest strategy of operator l for the chain row..l
#pragma unroll
        for (int q = 0; q < kIcSlots; ++q) {
            if (q < n_act) {
                double m = V[q][0];
#pragma unroll
                for (int k = 1; k < G::CPT; ++k) m = __builtin_fmin(m, V[q][k]);
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) m = __builtin_fmin(m, __shfl_xor(m, off, 64));
                if (lane == 0) T[(int64_t)row[q] * ldT + l + 1] = (int64_t)m;
            }
        }
        if (l == L - 1) break;

        double acc[kIcSlots][G::CPT];
#pragma unroll
        for (int q = 0; q < kIcSlots; ++q)
#pragma unroll
            for (int k = 0; k < G::CPT; ++k) acc[q][k] = kInfD;
        for (int ch = 0; ch < G::NCH; ++ch, ++g) {
            const bool more = g + 1 < n_pieces;
            if (more) fetch(g + 1);               // in flight during the arithmetic
            const double* piece = lds + (g & 1) * kPiece;
            switch (n_act) {
                case 1: relax_piece<KP, 1>(piece, col, ch, V, acc); break;
                case 2: relax_piece<KP, 2>(piece, col, ch, V, acc); break;
                case 3: relax_piece<KP, 3>(piece, col, ch, V, acc); break;
                case 4: relax_piece<KP, 4>(piece, col, ch, V, acc); break;
                default: break;
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
            cC[k] = load_c(l + 3, k);
        }
    }
}

}  // namespace

hipError_t launch_interval_costs(int32_t B, int32_t L, int32_t Kp, const int64_t* c, int64_t c_bs, const int64_t* R,
                                 int64_t R_bs, int64_t ldT, int64_t* T, int64_t T_bs, hipStream_t stream) {
    if (B == 0) return hipSuccess;
    const int NW = (L + kIcRows - 1) / kIcRows;
    const size_t lds = 2 * kPiece * sizeof(double);
    const dim3 grid((unsigned)NW, (unsigned)B);
#define RH_IC(KP)                                                                                                  \
    do {                                                                                                           \
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(interval_costs_kernel<KP>),               \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                  \
        if (e != hipSuccess) return e;                                                                             \
        hipLaunchKernelGGL((interval_costs_kernel<KP>), grid, dim3(kIcThreads), lds, stream, L, NW, c, c_bs, R,    \
                           R_bs, ldT, T, T_bs);                                                                    \
    } while (0)
    switch (Kp) {
        case 16: RH_IC(16); break;
        case 32: RH_IC(32); break;
        case 64: RH_IC(64); break;
        case 128: RH_IC(128); break;
        case 256: RH_IC(256); break;
        default: return hipErrorInvalidValue;
    }
#undef RH_IC
    return hipGetLastError();
}

}  // namespace rh

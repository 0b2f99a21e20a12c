// Balanced pipeline stages (Sec. 2.1, Sec. 5.1-5.2) for chains of up to 6143 segments, exact and
// without visiting every (i, j) cell.  In dp[s][j] = min_{s-1<=i<j} max(dp[s-1][i], P(j)-P(i))
// the first argument never decreases with i and the second never increases, so with
//     i* = first i in [s-1, j) with dp[s-1][i] + P(i) >= P(j)
// the minimum over i >= i* is dp[s-1][i*] (lowest index i*), the minimum over i < i* is
// P(j) - P(i*-1), reached first at the lowest i with P(i) = P(i*-1) (segments of cost 0 make
// plateaus), and the smaller of the two wins, the left one on ties because its index is lower.
// That is the same value and the same lowest minimising i as the full scan.
//
// One workgroup per problem keeps P, G[s-1] = dp[s-1] + P and G[s] in LDS.  A thread owns up to
// six consecutive j.  i*(j) never decreases with j, nor with s (more stages never cost more, so
// G[s] <= G[s-1] pointwise): the first j of a thread gallops forward from its own i* of the
// stage count before, each further j from its predecessor's i* (two LDS reads when i* advances
// by one).  The plateau search runs only when a segment of cost 0 sits left of i*.  One
// LDS-only workgroup barrier per stage count: the cut entries drain to memory behind it.
#include "kernels.h"

namespace rh {
namespace {

constexpr int kFastThreads = 1024;
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

constexpr int kFastMaxL = 6143;     // 3 * (L+1) * 8 bytes of LDS = 144 KiB at most, plus 8 KiB for the scan

__global__ void __launch_bounds__(kFastThreads)
stage_fast_kernel(int32_t L, int32_t S, const int64_t* __restrict__ cost, int64_t* __restrict__ bottleneck,
                  int32_t* __restrict__ cut, int32_t s_query, int32_t* __restrict__ bounds) {
    extern __shared__ int64_t sm[];
    int64_t* P = sm;                  // [L+1]
    int64_t* A = sm + (L + 1);        // G[s-1][i] = dp[s-1][i] + P(i)
    int64_t* C = A + (L + 1);         // G[s]
    __shared__ int64_t part[kFastThreads];

    const int p = blockIdx.x, t = threadIdx.x;
    const int64_t* cs = cost + (int64_t)p * L;
    int32_t* ct = cut + (int64_t)p * S * (L + 1);

    // prefix sums: every thread sums a contiguous slice, the slice totals are scanned in LDS
    const int per = (L + kFastThreads - 1) / kFastThreads;
    const int lo = t * per < L ? t * per : L;
    const int hi = lo + per < L ? lo + per : L;
    int64_t sum = 0;
    for (int l = lo; l < hi; ++l) sum += cs[l];
    part[t] = sum;
    __syncthreads();
    for (int off = 1; off < kFastThreads; off <<= 1) {
        const int64_t add = t >= off ? part[t - off] : 0;
        __syncthreads();
        part[t] += add;
        __syncthreads();
    }
    int64_t run = part[t] - sum;      // exclusive
    if (t == 0) P[0] = 0;
    for (int l = lo; l < hi; ++l) {
        run += cs[l];
        P[l + 1] = run;
    }
    __syncthreads();
    for (int j = t; j <= L; j += kFastThreads) {
        A[j] = 2 * P[j];              // G[1][j] = dp[1][j] + P(j) = 2 P(j)
        ct[j] = j >= 1 ? 0 : -1;
    }
    if (t == 0) bottleneck[(int64_t)p * S] = P[L];
    __syncthreads();

    const int m = (L + kFastThreads) / kFastThreads;   // consecutive j per thread, ceil((L+1) / threads)
    const int j0 = t * m;
    int carry = -1;                    // i* of this thread's first live j at the stage count before
    for (int s = 2; s <= S; ++s) {
        int32_t* cts = ct + (int64_t)(s - 1) * (L + 1);
        const int first = s - 1;
        int from = carry < first ? (carry < 0 ? -1 : first) : carry;
        bool head = true;
        for (int q = 0; q < m; ++q) {
            const int j = j0 + q;
            if (j > L) break;
            if (j < s) {
                C[j] = kInf + P[j];
                cts[j] = -1;
                continue;
            }
            const int64_t Pj = P[j];
            // i* = first i in [first, j) with G[s-1][i] >= P(j), j if none
            int a = first, b = j;
            if (from >= 0) {
                // every i in [first, from) has G < P(j); stop at the first probe that does not, or at j
                a = b = from;
                int step = 1;
                while (b < j && A[b] < Pj) {
                    a = b + 1;
                    b += step;
                    step <<= 1;
                }
                b = b < j ? b : j;
            }
            while (a < b) {
                const int mid = (a + b) >> 1;
                if (A[mid] < Pj) a = mid + 1; else b = mid;
            }
            const int istar = a;
            from = istar;
            if (head) {
                // the same j at s+1 starts here if it is still the first live one (j >= s+1), which
                // holds unless j == s; then the head of s+1 is j+1, whose i* is at least this one too
                carry = istar;
                head = false;
            }
            // the four words the decision needs, fetched together (indices clamped into the range)
            const bool has_r = istar < j, has_l = istar > first;
            const int ir = has_r ? istar : first;
            const int il1 = has_l ? istar - 1 : first;
            const int il2 = il1 > first ? il1 - 1 : first;
            const int64_t gr = A[ir], pr = P[ir], pl = P[il1], pl2 = P[il2];
            int64_t best = has_r ? gr - pr : INT64_MAX;
            int besti = has_r ? istar : -1;
            const int64_t left = Pj - pl;
            if (has_l && left <= best) {          // on a tie the left candidate wins: its index is lower
                int il = il1;
                if (il1 > first && pl2 == pl) {
                    int a2 = first, b2 = il1;     // lowest i in [first, i*-1] with P(i) = P(i*-1)
                    while (a2 < b2) {
                        const int mid = (a2 + b2) >> 1;
                        if (P[mid] >= pl) b2 = mid; else a2 = mid + 1;
                    }
                    il = a2;
                }
                best = left;
                besti = il;
            }
            C[j] = best + Pj;
            cts[j] = besti;
            if (j == L) bottleneck[(int64_t)p * S + (s - 1)] = best;
        }
        lds_barrier();     // G[s] complete; G[s-1] has been read for the last time, so it can take G[s+1]
        int64_t* tmp = A; A = C; C = tmp;
    }
    __syncthreads();       // the cut table is in memory for the walk below

    if (s_query > 0 && bounds != nullptr && t == 0) {
        // the cut table was written by this workgroup and the barriers above made it visible to this thread
        int32_t* bd = bounds + (int64_t)p * (s_query + 1);
        int32_t x = L;
        bd[s_query] = x;
        for (int q = s_query; q >= 1; --q) {
            x = ct[(int64_t)(q - 1) * (L + 1) + x];
            x = x < 0 ? 0 : (x > L ? L : x);
            bd[q - 1] = x;
        }
    }
}

}  // namespace

bool stage_fast_applies(int32_t L) { return L <= kFastMaxL; }

hipError_t launch_stage_fast(int32_t B, int32_t L, int32_t S, const int64_t* seg_cost, int64_t* bottleneck,
                             int32_t* cut, int32_t s_query, int32_t* bounds, hipStream_t stream) {
    if (B == 0) return hipSuccess;
    const size_t lds = 3 * ((size_t)L + 1) * sizeof(int64_t);
    // always the kernel's largest size, never this call's own: the attribute is shared by every caller of the
    // process, and a smaller value set by one thread would refuse the launch of another
    constexpr size_t kMaxLds = 3 * ((size_t)kFastMaxL + 1) * sizeof(int64_t);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(stage_fast_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(stage_fast_kernel, dim3(B), dim3(kFastThreads), lds, stream, L, S, seg_cost, bottleneck, cut,
                       s_query, bounds);
    return hipGetLastError();
}

}  // namespace rh

// Joining the branches of cones at their roots (Sec. 4.3.2, level 1).  A cone is one root
// operator with several inputs whose other nodes have one input each, so its branches are
// chains; rh_minplus_chain leaves, per branch and root strategy r, the branch's best cost
// w[b][r].  Here: table[q][r] = c_root[q][r] + sum_b w[b][r], the best root strategy, and the
// starting point of every branch's backtrack.  One wavefront per cone, lanes over r, rows of w
// read coalesced exactly once: a small HBM streamer.
#include "kernels.h"

namespace rh {
namespace {

constexpr int kConesPerBlock = 4;

template <int CPL>   // columns per lane = ceil(Kp / 64)
__global__ void __launch_bounds__(kConesPerBlock * 64)
cone_merge_kernel(int32_t n_cones, int32_t n_branches, int32_t Kp, const int32_t* __restrict__ branch_start,
                  const int64_t* __restrict__ w, const int64_t* __restrict__ c_root,
                  int64_t* __restrict__ table, int64_t* __restrict__ total,
                  int32_t* __restrict__ root_choice, int32_t* __restrict__ branch_last) {
    const int lane = threadIdx.x & 63;
    const int q = blockIdx.x * kConesPerBlock + (threadIdx.x >> 6);
    if (q >= n_cones) return;
    int b0 = branch_start[q], b1 = branch_start[q + 1];
    b0 = b0 < 0 ? 0 : (b0 > n_branches ? n_branches : b0);      // a malformed offset table must not
    b1 = b1 < b0 ? b0 : (b1 > n_branches ? n_branches : b1);    // lead outside the branch batch
    int64_t acc[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        const int r = lane + 64 * k;
        const int64_t x = r < Kp ? c_root[(int64_t)q * Kp + r] : kInf;
        acc[k] = x < kInf ? x : kInf;
    }
    for (int b = b0; b < b1; ++b) {
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const int r = lane + 64 * k;
            if (r < Kp) {
                const int64_t x = w[(int64_t)b * Kp + r];
                const int64_t s = acc[k] + (x < kInf ? x : kInf);   // both <= 2^52: no overflow
                acc[k] = s < kInf ? s : kInf;
            }
        }
    }
    unsigned long long key = ~0ull;
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        const int r = lane + 64 * k;
        if (r < Kp) {
            if (table != nullptr) table[(int64_t)q * Kp + r] = acc[k];
            const unsigned long long kk = ((unsigned long long)acc[k] << 10) | (unsigned long long)r;
            key = kk < key ? kk : key;
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long o = __shfl_xor(key, off, 64);
        key = o < key ? o : key;
    }
    const int32_t choice = (int32_t)(key & 1023u);
    if (lane == 0) {
        total[q] = (int64_t)(key >> 10);
        root_choice[q] = choice;
    }
    if (branch_last != nullptr)
        for (int b = b0 + lane; b < b1; b += 64) branch_last[b] = choice;
}

}  // namespace

hipError_t launch_cone_merge(int32_t n_cones, int32_t n_branches, int32_t Kp, const int32_t* branch_start,
                             const int64_t* w, const int64_t* c_root, int64_t* table, int64_t* total,
                             int32_t* root_choice, int32_t* branch_last, hipStream_t stream) {
    if (n_cones == 0) return hipSuccess;
    const dim3 grid((unsigned)((n_cones + kConesPerBlock - 1) / kConesPerBlock)), block(kConesPerBlock * 64);
#define RH_CONE(CPL)                                                                                         \
    hipLaunchKernelGGL(cone_merge_kernel<CPL>, grid, block, 0, stream, n_cones, n_branches, Kp, branch_start, \
                       w, c_root, table, total, root_choice, branch_last)
    if (Kp <= 64) RH_CONE(1);
    else if (Kp == 128) RH_CONE(2);
    else if (Kp == 256) RH_CONE(4);
    else if (Kp == 512) RH_CONE(8);
    else RH_CONE(16);
#undef RH_CONE
    return hipGetLastError();
}

}  // namespace rh

// Min-plus chain DP for a handful of problems: eight workgroups (a gang; four when there are more
// than 32 problems) share one problem.
//
// A single workgroup cannot pull more than about 55 GB/s through its CU, so one long chain
// (the search over one model graph, Sec. 4.3.2) is latency-bound there.  Here every workgroup
// of the gang streams an eighth of the rows of each edge table, reduces them for all columns,
// and the gang exchanges one packed (cost << 10 | a) key per column and workgroup through a
// small buffer in device memory once per edge.  Every workgroup then finishes v_{i+1} for all
// columns itself; workgroup 0 writes the outputs.
//
// The exchange uses relaxed device-scope atomic stores and loads of single 64-bit words, and
// the words carry their own "ready" mark: a key is below 2^63, so bit 63 holds a tag that
// flips every time a slot is rewritten, and a reader simply polls the eight words of its column
// until all show the tag of the current edge.  Two key buffers alternate by edge parity: a
// workgroup can publish edge i+2 into the slots of edge i only after it has read every
// workgroup's keys of edge i+1, which those publish only after they have read edge i.  The
// gang must be resident at once (the launcher asks the device for its number of compute units and sizes the gangs
// so that every workgroup of the launch has a compute unit of its own; more problems than that take the
// one-workgroup kernel); the poll is bounded all the same, and a problem whose gang gave up reports total = -1.
#include "kernels.h"

namespace rh {
namespace {

typedef long long ll2 __attribute__((ext_vector_type(2)));
typedef unsigned long long u64;

constexpr int kMaxGang = 8;              // workgroups per problem: 8 or 4
constexpr int kW = 16;                   // waves per workgroup
constexpr int kEdgesAhead = 4;           // edges whose rows are in flight per wave
constexpr uint32_t kSpinLimit = 1u << 22;

__device__ __forceinline__ ll2 ld_stream(const char* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const ll2*>(p));
}

__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Every slot starts with tag 1 (edges 0 and 1 publish tag 0); the per-problem failure flags start at 0.
__global__ void __launch_bounds__(256) gang_clear_kernel(uint32_t* failed, int32_t n_flags, u64* xbuf, int64_t n_words) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n_flags) failed[t] = 0;
    if (t < n_words) xbuf[t] = ~0ull;
}

template <int KP, int kGang>
__global__ void __launch_bounds__(kW * 64)
chain_gang_kernel(int32_t N, const int64_t* __restrict__ c, int64_t c_bs, const int64_t* __restrict__ R,
                  int64_t R_bs, uint16_t* __restrict__ arg, int64_t* __restrict__ vfinal,
                  int64_t* __restrict__ total, int32_t* __restrict__ last, u64* __restrict__ xbuf,
                  uint32_t* __restrict__ failed_flags) {
    constexpr int LPG = KP / 128;            // 16-byte loads per lane per row
    constexpr int CPL = 2 * LPG;             // columns owned by a lane
    constexpr int RW = KP / kGang;           // rows of every edge table this workgroup reduces
    constexpr int RPW = RW / kW;             // rows per wave per edge
    static_assert(KP >= 128 && RPW >= 1 && RPW * kW * kGang == KP, "tile does not fit the gang");
    // the rows in flight must fit the registers (more than 32 live there, and every wait for a scratch access
    // drains the loads that run ahead): at most 8 sixteen-byte words per lane, 4 in a gang of eight, whose exchange
    // holds more registers.  One edge ahead is already 64 KiB or more in flight per workgroup, plenty for a step of
    // several microseconds.
    constexpr int kEdgeWords = (KP / kGang / kW) * (KP / 128);      // words per lane and edge
    constexpr int kBudget = kGang == 8 ? 4 : 8;
    constexpr int EA = kBudget / kEdgeWords >= kEdgesAhead ? kEdgesAhead : (kBudget / kEdgeWords >= 1 ? kBudget / kEdgeWords : 1);
    static_assert(kEdgeWords <= kBudget, "an edge's rows do not fit the registers of this gang size");

    __shared__ int64_t vs[KP];
    __shared__ u64 pkey[kW][KP];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int p = blockIdx.x / kGang;
    const int g = blockIdx.x - p * kGang;
    const int64_t* cp = c + (int64_t)p * c_bs;
    const bool merger = tid < KP / 2;        // thread t finishes columns 2t, 2t+1 of every edge
    u64* xp = xbuf + (size_t)p * 2 * kGang * KP;          // [parity][workgroup][column]
    uint32_t* failed = failed_flags + p;     // set by any thread of the gang that gave up waiting
    bool gave_up = false;

    if (merger) {
        ll2 c0 = *reinterpret_cast<const ll2*>(cp + 2 * tid);
        c0.x = c0.x < kInf ? c0.x : kInf;
        c0.y = c0.y < kInf ? c0.y : kInf;
        *reinterpret_cast<ll2*>(vs + 2 * tid) = c0;
    }
    lds_barrier();

    if (N > 1) {
        const int last_edge = N - 2;
        constexpr uint64_t kTileBytes = (uint64_t)KP * KP * 8;
        // this wave's rows of an edge table: g*RW + kk*kW + wave, kk < RPW
        const char* Rw = reinterpret_cast<const char*>(R + (int64_t)p * R_bs) +
                         (uint64_t)(g * RW + wave) * (KP * 8);               // wave-uniform
        const uint32_t lane_off = (uint32_t)lane * 16u;
        uint16_t* argp = arg + (int64_t)p * (N - 1) * KP;

        ll2 buf[EA][RPW][LPG];
#pragma unroll
        for (int e = 0; e < EA; ++e) {
            const int ie = e < last_edge ? e : last_edge;
#pragma unroll
            for (int kk = 0; kk < RPW; ++kk) {
#pragma unroll
                for (int k = 0; k < LPG; ++k)
                    buf[e][kk][k] = ld_stream(Rw + (uint64_t)ie * kTileBytes + (uint64_t)kk * (kW * KP * 8) +
                                              lane_off + 1024u * k);
                __builtin_amdgcn_sched_barrier(0);
            }
        }

#pragma unroll 1
        for (int i0 = 0; i0 < N - 1; i0 += EA) {
#pragma unroll
            for (int e = 0; e < EA; ++e) {
                const int i = i0 + e;
                if (i >= N - 1) break;

                int64_t best[CPL];
                int32_t bidx[CPL];
#pragma unroll
                for (int j = 0; j < CPL; ++j) {
                    best[j] = INT64_MAX;
                    bidx[j] = 0;
                }
                ll2 cn = {0, 0};
                if (merger) cn = *reinterpret_cast<const ll2*>(cp + (int64_t)(i + 1) * KP + 2 * tid);

                const int inext = i + EA < last_edge ? i + EA : last_edge;
                const char* src = Rw + (uint64_t)inext * kTileBytes;
#pragma unroll
                for (int kk = 0; kk < RPW; ++kk) {
                    const int a = g * RW + kk * kW + wave;
                    const int64_t va = vs[a];
#pragma unroll
                    for (int k = 0; k < LPG; ++k) {
                        const int64_t k0 = va + buf[e][kk][k].x;
                        const int64_t k1 = va + buf[e][kk][k].y;
                        const bool l0 = k0 < best[2 * k];
                        const bool l1 = k1 < best[2 * k + 1];
                        best[2 * k] = l0 ? k0 : best[2 * k];
                        bidx[2 * k] = l0 ? a : bidx[2 * k];
                        best[2 * k + 1] = l1 ? k1 : best[2 * k + 1];
                        bidx[2 * k + 1] = l1 ? a : bidx[2 * k + 1];
                    }
#pragma unroll
                    for (int k = 0; k < LPG; ++k)
                        buf[e][kk][k] = ld_stream(src + (uint64_t)kk * (kW * KP * 8) + lane_off + 1024u * k);
                    __builtin_amdgcn_sched_barrier(0);
                }

                // costs are cut off at RH_INF (an infeasible sum can reach 2^53), so keys stay below 2^63 and
                // bit 63 is free for the tag; comparing keys compares (cost, a) lexicographically
#pragma unroll
                for (int k = 0; k < LPG; ++k) {
                    const int64_t v0 = best[2 * k] < kInf ? best[2 * k] : kInf;
                    const int64_t v1 = best[2 * k + 1] < kInf ? best[2 * k + 1] : kInf;
                    ll2 pk;
                    pk.x = (long long)(((u64)v0 << 10) | (u64)bidx[2 * k]);
                    pk.y = (long long)(((u64)v1 << 10) | (u64)bidx[2 * k + 1]);
                    *reinterpret_cast<ll2*>(&pkey[wave][2 * lane + 128 * k]) = pk;
                }
                lds_barrier();   // the waves' keys are in LDS; every read of v_i is done

                u64* xw = xp + (size_t)(i & 1) * kGang * KP;
                if (merger) {
                    const u64 tag = (u64)((i >> 1) & 1) << 63;
                    u64 m0 = pkey[0][2 * tid], m1 = pkey[0][2 * tid + 1];
#pragma unroll 4
                    for (int w = 1; w < kW; ++w) {   // (a few at a time: the rows in flight hold most registers)
                        const u64 o0 = pkey[w][2 * tid], o1 = pkey[w][2 * tid + 1];
                        m0 = o0 < m0 ? o0 : m0;
                        m1 = o1 < m1 ? o1 : m1;
                    }
                    __hip_atomic_store(xw + (size_t)g * KP + 2 * tid, m0 | tag, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(xw + (size_t)g * KP + 2 * tid + 1, m1 | tag, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                    // poll the gang's words for these two columns until all carry this edge's tag
                    u64 k0[kGang], k1[kGang];
                    uint32_t spins = 0;
                    for (;;) {
                        u64 stale = 0;
#pragma unroll
                        for (int gg = 0; gg < kGang; ++gg) {
                            k0[gg] = __hip_atomic_load(xw + (size_t)gg * KP + 2 * tid, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
                            k1[gg] = __hip_atomic_load(xw + (size_t)gg * KP + 2 * tid + 1, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
                            stale |= (k0[gg] ^ tag) | (k1[gg] ^ tag);
                        }
                        if ((stale >> 63) == 0 || gave_up) break;
                        if (++spins > kSpinLimit) {   // stop waiting, here and from now on
                            gave_up = true;
                            // the flag reaches device memory before anything this thread publishes afterwards
                            __hip_atomic_store(failed, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
                            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "agent");
                        }
                        __builtin_amdgcn_s_sleep(1);
                    }
                    m0 = ~0ull;
                    m1 = ~0ull;
#pragma unroll
                    for (int gg = 0; gg < kGang; ++gg) {
                        const u64 o0 = k0[gg] & ~(1ull << 63), o1 = k1[gg] & ~(1ull << 63);
                        m0 = o0 < m0 ? o0 : m0;
                        m1 = o1 < m1 ? o1 : m1;
                    }
                    const int64_t b0 = (int64_t)(m0 >> 10), b1 = (int64_t)(m1 >> 10);
                    const bool d0 = b0 >= kInf, d1 = b1 >= kInf;         // no feasible predecessor
                    ll2 nv;
                    nv.x = cn.x + (d0 ? kInf : b0);
                    nv.y = cn.y + (d1 ? kInf : b1);
                    nv.x = nv.x < kInf ? nv.x : kInf;
                    nv.y = nv.y < kInf ? nv.y : kInf;
                    *reinterpret_cast<ll2*>(vs + 2 * tid) = nv;
                    if (g == 0) {
                        const uint32_t packed = (d0 ? 0u : (uint32_t)(m0 & 1023u)) |
                                                ((d1 ? 0u : (uint32_t)(m1 & 1023u)) << 16);
                        *reinterpret_cast<uint32_t*>(argp + (int64_t)i * KP + 2 * tid) = packed;
                    }
                }
                lds_barrier();   // v_{i+1} visible
            }
        }
    }

    if (g != 0) return;
    if (merger && vfinal != nullptr)
        *reinterpret_cast<ll2*>(vfinal + (int64_t)p * KP + 2 * tid) = *reinterpret_cast<const ll2*>(vs + 2 * tid);
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
            // a thread that gave up flagged the problem before it published anything further
            const bool bad = gave_up || __hip_atomic_load(failed, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) != 0;
            total[p] = bad ? -1 : (int64_t)(key >> 10);
            last[p] = (int32_t)(key & 1023u);
        }
    }
}

}  // namespace

// Workgroups per problem: as many as keep all gangs resident together (one workgroup of 1024 threads per compute
// unit), four at least (two do not beat a workgroup on its own: measured at Kp = 128; at Kp = 256 their rows would
// not fit the registers).  0 = the route is not taken.
int gang_workgroups(int32_t B, int32_t compute_units) {
    if (B < 1) return 0;
    for (int g = kMaxGang; g >= 4; g /= 2)
        if ((int64_t)B * g <= compute_units) return g;
    return 0;
}

// Compute units of the current device; 0 if there is none to ask (then the route is never taken).
static int device_compute_units() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return n;
}

size_t gang_workspace_bytes(int32_t B, int32_t N, int32_t Kp) {
    // worth it only for long chains of wide tables, and safe only while every gang is resident
    if (B < 1 || N < 64 || (Kp != 128 && Kp != 256)) return 0;
    const int g = gang_workgroups(B, device_compute_units());
    if (g == 0) return 0;
    return (size_t)B * 2 * g * Kp * sizeof(u64) + (((size_t)B * 4 + 255) & ~(size_t)255);
}

hipError_t launch_chain_gang(int32_t B, int32_t N, int32_t Kp, const int64_t* c, int64_t c_bs,
                             const int64_t* R, int64_t R_bs, uint16_t* arg, int64_t* vfinal,
                             int64_t* total, int32_t* last, void* workspace, hipStream_t stream) {
    const int g = gang_workgroups(B, device_compute_units());
    if (g == 0) return hipErrorInvalidValue;
    char* wsb = static_cast<char*>(workspace);
    uint32_t* counters = reinterpret_cast<uint32_t*>(wsb);   // one failure flag per problem
    u64* xbuf = reinterpret_cast<u64*>(wsb + (((size_t)B * 4 + 255) & ~(size_t)255));
    const int64_t n_words = (int64_t)B * 2 * g * Kp;
    hipLaunchKernelGGL(gang_clear_kernel, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, stream, counters, B,
                       xbuf, n_words);
    const dim3 grid((unsigned)(B * g));
#define RH_GANG(KP, G)                                                                                             \
    hipLaunchKernelGGL((chain_gang_kernel<KP, G>), grid, dim3(kW * 64), 0, stream, N, c, c_bs, R, R_bs, arg, vfinal, \
                       total, last, xbuf, counters)
    if (Kp == 128 && g == 8) RH_GANG(128, 8);
    else if (Kp == 128) RH_GANG(128, 4);
    else if (g == 8) RH_GANG(256, 8);
    else RH_GANG(256, 4);
#undef RH_GANG
    return hipGetLastError();
}

}  // namespace rh

// Min-plus chain DP on gfx950: v_{i+1}[b] = c_{i+1}[b] + min_a (v_i[a] + R_i[a][b]),
// the dynamic program that stitches candidate strategies along a chain of
// operators / segments (Sec. 4.3.2) and minimises the objective C of Sec. 4.2.
//
// The edge tables R are read exactly once and dominate the traffic, so the
// kernel is an HBM streamer.  One wavefront owns one problem and walks its
// edges in order.  R_i is row-major with the consumer index b contiguous, so a
// lane owns fixed columns b and reduces over the rows a in registers: no
// cross-lane traffic in the inner loop, and a row (or a few short rows) is one
// fully coalesced 16-byte-per-lane load.  All edge tables of a problem are
// contiguous, so the rows form one flat stream that is prefetched DEPTH row
// groups ahead, across edge boundaries, independent of the DP state.  v_i lives
// in LDS and is read as a broadcast.
#include "kernels.h"

namespace rh {
namespace {

typedef long long ll2 __attribute__((ext_vector_type(2)));

constexpr int kWavesPerBlock = 4;   // independent problems per workgroup

template <int KP>
struct Geo {
    static constexpr int LPR = KP >= 128 ? 64 : KP / 2;     // lanes that cover one row
    static constexpr int RPG = 64 / LPR;                    // rows per row group
    static constexpr int LPG = KP >= 128 ? KP / 128 : 1;    // 16-byte loads per lane per group
    static constexpr int CPL = 2 * LPG;                     // columns owned by a lane
    static constexpr int NG = KP / RPG;                     // row groups per edge table
    static constexpr int D0 = 16 / LPG > 0 ? 16 / LPG : 1;
    static constexpr int DEPTH = D0 < NG ? D0 : NG;         // row groups in flight
    static constexpr int GE = RPG * KP;                     // elements per row group
};

__device__ __forceinline__ ll2 ld_stream(const char* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const ll2*>(p));
}

// Orders this wave's LDS traffic in program order for the compiler; the
// hardware already executes one wave's LDS instructions in order.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int KP>
__global__ void __launch_bounds__(kWavesPerBlock * 64)
chain_wave_kernel(int32_t B, int32_t N, const int64_t* __restrict__ c, int64_t c_bs,
                  const int64_t* __restrict__ R, int64_t R_bs, uint16_t* __restrict__ arg,
                  int64_t* __restrict__ vfinal, int64_t* __restrict__ total,
                  int32_t* __restrict__ last) {
    using G = Geo<KP>;
    __shared__ int64_t vs_all[kWavesPerBlock][KP];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int p = blockIdx.x * kWavesPerBlock + wave;
    if (p >= B) return;   // no workgroup barrier is used below

    int64_t* vs = vs_all[wave];
    const int h = lane / G::LPR;      // row of the group this lane reads
    const int lc = lane % G::LPR;     // column pair (2*lc, 2*lc+1), then every 128 columns
    const int64_t* cp = c + (int64_t)p * c_bs;

    // v_0 = c_0
#pragma unroll
    for (int k = 0; k < G::LPG; ++k) {
        ll2 c0 = *reinterpret_cast<const ll2*>(cp + 2 * lc + 128 * k);
        c0.x = c0.x < kInf ? c0.x : kInf;
        c0.y = c0.y < kInf ? c0.y : kInf;
        if (h == 0) *reinterpret_cast<ll2*>(vs + 2 * lc + 128 * k) = c0;
    }
    wave_sync();

    if (N > 1) {
        const uint32_t last_group = (uint32_t)(N - 1) * G::NG - 1;
        const char* Rp = reinterpret_cast<const char*>(R + (int64_t)p * R_bs);   // wave-uniform
        const uint32_t lane_off = (uint32_t)(h * KP + 2 * lc) * 8u;             // bytes
        uint16_t* argp = arg + (int64_t)p * (N - 1) * KP;

        ll2 buf[G::DEPTH][G::LPG];
#pragma unroll
        for (int d = 0; d < G::DEPTH; ++d) {
#pragma unroll
            for (int k = 0; k < G::LPG; ++k)
                buf[d][k] = ld_stream(Rp + (uint64_t)d * (G::GE * 8) + lane_off + 1024u * k);
            __builtin_amdgcn_sched_barrier(0);   // issue in slot order, as the main loop does
        }

        for (int i = 0; i < N - 1; ++i) {
            int64_t best[G::CPL];
            int32_t bidx[G::CPL];
#pragma unroll
            for (int j = 0; j < G::CPL; ++j) {
                best[j] = INT64_MAX;
                bidx[j] = 0;
            }
            ll2 cn[G::LPG];
#pragma unroll
            for (int k = 0; k < G::LPG; ++k)
                cn[k] = *reinterpret_cast<const ll2*>(cp + (int64_t)(i + 1) * KP + 2 * lc + 128 * k);

            const uint32_t gnext = (uint32_t)i * G::NG + G::DEPTH;
#pragma unroll 1
            for (int gb = 0; gb < G::NG; gb += G::DEPTH) {
                int64_t va[G::DEPTH];
#pragma unroll
                for (int d = 0; d < G::DEPTH; ++d) va[d] = vs[(gb + d) * G::RPG + h];
#pragma unroll
                for (int d = 0; d < G::DEPTH; ++d) {
                    const int a = (gb + d) * G::RPG + h;
#pragma unroll
                    for (int k = 0; k < G::LPG; ++k) {
                        const int64_t k0 = va[d] + buf[d][k].x;
                        const int64_t k1 = va[d] + buf[d][k].y;
                        const bool l0 = k0 < best[2 * k];
                        const bool l1 = k1 < best[2 * k + 1];
                        best[2 * k] = l0 ? k0 : best[2 * k];
                        bidx[2 * k] = l0 ? a : bidx[2 * k];
                        best[2 * k + 1] = l1 ? k1 : best[2 * k + 1];
                        bidx[2 * k + 1] = l1 ? a : bidx[2 * k + 1];
                    }
                    // refill the slot with the group DEPTH ahead; past the end of the stream the
                    // last group is read again instead of branching
                    uint32_t nxt = gnext + (uint32_t)(gb + d);
                    nxt = nxt < last_group ? nxt : last_group;
                    const char* src = Rp + (uint64_t)nxt * (G::GE * 8);
#pragma unroll
                    for (int k = 0; k < G::LPG; ++k) buf[d][k] = ld_stream(src + lane_off + 1024u * k);
                    // keep "consume slot d, then refill slot d" in this order: ALU and LDS may
                    // move across, memory reads may not
                    __builtin_amdgcn_sched_barrier(0);
                }
            }

            // lanes that read different rows of the same columns: merge, lowest a on ties
#pragma unroll
            for (int off = G::LPR; off < 64; off <<= 1) {
#pragma unroll
                for (int j = 0; j < G::CPL; ++j) {
                    const int64_t ob = __shfl_xor(best[j], off, 64);
                    const int32_t oi = __shfl_xor(bidx[j], off, 64);
                    const bool take = ob < best[j] || (ob == best[j] && oi < bidx[j]);
                    best[j] = take ? ob : best[j];
                    bidx[j] = take ? oi : bidx[j];
                }
            }

            wave_sync();   // every read of v_i is issued before v_{i+1} is written
            if (h == 0) {
#pragma unroll
                for (int k = 0; k < G::LPG; ++k) {
                    ll2 nv;
                    uint32_t packed = 0;
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int j = 2 * k + e;
                        const bool dead = best[j] >= kInf;          // no feasible predecessor
                        const int64_t bv = dead ? kInf : best[j];
                        const uint32_t bi = dead ? 0u : (uint32_t)bidx[j];
                        int64_t s = (e == 0 ? cn[k].x : cn[k].y) + bv;
                        s = s < kInf ? s : kInf;
                        if (e == 0) nv.x = s; else nv.y = s;
                        packed |= bi << (16 * e);
                    }
                    *reinterpret_cast<ll2*>(vs + 2 * lc + 128 * k) = nv;
                    *reinterpret_cast<uint32_t*>(argp + (int64_t)i * KP + 2 * lc + 128 * k) = packed;
                }
            }
            wave_sync();
        }
    }

    // total = min_b v_{N-1}[b], lowest b on ties: one packed (cost << 10 | b) key per lane,
    // then a butterfly over the wave
    uint64_t key = ~0ull;
#pragma unroll
    for (int k = 0; k < G::LPG; ++k) {
        const int col = 2 * lc + 128 * k;
        const ll2 v2 = *reinterpret_cast<const ll2*>(vs + col);
        if (vfinal != nullptr && h == 0) *reinterpret_cast<ll2*>(vfinal + (int64_t)p * KP + col) = v2;
        const uint64_t k0 = ((uint64_t)v2.x << 10) | (uint64_t)col;
        const uint64_t k1 = ((uint64_t)v2.y << 10) | (uint64_t)(col + 1);
        key = k0 < key ? k0 : key;
        key = k1 < key ? k1 : key;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint64_t o = __shfl_xor(key, off, 64);
        key = o < key ? o : key;
    }
    if (lane == 0) {
        total[p] = (int64_t)(key >> 10);
        last[p] = (int32_t)(key & 1023u);
    }
}

// ---------------------------------------------------------------------------------------
// Few problems: one workgroup of W waves per problem.  The row groups of the flat stream are
// dealt to the waves round-robin (at any moment the W waves read W consecutive groups), every
// wave keeps its own register ring over its share and reduces its rows for all the columns it
// owns; the W partial (min, argmin) pairs per column meet in LDS once per edge.  The barriers
// only order LDS traffic, so the prefetched loads stay in flight across them.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int KP, int W>
struct CoopGeo {
    using G = Geo<KP>;
    static constexpr int GPW = G::NG / W;                    // row groups per wave per edge
    static constexpr int DEPTH = G::D0 < GPW ? G::D0 : GPW;  // row groups in flight per wave
    static_assert(GPW >= 1 && GPW * W == G::NG && GPW % DEPTH == 0, "wave count does not fit the tile");
};

template <int KP, int W>
__global__ void __launch_bounds__(W * 64)
chain_coop_kernel(int32_t N, const int64_t* __restrict__ c, int64_t c_bs, const int64_t* __restrict__ R,
                  int64_t R_bs, uint16_t* __restrict__ arg, int64_t* __restrict__ vfinal,
                  int64_t* __restrict__ total, int32_t* __restrict__ last) {
    using G = Geo<KP>;
    using CG = CoopGeo<KP, W>;
    __shared__ int64_t vs[KP];
    __shared__ int64_t pval[W][KP];
    __shared__ int32_t pidx[W][KP];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int p = blockIdx.x;
    const int h = lane / G::LPR;
    const int lc = lane % G::LPR;
    const int64_t* cp = c + (int64_t)p * c_bs;
    // column pairs (2t, 2t+1) are finished, once per edge, by thread t (mod the workgroup size)
    constexpr int kThreads = W * 64;
    constexpr int MP = (KP / 2 + kThreads - 1) / kThreads;

#pragma unroll
    for (int m = 0; m < MP; ++m) {
        const int t = tid + m * kThreads;
        if (t < KP / 2) {
            ll2 c0 = *reinterpret_cast<const ll2*>(cp + 2 * t);
            c0.x = c0.x < kInf ? c0.x : kInf;
            c0.y = c0.y < kInf ? c0.y : kInf;
            *reinterpret_cast<ll2*>(vs + 2 * t) = c0;
        }
    }
    lds_barrier();

    if (N > 1) {
        const uint32_t last_k = (uint32_t)(N - 1) * CG::GPW - 1;   // this wave's last group, in its own count
        const char* Rp = reinterpret_cast<const char*>(R + (int64_t)p * R_bs) +
                         (uint64_t)wave * (G::GE * 8);             // wave-uniform
        const uint32_t lane_off = (uint32_t)(h * KP + 2 * lc) * 8u;
        constexpr uint64_t kStride = (uint64_t)W * G::GE * 8;      // bytes between a wave's groups
        uint16_t* argp = arg + (int64_t)p * (N - 1) * KP;

        ll2 buf[CG::DEPTH][G::LPG];
#pragma unroll
        for (int d = 0; d < CG::DEPTH; ++d) {
#pragma unroll
            for (int k = 0; k < G::LPG; ++k) buf[d][k] = ld_stream(Rp + d * kStride + lane_off + 1024u * k);
            __builtin_amdgcn_sched_barrier(0);
        }

        for (int i = 0; i < N - 1; ++i) {
            int64_t best[G::CPL];
            int32_t bidx[G::CPL];
#pragma unroll
            for (int j = 0; j < G::CPL; ++j) {
                best[j] = INT64_MAX;
                bidx[j] = 0;
            }
            ll2 cn[MP];
#pragma unroll
            for (int m = 0; m < MP; ++m) {
                const int t = tid + m * kThreads;
                cn[m] = ll2{0, 0};
                if (t < KP / 2) cn[m] = *reinterpret_cast<const ll2*>(cp + (int64_t)(i + 1) * KP + 2 * t);
            }

            const uint32_t knext = (uint32_t)i * CG::GPW + CG::DEPTH;
#pragma unroll 1
            for (int kb = 0; kb < CG::GPW; kb += CG::DEPTH) {
                int64_t va[CG::DEPTH];
#pragma unroll
                for (int d = 0; d < CG::DEPTH; ++d) va[d] = vs[((kb + d) * W + wave) * G::RPG + h];
#pragma unroll
                for (int d = 0; d < CG::DEPTH; ++d) {
                    const int a = ((kb + d) * W + wave) * G::RPG + h;
#pragma unroll
                    for (int k = 0; k < G::LPG; ++k) {
                        const int64_t k0 = va[d] + buf[d][k].x;
                        const int64_t k1 = va[d] + buf[d][k].y;
                        const bool l0 = k0 < best[2 * k];
                        const bool l1 = k1 < best[2 * k + 1];
                        best[2 * k] = l0 ? k0 : best[2 * k];
                        bidx[2 * k] = l0 ? a : bidx[2 * k];
                        best[2 * k + 1] = l1 ? k1 : best[2 * k + 1];
                        bidx[2 * k + 1] = l1 ? a : bidx[2 * k + 1];
                    }
                    uint32_t nxt = knext + (uint32_t)(kb + d);
                    nxt = nxt < last_k ? nxt : last_k;
                    const char* src = Rp + (uint64_t)nxt * kStride;
#pragma unroll
                    for (int k = 0; k < G::LPG; ++k) buf[d][k] = ld_stream(src + lane_off + 1024u * k);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }

#pragma unroll
            for (int off = G::LPR; off < 64; off <<= 1) {
#pragma unroll
                for (int j = 0; j < G::CPL; ++j) {
                    const int64_t ob = __shfl_xor(best[j], off, 64);
                    const int32_t oi = __shfl_xor(bidx[j], off, 64);
                    const bool take = ob < best[j] || (ob == best[j] && oi < bidx[j]);
                    best[j] = take ? ob : best[j];
                    bidx[j] = take ? oi : bidx[j];
                }
            }
            if (h == 0) {
#pragma unroll
                for (int k = 0; k < G::LPG; ++k) {
                    ll2 pv;
                    pv.x = best[2 * k];
                    pv.y = best[2 * k + 1];
                    int2 pi;
                    pi.x = bidx[2 * k];
                    pi.y = bidx[2 * k + 1];
                    *reinterpret_cast<ll2*>(&pval[wave][2 * lc + 128 * k]) = pv;
                    *reinterpret_cast<int2*>(&pidx[wave][2 * lc + 128 * k]) = pi;
                }
            }
            lds_barrier();   // partials visible; every read of v_i is done
#pragma unroll
            for (int m = 0; m < MP; ++m) {
                const int t = tid + m * kThreads;
                if (t >= KP / 2) continue;
                ll2 bv = *reinterpret_cast<const ll2*>(&pval[0][2 * t]);
                int2 bi = *reinterpret_cast<const int2*>(&pidx[0][2 * t]);
#pragma unroll
                for (int w = 1; w < W; ++w) {
                    const ll2 ov = *reinterpret_cast<const ll2*>(&pval[w][2 * t]);
                    const int2 oi = *reinterpret_cast<const int2*>(&pidx[w][2 * t]);
                    const bool t0 = ov.x < bv.x || (ov.x == bv.x && oi.x < bi.x);   // rows interleave over
                    const bool t1 = ov.y < bv.y || (ov.y == bv.y && oi.y < bi.y);   // waves: compare indices
                    bv.x = t0 ? ov.x : bv.x;
                    bi.x = t0 ? oi.x : bi.x;
                    bv.y = t1 ? ov.y : bv.y;
                    bi.y = t1 ? oi.y : bi.y;
                }
                const bool d0 = bv.x >= kInf, d1 = bv.y >= kInf;     // no feasible predecessor
                ll2 nv;
                nv.x = cn[m].x + (d0 ? kInf : bv.x);
                nv.y = cn[m].y + (d1 ? kInf : bv.y);
                nv.x = nv.x < kInf ? nv.x : kInf;
                nv.y = nv.y < kInf ? nv.y : kInf;
                *reinterpret_cast<ll2*>(vs + 2 * t) = nv;
                const uint32_t packed = (d0 ? 0u : (uint32_t)bi.x) | ((d1 ? 0u : (uint32_t)bi.y) << 16);
                *reinterpret_cast<uint32_t*>(argp + (int64_t)i * KP + 2 * t) = packed;
            }
            lds_barrier();   // v_{i+1} visible
        }
    }

    if (vfinal != nullptr) {
#pragma unroll
        for (int m = 0; m < MP; ++m) {
            const int t = tid + m * kThreads;
            if (t < KP / 2)
                *reinterpret_cast<ll2*>(vfinal + (int64_t)p * KP + 2 * t) = *reinterpret_cast<const ll2*>(vs + 2 * t);
        }
    }
    if (wave == 0) {
        uint64_t key = ~0ull;
        for (int col = lane; col < KP; col += 64) {
            const uint64_t k0 = ((uint64_t)vs[col] << 10) | (uint64_t)col;
            key = k0 < key ? k0 : key;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const uint64_t o = __shfl_xor(key, off, 64);
            key = o < key ? o : key;
        }
        if (lane == 0) {
            total[p] = (int64_t)(key >> 10);
            last[p] = (int32_t)(key & 1023u);
        }
    }
}

template <int KP, int W>
hipError_t launch_coop(int32_t B, int32_t N, const int64_t* c, int64_t c_bs, const int64_t* R,
                       int64_t R_bs, uint16_t* arg, int64_t* vfinal, int64_t* total, int32_t* last,
                       hipStream_t stream) {
    hipLaunchKernelGGL((chain_coop_kernel<KP, W>), dim3(B), dim3(W * 64), 0, stream, N, c, c_bs, R, R_bs, arg,
                       vfinal, total, last);
    return hipGetLastError();
}

template <int KP>
hipError_t launch_wave(int32_t B, int32_t N, const int64_t* c, int64_t c_bs, const int64_t* R,
                       int64_t R_bs, uint16_t* arg, int64_t* vfinal, int64_t* total,
                       int32_t* last, hipStream_t stream) {
    const int grid = (B + kWavesPerBlock - 1) / kWavesPerBlock;
    hipLaunchKernelGGL(chain_wave_kernel<KP>, dim3(grid), dim3(kWavesPerBlock * 64), 0, stream, B, N,
                       c, c_bs, R, R_bs, arg, vfinal, total, last);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_chain(int32_t B, int32_t N, int32_t Kp, const int64_t* c, int64_t c_bs,
                        const int64_t* R, int64_t R_bs, uint16_t* arg, int64_t* vfinal,
                        int64_t* total, int32_t* last, hipStream_t stream) {
    if (B == 0) return hipSuccess;
    // One workgroup of W waves per problem wherever the tile is tall enough: W waves reading W
    // consecutive row groups keep the DRAM accesses of a CU contiguous (16 KiB at a time for
    // W = 16), which measures faster than 4096 independent 1 KiB streams even when there are
    // thousands of problems.  Narrow tiles, and wide ones whose partials would not fit LDS at a
    // useful W, run one wave per problem once there are enough problems to fill the chip.
    const bool few = B < 2048;
#define RH_ARGS B, N, c, c_bs, R, R_bs, arg, vfinal, total, last, stream
    switch (Kp) {
        case 16: return launch_wave<16>(RH_ARGS);
        case 32: return few ? launch_coop<32, 4>(RH_ARGS) : launch_wave<32>(RH_ARGS);
        case 64: return few ? launch_coop<64, 8>(RH_ARGS) : launch_wave<64>(RH_ARGS);
        case 128: return launch_coop<128, 16>(RH_ARGS);
        case 256: return launch_coop<256, 16>(RH_ARGS);
        case 512: return few ? launch_coop<512, 8>(RH_ARGS) : launch_wave<512>(RH_ARGS);
        case 1024: return few ? launch_coop<1024, 4>(RH_ARGS) : launch_wave<1024>(RH_ARGS);
        default: return hipErrorInvalidValue;
    }
#undef RH_ARGS
}

}  // namespace rh

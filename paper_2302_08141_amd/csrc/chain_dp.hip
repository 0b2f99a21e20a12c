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
    switch (Kp) {
#define RH_CASE(KP) \
    case KP:        \
        return launch_wave<KP>(B, N, c, c_bs, R, R_bs, arg, vfinal, total, last, stream);
        RH_CASE(16)
        RH_CASE(32)
        RH_CASE(64)
        RH_CASE(128)
        RH_CASE(256)
        RH_CASE(512)
        RH_CASE(1024)
#undef RH_CASE
        default:
            return hipErrorInvalidValue;
    }
}

}  // namespace rh

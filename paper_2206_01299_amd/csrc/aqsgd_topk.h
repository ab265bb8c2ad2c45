// Sparsified backward message ("bw8[0.2]", Appendix H.6 of the paper): per group
// of G gradient entries only the `keep` largest magnitudes travel, as 8-bit
// levels of Q with the group's max-abs scale, plus one bit per entry that says
// which ones.  Equal magnitudes: the lower index survives first.
//
// One wave owns a group (G <= 2048).  The threshold is the keep-th largest
// magnitude, found on the magnitudes' bit patterns (which order like unsigned
// integers) by building it bit by bit from the top: a bit stays set if at least
// `keep` entries are >= the candidate.  Every count is a wave ballot and a scalar
// population count, so a pass costs one vector compare per entry held by a lane.
// Positions in the compacted byte string come from the same ballots through
// mbcnt (set bits in lower lanes).  The kept bytes are gathered in LDS and leave
// as full-width stores; the receiver stages them the same way.
#pragma once

#include "aqsgd_kernels.h"

namespace aqsgd {

struct TopkArgs {
    const void* grad;          // sender: [n]
    void* out;                 // receiver: [n]
    uint8_t* bitmap;           // [n / 8], entry j at bit j % 8 of byte j / 8
    uint8_t* codes;            // [n_groups * keep], a group's levels in ascending entry order
    float* scales;             // [n_groups]
    int64_t n_groups;
    int32_t group;
    int32_t cpg;               // chunks of eight entries per group
    int32_t keep;
    int32_t stochastic;
    uint64_t seed;
};

constexpr int kTopkMaxGroup = 2048;
constexpr int kTopkBits = 8;

// Number of magnitude bits that can differ between two entries of the dtype.
template <int DT> struct KeyBits { static constexpr int value = 15; };
template <> struct KeyBits<AQSGD_F32> { static constexpr int value = 31; };

// Magnitude bit patterns of a chunk, straight from storage: the 15 low bits of a
// half or bfloat16, the 31 low bits of a binary32.
template <int DT>
__device__ __forceinline__ void magnitude_keys(const Raw<DT>& r, uint32_t (&u)[kChunk]) {
    if constexpr (DT == AQSGD_F32) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            u[i] = __float_as_uint(r.lo[i]) & 0x7fffffffu;
            u[4 + i] = __float_as_uint(r.hi[i]) & 0x7fffffffu;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            u[2 * i] = r.v[i] & 0x7fffu;
            u[2 * i + 1] = (r.v[i] >> 16) & 0x7fffu;
        }
    }
}

__device__ __forceinline__ int wave_count(uint64_t ballot) { return __builtin_popcountll(ballot); }

// acc + number of set ballot bits that belong to lower lanes
__device__ __forceinline__ uint32_t lower_lanes(uint64_t ballot, uint32_t acc) {
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(ballot >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(ballot), acc));
}

// LDS traffic of one wave: later reads must see earlier writes of other lanes.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int DT, int CPL>
__device__ __forceinline__ void topk_quant_group(const TopkArgs& a, int64_t g, const uint32_t (&cc)[CPL],
                                                 const bool (&valid)[CPL], int lane, uint8_t* stage) {
    constexpr int kEB = ElemBytes<DT>::value;
    constexpr int kChunkBytes = kChunk * kEB;
    const int64_t e0 = g * a.group;                      // first entry of the group in the call tensor
    const char* src = static_cast<const char*>(a.grad) + e0 * kEB;

    Raw<DT> raw[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) raw[k] = load_raw_at<DT>(src + cc[k] * kChunkBytes);
    __builtin_amdgcn_sched_barrier(0);

    float f[CPL][kChunk];
    uint32_t u[CPL][kChunk];
    float mx = 0.0f;
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        unpack_raw<DT>(raw[k], f[k]);
        magnitude_keys<DT>(raw[k], u[k]);
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
            mx = __builtin_fmaxf(mx, __builtin_fabsf(f[k][e]));      // a clamped lane repeats a real chunk
            if (!valid[k]) u[k][e] = 0;                               // ... and must not be counted
        }
    }
    mx = team_max<kWave>(mx);
    const GroupScale sc = make_scale<kTopkBits>(mx);

    // ---- threshold: the keep-th largest key -----------------------------------------
    uint32_t threshold = 0;
    for (int b = KeyBits<DT>::value - 1; b >= 0; --b) {
        const uint32_t candidate = threshold | (1u << b);
        int at_least = 0;
#pragma unroll
        for (int k = 0; k < CPL; ++k)
#pragma unroll
            for (int e = 0; e < kChunk; ++e) at_least += wave_count(__ballot(u[k][e] >= candidate));
        if (at_least >= a.keep) threshold = candidate;
    }
    int above = 0;
#pragma unroll
    for (int k = 0; k < CPL; ++k)
#pragma unroll
        for (int e = 0; e < kChunk; ++e) above += wave_count(__ballot(u[k][e] > threshold));
    int ties_left = a.keep - above;                      // entries equal to the threshold still to keep

    // ---- keep flags, positions, levels -------------------------------------------------
    int kept_before = 0;                                 // kept entries of earlier chunk rows
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        uint32_t gtb = 0, eqb = 0, ties_below = 0;
        int ties_here = 0;
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
            const bool gt = u[k][e] > threshold;
            const bool eq = valid[k] && u[k][e] == threshold;
            gtb |= static_cast<uint32_t>(gt) << e;
            eqb |= static_cast<uint32_t>(eq) << e;
            const uint64_t m = __ballot(eq);
            ties_below = lower_lanes(m, ties_below);
            ties_here += wave_count(m);
        }
        const int allowed = ties_left - static_cast<int>(ties_below);   // ties this lane may still keep
        uint32_t keepb = gtb;
        int seen = 0;
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
            const bool eq = (eqb >> e) & 1u;
            if (eq && seen < allowed) keepb |= 1u << e;
            seen += eq;
        }
        ties_left = max(ties_left - ties_here, 0);

        uint32_t kept_below = 0;
        int kept_here = 0;
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
            const uint64_t m = __ballot((keepb >> e) & 1u);
            kept_below = lower_lanes(m, kept_below);
            kept_here += wave_count(m);
        }
        uint32_t pos = static_cast<uint32_t>(kept_before) + kept_below;

        float r[kChunk];
        if (a.stochastic) {
            chunk_uniforms(a.seed, static_cast<uint64_t>(e0) + static_cast<uint64_t>(cc[k]) * kChunk, r);
        } else {
#pragma unroll
            for (int e = 0; e < kChunk; ++e) r[e] = 0.5f;
        }
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
            const float q = level_of<kTopkBits, AQSGD_ROUND_STOCHASTIC>(f[k][e], sc, r[e]);
            if ((keepb >> e) & 1u) {
                stage[pos] = static_cast<uint8_t>(static_cast<uint32_t>(q));
                ++pos;
            }
        }
        if (valid[k]) a.bitmap[e0 / kChunk + cc[k]] = static_cast<uint8_t>(keepb);
        kept_before += kept_here;
    }

    // ---- the group's bytes leave LDS ------------------------------------------------------
    wave_lds_sync();
    uint8_t* dst = a.codes + g * a.keep;
    if (a.keep % 16 == 0) {
        for (int i = lane; i < a.keep / 16; i += kWave)
            *reinterpret_cast<u32x4_t*>(dst + 16 * i) = *reinterpret_cast<const u32x4_t*>(stage + 16 * i);
    } else {
        for (int i = lane; i < a.keep; i += kWave) dst[i] = stage[i];
    }
    if (lane == 0) a.scales[g] = sc.s_tx;
    wave_lds_sync();                                     // the next group reuses the staging bytes
}

template <int DT, int CPL>
__device__ __forceinline__ void topk_dequant_group(const TopkArgs& a, int64_t g, const uint32_t (&cc)[CPL],
                                                   const bool (&valid)[CPL], int lane, uint8_t* stage) {
    constexpr int kEB = ElemBytes<DT>::value;
    constexpr int kChunkBytes = kChunk * kEB;
    const int64_t e0 = g * a.group;
    char* dst = static_cast<char*>(a.out) + e0 * kEB;

    uint32_t bm[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) bm[k] = a.bitmap[e0 / kChunk + cc[k]];
    const float s_tx = a.scales[g];
    const uint8_t* src = a.codes + g * a.keep;
    if (a.keep % 16 == 0) {
        for (int i = lane; i < a.keep / 16; i += kWave)
            *reinterpret_cast<u32x4_t*>(stage + 16 * i) = *reinterpret_cast<const u32x4_t*>(src + 16 * i);
    } else {
        for (int i = lane; i < a.keep; i += kWave) stage[i] = src[i];
    }
    wave_lds_sync();

    const GroupScale sc = scale_from_wire<kTopkBits>(s_tx);
    int kept_before = 0;
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        const uint32_t mine = valid[k] ? bm[k] : 0u;
        uint32_t kept_below = 0;
        int kept_here = 0;
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
            const uint64_t m = __ballot((mine >> e) & 1u);
            kept_below = lower_lanes(m, kept_below);
            kept_here += wave_count(m);
        }
        uint32_t pos = static_cast<uint32_t>(kept_before) + kept_below;
        float x[kChunk];
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
            x[e] = 0.0f;
            if ((mine >> e) & 1u) {
                x[e] = value_of(static_cast<float>(stage[pos]), sc);   // pos < G <= the staging bytes
                ++pos;
            }
        }
        if (valid[k]) store_raw_at<DT>(dst + cc[k] * kChunkBytes, pack_raw<DT>(x));
        kept_before += kept_here;
    }
    wave_lds_sync();
}

template <int DT, int CPL, bool SENDER>
__global__ __launch_bounds__(kBlock)
void topk_kernel(const TopkArgs a) {
    constexpr int kWaves = kBlock / kWave;
    __shared__ __align__(16) uint8_t stage_all[kWaves][kTopkMaxGroup];

    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    uint32_t cc[CPL];
    bool valid[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        const int c = k * kWave + lane;
        valid[k] = c < a.cpg;
        cc[k] = static_cast<uint32_t>(min(c, a.cpg - 1));
    }
    for (int64_t g = static_cast<int64_t>(blockIdx.x) * kWaves + wave; g < a.n_groups;
         g += static_cast<int64_t>(gridDim.x) * kWaves) {
        if constexpr (SENDER) topk_quant_group<DT, CPL>(a, g, cc, valid, lane, stage_all[wave]);
        else topk_dequant_group<DT, CPL>(a, g, cc, valid, lane, stage_all[wave]);
    }
}

// chunks per lane: 1, 2 or 4 (groups of up to 512, 1024, 2048 entries)
hipError_t launch_topk(int dtype, int cpl, bool sender, unsigned blocks, const TopkArgs& a, hipStream_t stream);

}  // namespace aqsgd

// Kernels of the AQ-SGD boundary codec (gfx950).  Included once per storage
// dtype by aqsgd_f32.hip / aqsgd_f16.hip / aqsgd_bf16.hip, which instantiate the
// launch tables for their dtype; aqsgd_api.hip holds the C ABI and the dispatch.
//
// Quantising side (encode, grad_quant): a TEAM of lanes owns one group.  Lane l
// of the team takes chunks l, l+TEAM, ... of the group (CPL of them), so every
// load instruction of a wavefront reads consecutive 16-byte pieces.  All loads
// are issued before anything is consumed; the deltas stay in registers while
// the team reduces max|delta|, so act and m are read from HBM exactly once and
// m and the codes are written exactly once.
//   TEAM <= 64: the team is a slice of one wavefront, reduced with DPP /
//               ds_bpermute; 256/TEAM teams per 256-thread workgroup.
//   TEAM  > 64: the team is a whole workgroup; wave maxima meet in LDS.
// Dequantising side (decode, grad_dequant): no reduction, one chunk per lane
// and step, flat over the sample.
// gridDim.y walks the samples of the call, gridDim.x the groups (or chunks)
// inside a sample, so no index needs a 64-bit division on the device.
#pragma once

#include "aqsgd_device.h"

namespace aqsgd {

struct QuantArgs {
    const void* src;           // act or grad  [batch, n_per]
    const int64_t* ids;        // sample ids, or nullptr (src rows are not gathered)
    void* m_buf;               // previous messages, or nullptr (direct quantisation)
    uint8_t* codes;
    float* scales;
    int64_t n_per;             // elements per sample
    int64_t gps;               // groups per sample
    int32_t batch;
    int32_t group;             // G
    int32_t cpg;               // chunks per group (G / 8), team kernels only
    uint64_t seed;
};

struct DequantArgs {
    const uint8_t* codes;
    const float* scales;
    const int64_t* ids;        // or nullptr
    void* m_buf;               // or nullptr: out = Q^-1 alone
    void* out;
    int64_t n_per;
    int64_t gps;
    int64_t cps;               // chunks per sample
    int32_t batch;
    int32_t group;
    int32_t cpg;
};

constexpr int kBlock = 256;

// ---------------------------------------------------------------------------
// encode / grad_quant, team kernel
// ---------------------------------------------------------------------------
template <int DT, int BITS, int ROUND, int TEAM, int CPL>
__global__ __launch_bounds__((TEAM > kBlock ? TEAM : kBlock))
void quant_team_kernel(const QuantArgs a) {
    constexpr bool kMultiWave = TEAM > kWave;
    constexpr int kThreads = TEAM > kBlock ? TEAM : kBlock;
    constexpr int kTeamsPerBlock = kMultiWave ? 1 : kThreads / TEAM;
    static_assert(!kMultiWave || TEAM == kThreads, "a multi-wave team is the whole workgroup");

    const int lane_in_team = threadIdx.x % TEAM;
    const int team = threadIdx.x / TEAM;
    const bool has_buf = a.m_buf != nullptr;
    [[maybe_unused]] __shared__ float wave_max[kThreads / kWave];

    for (int i = blockIdx.y; i < a.batch; i += gridDim.y) {
        const int64_t row = a.ids ? a.ids[i] : static_cast<int64_t>(i);
        const int64_t src0 = static_cast<int64_t>(i) * a.n_per;      // flat offset of sample i
        const int64_t m0 = row * a.n_per;

        for (int64_t gbase = static_cast<int64_t>(blockIdx.x) * kTeamsPerBlock; gbase < a.gps;
             gbase += static_cast<int64_t>(gridDim.x) * kTeamsPerBlock) {
            const int64_t gs = gbase + team;                 // group within the sample
            const bool group_ok = gs < a.gps;
            const int64_t goff = gs * a.group;               // element offset within the sample

            // ---- issue every load of the group -------------------------------
            Raw<DT> ra[CPL], rm[CPL];
            bool ok[CPL];
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
                const int c = k * TEAM + lane_in_team;
                ok[k] = group_ok && c < a.cpg;
                ra[k] = zero_raw<DT>();
                rm[k] = zero_raw<DT>();
                if (ok[k]) {
                    ra[k] = load_raw<DT>(a.src, src0 + goff + static_cast<int64_t>(c) * kChunk);
                    if (has_buf) rm[k] = load_raw<DT>(a.m_buf, m0 + goff + static_cast<int64_t>(c) * kChunk);
                }
            }

            // ---- delta and the group's max-abs -----------------------------------
            float d[CPL][kChunk], m_old[CPL][kChunk];
            float mx = 0.0f;
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
                float av[kChunk];
                unpack_raw<DT>(ra[k], av);
                unpack_raw<DT>(rm[k], m_old[k]);
#pragma unroll
                for (int e = 0; e < kChunk; ++e) {
                    d[k][e] = av[e] - m_old[k][e];
                    mx = __builtin_fmaxf(mx, __builtin_fabsf(d[k][e]));
                }
            }
            mx = team_max<(TEAM < kWave ? TEAM : kWave)>(mx);
            if constexpr (kMultiWave) {
                __syncthreads();                                 // previous round's readers are done
                if (threadIdx.x % kWave == 0) wave_max[threadIdx.x / kWave] = mx;
                __syncthreads();
#pragma unroll
                for (int w = 0; w < kThreads / kWave; ++w) mx = __builtin_fmaxf(mx, wave_max[w]);
            }
            const GroupScale sc = make_scale<BITS>(mx);
            const bool live = sc.s_tx != 0.0f;

            // ---- quantise, pack, update m ----------------------------------------
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
                const int c = k * TEAM + lane_in_team;
                const int64_t e0 = goff + static_cast<int64_t>(c) * kChunk;   // within the sample
                float r[kChunk];
                if constexpr (ROUND == AQSGD_ROUND_STOCHASTIC) {
                    chunk_uniforms(a.seed, static_cast<uint64_t>(src0 + e0), r);
                } else {
#pragma unroll
                    for (int e = 0; e < kChunk; ++e) r[e] = 0.5f;
                }
                int q[kChunk];
                float m_new[kChunk];
#pragma unroll
                for (int e = 0; e < kChunk; ++e) {
                    const int kq = level_of<BITS>(d[k][e], sc.inv, r[e]);
                    q[e] = live ? kq : 0;
                    const float dh = live ? value_of<BITS>(kq, sc.step) : 0.0f;
                    m_new[e] = m_old[k][e] + dh;
                }
                if (ok[k]) {
                    store_codes<BITS>(a.codes, (src0 + e0) / kChunk, pack_levels<BITS>(q));
                    if (has_buf) store_raw<DT>(a.m_buf, m0 + e0, pack_raw<DT>(m_new));
                }
            }
            if (group_ok && lane_in_team == 0)
                a.scales[static_cast<int64_t>(i) * a.gps + gs] = sc.s_tx;
        }
    }
}

// ---------------------------------------------------------------------------
// decode / grad_dequant, flat chunk kernel: UNROLL chunks per lane and step.
// ---------------------------------------------------------------------------
template <int DT, int BITS, int UNROLL>
__global__ __launch_bounds__(kBlock)
void dequant_flat_kernel(const DequantArgs a) {
    const bool has_buf = a.m_buf != nullptr;
    const uint32_t cpg = static_cast<uint32_t>(a.cpg);
    for (int i = blockIdx.y; i < a.batch; i += gridDim.y) {
        const int64_t row = a.ids ? a.ids[i] : static_cast<int64_t>(i);
        const int64_t out0 = static_cast<int64_t>(i) * a.n_per;
        const int64_t m0 = row * a.n_per;
        const float* scales_i = a.scales + static_cast<int64_t>(i) * a.gps;

        for (int64_t cbase = static_cast<int64_t>(blockIdx.x) * (kBlock * UNROLL); cbase < a.cps;
             cbase += static_cast<int64_t>(gridDim.x) * (kBlock * UNROLL)) {
            uint64_t w[UNROLL];
            float scale[UNROLL];
            Raw<DT> rm[UNROLL];
            bool ok[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int64_t cs = cbase + u * kBlock + threadIdx.x;       // chunk within the sample
                ok[u] = cs < a.cps;
                w[u] = 0; scale[u] = 0.0f; rm[u] = zero_raw<DT>();
                if (ok[u]) {
                    w[u] = load_codes<BITS>(a.codes, out0 / kChunk + cs);
                    scale[u] = scales_i[static_cast<uint32_t>(cs) / cpg];
                    if (has_buf) rm[u] = load_raw<DT>(a.m_buf, m0 + cs * kChunk);
                }
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int64_t cs = cbase + u * kBlock + threadIdx.x;
                const bool live = scale[u] != 0.0f;
                const float step = (live ? scale[u] : 1.0f) / Levels<BITS>::half;
                int q[kChunk];
                unpack_levels<BITS>(w[u], q);
                float m_old[kChunk], m_new[kChunk];
                unpack_raw<DT>(rm[u], m_old);
#pragma unroll
                for (int e = 0; e < kChunk; ++e) {
                    const float dh = live ? value_of<BITS>(q[e], step) : 0.0f;
                    m_new[e] = has_buf ? m_old[e] + dh : dh;
                }
                if (ok[u]) {
                    const Raw<DT> packed = pack_raw<DT>(m_new);
                    if (has_buf) store_raw<DT>(a.m_buf, m0 + cs * kChunk, packed);
                    store_raw<DT>(a.out, out0 + cs * kChunk, packed);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Any-shape fallbacks: one thread per group, scalar accesses.  Used when the
// group size is not a multiple of 8 or too large for a workgroup's registers;
// correct for every shape the ABI admits, not tuned.
// ---------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(kBlock)
void quant_anyshape_kernel(const QuantArgs a, const int bits, const int rounding) {
    const int L = (1 << bits) - 1;
    const float hL = static_cast<float>(L) / 2.0f;
    const bool has_buf = a.m_buf != nullptr;
    for (int i = blockIdx.y; i < a.batch; i += gridDim.y) {
        const int64_t row = a.ids ? a.ids[i] : static_cast<int64_t>(i);
        const int64_t src0 = static_cast<int64_t>(i) * a.n_per;
        const int64_t m0 = row * a.n_per;
        for (int64_t gs = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; gs < a.gps;
             gs += static_cast<int64_t>(gridDim.x) * kBlock) {
            const int64_t goff = gs * a.group;
            float mx = 0.0f;
            for (int e = 0; e < a.group; ++e) {
                const float m_old = has_buf ? load_elem<DT>(a.m_buf, m0 + goff + e) : 0.0f;
                const float d = load_elem<DT>(a.src, src0 + goff + e) - m_old;
                mx = __builtin_fmaxf(mx, __builtin_fabsf(d));
            }
            const bool live = !(mx < 0x1p-120f);
            const float s_tx = live ? mx : 0.0f;
            const float denom = live ? mx : 1.0f;
            const float inv = hL / denom;
            const float step = denom / hL;
            uint8_t* out = a.codes + (src0 + goff) * bits / 8;   // whole bytes: (G*bits) % 8 == 0
            uint32_t acc = 0;
            int filled = 0;
            for (int e = 0; e < a.group; ++e) {
                const float m_old = has_buf ? load_elem<DT>(a.m_buf, m0 + goff + e) : 0.0f;
                const float d = load_elem<DT>(a.src, src0 + goff + e) - m_old;
                float r = 0.5f;
                if (rounding == AQSGD_ROUND_STOCHASTIC) {
                    const uint64_t j = static_cast<uint64_t>(src0 + goff + e);
                    uint32_t w[4];
                    philox4x32_10(static_cast<uint32_t>(j >> 2), static_cast<uint32_t>(j >> 34),
                                  static_cast<uint32_t>(a.seed), static_cast<uint32_t>(a.seed >> 32), w);
                    r = uniform_from_word(w[j & 3]);
                }
                float t = d * inv;
                t = t + hL;
                const float y = t + r;
                int k = static_cast<int>(__builtin_floorf(y));
                k = min(max(k, 0), L);
                if (!live) k = 0;
                const float dh = live ? (static_cast<float>(k) - hL) * step : 0.0f;
                if (has_buf) store_elem<DT>(a.m_buf, m0 + goff + e, m_old + dh);
                acc |= static_cast<uint32_t>(k) << filled;
                filled += bits;
                while (filled >= 8) {
                    *out++ = static_cast<uint8_t>(acc);
                    acc >>= 8;
                    filled -= 8;
                }
            }
            a.scales[static_cast<int64_t>(i) * a.gps + gs] = s_tx;
        }
    }
}

template <int DT>
__global__ __launch_bounds__(kBlock)
void dequant_anyshape_kernel(const DequantArgs a, const int bits) {
    const int L = (1 << bits) - 1;
    const float hL = static_cast<float>(L) / 2.0f;
    const bool has_buf = a.m_buf != nullptr;
    for (int i = blockIdx.y; i < a.batch; i += gridDim.y) {
        const int64_t row = a.ids ? a.ids[i] : static_cast<int64_t>(i);
        const int64_t out0 = static_cast<int64_t>(i) * a.n_per;
        const int64_t m0 = row * a.n_per;
        for (int64_t gs = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; gs < a.gps;
             gs += static_cast<int64_t>(gridDim.x) * kBlock) {
            const int64_t goff = gs * a.group;
            const float scale = a.scales[static_cast<int64_t>(i) * a.gps + gs];
            const bool live = scale != 0.0f;
            const float step = (live ? scale : 1.0f) / hL;
            const uint8_t* in = a.codes + (out0 + goff) * bits / 8;
            uint32_t acc = 0;
            int have = 0;
            for (int e = 0; e < a.group; ++e) {
                while (have < bits) {
                    acc |= static_cast<uint32_t>(*in++) << have;
                    have += 8;
                }
                const int k = static_cast<int>(acc & static_cast<uint32_t>(L));
                acc >>= bits;
                have -= bits;
                const float dh = live ? (static_cast<float>(k) - hL) * step : 0.0f;
                float v = dh;
                if (has_buf) {
                    v = load_elem<DT>(a.m_buf, m0 + goff + e) + dh;
                    store_elem<DT>(a.m_buf, m0 + goff + e, v);
                }
                store_elem<DT>(a.out, out0 + goff + e, v);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Launch tables, one set per dtype translation unit.
// ---------------------------------------------------------------------------
struct LaunchGeom { unsigned grid_x, grid_y; };

// Team shapes the dispatcher may pick; index into the table below.
enum TeamShape {
    kTeam8x1 = 0, kTeam16x1, kTeam32x1, kTeam64x1, kTeam64x2, kTeam64x3, kTeam64x4,
    kTeam256x2, kTeam256x4, kTeam1024x2, kTeam1024x4, kNumTeamShapes
};

hipError_t launch_quant_team(int dtype, int bits, int rounding, int shape, LaunchGeom g,
                             const QuantArgs& a, hipStream_t stream);
hipError_t launch_dequant_flat(int dtype, int bits, int unroll, LaunchGeom g, const DequantArgs& a,
                               hipStream_t stream);
hipError_t launch_quant_anyshape(int dtype, int bits, int rounding, LaunchGeom g, const QuantArgs& a,
                                 hipStream_t stream);
hipError_t launch_dequant_anyshape(int dtype, int bits, LaunchGeom g, const DequantArgs& a,
                                   hipStream_t stream);

// Per-dtype pieces (defined by AQSGD_INSTANTIATE_DTYPE in the dtype's .hip file).
template <int DT> hipError_t launch_quant_team_dt(int bits, int rounding, int shape, LaunchGeom g,
                                                  const QuantArgs& a, hipStream_t stream);
template <int DT> hipError_t launch_dequant_flat_dt(int bits, int unroll, LaunchGeom g,
                                                    const DequantArgs& a, hipStream_t stream);
template <int DT> hipError_t launch_quant_anyshape_dt(int bits, int rounding, LaunchGeom g,
                                                      const QuantArgs& a, hipStream_t stream);
template <int DT> hipError_t launch_dequant_anyshape_dt(int bits, LaunchGeom g, const DequantArgs& a,
                                                        hipStream_t stream);

}  // namespace aqsgd

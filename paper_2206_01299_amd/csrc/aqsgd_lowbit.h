// Codec kernels for previous messages kept at low precision ("m z", Appendix
// H.5 of the paper): m(xi) lives in HBM as z-bit levels plus one binary32 scale
// per group instead of the activation dtype, which cuts both the footprint and
// the dominant traffic of the boundary (config 2 at z = 8: 4.5 instead of 6.5
// bytes per element and call).
//
// Both machines work from the stored value m^ = Q_z^-1(stored):
//     sender:    Delta m = Q_b(a - m^)           -> codes, scales on the wire
//     both:      v = m^ + Delta m  (binary32);   store Q_z(v), nearest rounding
//     receiver:  out = dtype(v)
// One team of lanes owns a group, as in the plain quantising kernel, and runs two
// max reductions: over |a - m^| for the wire scale and over |v| for the storage
// scale.  Everything between the loads and the stores stays in registers.
#pragma once

#include "aqsgd_kernels.h"

namespace aqsgd {

struct LowbitArgs {
    const void* act;           // sender: [batch, n_per]; receiver: unused
    void* out;                 // receiver: [batch, n_per]; sender: unused
    const int64_t* ids;
    uint8_t* m_codes;          // [n_samples, n_per * MBITS / 8]
    float* m_scales;           // [n_samples, gps]
    uint8_t* codes;            // the message: written by the sender, read by the receiver
    float* scales;
    int64_t n_per;
    int64_t gps;
    int32_t batch;
    int32_t group;
    int32_t cpg;
    int32_t stochastic;        // sender: rounding mode of the message
    uint64_t seed;
};

template <int TEAM, int KIND>
__device__ __forceinline__ float team_max_all(float mx, float* wave_max) {
    constexpr bool kMultiWave = TEAM > kWave;
    constexpr int kThreads = TEAM > kWave ? TEAM : kBlock;
    mx = team_max<(TEAM < kWave ? TEAM : kWave)>(mx);
    if constexpr (kMultiWave) {
        float* slot = wave_max + KIND * (kThreads / kWave);      // one array per reduction
        __syncthreads();
        if (threadIdx.x % kWave == 0) slot[threadIdx.x / kWave] = mx;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < kThreads / kWave; ++w) mx = __builtin_fmaxf(mx, slot[w]);
    }
    return mx;
}

// Tells the compiler nothing about a packed word's value from here on, so that what is
// derived from it afterwards is computed afresh instead of being kept in registers.
__device__ __forceinline__ void forget(uint64_t& w) {
    uint32_t lo = static_cast<uint32_t>(w), hi = static_cast<uint32_t>(w >> 32);
    asm volatile("" : "+v"(lo), "+v"(hi));
    w = (static_cast<uint64_t>(hi) << 32) | lo;
}
template <int DT>
__device__ __forceinline__ void forget(Raw<DT>& r) {
    if constexpr (DT == AQSGD_F32) {
        asm volatile("" : "+v"(r.lo), "+v"(r.hi));
    } else {
        asm volatile("" : "+v"(r.v));
    }
}

// m^ of one chunk from its stored levels.
template <int MBITS>
__device__ __forceinline__ void stored_values(uint64_t mw, const GroupScale& msc, float (&m)[kChunk]) {
    float q[kChunk];
    unpack_levels<MBITS>(mw, q);
#pragma unroll
    for (int e = 0; e < kChunk; ++e) m[e] = value_of(q[e], msc);
}

// ---------------------------------------------------------------------------
// A last round of at most eight chunks taken as one element per lane.  A 1600-element
// group is three rounds of one chunk per lane and 64 more elements; with whole chunks
// those 64 cost every lane a fourth round of eight elements' arithmetic, and this kernel
// is bound by arithmetic.  b-bit levels of eight neighbouring lanes make one chunk's b
// bytes: they meet in the first of the eight lanes through three row shifts.
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_from_higher_lane(uint32_t v) {
    // lane l reads lane l + n of its row of 16 (row_shl:n); lanes without a source read zero
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xf, 0xf, true));
}

constexpr bool tail_bits_ok(int b) { return b == 2 || b == 4 || b == 8; }

// Every lane calls it (the shifts read the neighbours); `level` must be 0 in lanes without
// an element.  base: the tail's first byte; the tail has tail_entries (a multiple of 8) elements.
template <int B>
__device__ __forceinline__ void store_tail_levels(uint8_t* base, uint32_t level, int lane, int tail_entries) {
    static_assert(tail_bits_ok(B), "single-element tails: 2, 4 or 8 bits");
    if constexpr (B == 8) {
        if (lane < tail_entries) base[lane] = static_cast<uint8_t>(level);
    } else {
        uint32_t x = level;
        x |= dpp_from_higher_lane<0x101>(x) << B;
        x |= dpp_from_higher_lane<0x102>(x) << (2 * B);
        x |= dpp_from_higher_lane<0x104>(x) << (4 * B);
        if (lane % 8 == 0 && lane < tail_entries) {
            if constexpr (B == 4) *reinterpret_cast<uint32_t*>(base + lane / 8 * 4) = x;
            else *reinterpret_cast<uint16_t*>(base + lane / 8 * 2) = static_cast<uint16_t>(x);
        }
    }
}

// The level of tail element l (l inside the tail).
template <int B>
__device__ __forceinline__ uint32_t load_tail_level(const uint8_t* base, int l) {
    static_assert(tail_bits_ok(B), "single-element tails: 2, 4 or 8 bits");
    if constexpr (B == 8) return base[l];
    else if constexpr (B == 4) return (static_cast<uint32_t>(base[l / 2]) >> (4 * (l & 1))) & 15u;
    else return (static_cast<uint32_t>(base[l / 4]) >> (2 * (l & 3))) & 3u;
}

// One group.  The kernel is bound by vector arithmetic, not by memory (two quantisers and
// a dequantiser per element), and registers decide how many waves a SIMD holds, so what is
// live across the two reductions is chosen by what is cheapest to form again.  Sender with
// 16-bit activations: m^ stays in registers, the change d = a - m^ is formed for the first
// reduction and again afterwards (one widening subtract per element from the activation as
// loaded), and v = m^ + Delta m takes over m^'s registers.  Sender with binary32
// activations: d stays across the first reduction and m^ is formed again from the stored
// levels when v is built.  Keeping d, m^ and v live all at once would cost a wave of
// occupancy per SIMD and with it the chance to hold a whole launch on the chip at a time.
// TAIL (one-wave teams, 16-bit activations, nearest rounding): the group is CPL whole rounds
// and `tail_entries` more elements, one per lane (see above).
template <int DT, int BITS, int MBITS, int ROUND, int TEAM, int CPL, bool SENDER, bool TAIL = false>
__device__ __forceinline__ void lowbit_team_group(const LowbitArgs& a, const char* act_s, char* out_s,
                                                  uint8_t* mcodes_s, float* mscales_s, uint8_t* codes_s,
                                                  float* scales_s, int64_t src0, int64_t g,
                                                  const uint32_t (&cc)[CPL], int lane_in_team,
                                                  float* wave_max, int tail_entries = 0) {
    static_assert(!TAIL || (TEAM == kWave && ElemBytes<DT>::value == 2 && ROUND == AQSGD_ROUND_NEAREST),
                  "single-element tails: one-wave teams, 16-bit activations, nearest rounding");
    constexpr int kEB = ElemBytes<DT>::value;
    constexpr int kChunkBytes = kChunk * kEB;
    const int64_t goff = g * a.group;                    // element offset within the sample
    const int64_t gchunk = goff / kChunk;
    // the group's own pointers (uniform over the team) + a lane's 32-bit byte offsets
    uint8_t* const m_group = mcodes_s + gchunk * MBITS;
    uint8_t* const c_group = codes_s + gchunk * BITS;

    // ---- issue every load of the group ------------------------------------------
    uint64_t mw[CPL], cw[CPL];
    Raw<DT> ra[CPL];
    const float m_scale = mscales_s[g];
    float wire_scale = 0.0f;
    if constexpr (!SENDER) wire_scale = scales_s[g];
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        mw[k] = load_codes_at<MBITS>(m_group + cc[k] * static_cast<uint32_t>(MBITS));
        if constexpr (SENDER) ra[k] = load_raw_at<DT>(act_s + goff * kEB + cc[k] * kChunkBytes);
        else cw[k] = load_codes_at<BITS>(c_group + cc[k] * static_cast<uint32_t>(BITS));
    }
    // the tail: element CPL * 64 * 8 + lane of the group (a lane past the end repeats the last one)
    [[maybe_unused]] const bool tail_valid = TAIL && lane_in_team < tail_entries;
    [[maybe_unused]] const int tail_l = min(lane_in_team, tail_entries - 1);
    [[maybe_unused]] const int64_t tail_e = goff + CPL * kWave * kChunk + tail_l;
    [[maybe_unused]] uint8_t* const m_tail = m_group + CPL * kWave * MBITS;
    [[maybe_unused]] uint8_t* const c_tail = c_group + CPL * kWave * BITS;
    [[maybe_unused]] uint32_t tail_m = 0, tail_c = 0;
    [[maybe_unused]] float tail_a = 0.0f, tail_v = 0.0f;
    if constexpr (TAIL) {
        tail_m = load_tail_level<MBITS>(m_tail, tail_l);
        if constexpr (SENDER) tail_a = load_elem<DT>(act_s, tail_e);
        else tail_c = load_tail_level<BITS>(c_tail, tail_l);
    }
    __builtin_amdgcn_sched_barrier(0);

    const GroupScale msc = scale_from_wire<MBITS>(m_scale);      // m^ = Q_z^-1(stored)
    if constexpr (TAIL) tail_v = value_of(static_cast<float>(tail_m), msc);     // m^ of the tail element
    float v[CPL][kChunk];                                        // m^ + Delta m
    float mx2 = 0.0f;                                            // max |v| for the storage scale

    if constexpr (SENDER && kEB == 2) {
        // ---- sixteen-bit activations: m^ stays, d = a - m^ is formed twice (one instruction
        // per element from the activation as loaded), v takes m^'s registers ----------------------
        float mx = 0.0f;
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            float d[kChunk];
            stored_values<MBITS>(mw[k], msc, v[k]);      // v holds m^ for now
            delta_from_values<DT>(ra[k], v[k], d);
#pragma unroll
            for (int e = 0; e < kChunk; ++e) mx = __builtin_fmaxf(mx, __builtin_fabsf(d[e]));
        }
        [[maybe_unused]] float tail_d = 0.0f;
        if constexpr (TAIL) {
            tail_d = tail_a - tail_v;
            mx = __builtin_fmaxf(mx, tail_valid ? __builtin_fabsf(tail_d) : 0.0f);
        }
        mx = team_max_all<TEAM, 0>(mx, wave_max);
        const GroupScale sc = make_scale<BITS>(mx);
        if constexpr (TAIL) {
            const float q = level_of<BITS, ROUND>(tail_d, sc, kNearestOffset32);
            tail_v = tail_v + value_of(q, sc);
            mx2 = __builtin_fmaxf(mx2, tail_valid ? __builtin_fabsf(tail_v) : 0.0f);
            store_tail_levels<BITS>(c_tail, tail_valid ? static_cast<uint32_t>(q) : 0u, lane_in_team, tail_entries);
        }
#pragma unroll
        for (int k = 0; k < CPL; ++k) forget(ra[k]);     // d is formed again below, not kept
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            float r[kChunk];
            if constexpr (ROUND == AQSGD_ROUND_STOCHASTIC) {
                chunk_uniforms(a.seed, static_cast<uint64_t>(src0 + goff) + cc[k] * kChunk, r);
            } else {
#pragma unroll
                for (int e = 0; e < kChunk; ++e) r[e] = kNearestOffset32;
            }
            float d[kChunk], q[kChunk];
            delta_from_values<DT>(ra[k], v[k], d);
#pragma unroll
            for (int e = 0; e < kChunk; ++e) {
                q[e] = level_of<BITS, ROUND>(d[e], sc, r[e]);
                v[k][e] = v[k][e] + value_of(q[e], sc);
                mx2 = __builtin_fmaxf(mx2, __builtin_fabsf(v[k][e]));
            }
            store_codes_at<BITS>(c_group + cc[k] * static_cast<uint32_t>(BITS), pack_levels<BITS>(q));
        }
        if (lane_in_team == 0) scales_s[g] = sc.s_tx;
    } else if constexpr (SENDER) {
        // ---- d = a - m^ and the wire scale ------------------------------------------------
        float d[CPL][kChunk];
        float mx = 0.0f;
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            float m[kChunk], av[kChunk];
            stored_values<MBITS>(mw[k], msc, m);
            unpack_raw<DT>(ra[k], av);
#pragma unroll
            for (int e = 0; e < kChunk; ++e) {
                d[k][e] = av[e] - m[e];
                mx = __builtin_fmaxf(mx, __builtin_fabsf(d[k][e]));
            }
        }
        mx = team_max_all<TEAM, 0>(mx, wave_max);
        const GroupScale sc = make_scale<BITS>(mx);
#pragma unroll
        for (int k = 0; k < CPL; ++k) forget(mw[k]);     // m^ is formed again below, not kept
        // ---- Delta m = Q_b(d): codes out; v = m^ + Delta m ----------------------------------
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            float r[kChunk];
            if constexpr (ROUND == AQSGD_ROUND_STOCHASTIC) {
                chunk_uniforms(a.seed, static_cast<uint64_t>(src0 + goff) + cc[k] * kChunk, r);
            } else {
#pragma unroll
                for (int e = 0; e < kChunk; ++e) r[e] = kNearestOffset32;
            }
            float m[kChunk], q[kChunk];
            stored_values<MBITS>(mw[k], msc, m);
#pragma unroll
            for (int e = 0; e < kChunk; ++e) {
                q[e] = level_of<BITS, ROUND>(d[k][e], sc, r[e]);
                v[k][e] = m[e] + value_of(q[e], sc);
                mx2 = __builtin_fmaxf(mx2, __builtin_fabsf(v[k][e]));
            }
            store_codes_at<BITS>(c_group + cc[k] * static_cast<uint32_t>(BITS), pack_levels<BITS>(q));
        }
        if (lane_in_team == 0) scales_s[g] = sc.s_tx;
    } else {
        const GroupScale wsc = scale_from_wire<BITS>(wire_scale);
        if constexpr (TAIL) {
            tail_v = tail_v + value_of(static_cast<float>(tail_c), wsc);
            mx2 = __builtin_fmaxf(mx2, tail_valid ? __builtin_fabsf(tail_v) : 0.0f);
        }
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            float m[kChunk], q[kChunk];
            stored_values<MBITS>(mw[k], msc, m);
            unpack_levels<BITS>(cw[k], q);
#pragma unroll
            for (int e = 0; e < kChunk; ++e) {
                v[k][e] = m[e] + value_of(q[e], wsc);
                mx2 = __builtin_fmaxf(mx2, __builtin_fabsf(v[k][e]));
            }
            __builtin_amdgcn_sched_barrier(0);           // one chunk's temporaries at a time
        }
    }

    // ---- store Q_z(v); the receiver also hands v on ------------------------------------
    mx2 = team_max_all<TEAM, 1>(mx2, wave_max);
    const GroupScale ssc = make_scale<MBITS>(mx2);
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        float q2[kChunk];
#pragma unroll
        for (int e = 0; e < kChunk; ++e) q2[e] = level_of<MBITS, AQSGD_ROUND_NEAREST>(v[k][e], ssc, kNearestOffset32);
        store_codes_at<MBITS>(m_group + cc[k] * static_cast<uint32_t>(MBITS), pack_levels<MBITS>(q2));
        if constexpr (!SENDER) store_raw_at<DT>(out_s + goff * kEB + cc[k] * kChunkBytes, pack_raw<DT>(v[k]));
    }
    if constexpr (TAIL) {
        const float q2 = level_of<MBITS, AQSGD_ROUND_NEAREST>(tail_v, ssc, kNearestOffset32);
        store_tail_levels<MBITS>(m_tail, tail_valid ? static_cast<uint32_t>(q2) : 0u, lane_in_team, tail_entries);
        if constexpr (!SENDER) {
            if (tail_valid) store_elem<DT>(out_s, tail_e, tail_v);
        }
    }
    if (lane_in_team == 0) mscales_s[g] = ssc.s_tx;
}

// MODE: which side and, for the sender, how the message is rounded.
enum LowbitMode { kLbReceiver = 0, kLbSenderNearest = 1, kLbSenderStochastic = 2 };

// Four waves per SIMD hold a whole GPT2-sized launch (one wave per row) on the chip at
// once; the hint makes the register allocator aim for that.
// TAILK: the launch's groups end in a last round of at most eight chunks, which is taken as one
// element per lane (the host picks this variant; see lowbit_tail_chunks).
template <int DT, int BITS, int MBITS, int TEAM, int CPL, int MODE, bool TAILK = false>
__global__ __launch_bounds__((TEAM > kWave ? TEAM : kBlock)) __attribute__((amdgpu_waves_per_eu(4)))
void lowbit_team_kernel(const LowbitArgs a) {
    constexpr bool SENDER = MODE != kLbReceiver;
    constexpr int ROUND = MODE == kLbSenderStochastic ? AQSGD_ROUND_STOCHASTIC : AQSGD_ROUND_NEAREST;
    constexpr bool kMultiWave = TEAM > kWave;
    constexpr int kThreads = TEAM > kWave ? TEAM : kBlock;
    constexpr int kTeamsPerBlock = kMultiWave ? 1 : kThreads / TEAM;
    constexpr int kEB = ElemBytes<DT>::value;
    [[maybe_unused]] __shared__ float wave_max[2 * (kThreads / kWave)];

    const int lane_in_team = threadIdx.x % TEAM;
    const int team = kMultiWave ? 0
                     : (TEAM == kWave ? __builtin_amdgcn_readfirstlane(threadIdx.x / kWave)
                                      : static_cast<int>(threadIdx.x / TEAM));
    uint32_t cc[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k)
        cc[k] = static_cast<uint32_t>(min(k * TEAM + lane_in_team, a.cpg - 1));

    for (int i = blockIdx.y; i < a.batch; i += gridDim.y) {
        const int64_t row = sample_id(a.ids, i);
        const int64_t src0 = static_cast<int64_t>(i) * a.n_per;
        const char* act_s = SENDER ? static_cast<const char*>(a.act) + src0 * kEB : nullptr;
        char* out_s = SENDER ? nullptr : static_cast<char*>(a.out) + src0 * kEB;
        uint8_t* mcodes_s = a.m_codes + row * (a.n_per / kChunk * MBITS);
        float* mscales_s = a.m_scales + row * a.gps;
        uint8_t* codes_s = a.codes + src0 / kChunk * BITS;
        float* scales_s = a.scales + static_cast<int64_t>(i) * a.gps;

        if constexpr (TAILK) {
            constexpr int kRounds = CPL - 1;
            const int tail_chunks = a.cpg - kRounds * kWave;         // 1..8: checked by the host
            uint32_t rc[kRounds];
#pragma unroll
            for (int k = 0; k < kRounds; ++k) rc[k] = static_cast<uint32_t>(k * kWave + lane_in_team);
            for (int64_t gbase = static_cast<int64_t>(blockIdx.x) * kTeamsPerBlock; gbase < a.gps;
                 gbase += static_cast<int64_t>(gridDim.x) * kTeamsPerBlock) {
                const int64_t g = gbase + team;
                if (g < a.gps)
                    lowbit_team_group<DT, BITS, MBITS, ROUND, TEAM, kRounds, SENDER, true>(
                        a, act_s, out_s, mcodes_s, mscales_s, codes_s, scales_s, src0, g, rc, lane_in_team,
                        wave_max, kChunk * tail_chunks);
            }
            continue;
        }
        for (int64_t gbase = static_cast<int64_t>(blockIdx.x) * kTeamsPerBlock; gbase < a.gps;
             gbase += static_cast<int64_t>(gridDim.x) * kTeamsPerBlock) {
            const int64_t g = gbase + team;
            if (g < a.gps)
                lowbit_team_group<DT, BITS, MBITS, ROUND, TEAM, CPL, SENDER>(a, act_s, out_s, mcodes_s,
                                                                             mscales_s, codes_s, scales_s, src0,
                                                                             g, cc, lane_in_team, wave_max);
        }
    }
}

// Team shapes of the low-precision-storage kernels (more live registers per
// element than the plain codec, so the widest shapes stop at two chunks per lane).
enum LowbitShape {
    kLb8x1 = 0, kLb16x1, kLb32x1, kLb64x1, kLb64x2, kLb64x3, kLb64x4, kLb256x2, kLb256x4, kLb1024x2, kNumLowbitShapes
};
constexpr int kMaxLowbitChunks = 2048;

hipError_t launch_lowbit(int dtype, int bits, int m_bits, int shape, bool sender, LaunchGeom g,
                         const LowbitArgs& a, hipStream_t stream);
template <int DT> hipError_t launch_lowbit_dt(int bits, int m_bits, int shape, bool sender, LaunchGeom g,
                                              const LowbitArgs& a, hipStream_t stream);

// The single-element-tail variant exists for 16-bit activations, wire levels of 2, 4 or 8 bits
// and everything but the stochastic sender; a launch takes it when its groups are cpl - 1 whole
// rounds of a wavefront's chunks plus one to eight more chunks.
template <int DT, int BITS, int MODE>
constexpr bool lowbit_tail_variant() {
    return ElemBytes<DT>::value == 2 && tail_bits_ok(BITS) && MODE != kLbSenderStochastic;
}
inline bool lowbit_tail_chunks(int cpg, int cpl) {
    const int t = cpg - (cpl - 1) * kWave;
    return t >= 1 && t <= 8;
}

// ---- launch table (instantiated per dtype in aqsgd_lowbit_<dtype>.hip) ----------------
template <int DT, int BITS, int MBITS, int MODE>
static hipError_t launch_lb_shape(int shape, LaunchGeom g, const LowbitArgs& a, hipStream_t s) {
    const dim3 grid(g.grid_x, g.grid_y);
    switch (shape) {
    case kLb8x1:    return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 8, 1, MODE>, grid, dim3(kBlock), s, a);
    case kLb16x1:   return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 16, 1, MODE>, grid, dim3(kBlock), s, a);
    case kLb32x1:   return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 32, 1, MODE>, grid, dim3(kBlock), s, a);
    case kLb64x1:   return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 64, 1, MODE>, grid, dim3(kBlock), s, a);
    case kLb64x2:
        if constexpr (lowbit_tail_variant<DT, BITS, MODE>()) {
            if (lowbit_tail_chunks(a.cpg, 2))
                return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 64, 2, MODE, true>, grid, dim3(kBlock), s, a);
        }
        return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 64, 2, MODE>, grid, dim3(kBlock), s, a);
    case kLb64x3:
        if constexpr (lowbit_tail_variant<DT, BITS, MODE>()) {
            if (lowbit_tail_chunks(a.cpg, 3))
                return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 64, 3, MODE, true>, grid, dim3(kBlock), s, a);
        }
        return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 64, 3, MODE>, grid, dim3(kBlock), s, a);
    case kLb64x4:
        if constexpr (lowbit_tail_variant<DT, BITS, MODE>()) {
            if (lowbit_tail_chunks(a.cpg, 4))
                return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 64, 4, MODE, true>, grid, dim3(kBlock), s, a);
        }
        return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 64, 4, MODE>, grid, dim3(kBlock), s, a);
    case kLb256x2:  return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 256, 2, MODE>, grid, dim3(256), s, a);
    case kLb256x4:  return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 256, 4, MODE>, grid, dim3(256), s, a);
    case kLb1024x2: return launch_kernel(lowbit_team_kernel<DT, BITS, MBITS, 1024, 2, MODE>, grid, dim3(1024), s, a);
    default:        return hipErrorInvalidValue;
    }
}

template <int DT, int BITS, int MBITS>
static hipError_t launch_lb_mode(int mode, int shape, LaunchGeom g, const LowbitArgs& a, hipStream_t s) {
    switch (mode) {
    case kLbReceiver:         return launch_lb_shape<DT, BITS, MBITS, kLbReceiver>(shape, g, a, s);
    case kLbSenderNearest:    return launch_lb_shape<DT, BITS, MBITS, kLbSenderNearest>(shape, g, a, s);
    case kLbSenderStochastic: return launch_lb_shape<DT, BITS, MBITS, kLbSenderStochastic>(shape, g, a, s);
    default:                  return hipErrorInvalidValue;
    }
}

template <int DT, int BITS>
static hipError_t launch_lb_mbits(int m_bits, int shape, bool sender, LaunchGeom g, const LowbitArgs& a,
                                  hipStream_t s) {
    const int mode = !sender ? kLbReceiver : (a.stochastic ? kLbSenderStochastic : kLbSenderNearest);
    if (m_bits == 8) return launch_lb_mode<DT, BITS, 8>(mode, shape, g, a, s);
    if (m_bits == 2) return launch_lb_mode<DT, BITS, 2>(mode, shape, g, a, s);
    return hipErrorInvalidValue;
}

template <int DT>
hipError_t launch_lowbit_dt(int bits, int m_bits, int shape, bool sender, LaunchGeom g, const LowbitArgs& a,
                            hipStream_t s) {
    switch (bits) {
    case 2: return launch_lb_mbits<DT, 2>(m_bits, shape, sender, g, a, s);
    case 3: return launch_lb_mbits<DT, 3>(m_bits, shape, sender, g, a, s);
    case 4: return launch_lb_mbits<DT, 4>(m_bits, shape, sender, g, a, s);
    case 6: return launch_lb_mbits<DT, 6>(m_bits, shape, sender, g, a, s);
    case 8: return launch_lb_mbits<DT, 8>(m_bits, shape, sender, g, a, s);
    default: return hipErrorInvalidValue;
    }
}

#define AQSGD_INSTANTIATE_LOWBIT_DTYPE(DT)                                                        \
    template hipError_t launch_lowbit_dt<DT>(int, int, int, bool, LaunchGeom, const LowbitArgs&,  \
                                             hipStream_t);

}  // namespace aqsgd

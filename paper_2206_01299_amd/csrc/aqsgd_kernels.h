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
//
// One launch carries a table of independent jobs (messages): the quantising
// jobs of one kernel configuration and any number of dequantising jobs.  A
// stage of a pipeline has both kinds to do at the same time (the sending stage
// encodes activations and reconstructs gradients, the receiving stage decodes
// activations and quantises gradients), and a launch of a few tens of MB spends
// a quarter of its time filling and draining the chip, so messages that are
// ready together go out as one grid.  Workgroup b of the grid finds its job from
// the jobs' first-workgroup numbers; inside a job the workgroups form a
// grid_x x grid_y rectangle, grid_y walking the samples of the call and grid_x
// the groups (or chunks) inside a sample, so no index needs a 64-bit division.
#pragma once

#include <hip/hip_ext.h>

#include <cstddef>
#include <tuple>
#include <utility>

#include "aqsgd_device.h"

namespace aqsgd {

template <typename Tuple, size_t... I>
void fill_arg_pointers(Tuple& t, void** argv, std::index_sequence<I...>) {
    ((argv[I] = static_cast<void*>(&std::get<I>(t))), ...);
}

// First-visit handling (Algorithm 1's branch for a sample without a previous
// message).  `seen` holds one 32-bit word per sample: 0 = never visited, else the
// stamp of the call that visited it first.  A call carries its own stamp, which no
// earlier call on this buffer used; a sample is new to the call if its word is 0
// or equal to the call's stamp.  The second case lets the workgroup that owns the
// sample's first piece write the stamp while other workgroups of the same launch
// still read the word: both values mean "new" to them, and to every later call
// the stamp means "seen".
struct QuantJob {
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
    int32_t bits;
    uint32_t grid_x, grid_y;   // its workgroups: grid_x per sample row, grid_y rows
    float rcp_grid_x;          // 1 / grid_x, for the workgroup's position in that rectangle
    uint64_t seed;
    uint32_t* seen;            // or nullptr: no first-visit handling
    int32_t* first;            // with seen: first[i] = 1 if sample i was new, else 0
    uint32_t stamp;            // with seen: this call's stamp (non-zero)
};

struct DequantJob {
    const uint8_t* codes;
    const float* scales;
    const int64_t* ids;        // or nullptr
    void* m_buf;               // or nullptr: out = Q^-1 alone
    void* out;
    const void* full;          // with seen: uncompressed rows of the call's new samples
    int64_t n_per;
    int64_t gps;
    int64_t cps;               // chunks per sample
    int32_t batch;
    int32_t group;
    int32_t cpg;
    int32_t bits;
    uint32_t grid_x, grid_y;
    float rcp_grid_x;
    uint32_t* seen;            // or nullptr
    uint32_t stamp;
};

constexpr int kMaxQuantJobs = 8;       // per launch
constexpr int kMaxDequantJobs = 8;

// The table is the kernel's argument.  A wave's first instructions fetch it from
// memory, and every fetch that depends on an earlier one adds its full latency to the
// start of every workgroup of the first wave of a launch.  So everything needed to
// find a workgroup's job sits in the header at fixed offsets, next to the first job
// of each kind, which is read at fixed offsets too; only a workgroup of a later job
// reads its job through a computed offset.
struct JobTable {
    int32_t n_quant, n_dequant;
    uint32_t dequant_block0;           // workgroups below this number belong to quantising jobs
    uint32_t total_blocks;
    uint32_t q_block0[kMaxQuantJobs];  // first workgroup of each job, ascending
    uint32_t d_block0[kMaxDequantJobs];
    QuantJob q[kMaxQuantJobs];
    DequantJob d[kMaxDequantJobs];
};

// Is sample `row` new to this call?  (see above; uniform over the workgroup)
__device__ __forceinline__ bool first_visit(const uint32_t* seen, int64_t row, uint32_t stamp) {
    const uint32_t w = seen[row];
    return w == 0u || w == stamp;
}

constexpr int kBlock = 256;

// Groups a team of the quantising kernel takes per step.  A lane of a small team holds
// one chunk of a group, so a workgroup step over one group per team would set up a
// workgroup (job lookup, sample id, row addresses) for eight elements per lane and keep
// two loads per lane in flight; such teams take four groups per step instead, all loads
// first, which is the register budget of the four-chunks-per-lane shapes.
__host__ __device__ constexpr int groups_per_team(int team, int cpl) {
    return (team < kWave && cpl == 1) ? 2 : 1;
}

// ---------------------------------------------------------------------------
// encode / grad_quant, team kernel.
//
// One step of a workgroup covers consecutive groups, groups_per_team() of them
// per team (NG below; a team's groups lie kTeamsPerBlock apart, so that the
// teams of a workgroup read consecutive groups with every load instruction).
// Lanes past the end of a group do not branch around their loads: they
// re-read the group's last chunk, whose values are already in the maximum, hold
// a copy of its results (loaded by the same instruction as the original) and
// store the same bytes to the same place.  Only a team past the last group of
// the sample (ragged last step) is switched off, as a whole.
// ---------------------------------------------------------------------------
template <int DT, int BITS, int ROUND, int TEAM, int CPL, bool HAS_BUF, int NG>
__device__ __forceinline__ void quant_team_group(const QuantJob& a, const char* src_s, char* m_s,
                                                 uint8_t* codes_s, float* scales_s, int64_t src0,
                                                 int64_t g0, int64_t gstride, const uint32_t (&cc)[CPL],
                                                 const uint32_t (&ua)[CPL], const uint32_t (&ub)[CPL],
                                                 int lane_in_team, float* wave_max) {
    constexpr bool kMultiWave = TEAM > kWave;
    constexpr int kThreads = TEAM > kWave ? TEAM : kBlock;
    constexpr int kEB = ElemBytes<DT>::value;
    constexpr int kChunkBytes = kChunk * kEB;
    constexpr int kUnitBytes = kUnit * kEB;
    constexpr bool kUnits = UnitLayout<DT, BITS>::value;   // float32: a chunk is two separate 16-byte units
    static_assert(NG == 1 || !kMultiWave, "several groups per step: teams inside a wavefront only");

    // The team takes NG groups per step, gstride apart: g0, g0 + gstride, ...
    // ---- issue every load of the groups -----------------------------------------
    int64_t goff[NG];                                    // element offsets within the sample
    Raw<DT> ra[NG][CPL], rm[NG][CPL];
#pragma unroll
    for (int u = 0; u < NG; ++u) {
        goff[u] = (g0 + u * gstride) * a.group;
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            if constexpr (kUnits) {
                ra[u][k] = load_raw_units(src_s + goff[u] * kEB + ua[k] * kUnitBytes,
                                          src_s + goff[u] * kEB + ub[k] * kUnitBytes);
                if constexpr (HAS_BUF)
                    rm[u][k] = load_raw_units(m_s + goff[u] * kEB + ua[k] * kUnitBytes,
                                              m_s + goff[u] * kEB + ub[k] * kUnitBytes);
                else rm[u][k] = zero_raw<DT>();
            } else {
                ra[u][k] = load_raw_at<DT>(src_s + goff[u] * kEB + cc[k] * kChunkBytes);
                if constexpr (HAS_BUF) rm[u][k] = load_raw_at<DT>(m_s + goff[u] * kEB + cc[k] * kChunkBytes);
                else rm[u][k] = zero_raw<DT>();
            }
        }
    }
    // Keep all of the loads ahead of the first use: the scheduler would otherwise
    // sink them next to their consumers and leave two or three in flight.
    __builtin_amdgcn_sched_barrier(0);

    // ---- rounding offsets: they depend on the element index only, so the generator
    //      runs while the loads are in flight (second barrier: it stays up here) -------
    float r[NG][CPL][kChunk];
#pragma unroll
    for (int u = 0; u < NG; ++u) {
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            if constexpr (ROUND == AQSGD_ROUND_STOCHASTIC) {
                if constexpr (kUnits)
                    units_uniforms(a.seed, static_cast<uint64_t>(src0 + goff[u]) + ua[k] * kUnit,
                                   static_cast<uint64_t>(src0 + goff[u]) + ub[k] * kUnit, r[u][k]);
                else
                    chunk_uniforms(a.seed, static_cast<uint64_t>(src0 + goff[u]) + cc[k] * kChunk, r[u][k]);
            } else {
#pragma unroll
                for (int e = 0; e < kChunk; ++e) r[u][k][e] = kNearestOffset32;
            }
        }
    }
    if constexpr (ROUND == AQSGD_ROUND_STOCHASTIC) __builtin_amdgcn_sched_barrier(0);

    // ---- delta and each group's max-abs ---------------------------------------------
    float d[NG][CPL][kChunk];
    GroupScale sc[NG];
#pragma unroll
    for (int u = 0; u < NG; ++u) {
        float mx = 0.0f;
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            delta_chunk<DT>(ra[u][k], rm[u][k], d[u][k]);
#pragma unroll
            for (int e = 0; e < kChunk; ++e) mx = __builtin_fmaxf(mx, __builtin_fabsf(d[u][k][e]));
        }
        mx = team_max<(TEAM < kWave ? TEAM : kWave)>(mx);
        if constexpr (kMultiWave) {                      // the whole workgroup is in here
            __syncthreads();                             // earlier readers of wave_max are done
            if (threadIdx.x % kWave == 0) wave_max[threadIdx.x / kWave] = mx;
            __syncthreads();
#pragma unroll
            for (int w = 0; w < kThreads / kWave; ++w) mx = __builtin_fmaxf(mx, wave_max[w]);
        }
        sc[u] = make_scale<BITS>(mx);
    }

    // ---- quantise, pack, update m ---------------------------------------------------
#pragma unroll
    for (int u = 0; u < NG; ++u) {
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            float q[kChunk], dh[kChunk];
#pragma unroll
            for (int e = 0; e < kChunk; ++e) {
                q[e] = level_of<BITS, ROUND>(d[u][k][e], sc[u], r[u][k][e]);
                dh[e] = value_of(q[e], sc[u]);
            }
            uint8_t* group_codes = codes_s + goff[u] / kChunk * BITS;
            if constexpr (kUnits) {
                const uint64_t w = pack_levels<BITS>(q);
                store_unit_codes<BITS>(group_codes + ua[k] * (BITS / 2), low_unit_codes<BITS>(w));
                store_unit_codes<BITS>(group_codes + ub[k] * (BITS / 2), high_unit_codes<BITS>(w));
                if constexpr (HAS_BUF)
                    store_raw_units(m_s + goff[u] * kEB + ua[k] * kUnitBytes, m_s + goff[u] * kEB + ub[k] * kUnitBytes,
                                    updated_chunk<DT>(rm[u][k], dh));
                continue;
            }
            if (BITS == 3 && TEAM % 4 == 0 && a.cpg % 4 == 0) {
                // whole quads of lanes are inside the group or past its end
                const bool inside = k * TEAM + lane_in_team < a.cpg;
                store_codes3_quad(group_codes + (cc[k] & ~3u) * 3, static_cast<uint32_t>(pack_levels<BITS>(q)),
                                  lane_in_team & 3, inside);
            } else {
                store_codes_at<BITS>(group_codes + cc[k] * BITS, pack_levels<BITS>(q));
            }
            if constexpr (HAS_BUF)
                store_raw_at<DT>(m_s + goff[u] * kEB + cc[k] * kChunkBytes, updated_chunk<DT>(rm[u][k], dh));
        }
        if (lane_in_team == 0) scales_s[g0 + u * gstride] = sc[u].s_tx;
    }
}

// First visit of a sample on the sender: the team's chunks of the group go from act
// to m unchanged (the activation itself is the message).  Same chunk ownership and
// clamping as above, so the two paths write a row with the same access pattern.
template <int DT, int BITS, int TEAM, int CPL>
__device__ __forceinline__ void copy_team_group(const QuantJob& a, const char* src_s, char* m_s, int64_t g,
                                                const uint32_t (&cc)[CPL], const uint32_t (&ua)[CPL],
                                                const uint32_t (&ub)[CPL]) {
    constexpr int kEB = ElemBytes<DT>::value;
    constexpr int kChunkBytes = kChunk * kEB;
    constexpr int kUnitBytes = kUnit * kEB;
    constexpr bool kUnits = UnitLayout<DT, BITS>::value;
    const int64_t goff = g * a.group;
    Raw<DT> ra[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        if constexpr (kUnits)
            ra[k] = load_raw_units(src_s + goff * kEB + ua[k] * kUnitBytes, src_s + goff * kEB + ub[k] * kUnitBytes);
        else
            ra[k] = load_raw_at<DT>(src_s + goff * kEB + cc[k] * kChunkBytes);
    }
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        if constexpr (kUnits)
            store_raw_units(m_s + goff * kEB + ua[k] * kUnitBytes, m_s + goff * kEB + ub[k] * kUnitBytes, ra[k]);
        else
            store_raw_at<DT>(m_s + goff * kEB + cc[k] * kChunkBytes, ra[k]);
    }
}

// Workgroup (bx, by) of a quantising job's grid_x x grid_y rectangle.
template <int DT, int BITS, int ROUND, int TEAM, int CPL, bool HAS_BUF>
__device__ __forceinline__ void quant_team_body(const QuantJob& a, uint32_t bx, uint32_t by, float* wave_max) {
    constexpr bool kMultiWave = TEAM > kWave;
    constexpr int kThreads = TEAM > kWave ? TEAM : kBlock;
    constexpr int kTeamsPerBlock = kMultiWave ? 1 : kThreads / TEAM;
    constexpr int kGroupsPerTeam = groups_per_team(TEAM, CPL);
    constexpr int kGroupsPerStep = kTeamsPerBlock * kGroupsPerTeam;
    constexpr int kEB = ElemBytes<DT>::value;

    const int lane_in_team = threadIdx.x % TEAM;
    // A team of at least one wavefront has a wave-uniform index: say so, and the
    // group's base addresses stay in scalar registers.
    const int team = kMultiWave ? 0
                     : (TEAM == kWave ? __builtin_amdgcn_readfirstlane(threadIdx.x / kWave)
                                      : static_cast<int>(threadIdx.x / TEAM));

    uint32_t cc[CPL];           // this lane's chunks within a group, clamped to the last one
#pragma unroll
    for (int k = 0; k < CPL; ++k)
        cc[k] = static_cast<uint32_t>(min(k * TEAM + lane_in_team, a.cpg - 1));
    // The same ownership in 16-byte units for the float32 layout: row k of the team
    // covers units [2k TEAM, 2(k+1) TEAM), a lane takes one from each half of the row;
    // past the group's end a lane repeats the last unit (same values, same stores).
    uint32_t ua[CPL], ub[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        ua[k] = static_cast<uint32_t>(min(2 * k * TEAM + lane_in_team, 2 * a.cpg - 1));
        ub[k] = static_cast<uint32_t>(min((2 * k + 1) * TEAM + lane_in_team, 2 * a.cpg - 1));
    }

    for (int i = by; i < a.batch; i += a.grid_y) {
        const int64_t row = a.ids ? sample_id(a.ids, i) : static_cast<int64_t>(i);
        const int64_t src0 = static_cast<int64_t>(i) * a.n_per;      // flat offset of sample i
        const char* src_s = static_cast<const char*>(a.src) + src0 * kEB;
        char* m_s = HAS_BUF ? static_cast<char*>(a.m_buf) + row * a.n_per * kEB : nullptr;
        uint8_t* codes_s = a.codes + src0 / kChunk * BITS;
        float* scales_s = a.scales + static_cast<int64_t>(i) * a.gps;

        bool fresh = false;
        if constexpr (HAS_BUF) {
            if (a.seen != nullptr) {
                fresh = __builtin_amdgcn_readfirstlane(first_visit(a.seen, row, a.stamp) ? 1 : 0) != 0;
                if (bx == 0 && threadIdx.x == 0) {       // one writer per sample
                    a.first[i] = fresh ? 1 : 0;
                    if (fresh) a.seen[row] = a.stamp;
                }
            }
        }

        // One step of the workgroup: kGroupsPerStep consecutive groups, kGroupsPerTeam per team.
        for (int64_t gbase = static_cast<int64_t>(bx) * kGroupsPerStep; gbase < a.gps;
             gbase += static_cast<int64_t>(a.grid_x) * kGroupsPerStep) {
            if constexpr (kGroupsPerTeam > 1) {
                if (!fresh && gbase + kGroupsPerStep <= a.gps) {         // uniform over the workgroup
                    quant_team_group<DT, BITS, ROUND, TEAM, CPL, HAS_BUF, kGroupsPerTeam>(
                        a, src_s, m_s, codes_s, scales_s, src0, gbase + team, kTeamsPerBlock, cc, ua, ub,
                        lane_in_team, wave_max);
                    continue;
                }
            }
            // a sample's ragged last step, first visits, and the shapes with one group per team
#pragma unroll 1
            for (int u = 0; u < kGroupsPerTeam; ++u) {
                const int64_t g = gbase + u * kTeamsPerBlock + team;     // uniform over the team
                if (g >= a.gps) continue;
                if constexpr (HAS_BUF) {
                    if (fresh) {                         // uniform over the workgroup
                        copy_team_group<DT, BITS, TEAM, CPL>(a, src_s, m_s, g, cc, ua, ub);
                        continue;
                    }
                }
                quant_team_group<DT, BITS, ROUND, TEAM, CPL, HAS_BUF, 1>(a, src_s, m_s, codes_s, scales_s, src0, g,
                                                                         0, cc, ua, ub, lane_in_team, wave_max);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// decode / grad_dequant, flat chunk body: UNROLL chunks per lane and step, all
// loads first.  The group of a chunk comes from one exact division per
// workgroup step plus a small per-lane correction.  THREADS is the size of the
// workgroup the body runs in (the hosting kernel's).
// ---------------------------------------------------------------------------
template <int DT, int BITS, int UNROLL, bool HAS_BUF, int THREADS>
__device__ __forceinline__ void dequant_flat_body(const DequantJob& a, uint32_t bx, uint32_t by) {
    constexpr int kEB = ElemBytes<DT>::value;
    constexpr int kChunkBytes = kChunk * kEB;
    constexpr uint32_t kStep = THREADS * UNROLL;
    const uint32_t cpg = static_cast<uint32_t>(a.cpg);
    const float rcp_cpg = 1.0f / static_cast<float>(cpg);
    const uint32_t cps = static_cast<uint32_t>(a.cps);
    for (int i = by; i < a.batch; i += a.grid_y) {
        const int64_t row = a.ids ? sample_id(a.ids, i) : static_cast<int64_t>(i);
        const int64_t out0 = static_cast<int64_t>(i) * a.n_per;
        char* out_s = static_cast<char*>(a.out) + out0 * kEB;
        char* m_s = HAS_BUF ? static_cast<char*>(a.m_buf) + row * a.n_per * kEB : nullptr;
        const uint8_t* codes_s = a.codes + out0 / kChunk * BITS;
        const float* scales_s = a.scales + static_cast<int64_t>(i) * a.gps;

        if constexpr (HAS_BUF) {
            if (a.seen != nullptr) {
                const bool fresh = __builtin_amdgcn_readfirstlane(first_visit(a.seen, row, a.stamp) ? 1 : 0) != 0;
                if (fresh && bx == 0 && threadIdx.x == 0) a.seen[row] = a.stamp;       // one writer per sample
                if (fresh) {             // first visit: the uncompressed row is the message
                    const char* full_s = static_cast<const char*>(a.full) + out0 * kEB;
                    for (uint32_t c = bx * THREADS + threadIdx.x; c < cps; c += a.grid_x * THREADS) {
                        const Raw<DT> v = load_raw_at<DT>(full_s + static_cast<uint64_t>(c) * kChunkBytes);
                        store_raw_at<DT>(m_s + static_cast<uint64_t>(c) * kChunkBytes, v);
                        store_raw_at<DT>(out_s + static_cast<uint64_t>(c) * kChunkBytes, v);
                    }
                    continue;
                }
            }
        }

        for (uint32_t cbase = bx * kStep; cbase < cps; cbase += a.grid_x * kStep) {
            // group and position of the step's first chunk (uniform), then per lane
            const uint32_t g0 = cbase / cpg;
            const uint32_t r0 = cbase - g0 * cpg;
            uint64_t w[UNROLL];
            float scale[UNROLL];
            Raw<DT> rm[UNROLL];
            uint32_t cs[UNROLL];
            bool ok[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t c = cbase + u * THREADS + threadIdx.x;      // chunk within the sample
                ok[u] = c < cps;
                cs[u] = ok[u] ? c : cps - 1;
                const uint32_t x = r0 + (cs[u] - cbase);                   // < cpg + kStep
                uint32_t dg;
                if (cpg >= kStep) {
                    dg = x >= cpg ? 1u : 0u;
                } else {                                                   // x < 2^23: float is exact enough
                    dg = static_cast<uint32_t>(static_cast<float>(x) * rcp_cpg);
                    if (dg * cpg > x) --dg;
                    else if ((dg + 1) * cpg <= x) ++dg;
                }
                if (BITS == 3 && cps % 4 == 0)           // quads of lanes never straddle the end
                    w[u] = load_codes3_quad(codes_s + static_cast<uint64_t>(cs[u] & ~3u) * 3, threadIdx.x & 3);
                else
                    w[u] = load_codes_at<BITS>(codes_s + static_cast<uint64_t>(cs[u]) * BITS);
                scale[u] = scales_s[g0 + dg];
                if constexpr (HAS_BUF) rm[u] = load_raw_at<DT>(m_s + static_cast<uint64_t>(cs[u]) * kChunkBytes);
            }
            __builtin_amdgcn_sched_barrier(0);           // every load is out before the first use
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const GroupScale sc = scale_from_wire<BITS>(scale[u]);
                float q[kChunk], dh[kChunk];
                unpack_levels<BITS>(w[u], q);
#pragma unroll
                for (int e = 0; e < kChunk; ++e) dh[e] = value_of(q[e], sc);
                if (ok[u]) {
                    Raw<DT> packed;
                    if constexpr (HAS_BUF) {
                        packed = updated_chunk<DT>(rm[u], dh);
                        store_raw_at<DT>(m_s + static_cast<uint64_t>(cs[u]) * kChunkBytes, packed);
                    } else {
                        packed = pack_raw<DT>(dh);
                    }
                    store_raw_at<DT>(out_s + static_cast<uint64_t>(cs[u]) * kChunkBytes, packed);
                }
            }
        }
    }
}

// The same for float32 in 16-byte units (see UnitLayout): one unit of four elements
// per lane and access, UNITS of them per step, so consecutive lanes touch
// consecutive 16 bytes of m, out and, b/2 bytes each, of the codes.
constexpr int64_t kMaxUnitChunks = int64_t{1} << 30;     // unit indices of a sample fit 32 bits

template <int BITS, int UNITS, bool HAS_BUF, int THREADS>
__device__ __forceinline__ void dequant_units_body(const DequantJob& a, uint32_t bx, uint32_t by) {
    constexpr int kUnitBytes = kUnit * 4;
    constexpr uint32_t kStep = THREADS * UNITS;
    const uint32_t upg = 2u * static_cast<uint32_t>(a.cpg);              // units per group
    const float rcp_upg = 1.0f / static_cast<float>(upg);
    const uint32_t ups = 2u * static_cast<uint32_t>(a.cps);              // units per sample
    for (int i = by; i < a.batch; i += a.grid_y) {
        const int64_t row = a.ids ? sample_id(a.ids, i) : static_cast<int64_t>(i);
        const int64_t out0 = static_cast<int64_t>(i) * a.n_per;
        char* out_s = static_cast<char*>(a.out) + out0 * 4;
        char* m_s = HAS_BUF ? static_cast<char*>(a.m_buf) + row * a.n_per * 4 : nullptr;
        const uint8_t* codes_s = a.codes + out0 / kChunk * BITS;
        const float* scales_s = a.scales + static_cast<int64_t>(i) * a.gps;

        if constexpr (HAS_BUF) {
            if (a.seen != nullptr) {
                const bool fresh = __builtin_amdgcn_readfirstlane(first_visit(a.seen, row, a.stamp) ? 1 : 0) != 0;
                if (fresh && bx == 0 && threadIdx.x == 0) a.seen[row] = a.stamp;       // one writer per sample
                if (fresh) {             // first visit: the uncompressed row is the message
                    const char* full_s = static_cast<const char*>(a.full) + out0 * 4;
                    for (uint32_t u = bx * THREADS + threadIdx.x; u < ups; u += a.grid_x * THREADS) {
                        const f32x4_t v = __builtin_nontemporal_load(
                            reinterpret_cast<const f32x4_t*>(full_s + static_cast<uint64_t>(u) * kUnitBytes));
                        store16_through(m_s + static_cast<uint64_t>(u) * kUnitBytes, v);
                        store16_through(out_s + static_cast<uint64_t>(u) * kUnitBytes, v);
                    }
                    continue;
                }
            }
        }

        for (uint32_t ubase = bx * kStep; ubase < ups; ubase += a.grid_x * kStep) {
            const uint32_t g0 = ubase / upg;
            const uint32_t r0 = ubase - g0 * upg;
            uint32_t w[UNITS];
            float scale[UNITS];
            f32x4_t rm[UNITS];
            uint32_t us[UNITS];
            bool ok[UNITS];
#pragma unroll
            for (int u = 0; u < UNITS; ++u) {
                const uint32_t unit = ubase + u * THREADS + threadIdx.x;   // unit within the sample
                ok[u] = unit < ups;
                us[u] = ok[u] ? unit : ups - 1;
                const uint32_t x = r0 + (us[u] - ubase);                   // < upg + kStep
                uint32_t dg;
                if (upg >= kStep) {
                    dg = x >= upg ? 1u : 0u;
                } else {                                                   // x < 2^23: float is exact enough
                    dg = static_cast<uint32_t>(static_cast<float>(x) * rcp_upg);
                    if (dg * upg > x) --dg;
                    else if ((dg + 1) * upg <= x) ++dg;
                }
                w[u] = load_unit_codes<BITS>(codes_s + static_cast<uint64_t>(us[u]) * (BITS / 2));
                scale[u] = scales_s[g0 + dg];
                if constexpr (HAS_BUF)
                    rm[u] = __builtin_nontemporal_load(
                        reinterpret_cast<const f32x4_t*>(m_s + static_cast<uint64_t>(us[u]) * kUnitBytes));
            }
            __builtin_amdgcn_sched_barrier(0);           // every load is out before the first use
#pragma unroll
            for (int u = 0; u < UNITS; ++u) {
                const GroupScale sc = scale_from_wire<BITS>(scale[u]);
                float q[kChunk];
                unpack_levels<BITS>(w[u], q);            // the unit's four levels are the word's first four
                f32x4_t v;
#pragma unroll
                for (int e = 0; e < kUnit; ++e) {
                    const float dh = value_of(q[e], sc);
                    if constexpr (HAS_BUF) v[e] = rm[u][e] + dh;
                    else v[e] = dh;
                }
                if (ok[u]) {
                    if constexpr (HAS_BUF) store16_through(m_s + static_cast<uint64_t>(us[u]) * kUnitBytes, v);
                    store16_through(out_s + static_cast<uint64_t>(us[u]) * kUnitBytes, v);
                }
            }
        }
    }
}

// One dequantising job in a workgroup of THREADS lanes: the body for its bit width
// and for with / without previous messages.
template <int DT, int BITS, int UNROLL, int THREADS>
__device__ __forceinline__ void dequant_job_bits(const DequantJob& a, uint32_t bx, uint32_t by) {
    if constexpr (UnitLayout<DT, BITS>::value) {
        if (a.cps <= kMaxUnitChunks) {                   // else the unit index would pass 32 bits
            if (a.m_buf) dequant_units_body<BITS, 2 * UNROLL, true, THREADS>(a, bx, by);
            else dequant_units_body<BITS, 2 * UNROLL, false, THREADS>(a, bx, by);
            return;
        }
    }
    if (a.m_buf) dequant_flat_body<DT, BITS, UNROLL, true, THREADS>(a, bx, by);
    else dequant_flat_body<DT, BITS, UNROLL, false, THREADS>(a, bx, by);
}

template <int DT, int UNROLL, int THREADS>
__device__ __forceinline__ void dequant_job(const DequantJob& a, uint32_t bx, uint32_t by) {
    switch (a.bits) {                                    // uniform over the workgroup
    case 2: dequant_job_bits<DT, 2, UNROLL, THREADS>(a, bx, by); break;
    case 3: dequant_job_bits<DT, 3, UNROLL, THREADS>(a, bx, by); break;
    case 4: dequant_job_bits<DT, 4, UNROLL, THREADS>(a, bx, by); break;
    case 6: dequant_job_bits<DT, 6, UNROLL, THREADS>(a, bx, by); break;
    default: dequant_job_bits<DT, 8, UNROLL, THREADS>(a, bx, by); break;
    }
}

// The compiler fetches a kernel argument where it is first used, behind whatever
// branch that is, and keeping a whole job in registers from the top would cost more
// registers than the kernels can spare.  A chain of such fetches, each missing the
// scalar cache, would open every workgroup of a launch's first wave.  touch_lines()
// reads one word of each 64-byte line that such a workgroup is going to need, all in
// one batch, so the misses overlap and the later fetches hit the cache.
__device__ __forceinline__ void touch_lines(const void* base, int first_byte, int last_byte) {
    const char* p = static_cast<const char*>(base);
    const int l0 = first_byte / 64, l1 = last_byte / 64;       // constants after inlining
    uint32_t w0 = *reinterpret_cast<const uint32_t*>(p + 64 * l0);
    uint32_t w1 = *reinterpret_cast<const uint32_t*>(p + 64 * (l0 + 1 <= l1 ? l0 + 1 : l1));
    uint32_t w2 = *reinterpret_cast<const uint32_t*>(p + 64 * (l0 + 2 <= l1 ? l0 + 2 : l1));
    uint32_t w3 = *reinterpret_cast<const uint32_t*>(p + 64 * (l0 + 3 <= l1 ? l0 + 3 : l1));
    asm volatile("" : : "s"(w0), "s"(w1), "s"(w2), "s"(w3));
}
static_assert(sizeof(QuantJob) <= 192 && sizeof(DequantJob) <= 192, "touch_lines covers four lines");

struct BlockStarts { u32x4_t lo, hi; };                  // first workgroup of jobs 0..3, 4..7
static_assert(kMaxQuantJobs == 8 && kMaxDequantJobs == 8, "BlockStarts holds eight");

__device__ __forceinline__ BlockStarts block_starts(const uint32_t (&b)[8]) {
    BlockStarts s;
    s.lo = u32x4_t{b[0], b[1], b[2], b[3]};
    s.hi = u32x4_t{b[4], b[5], b[6], b[7]};
    return s;
}

// Workgroup number -> job from the first-workgroup numbers (ascending).
__device__ __forceinline__ int job_of_block(const BlockStarts& s, int n, uint32_t b) {
    int j = 0;
#pragma unroll
    for (int k = 1; k < 8; ++k) {
        const uint32_t start = k < 4 ? s.lo[k] : s.hi[k - 4];
        if (k < n && b >= start) j = k;
    }
    return j;
}

__device__ __forceinline__ uint32_t start_of_job(const BlockStarts& s, int j) {
    uint32_t v = s.lo[0];
#pragma unroll
    for (int k = 1; k < 8; ++k)
        if (j == k) v = k < 4 ? s.lo[k] : s.hi[k - 4];
    return v;
}

// Position of workgroup `local` in a job's grid_x x grid_y rectangle (local < 2^24).
__device__ __forceinline__ void place_in_job(uint32_t local, uint32_t grid_x, float rcp_grid_x, uint32_t& bx,
                                             uint32_t& by) {
    uint32_t y = static_cast<uint32_t>(static_cast<float>(local) * rcp_grid_x);
    if (y * grid_x > local) --y;
    else if ((y + 1) * grid_x <= local) ++y;
    by = y;
    bx = local - y * grid_x;
}

constexpr int kHostedDequantUnroll = 2;      // dequantising jobs inside a quantising kernel's launch

// One quantising job in a team kernel: the body for its bit width and for with /
// without previous messages.  The 3-bit bodies (codes leave through a lane
// transpose) need a sixth more registers than the others, which would cost every
// launch a wave of occupancy per SIMD, so the kernel comes in two variants: without
// them (THREE = false: 2, 4, 6 and 8 bits), and with them for a table in which at
// least one quantising job is 3-bit (THREE = true: every width, at the 3-bit bodies'
// register count).
template <int DT, int BITS, int ROUND, int TEAM, int CPL>
__device__ __forceinline__ void quant_job_bits(const QuantJob& a, uint32_t bx, uint32_t by, float* wave_max) {
    if (a.m_buf) quant_team_body<DT, BITS, ROUND, TEAM, CPL, true>(a, bx, by, wave_max);
    else quant_team_body<DT, BITS, ROUND, TEAM, CPL, false>(a, bx, by, wave_max);
}

template <int DT, int ROUND, int TEAM, int CPL, bool THREE>
__device__ __forceinline__ void quant_job(const QuantJob& a, uint32_t bx, uint32_t by, float* wave_max) {
    if constexpr (THREE) {
        if (a.bits == 3) {                               // uniform over the workgroup
            quant_job_bits<DT, 3, ROUND, TEAM, CPL>(a, bx, by, wave_max);
            return;
        }
    }
    switch (a.bits) {
    case 2: quant_job_bits<DT, 2, ROUND, TEAM, CPL>(a, bx, by, wave_max); break;
    case 4: quant_job_bits<DT, 4, ROUND, TEAM, CPL>(a, bx, by, wave_max); break;
    case 6: quant_job_bits<DT, 6, ROUND, TEAM, CPL>(a, bx, by, wave_max); break;
    default: quant_job_bits<DT, 8, ROUND, TEAM, CPL>(a, bx, by, wave_max); break;
    }
}

// The quantising jobs of one rounding mode and team shape (THREE: 3-bit ones among them)
// plus any dequantising jobs.
template <int DT, int ROUND, int TEAM, int CPL, bool THREE>
__global__ __launch_bounds__((TEAM > kWave ? TEAM : kBlock))
void codec_jobs_kernel(const JobTable t) {
    constexpr int kThreads = TEAM > kWave ? TEAM : kBlock;
    static_assert(TEAM <= kWave || TEAM == kThreads, "a multi-wave team is the whole workgroup");
    [[maybe_unused]] __shared__ float wave_max[kThreads / kWave];
    const uint32_t b = blockIdx.x;
    // header (job counts, first workgroups) and the first quantising job: the workgroups
    // of a launch's first wave belong to it
    touch_lines(&t, 0, 63);
    touch_lines(&t, offsetof(JobTable, q), offsetof(JobTable, q) + sizeof(QuantJob) - 1);
    uint32_t bx, by;
    if (b < t.dequant_block0) {
        const BlockStarts qs = block_starts(t.q_block0);
        const int j = job_of_block(qs, t.n_quant, b);
        const QuantJob& a = t.q[j];
        place_in_job(b - start_of_job(qs, j), a.grid_x, a.rcp_grid_x, bx, by);
        quant_job<DT, ROUND, TEAM, CPL, THREE>(a, bx, by, wave_max);
    } else {
        const BlockStarts ds = block_starts(t.d_block0);
        const int j = job_of_block(ds, t.n_dequant, b);
        const DequantJob& d = t.d[j];
        place_in_job(b - start_of_job(ds, j), d.grid_x, d.rcp_grid_x, bx, by);
        dequant_job<DT, kHostedDequantUnroll, kThreads>(d, bx, by);
    }
}

// Dequantising jobs alone.
template <int DT, int UNROLL>
__global__ __launch_bounds__(kBlock)
void dequant_jobs_kernel(const JobTable t) {
    const uint32_t b = blockIdx.x;
    touch_lines(&t, 0, 63);
    touch_lines(&t, offsetof(JobTable, d), offsetof(JobTable, d) + sizeof(DequantJob) - 1);
    const BlockStarts ds = block_starts(t.d_block0);
    const int j = job_of_block(ds, t.n_dequant, b);
    const DequantJob& a = t.d[j];
    uint32_t bx, by;
    place_in_job(b - start_of_job(ds, j), a.grid_x, a.rcp_grid_x, bx, by);
    dequant_job<DT, UNROLL, kBlock>(a, bx, by);
}

// ---------------------------------------------------------------------------
// Any-shape fallbacks: one thread per group, scalar accesses.  Used when the
// group size is not a multiple of 8 or too large for a workgroup's registers;
// correct for every shape the ABI admits, not tuned.
// ---------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(kBlock)
void quant_anyshape_kernel(const QuantJob a, const int bits, const int rounding) {
    const int L = (1 << bits) - 1;
    const float hL = static_cast<float>(L) / 2.0f;
    const bool has_buf = a.m_buf != nullptr;
    for (int i = blockIdx.y; i < a.batch; i += gridDim.y) {
        const int64_t row = a.ids ? sample_id(a.ids, i) : static_cast<int64_t>(i);
        const int64_t src0 = static_cast<int64_t>(i) * a.n_per;
        const int64_t m0 = row * a.n_per;
        bool fresh = false;
        if (has_buf && a.seen != nullptr) {
            fresh = first_visit(a.seen, row, a.stamp);
            if (blockIdx.x == 0 && threadIdx.x == 0) {           // one writer per sample
                a.first[i] = fresh ? 1 : 0;
                if (fresh) a.seen[row] = a.stamp;
            }
        }
        for (int64_t gs = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; gs < a.gps;
             gs += static_cast<int64_t>(gridDim.x) * kBlock) {
            const int64_t goff = gs * a.group;
            if (fresh) {                                         // first visit: the row itself is the message
                for (int e = 0; e < a.group; ++e)
                    store_elem<DT>(a.m_buf, m0 + goff + e, load_elem<DT>(a.src, src0 + goff + e));
                continue;
            }
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
void dequant_anyshape_kernel(const DequantJob a) {
    const int bits = a.bits;
    const int L = (1 << bits) - 1;
    const float hL = static_cast<float>(L) / 2.0f;
    const bool has_buf = a.m_buf != nullptr;
    for (int i = blockIdx.y; i < a.batch; i += gridDim.y) {
        const int64_t row = a.ids ? sample_id(a.ids, i) : static_cast<int64_t>(i);
        const int64_t out0 = static_cast<int64_t>(i) * a.n_per;
        const int64_t m0 = row * a.n_per;
        bool fresh = false;
        if (has_buf && a.seen != nullptr) {
            fresh = first_visit(a.seen, row, a.stamp);
            if (fresh && blockIdx.x == 0 && threadIdx.x == 0) a.seen[row] = a.stamp;   // one writer per sample
        }
        for (int64_t gs = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; gs < a.gps;
             gs += static_cast<int64_t>(gridDim.x) * kBlock) {
            const int64_t goff = gs * a.group;
            if (fresh) {                                         // first visit: the uncompressed row arrives
                for (int e = 0; e < a.group; ++e) {
                    const float v = load_elem<DT>(a.full, out0 + goff + e);
                    store_elem<DT>(a.m_buf, m0 + goff + e, v);
                    store_elem<DT>(a.out, out0 + goff + e, v);
                }
                continue;
            }
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

struct LaunchGeom { uint32_t grid_x, grid_y; };

// Optional timing of the next launch made by this host thread: when set (see
// aqsgd_profile_next_launch) the kernel goes out through hipExtLaunchKernel,
// which stamps the two events with the kernel's own start and end, and the
// request is cleared.
struct ProfileRequest { hipEvent_t start, stop; };
extern thread_local ProfileRequest g_profile_request;

// Returns the status of this launch alone (an earlier error that the calling
// thread has not collected is neither reported here nor cleared).
template <typename... KArgs, typename... Args>
hipError_t launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t stream,
                         Args... args) {
    std::tuple<KArgs...> held(args...);
    void* argv[sizeof...(KArgs)];
    fill_arg_pointers(held, argv, std::index_sequence_for<KArgs...>{});
    ProfileRequest& pr = g_profile_request;
    if (pr.start || pr.stop) {
        const hipError_t err = hipExtLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, argv,
                                                  0, stream, pr.start, pr.stop, 0);
        pr.start = nullptr;
        pr.stop = nullptr;
        return err;
    }
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, argv, 0, stream);
}

// Team shapes the dispatcher may pick; index into the table below.
enum TeamShape {
    kTeam8x1 = 0, kTeam16x1, kTeam32x1, kTeam64x1, kTeam64x2, kTeam64x3, kTeam64x4,
    kTeam256x2, kTeam256x4, kTeam1024x2, kTeam1024x4, kNumTeamShapes
};

// A launch of codec_jobs_kernel (the table's quantising jobs all have this rounding
// mode and team shape; `three`: at least one of them is 3-bit) or, with no quantising
// job, of dequant_jobs_kernel.
hipError_t launch_codec_jobs(int dtype, int rounding, int shape, bool three, const JobTable& t,
                             hipStream_t stream);
hipError_t launch_dequant_jobs(int dtype, int unroll, const JobTable& t, hipStream_t stream);
hipError_t launch_quant_anyshape(int dtype, int bits, int rounding, const QuantJob& a, hipStream_t stream);
hipError_t launch_dequant_anyshape(int dtype, const DequantJob& a, hipStream_t stream);

// Per-dtype pieces (defined by AQSGD_INSTANTIATE_DTYPE in the dtype's .hip file).
template <int DT> hipError_t launch_codec_jobs_dt(int rounding, int shape, bool three, const JobTable& t,
                                                  hipStream_t stream);
template <int DT> hipError_t launch_dequant_jobs_dt(int unroll, const JobTable& t, hipStream_t stream);
template <int DT> hipError_t launch_quant_anyshape_dt(int bits, int rounding, const QuantJob& a,
                                                      hipStream_t stream);
template <int DT> hipError_t launch_dequant_anyshape_dt(const DequantJob& a, hipStream_t stream);

}  // namespace aqsgd

// Sparsified backward message ("bw8[0.2]", Appendix H.6 of the paper): per group
// of G gradient entries only the `keep` largest magnitudes travel, as 8-bit
// levels of Q with the group's max-abs scale, plus one bit per entry that says
// which ones.  Equal magnitudes: the lower index survives first.
//
// One wave owns a group (G <= 2048) and keeps it in registers.  The threshold is
// the keep-th largest magnitude, found on the magnitudes' bit patterns (which
// order like unsigned integers) by a radix select, one byte per level: the wave
// histograms the byte in 256 LDS counters, a prefix sum over the lanes (each
// holding four counters) finds the counter that contains the wanted rank, and the
// next level only looks at entries that share the bytes decided so far.  Two
// levels for the 16-bit types, four for binary32.  Positions in the compacted
// byte string come from per-lane population counts and the same wave prefix sum.
// The kept bytes are gathered in LDS and leave as full-width stores; the receiver
// stages them the same way.
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
constexpr int kTopkBins = 256;
constexpr int kTopkStageBytes = kTopkMaxGroup + kWave;   // + one spare byte per lane for entries not kept

// One wave per workgroup: a group is a wave's work and the waves share nothing, and with a
// single TopkLds per workgroup every LDS address is an instruction offset instead of a
// register sum (one vector instruction less per histogram update and per staged entry).
constexpr int kTopkBlock = kWave;

// LDS of one wave.  (One histogram per row of 16 lanes, added up when read, was tried
// against the bank conflicts of the counting and did not remove them: 64 lanes updating
// counters picked by the data fall several to a bank however the counters are laid out,
// and the extra clearing and reading made the kernel slower.)
struct TopkLds {
    uint32_t bins[kTopkBins + kWave];                    // 256 counters + one spare per lane
    uint8_t stage[kTopkStageBytes];
    uint16_t stage16[kTopkMaxGroup + kWave];             // kept entries as stored, + one spare per lane
};

// Bytes of a magnitude key: the key is the magnitude's bit pattern shifted left by
// one, so it fills 2 (half, bfloat16) or 4 (binary32) whole bytes.
template <int DT> struct KeyBytes { static constexpr int value = 2; };
template <> struct KeyBytes<AQSGD_F32> { static constexpr int value = 4; };

template <int DT>
__device__ __forceinline__ void magnitude_keys(const Raw<DT>& r, uint32_t (&u)[kChunk]) {
    if constexpr (DT == AQSGD_F32) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            u[i] = __float_as_uint(r.lo[i]) << 1;
            u[4 + i] = __float_as_uint(r.hi[i]) << 1;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            u[2 * i] = (r.v[i] << 1) & 0xfffeu;
            u[2 * i + 1] = (r.v[i] >> 15) & 0xfffeu;
        }
    }
}

// LDS traffic of one wave: later reads must see earlier writes of other lanes.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_shifted_or_zero(uint32_t v) {
    // lanes without a source lane in their row of 16 read zero
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xf, 0xf, true));
}

// Inclusive prefix sum over the 64 lanes (lane order); `total` = the sum of all lanes.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t x, int lane, uint32_t& total) {
    x += dpp_shifted_or_zero<0x111>(x);                  // row_shr:1
    x += dpp_shifted_or_zero<0x112>(x);                  // row_shr:2
    x += dpp_shifted_or_zero<0x114>(x);                  // row_shr:4
    x += dpp_shifted_or_zero<0x118>(x);                  // row_shr:8 -> prefix within each row of 16
    const uint32_t r0 = __builtin_amdgcn_readlane(x, 15);
    const uint32_t r1 = __builtin_amdgcn_readlane(x, 31);
    const uint32_t r2 = __builtin_amdgcn_readlane(x, 47);
    const uint32_t r3 = __builtin_amdgcn_readlane(x, 63);
    total = r0 + r1 + r2 + r3;
    const uint32_t before = lane < 16 ? 0u : (lane < 32 ? r0 : (lane < 48 ? r0 + r1 : r0 + r1 + r2));
    return x + before;
}

// The keep-th largest key of the group and how many entries equal to it are kept.
// `equal_total` = number of entries equal to the threshold.
// TAIL: the lane's single entry of a last round taken entry by entry (key tail_u, counted if tail_valid).
template <int DT, int CPL, bool TAIL>
__device__ __forceinline__ void kth_largest(const uint32_t (&u)[CPL][kChunk], const bool (&valid)[CPL],
                                            uint32_t tail_u, bool tail_valid,
                                            int keep, int lane, uint32_t* bins, uint32_t& threshold,
                                            int& equal_kept, int& equal_total) {
    uint32_t prefix = 0;                                 // bytes of the threshold decided so far
    uint32_t need = static_cast<uint32_t>(keep);         // rank of the threshold among entries sharing them
    uint32_t in_bin = 0;
#pragma unroll
    for (int level = KeyBytes<DT>::value - 1; level >= 0; --level) {
        const int shift = 8 * level;
        const u32x4_t zero = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4_t*>(bins + 4 * lane) = zero;
        const uint32_t spare = static_cast<uint32_t>(kTopkBins + lane);
        wave_lds_sync();
        // Below the top level only entries that share the decided bytes count.  With
        // those bytes cancelled by an exclusive-or, a sharing entry is left with its
        // byte (< 256) and every other entry with something larger, which min() sends
        // to the lane's spare counter behind the 256 real ones (never read).
        const uint32_t decided = level == KeyBytes<DT>::value - 1 ? 0u : prefix << ((shift + 8) & 31);
#pragma unroll
        for (int k = 0; k < CPL; ++k)
            if (valid[k]) {
#pragma unroll
                for (int e = 0; e < kChunk; ++e) {
                    const uint32_t digit = (u[k][e] ^ decided) >> shift;
                    atomicAdd(&bins[min(digit, spare)], 1u);
                }
            }
        if constexpr (TAIL) {
            if (tail_valid) atomicAdd(&bins[min((tail_u ^ decided) >> shift, spare)], 1u);
        }
        wave_lds_sync();
        const u32x4_t c = *reinterpret_cast<const u32x4_t*>(bins + 4 * lane);
        const uint32_t mine = c[0] + c[1] + c[2] + c[3];
        uint32_t total;
        const uint32_t upto = wave_inclusive_sum(mine, lane, total);
        // entries in counters above this lane's four, then above each of its counters
        const uint32_t a3 = total - upto;
        const uint32_t a2 = a3 + c[3], a1 = a2 + c[2], a0 = a1 + c[1];
        const bool here = a3 < need && need <= a3 + mine;            // exactly one lane
        const int sel = need <= a2 ? 3 : (need <= a1 ? 2 : (need <= a0 ? 1 : 0));
        const uint32_t above = sel == 3 ? a3 : (sel == 2 ? a2 : (sel == 1 ? a1 : a0));
        const uint32_t count = sel == 3 ? c[3] : (sel == 2 ? c[2] : (sel == 1 ? c[1] : c[0]));
        const uint64_t who = __ballot(here);
        const int src = who ? __builtin_ctzll(who) : 0;
        const uint32_t digit = __builtin_amdgcn_readlane(static_cast<uint32_t>(4 * lane + sel), src);
        need -= __builtin_amdgcn_readlane(above, src);
        in_bin = __builtin_amdgcn_readlane(count, src);
        prefix = (prefix << 8) | digit;
    }
    threshold = prefix;
    equal_kept = static_cast<int>(need);
    equal_total = static_cast<int>(in_bin);
}

// Bit e of the result: key e is greater than (STRICT) / at least the threshold.
template <int DT, bool STRICT>
__device__ __forceinline__ uint32_t chunk_mask(const uint32_t (&u)[kChunk], uint32_t t) {
    uint32_t m = 0;
    if constexpr (KeyBytes<DT>::value == 2) {
        // Keys below 2^16: the sign bit of a difference is the comparison, and alignbit
        // shifts it into the mask ((m << 1) | (d >> 31)), last entry first.
#pragma unroll
        for (int e = kChunk - 1; e >= 0; --e) {
            const uint32_t d = STRICT ? t - u[e] : u[e] - t;          // sign set: u > t / u < t
            m = __builtin_amdgcn_alignbit(m, d, 31);
        }
        return STRICT ? m : ~m & 0xffu;
    } else {
#pragma unroll
        for (int e = 0; e < kChunk; ++e)
            m |= static_cast<uint32_t>(STRICT ? u[e] > t : u[e] >= t) << e;
        return m;
    }
}

// Exclusive prefix over the lanes of up to four per-lane counts (each < 2^16 in
// total), two per scanned register; totals[k] = sum over all lanes.
template <int CPL>
__device__ __forceinline__ void lanes_before(const uint32_t (&cnt)[CPL], int lane, uint32_t (&before)[CPL],
                                             uint32_t (&totals)[CPL]) {
#pragma unroll
    for (int k = 0; k < CPL; k += 2) {
        const int k1 = k + 1 < CPL ? k + 1 : k;         // second count of the pair, if there is one
        const uint32_t packed = cnt[k] | (k1 != k ? cnt[k1] << 16 : 0u);
        uint32_t tot;
        const uint32_t excl = wave_inclusive_sum(packed, lane, tot) - packed;
        before[k] = excl & 0xffffu;
        totals[k] = tot & 0xffffu;
        if (k1 != k) {
            before[k1] = excl >> 16;
            totals[k1] = tot >> 16;
        }
    }
}

// ---------------------------------------------------------------------------
// Sixteen-bit types with nearest rounding: the sender works on the magnitudes as they
// sit in memory, two per register (packed 16-bit integer operations), and quantises
// only the entries that are kept.  The kernel is bound by vector arithmetic (a wave64
// instruction occupies its SIMD for four cycles, and a group is a thousand of them in
// the general path below), so instructions are what this path saves: no conversion of
// all entries to binary32, no unpacked keys, each digit of the radix select a byte of
// the packed word (magnitudes are held doubled for that), masks from the sign bits of
// packed differences, and one quantisation per kept entry instead of one per entry.
// ---------------------------------------------------------------------------
typedef unsigned short u16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2_t, a),
                                                                  __builtin_bit_cast(u16x2_t, b)));
}
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2_t, a),
                                                                  __builtin_bit_cast(u16x2_t, b)));
}
__device__ __forceinline__ uint32_t pk_add_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2_t, a) + __builtin_bit_cast(u16x2_t, b));
}
__device__ __forceinline__ uint32_t pk_sub_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2_t, a) - __builtin_bit_cast(u16x2_t, b));
}

// binary32 value of a 16-bit storage pattern.
template <int DT>
__device__ __forceinline__ float f32_of_bits16(uint32_t h) {
    if constexpr (DT == AQSGD_F16) return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)));
    else return bf16_bits_to_f32(h);
}

// One level of the radix select for packed magnitudes held doubled (m2 = 2 * magnitude:
// adding a stored pattern to itself drops the sign bit, and it leaves the magnitude's top
// eight bits in a byte of their own, which a counter's address is one instruction away
// from).  LEVEL 1 counts that byte for every entry; LEVEL 0 counts the other byte (twice
// the low seven bits: even counters only) for the entries whose top byte is `prefix`: with
// that byte cancelled by an exclusive-or a sharing entry is left below 256 and every other
// entry at 256 or above, where min() caps it at the lane's spare counter (counters from
// 256 on are never read).  Returns the digit that holds rank `need` and updates need / in_bin.
template <int CPL, int LEVEL, bool TAIL>
__device__ __forceinline__ uint32_t radix_level16(const uint32_t (&m)[CPL][4], const bool (&valid)[CPL],
                                                  uint32_t tail_m2, bool tail_valid, uint32_t prefix, int lane,
                                                  uint32_t* bins, uint32_t& need, uint32_t& in_bin) {
    const u32x4_t zero = {0u, 0u, 0u, 0u};
    *reinterpret_cast<u32x4_t*>(bins + 4 * lane) = zero;
    wave_lds_sync();
    const uint32_t spare = static_cast<uint32_t>(kTopkBins + lane);
    const uint32_t cancel = (prefix << 8) | (prefix << 24);
    const uint32_t spare2 = spare | (spare << 16);
#pragma unroll
    for (int k = 0; k < CPL; ++k)
        if (valid[k]) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (LEVEL == 1) {
                    atomicAdd(&bins[(m[k][i] >> 8) & 0xffu], 1u);
                    atomicAdd(&bins[m[k][i] >> 24], 1u);
                } else {
                    const uint32_t y = pk_min_u16(m[k][i] ^ cancel, spare2);
                    atomicAdd(&bins[y & 0xffffu], 1u);
                    atomicAdd(&bins[y >> 16], 1u);
                }
            }
        }
    if constexpr (TAIL) {                                // the lane's single entry of the last round
        if (tail_valid) {
            if constexpr (LEVEL == 1) atomicAdd(&bins[tail_m2 >> 8], 1u);
            else atomicAdd(&bins[min(tail_m2 ^ (prefix << 8), spare)], 1u);
        }
    }
    wave_lds_sync();
    u32x4_t c = *reinterpret_cast<const u32x4_t*>(bins + 4 * lane);
    const uint32_t mine = c[0] + c[1] + c[2] + c[3];
    uint32_t total;
    const uint32_t upto = wave_inclusive_sum(mine, lane, total);
    // entries in counters above this lane's four, then above each of its counters
    const uint32_t a3 = total - upto;
    const uint32_t a2 = a3 + c[3], a1 = a2 + c[2], a0 = a1 + c[1];
    const bool here = a3 < need && need <= a3 + mine;                // exactly one lane
    const int sel = need <= a2 ? 3 : (need <= a1 ? 2 : (need <= a0 ? 1 : 0));
    const uint32_t above = sel == 3 ? a3 : (sel == 2 ? a2 : (sel == 1 ? a1 : a0));
    const uint32_t count = sel == 3 ? c[3] : (sel == 2 ? c[2] : (sel == 1 ? c[1] : c[0]));
    const uint64_t who = __ballot(here);
    const int src = who ? __builtin_ctzll(who) : 0;
    const uint32_t digit = __builtin_amdgcn_readlane(static_cast<uint32_t>(4 * lane + sel), src);
    need -= __builtin_amdgcn_readlane(above, src);
    in_bin = __builtin_amdgcn_readlane(count, src);
    return digit;
}

// Bit e of the result: entry e of the chunk has its sign bit set in the packed
// differences d[0..3] (entry 2i in the low half of d[i], entry 2i+1 in the high half).
__device__ __forceinline__ uint32_t sign_mask16(const uint32_t (&d)[4]) {
    uint32_t mask = 0;
#pragma unroll
    for (int i = 3; i >= 0; --i) {                       // last entry first: (mask << 1) | sign
        mask = __builtin_amdgcn_alignbit(mask, d[i], 31);
        mask = __builtin_amdgcn_alignbit(mask, d[i] << 16, 31);
    }
    return mask;
}

// The group's entries as stored, one chunk per lane and row.
template <int DT, int CPL>
__device__ __forceinline__ void load_group16(const TopkArgs& a, int64_t g, const uint32_t (&cc)[CPL],
                                             Raw<DT> (&raw)[CPL]) {
    const char* src = static_cast<const char*>(a.grad) + g * a.group * 2;
#pragma unroll
    for (int k = 0; k < CPL; ++k) raw[k] = load_raw_at<DT>(src + cc[k] * (kChunk * 2));
}

// Entries of a 64-bit lane mask below this lane.
__device__ __forceinline__ int lanes_set_below(uint64_t mask) {
    return static_cast<int>(__builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                                      __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u)));
}

// TAIL: the group is CPL full rounds of chunks (one chunk per lane and round) followed by at
// most eight more chunks, i.e. at most one entry per lane, which the lanes take as single
// entries (`tail_raw`: the entry as stored; `tail_valid`: the lane has one) instead of
// eight lanes taking a chunk each through one more round of whole-chunk work for everyone
// - a 1600-entry group is three rounds and one such entry, not four rounds.  Ballots give
// the tail's bitmap bytes and positions directly.
template <int DT, int CPL, bool TAIL>
__device__ __forceinline__ void topk_quant_group16(const TopkArgs& a, int64_t g, const Raw<DT> (&raw)[CPL],
                                                   uint32_t tail_raw, bool tail_valid,
                                                   const uint32_t (&cc)[CPL], const bool (&valid)[CPL], int lane,
                                                   TopkLds& lds) {
    const int64_t e0 = g * a.group;                      // first entry of the group in the call tensor

    // ---- doubled magnitudes (two per register) and the group's largest ------------------------
    uint32_t m2[CPL][4];
    uint32_t top = 0;
#pragma unroll
    for (int k = 0; k < CPL; ++k)
#pragma unroll
        for (int i = 0; i < 4; ++i) {                    // a clamped lane repeats a real chunk: harmless here
            m2[k][i] = pk_add_u16(raw[k].v[i], raw[k].v[i]);
            top = pk_max_u16(top, m2[k][i]);
        }
    uint32_t tail_m2 = 0;
    if constexpr (TAIL) {
        tail_m2 = tail_valid ? (tail_raw + tail_raw) & 0xffffu : 0u;
        top = pk_max_u16(top, tail_m2);
    }
    top = max(top & 0xffffu, top >> 16) >> 1;
    top = __float_as_uint(team_max<kWave>(__uint_as_float(top)));    // an integer maximum over the lanes
    const GroupScale sc = make_scale<kTopkBits>(f32_of_bits16<DT>(top));

    // ---- the keep-th largest magnitude: two levels, eight then seven bits ---------------------
    uint32_t need = static_cast<uint32_t>(a.keep), in_bin = 0;
    const uint32_t hi8 = radix_level16<CPL, 1, TAIL>(m2, valid, tail_m2, tail_valid, 0u, lane, lds.bins, need, in_bin);
    const uint32_t lo7x2 = radix_level16<CPL, 0, TAIL>(m2, valid, tail_m2, tail_valid, hi8, lane, lds.bins, need, in_bin);
    const uint32_t threshold = ((hi8 << 8) | lo7x2) >> 1;
    const int equal_kept = static_cast<int>(need), equal_total = static_cast<int>(in_bin);
    const uint32_t tt = threshold | (threshold << 16);

    // ---- keep flags: everything above the threshold, and the first equal_kept entries equal to it
    uint32_t geb[CPL];                                   // bit e: entry e is >= the threshold
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        uint32_t d[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) d[i] = pk_sub_u16(raw[k].v[i] & 0x7fff7fffu, tt);   // sign set: below the threshold
        geb[k] = valid[k] ? ~sign_mask16(d) & 0xffu : 0u;
    }
    const uint32_t tail_mag = tail_raw & 0x7fffu;
    const bool tail_ge = TAIL && tail_valid && tail_mag >= threshold;
    bool tail_keep = tail_ge;
    uint32_t keepb[CPL];
    if (equal_kept == equal_total) {                     // no choice to make among equals (wave-uniform)
#pragma unroll
        for (int k = 0; k < CPL; ++k) keepb[k] = geb[k];
    } else {
        uint32_t gtb[CPL], eqb[CPL], ties[CPL], ties_below[CPL], ties_total[CPL];
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            uint32_t d[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) d[i] = pk_sub_u16(tt, raw[k].v[i] & 0x7fff7fffu);   // sign set: above the threshold
            gtb[k] = sign_mask16(d) & geb[k];
            eqb[k] = geb[k] & ~gtb[k];
            ties[k] = __builtin_popcount(eqb[k]);
        }
        lanes_before<CPL>(ties, lane, ties_below, ties_total);
        int left = equal_kept;                           // equals still to keep when chunk row k starts
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const int allowed = left - static_cast<int>(ties_below[k]);   // ... when this lane's chunk starts
            // all of the chunk's equals, or none of them, unless the cut falls inside the chunk
            uint32_t kb = gtb[k] | (static_cast<int>(ties[k]) <= allowed ? eqb[k] : 0u);
            if (allowed > 0 && allowed < static_cast<int>(ties[k])) {    // rare: at most one lane per row
                int seen = 0;
#pragma unroll
                for (int e = 0; e < kChunk; ++e) {
                    const uint32_t eq = (eqb[k] >> e) & 1u;
                    if (eq && seen < allowed) kb |= 1u << e;
                    seen += static_cast<int>(eq);
                }
            }
            keepb[k] = kb;
            left = max(left - static_cast<int>(ties_total[k]), 0);
        }
        if constexpr (TAIL) {                            // the tail's entries come last in entry order
            const bool tail_eq = tail_ge && tail_mag == threshold;
            tail_keep = tail_ge && (!tail_eq || lanes_set_below(__ballot(tail_eq)) < left);
        }
    }

    // ---- the kept entries, as stored, in entry order into LDS ----------------------------------
    uint32_t kept[CPL], kept_below[CPL], kept_total[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) kept[k] = __builtin_popcount(keepb[k]);
    lanes_before<CPL>(kept, lane, kept_below, kept_total);
    // An entry that is not kept lands in the lane's spare slot behind the staged ones.  Byte
    // offsets, and the choice written as spare + on * (position - spare): three vector
    // instructions per entry (extract, multiply-add, advance) where compare + select took five.
    char* const stage16 = reinterpret_cast<char*>(lds.stage16);
    const int spare = 2 * (kTopkMaxGroup + lane);
    uint32_t row_start = 0;
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        int ahead = 2 * static_cast<int>(row_start + kept_below[k]) - spare;     // negative: the spares come last
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
            const int on = static_cast<int>((keepb[k] >> e) & 1u);
            const uint32_t w = raw[k].v[e / 2];
            *reinterpret_cast<uint16_t*>(stage16 + (__mul24(on, ahead) + spare)) =
                static_cast<uint16_t>(e % 2 ? w >> 16 : w);
            ahead += 2 * on;
            asm volatile("" : "+v"(ahead));              // keeps the running difference in its register
        }
        if (valid[k]) a.bitmap[e0 / kChunk + cc[k]] = static_cast<uint8_t>(keepb[k]);
        row_start += kept_total[k];
    }
    if constexpr (TAIL) {
        const uint64_t km = __ballot(tail_keep);         // bit l: lane l's entry, which is entry 64 * 8 * CPL + l
        if (tail_keep) lds.stage16[row_start + static_cast<uint32_t>(lanes_set_below(km))] = static_cast<uint16_t>(tail_raw);
        const int tail_chunks = a.cpg - CPL * kWave;
        if (lane < tail_chunks)
            a.bitmap[e0 / kChunk + CPL * kWave + lane] = static_cast<uint8_t>(km >> (8 * lane));
    }
    wave_lds_sync();

    // ---- quantise the kept entries: lane l takes a run of consecutive positions ---------------
    const int run = (a.keep + kWave - 1) / kWave;
    for (int j = 0; j < run; ++j) {
        const int p = lane * run + j;
        if (p < a.keep) {
            const float f = f32_of_bits16<DT>(lds.stage16[p]);
            const float q = level_of<kTopkBits, AQSGD_ROUND_NEAREST>(f, sc, kNearestOffset32);
            lds.stage[p] = static_cast<uint8_t>(__builtin_amdgcn_cvt_pk_u8_f32(q, 0, 0));
        }
    }
    wave_lds_sync();

    // ---- the group's bytes leave LDS ------------------------------------------------------
    uint8_t* dst = a.codes + g * a.keep;
    if (a.keep % 16 == 0) {
        for (int i = lane; i < a.keep / 16; i += kWave)
            *reinterpret_cast<u32x4_t*>(dst + 16 * i) = *reinterpret_cast<const u32x4_t*>(lds.stage + 16 * i);
    } else {
        for (int i = lane; i < a.keep; i += kWave) dst[i] = lds.stage[i];
    }
    if (lane == 0) a.scales[g] = sc.s_tx;
    wave_lds_sync();                                     // the next group reuses the staging bytes
}

// TAIL as in topk_quant_group16: CPL whole rounds of chunks, then at most eight more chunks
// taken as one entry per lane (`tail_entries` of them).
template <int DT, int CPL, int ROUND, bool TAIL>
__device__ __forceinline__ void topk_quant_group(const TopkArgs& a, int64_t g, const uint32_t (&cc)[CPL],
                                                 const bool (&valid)[CPL], int lane, TopkLds& lds,
                                                 int tail_entries = 0) {
    constexpr int kEB = ElemBytes<DT>::value;
    constexpr int kChunkBytes = kChunk * kEB;
    const int64_t e0 = g * a.group;                      // first entry of the group in the call tensor
    const char* src = static_cast<const char*>(a.grad) + e0 * kEB;

    Raw<DT> raw[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) raw[k] = load_raw_at<DT>(src + cc[k] * kChunkBytes);
    // the tail: entry CPL * 64 * 8 + lane of the group (a lane past the end repeats the last one)
    [[maybe_unused]] const bool tail_valid = TAIL && lane < tail_entries;
    [[maybe_unused]] const int tail_j = CPL * kWave * kChunk + min(lane, tail_entries - 1);
    [[maybe_unused]] float tail_f = 0.0f;
    if constexpr (TAIL) tail_f = load_elem<DT>(src, tail_j);
    __builtin_amdgcn_sched_barrier(0);

    float f[CPL][kChunk];
    uint32_t u[CPL][kChunk];
    float mx = 0.0f;
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        unpack_raw<DT>(raw[k], f[k]);
        magnitude_keys<DT>(raw[k], u[k]);
#pragma unroll
        for (int e = 0; e < kChunk; ++e)                 // a clamped lane repeats a real chunk: harmless here
            mx = __builtin_fmaxf(mx, __builtin_fabsf(f[k][e]));
    }
    // the tail entry's key: as magnitude_keys makes them (the storage pattern's magnitude, doubled)
    [[maybe_unused]] uint32_t tail_u = 0;
    if constexpr (TAIL) {
        if constexpr (DT == AQSGD_F32) tail_u = __float_as_uint(tail_f) << 1;
        else if constexpr (DT == AQSGD_F16)
            tail_u = (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, static_cast<_Float16>(tail_f))) << 1) & 0xfffeu;
        else tail_u = (__float_as_uint(tail_f) >> 15) & 0xfffeu;
        mx = __builtin_fmaxf(mx, __builtin_fabsf(tail_f));           // a repeated entry: harmless here
    }
    mx = team_max<kWave>(mx);
    const GroupScale sc = make_scale<kTopkBits>(mx);

    uint32_t threshold;
    int equal_kept, equal_total;
    kth_largest<DT, CPL, TAIL>(u, valid, tail_u, tail_valid, a.keep, lane, lds.bins, threshold, equal_kept, equal_total);

    // ---- keep flags: everything above the threshold, and the first equal_kept entries equal to it
    uint32_t geb[CPL];                                   // bit e: entry e is >= the threshold
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        geb[k] = chunk_mask<DT, false>(u[k], threshold);
        if (!valid[k]) geb[k] = 0;
    }
    const bool tail_ge = TAIL && tail_valid && tail_u >= threshold;
    bool tail_keep = tail_ge;
    uint32_t keepb[CPL];
    if (equal_kept == equal_total) {                     // no choice to make among equals (wave-uniform)
#pragma unroll
        for (int k = 0; k < CPL; ++k) keepb[k] = geb[k];
    } else {
        uint32_t gtb[CPL], eqb[CPL], ties[CPL], ties_below[CPL], ties_total[CPL];
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            gtb[k] = chunk_mask<DT, true>(u[k], threshold) & geb[k];
            eqb[k] = geb[k] & ~gtb[k];
            ties[k] = __builtin_popcount(eqb[k]);
        }
        lanes_before<CPL>(ties, lane, ties_below, ties_total);
        int left = equal_kept;                           // equals still to keep when chunk row k starts
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const int allowed = left - static_cast<int>(ties_below[k]);   // ... when this lane's chunk starts
            // all of the chunk's equals, or none of them, unless the cut falls inside the chunk
            uint32_t kb = gtb[k] | (static_cast<int>(ties[k]) <= allowed ? eqb[k] : 0u);
            if (allowed > 0 && allowed < static_cast<int>(ties[k])) {    // rare: at most one lane per row
                int seen = 0;
#pragma unroll
                for (int e = 0; e < kChunk; ++e) {
                    const uint32_t eq = (eqb[k] >> e) & 1u;
                    if (eq && seen < allowed) kb |= 1u << e;
                    seen += static_cast<int>(eq);
                }
            }
            keepb[k] = kb;
            left = max(left - static_cast<int>(ties_total[k]), 0);
        }
        if constexpr (TAIL) {                            // the tail's entries come last in entry order
            const bool tail_eq = tail_ge && tail_u == threshold;
            tail_keep = tail_ge && (!tail_eq || lanes_set_below(__ballot(tail_eq)) < left);
        }
    }

    // ---- positions in the group's byte string, levels, staging ------------------------------
    uint32_t kept[CPL], kept_below[CPL], kept_total[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) kept[k] = __builtin_popcount(keepb[k]);
    lanes_before<CPL>(kept, lane, kept_below, kept_total);
    uint32_t row_start = 0;
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        uint32_t pos = row_start + kept_below[k];
        float r[kChunk];
        if constexpr (ROUND == AQSGD_ROUND_STOCHASTIC) {
            chunk_uniforms(a.seed, static_cast<uint64_t>(e0) + static_cast<uint64_t>(cc[k]) * kChunk, r);
        } else {
#pragma unroll
            for (int e = 0; e < kChunk; ++e) r[e] = kNearestOffset32;
        }
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
            const float q = level_of<kTopkBits, ROUND>(f[k][e], sc, r[e]);
            const uint32_t on = (keepb[k] >> e) & 1u;
            // entries that are not kept write this lane's spare byte
            lds.stage[on ? pos : static_cast<uint32_t>(kTopkMaxGroup + lane)] =
                static_cast<uint8_t>(__builtin_amdgcn_cvt_pk_u8_f32(q, 0, 0));
            pos += on;
        }
        if (valid[k]) a.bitmap[e0 / kChunk + cc[k]] = static_cast<uint8_t>(keepb[k]);
        row_start += kept_total[k];
    }
    if constexpr (TAIL) {
        float r = kNearestOffset32;
        if constexpr (ROUND == AQSGD_ROUND_STOCHASTIC) {             // the entry's own draw (word j mod 4 of block j / 4)
            const uint64_t j = static_cast<uint64_t>(e0) + static_cast<uint64_t>(tail_j);
            uint32_t w[4];
            philox4x32_10(static_cast<uint32_t>(j >> 2), static_cast<uint32_t>(j >> 34),
                          static_cast<uint32_t>(a.seed), static_cast<uint32_t>(a.seed >> 32), w);
            const uint32_t sel = static_cast<uint32_t>(j) & 3u;
            r = offset32_from_word(sel == 0 ? w[0] : (sel == 1 ? w[1] : (sel == 2 ? w[2] : w[3])));
        }
        const float q = level_of<kTopkBits, ROUND>(tail_f, sc, r);
        const uint64_t km = __ballot(tail_keep);         // bit l: lane l's entry, which is entry 64 * 8 * CPL + l
        if (tail_keep)
            lds.stage[row_start + static_cast<uint32_t>(lanes_set_below(km))] =
                static_cast<uint8_t>(__builtin_amdgcn_cvt_pk_u8_f32(q, 0, 0));
        if (lane < tail_entries / kChunk)
            a.bitmap[e0 / kChunk + CPL * kWave + lane] = static_cast<uint8_t>(km >> (8 * lane));
    }

    // ---- the group's bytes leave LDS ------------------------------------------------------
    wave_lds_sync();
    uint8_t* dst = a.codes + g * a.keep;
    if (a.keep % 16 == 0) {
        for (int i = lane; i < a.keep / 16; i += kWave)
            *reinterpret_cast<u32x4_t*>(dst + 16 * i) = *reinterpret_cast<const u32x4_t*>(lds.stage + 16 * i);
    } else {
        for (int i = lane; i < a.keep; i += kWave) dst[i] = lds.stage[i];
    }
    if (lane == 0) a.scales[g] = sc.s_tx;
    wave_lds_sync();                                     // the next group reuses the staging bytes
}

template <int DT, int CPL>
__device__ __forceinline__ void topk_dequant_group(const TopkArgs& a, int64_t g, const uint32_t (&cc)[CPL],
                                                   const bool (&valid)[CPL], int lane, TopkLds& lds) {
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
            *reinterpret_cast<u32x4_t*>(lds.stage + 16 * i) = *reinterpret_cast<const u32x4_t*>(src + 16 * i);
    } else {
        for (int i = lane; i < a.keep; i += kWave) lds.stage[i] = src[i];
    }
    wave_lds_sync();

    const GroupScale sc = scale_from_wire<kTopkBits>(s_tx);
    uint32_t kept[CPL], kept_below[CPL], kept_total[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        if (!valid[k]) bm[k] = 0;
        kept[k] = __builtin_popcount(bm[k]);
    }
    lanes_before<CPL>(kept, lane, kept_below, kept_total);
    uint32_t row_start = 0;
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        uint32_t pos = row_start + kept_below[k];
        float x[kChunk];
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
            const uint32_t on = (bm[k] >> e) & 1u;
            // pos never passes the number of set bits of the group (<= G), so the read stays
            // inside the staging bytes even for a bitmap that disagrees with `keep`
            const float v = value_of(static_cast<float>(lds.stage[pos]), sc);
            x[e] = on ? v : 0.0f;
            pos += on;
        }
        if (valid[k]) store_raw_at<DT>(dst + cc[k] * kChunkBytes, pack_raw<DT>(x));
        row_start += kept_total[k];
    }
    wave_lds_sync();
}

// Workgroups are handed to the chip's eight XCDs in turn (workgroup b runs on XCD b % 8),
// each with its own L2.  A group's bitmap and code bytes do not fill whole cache lines,
// so neighbouring groups share lines: the numbering below gives every XCD one contiguous
// run of the launch's workgroup slots, which keeps the two halves of such a line in one L2
// (written back once) instead of in two.  A bijection of [0, n_blocks) for any n_blocks.
constexpr uint32_t kXcds = 8;
__device__ __forceinline__ uint32_t xcd_contiguous_slot(uint32_t block, uint32_t n_blocks) {
    const uint32_t xcd = block % kXcds, turn = block / kXcds;
    const uint32_t base = n_blocks / kXcds, extra = n_blocks % kXcds;     // the first `extra` XCDs get one more
    return xcd * base + min(xcd, extra) + turn;
}

// MODE: 0 receiver, 1 sender with nearest rounding, 2 sender with stochastic rounding.
template <int DT, int CPL, int MODE>
__global__ __launch_bounds__(kTopkBlock)
void topk_kernel(const TopkArgs a) {
    constexpr int kWaves = kTopkBlock / kWave;
    __shared__ __align__(16) TopkLds lds_all[kWaves];

    const int lane = threadIdx.x % kWave;
    const int wave = kWaves == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t slot = xcd_contiguous_slot(blockIdx.x, gridDim.x);
    uint32_t cc[CPL];
    bool valid[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        const int c = k * kWave + lane;
        valid[k] = c < a.cpg;
        cc[k] = static_cast<uint32_t>(min(c, a.cpg - 1));
    }
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kWaves;
    int64_t g = static_cast<int64_t>(slot) * kWaves + wave;
    if constexpr (MODE == 1 && KeyBytes<DT>::value == 2) {
        // The loads of the wave's first group go out before anything else: a launch is one
        // round of waves that all start by waiting for memory, and whatever does not depend
        // on the data (lane constants, clearing counters) is then worked off during that wait.
        if (g >= a.n_groups) return;
        if constexpr (CPL >= 2) {
            // a last round of at most eight chunks is taken as one entry per lane (see above)
            constexpr int kRounds = CPL - 1;
            const int tail_chunks = a.cpg - kRounds * kWave;
            if (tail_chunks >= 1 && tail_chunks <= 8) {              // uniform over the launch
                uint32_t rc[kRounds];
                bool all[kRounds];
#pragma unroll
                for (int k = 0; k < kRounds; ++k) {
                    rc[k] = static_cast<uint32_t>(k * kWave + lane);
                    all[k] = true;
                }
                const bool tail_valid = lane < kChunk * tail_chunks;
                const int64_t tail_at = 2 * (kRounds * kWave * kChunk + min(lane, kChunk * tail_chunks - 1));
                auto tail_of = [&](int64_t group) {
                    return static_cast<uint32_t>(*reinterpret_cast<const uint16_t*>(
                        static_cast<const char*>(a.grad) + group * a.group * 2 + tail_at));
                };
                Raw<DT> raw[kRounds];
                load_group16<DT, kRounds>(a, g, rc, raw);
                uint32_t tail_raw = tail_of(g);
                __builtin_amdgcn_sched_barrier(0);
                for (;;) {
                    topk_quant_group16<DT, kRounds, true>(a, g, raw, tail_raw, tail_valid, rc, all, lane, lds_all[wave]);
                    g += stride;
                    if (g >= a.n_groups) break;
                    load_group16<DT, kRounds>(a, g, rc, raw);
                    tail_raw = tail_of(g);
                }
                return;
            }
        }
        Raw<DT> raw[CPL];
        load_group16<DT, CPL>(a, g, cc, raw);
        __builtin_amdgcn_sched_barrier(0);
        for (;;) {
            topk_quant_group16<DT, CPL, false>(a, g, raw, 0u, false, cc, valid, lane, lds_all[wave]);
            g += stride;
            if (g >= a.n_groups) break;
            load_group16<DT, CPL>(a, g, cc, raw);
        }
    } else {
        if constexpr (MODE != 0 && CPL >= 2) {
            // the general sender (binary32 entries, stochastic rounding): the same last round as single entries
            constexpr int kRounds = CPL - 1;
            constexpr int kRound = MODE == 2 ? AQSGD_ROUND_STOCHASTIC : AQSGD_ROUND_NEAREST;
            const int tail_chunks = a.cpg - kRounds * kWave;
            if (tail_chunks >= 1 && tail_chunks <= 8) {              // uniform over the launch
                uint32_t rc[kRounds];
                bool all[kRounds];
#pragma unroll
                for (int k = 0; k < kRounds; ++k) {
                    rc[k] = static_cast<uint32_t>(k * kWave + lane);
                    all[k] = true;
                }
                for (; g < a.n_groups; g += stride)
                    topk_quant_group<DT, kRounds, kRound, true>(a, g, rc, all, lane, lds_all[wave], kChunk * tail_chunks);
                return;
            }
        }
        for (; g < a.n_groups; g += stride) {
            if constexpr (MODE == 1) topk_quant_group<DT, CPL, AQSGD_ROUND_NEAREST, false>(a, g, cc, valid, lane, lds_all[wave]);
            else if constexpr (MODE == 2) topk_quant_group<DT, CPL, AQSGD_ROUND_STOCHASTIC, false>(a, g, cc, valid, lane, lds_all[wave]);
            else topk_dequant_group<DT, CPL>(a, g, cc, valid, lane, lds_all[wave]);
        }
    }
}

// chunks per lane: 1, 2, 3 or 4 (groups of up to 512, 1024, 1536, 2048 entries)
hipError_t launch_topk(int dtype, int cpl, bool sender, unsigned blocks, const TopkArgs& a, hipStream_t stream);

}  // namespace aqsgd

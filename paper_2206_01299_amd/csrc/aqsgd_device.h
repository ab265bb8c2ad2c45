// Device-side building blocks of the AQ-SGD boundary codec for gfx950 (CDNA4).
//
// Work is organised in "chunks" of 8 consecutive elements: 16 bytes of
// float16/bfloat16 (one 128-bit access per lane, fully coalesced across a
// wavefront) or 32 bytes of float32.  Eight b-bit codes are b whole bytes, so a
// lane's codes never share a byte with a neighbour's.  The main kernels hold a
// float32 lane's eight elements as two separate 16-byte units instead (end of
// this file), which gives float32 the same access shape as the 16-bit types.
//
// All arithmetic is binary32 with one rounding per operation (the translation
// unit is compiled with floating-point contraction off); the order of the
// operations below is part of the wire format: sender, receiver and any other
// implementation must round in the same places to stay bit-identical.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "aqsgd.h"

namespace aqsgd {

constexpr int kChunk = 8;          // elements per lane-chunk
constexpr int kWave = 64;          // CDNA wavefront

// ---------------------------------------------------------------------------
// Storage formats
// ---------------------------------------------------------------------------
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <int DT> struct ElemBytes { static constexpr int value = 2; };
template <> struct ElemBytes<AQSGD_F32> { static constexpr int value = 4; };

// One chunk as it sits in memory.
template <int DT> struct Raw { u32x4_t v; };
template <> struct Raw<AQSGD_F32> { f32x4_t lo, hi; };

// One chunk from / to a byte address.
template <int DT>
__device__ __forceinline__ Raw<DT> load_raw_at(const char* p) {
    Raw<DT> r;
    if constexpr (DT == AQSGD_F32) {
        const f32x4_t* q = reinterpret_cast<const f32x4_t*>(p);
        r.lo = __builtin_nontemporal_load(q);
        r.hi = __builtin_nontemporal_load(q + 1);
    } else {
        r.v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    }
    return r;
}

// A 16-byte streaming store that is also written through the L2 at system scope (nt with
// sc0 sc1).  The launches here end with tens of MB of freshly written lines, and lines
// that only stream (nt) still wait in the eight L2s for the write-back at the end of the
// kernel; written through, they leave while the kernel is still reading.  Measured on the
// GPT2 boundary: forward pair in the pipelined schedule 13.9-14.2 -> 13.3-13.4 us, DeBERTa
// step 36.7 -> 35.6 us.  The compiler has no spelling for this combination on a 16-byte
// store, so the instruction is written out; the data registers of a store of more than
// eight bytes must not be overwritten in the next two cycles, which the compiler's hazard
// pass cannot see through the asm statement, hence the s_nop.
template <typename V>
__device__ __forceinline__ void store16_through(void* p, const V& v) {
    static_assert(sizeof(V) == 16, "one 16-byte piece");
#if defined(AQSGD_PLAIN_STREAMING_STORES)
    __builtin_nontemporal_store(v, reinterpret_cast<V*>(p));
#else
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 2" : : "v"(p), "v"(v) : "memory");
#endif
}

// A float32 chunk is two 16-byte stores per lane, 32 bytes apart between lanes:
// each instruction fills half of every cache line.  Streaming (nontemporal)
// stores of that shape reach 2.4 TB/s, ordinary stores, which L2 merges, 6.6;
// the contiguous 16-byte-per-lane stores of the 16-bit types stream at full rate.
template <int DT>
__device__ __forceinline__ void store_raw_at(char* p, const Raw<DT>& r) {
    if constexpr (DT == AQSGD_F32) {
        f32x4_t* q = reinterpret_cast<f32x4_t*>(p);
        q[0] = r.lo;
        q[1] = r.hi;
    } else {
        store16_through(p, r.v);
    }
}

template <int DT>
__device__ __forceinline__ Raw<DT> zero_raw() {
    Raw<DT> r;
    if constexpr (DT == AQSGD_F32) { r.lo = f32x4_t{0, 0, 0, 0}; r.hi = r.lo; }
    else { r.v = u32x4_t{0, 0, 0, 0}; }
    return r;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// binary32 -> bfloat16, round to nearest even (the top 16 bits of the pattern,
// rounded on the lower 16; a carry walks into the exponent as it should).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Two binary32 -> two bfloat16 in one register with gfx950's packed convert (round
// to nearest even; checked equal to f32_to_bf16_bits on all 2^32 inputs).
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
    uint32_t r;
    asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
    return r;
}

template <int DT>
__device__ __forceinline__ void unpack_raw(const Raw<DT>& r, float (&f)[kChunk]) {
    if constexpr (DT == AQSGD_F32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) { f[e] = r.lo[e]; f[4 + e] = r.hi[e]; }
    } else if constexpr (DT == AQSGD_F16) {
        half8_t h = __builtin_bit_cast(half8_t, r.v);
#pragma unroll
        for (int e = 0; e < kChunk; ++e) f[e] = static_cast<float>(h[e]);   // exact
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[2 * e] = bf16_bits_to_f32(r.v[e] & 0xffffu);
            f[2 * e + 1] = __uint_as_float(r.v[e] & 0xffff0000u);
        }
    }
}

template <int DT>
__device__ __forceinline__ Raw<DT> pack_raw(const float (&f)[kChunk]) {
    Raw<DT> r;
    if constexpr (DT == AQSGD_F32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) { r.lo[e] = f[e]; r.hi[e] = f[4 + e]; }
    } else if constexpr (DT == AQSGD_F16) {
        half8_t h;
#pragma unroll
        for (int e = 0; e < kChunk; ++e) h[e] = static_cast<_Float16>(f[e]);  // RNE
        r.v = __builtin_bit_cast(u32x4_t, h);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) r.v[e] = f32x2_to_bf16x2(f[2 * e], f[2 * e + 1]);
    }
    return r;
}

// float16 operands enter binary32 arithmetic through v_fma_mix_f32, which widens
// a half (low or high 16 bits of a register) on the fly: x * 1.0 + y is exact in
// the product and rounds the sum once, so it is the same binary32 add/subtract,
// without a separate conversion instruction per operand.
__device__ __forceinline__ float f16lo_minus_f16lo(uint32_t a, uint32_t m) {
    float d;
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel_hi:[1,0,1]" : "=v"(d) : "v"(a), "v"(m));
    return d;
}
__device__ __forceinline__ float f16hi_minus_f16hi(uint32_t a, uint32_t m) {
    float d;
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[1,0,1] op_sel_hi:[1,0,1]" : "=v"(d) : "v"(a), "v"(m));
    return d;
}
__device__ __forceinline__ float f32_plus_f16lo(float x, uint32_t m) {
    float d;
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel_hi:[0,0,1]" : "=v"(d) : "v"(x), "v"(m));
    return d;
}
__device__ __forceinline__ float f32_plus_f16hi(float x, uint32_t m) {
    float d;
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[0,0,1] op_sel_hi:[0,0,1]" : "=v"(d) : "v"(x), "v"(m));
    return d;
}

__device__ __forceinline__ float f16lo_minus_f32(uint32_t a, float m) {
    float d;
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel_hi:[1,0,0]" : "=v"(d) : "v"(a), "v"(m));
    return d;
}
__device__ __forceinline__ float f16hi_minus_f32(uint32_t a, float m) {
    float d;
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(a), "v"(m));
    return d;
}

// d[e] = binary32(a[e]) - m[e] for one chunk, m already in binary32.
template <int DT>
__device__ __forceinline__ void delta_from_values(const Raw<DT>& a, const float (&m)[kChunk], float (&d)[kChunk]) {
    if constexpr (DT == AQSGD_F16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            d[2 * e] = f16lo_minus_f32(a.v[e], m[2 * e]);
            d[2 * e + 1] = f16hi_minus_f32(a.v[e], m[2 * e + 1]);
        }
    } else {
        float av[kChunk];
        unpack_raw<DT>(a, av);
#pragma unroll
        for (int e = 0; e < kChunk; ++e) d[e] = av[e] - m[e];
    }
}

// d[e] = binary32(a[e]) - binary32(m[e]) for one chunk.
template <int DT>
__device__ __forceinline__ void delta_chunk(const Raw<DT>& a, const Raw<DT>& m, float (&d)[kChunk]) {
    if constexpr (DT == AQSGD_F16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            d[2 * e] = f16lo_minus_f16lo(a.v[e], m.v[e]);
            d[2 * e + 1] = f16hi_minus_f16hi(a.v[e], m.v[e]);
        }
    } else {
        float av[kChunk], mv[kChunk];
        unpack_raw<DT>(a, av);
        unpack_raw<DT>(m, mv);
#pragma unroll
        for (int e = 0; e < kChunk; ++e) d[e] = av[e] - mv[e];
    }
}

// storage(binary32(m[e]) + x[e]) for one chunk.
template <int DT>
__device__ __forceinline__ Raw<DT> updated_chunk(const Raw<DT>& m, const float (&x)[kChunk]) {
    float s[kChunk];
    if constexpr (DT == AQSGD_F16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            s[2 * e] = f32_plus_f16lo(x[2 * e], m.v[e]);
            s[2 * e + 1] = f32_plus_f16hi(x[2 * e + 1], m.v[e]);
        }
    } else {
        float mv[kChunk];
        unpack_raw<DT>(m, mv);
#pragma unroll
        for (int e = 0; e < kChunk; ++e) s[e] = mv[e] + x[e];
    }
    return pack_raw<DT>(s);
}

// Scalar element access for the any-shape fallback kernels.
template <int DT>
__device__ __forceinline__ float load_elem(const void* base, int64_t idx) {
    if constexpr (DT == AQSGD_F32) return static_cast<const float*>(base)[idx];
    else if constexpr (DT == AQSGD_F16) return static_cast<float>(static_cast<const _Float16*>(base)[idx]);
    else return bf16_bits_to_f32(static_cast<const uint16_t*>(base)[idx]);
}

template <int DT>
__device__ __forceinline__ void store_elem(void* base, int64_t idx, float v) {
    if constexpr (DT == AQSGD_F32) static_cast<float*>(base)[idx] = v;
    else if constexpr (DT == AQSGD_F16) static_cast<_Float16*>(base)[idx] = static_cast<_Float16>(v);
    else static_cast<uint16_t*>(base)[idx] = static_cast<uint16_t>(f32_to_bf16_bits(v));
}

// A call's sample ids are its input: nothing writes them while a kernel of the call runs.
// Reading them as constant memory lets the compiler fetch an id with a scalar load (the
// index is the same for every lane), which comes back sooner than a vector load does and
// needs no readfirstlane; the row's loads can only be issued once the id is there.
__device__ __forceinline__ int64_t sample_id(const int64_t* ids, int64_t i) {
    typedef const int64_t __attribute__((address_space(4))) * constant_ids;
    return reinterpret_cast<constant_ids>(reinterpret_cast<uintptr_t>(ids))[i];
}

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): counter-based, so element j of a call
// gets the same draw whatever lane, wave or launch shape computes it.
// ---------------------------------------------------------------------------
// a ^ b ^ c in one instruction (v_bitop3_b32 with the truth table of a three-input xor;
// the compiler does not form it from two xors by itself).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1,
                                              uint32_t (&out)[4]) {
    uint32_t c2 = 0u, c3 = 0u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c0;
        const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c2;
        const uint32_t n0 = xor3(static_cast<uint32_t>(p1 >> 32), c1, k0);
        const uint32_t n1 = static_cast<uint32_t>(p1);
        const uint32_t n2 = xor3(static_cast<uint32_t>(p0 >> 32), c3, k1);
        const uint32_t n3 = static_cast<uint32_t>(p0);
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ __forceinline__ float uniform_from_word(uint32_t w) {
    return static_cast<float>(w >> 8) * 0x1p-24f;      // 24 bits: exact in binary32
}

// The vector kernels carry a rounding offset r as r * 2^32, which for the uniform
// draw is the Philox word with its low byte cleared (24 significant bits: exact in
// binary32) and for nearest rounding 2^31.  level_of() adds it to t with one fused
// multiply-add, RN(r32 * 2^-32 + t): the product is exact, so this is the single
// rounding of t + r that the wire format prescribes, without forming r first.
constexpr float kNearestOffset32 = 0x1p31f;
__device__ __forceinline__ float offset32_from_word(uint32_t w) {
    return static_cast<float>(w & 0xffffff00u);
}

// Rounding offsets (times 2^32) of one chunk whose first element has flat index j0
// (a multiple of 8): block j0/4 feeds elements 0..3, block j0/4 + 1 elements 4..7.
__device__ __forceinline__ void chunk_uniforms(uint64_t seed, uint64_t j0, float (&r)[kChunk]) {
    const uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
    const uint64_t blk = j0 >> 2;
    uint32_t w[4];
    philox4x32_10(static_cast<uint32_t>(blk), static_cast<uint32_t>(blk >> 32), k0, k1, w);
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = offset32_from_word(w[e]);
    const uint64_t blk1 = blk + 1;
    philox4x32_10(static_cast<uint32_t>(blk1), static_cast<uint32_t>(blk1 >> 32), k0, k1, w);
#pragma unroll
    for (int e = 0; e < 4; ++e) r[4 + e] = offset32_from_word(w[e]);
}

// ---------------------------------------------------------------------------
// Max over the TEAM consecutive lanes a lane belongs to (TEAM = 1..64, power of
// two).  The first four steps are DPP lane permutations inside a 16-lane row;
// the last two cross rows through ds_bpermute.  The values are magnitudes, so
// their bit patterns order like unsigned integers and the reduction runs on
// those (an integer max has no NaN quieting to do and fuses with the DPP move).
// Max is exact and order-free, so any tree gives the same bits.
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_max_step(uint32_t v) {
    const uint32_t other = static_cast<uint32_t>(
        __builtin_amdgcn_update_dpp(static_cast<int>(v), static_cast<int>(v), CTRL, 0xf, 0xf, false));
    return max(v, other);
}

template <int TEAM>
__device__ __forceinline__ float team_max(float magnitude) {
    uint32_t v = __float_as_uint(magnitude);
    if constexpr (TEAM >= 2) v = dpp_max_step<0xB1>(v);     // quad_perm [1,0,3,2]
    if constexpr (TEAM >= 4) v = dpp_max_step<0x4E>(v);     // quad_perm [2,3,0,1]
    if constexpr (TEAM >= 8) v = dpp_max_step<0x141>(v);    // row_half_mirror
    if constexpr (TEAM >= 16) v = dpp_max_step<0x140>(v);   // row_mirror
    if constexpr (TEAM >= 32) v = max(v, static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), 16, kWave)));
    if constexpr (TEAM >= 64) v = max(v, static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), 32, kWave)));
    return __uint_as_float(v);
}

// ---------------------------------------------------------------------------
// The quantiser Q on values held in registers.
// ---------------------------------------------------------------------------
template <int BITS> struct Levels {
    static constexpr int top = (1 << BITS) - 1;                         // L
    static constexpr float half = static_cast<float>((1 << BITS) - 1) / 2.0f;   // L/2, exact
};

// Per-group constants.  A group whose max-abs is below 2^-120 sends scale 0,
// level 0 everywhere and reconstructs +0: with inv = offset = step = 0 the
// element formulas below give exactly that (0*d + 0 + r < 1 -> level 0;
// (0 - 0) * 0 = +0), so the per-element code carries no special case.
struct GroupScale {
    float s_tx;     // transmitted scale (0 = nothing to send)
    float inv;      // (L/2) / s
    float offset;   // L/2: position of value 0 on the level axis
    float step;     // s / (L/2): level spacing
};

template <int BITS>
__device__ __forceinline__ GroupScale make_scale(float max_abs) {
    GroupScale g;
    const bool live = !(max_abs < 0x1p-120f);
    const float denom = live ? max_abs : 1.0f;           // keep the divisions finite
    const float inv = Levels<BITS>::half / denom;        // IEEE-rounded divisions
    const float step = denom / Levels<BITS>::half;
    g.s_tx = live ? max_abs : 0.0f;
    g.inv = live ? inv : 0.0f;
    g.offset = live ? Levels<BITS>::half : 0.0f;
    g.step = live ? step : 0.0f;
    return g;
}

// Receiver's view: the same constants from the transmitted scale.
template <int BITS>
__device__ __forceinline__ GroupScale scale_from_wire(float s_tx) {
    GroupScale g;
    const bool live = s_tx != 0.0f;
    g.s_tx = s_tx;
    g.inv = 0.0f;
    g.offset = live ? Levels<BITS>::half : 0.0f;
    g.step = live ? s_tx / Levels<BITS>::half : 0.0f;
    return g;
}

// Level of one value, kept as a float (an exact small integer); the rounding offset
// r = 1/2 (nearest, ties upwards) or U[0,1) arrives as r32 = r * 2^32 (see above).
// y = ((d * inv) + L/2) + r is never below -2^-20, so rounding towards zero is
// floor() followed by the clamp at 0 (a result of -0 counts as level 0 in all
// that follows).  With r = 1/2, |d| <= s bounds y below L + 1, so no upper clamp
// is needed; a stochastic r can reach L + 1.
template <int BITS, int ROUND>
__device__ __forceinline__ float level_of(float d, const GroupScale& g, float r32) {
    float t = d * g.inv;
    t = t + g.offset;
    if constexpr (ROUND == AQSGD_ROUND_STOCHASTIC) {
        const float y = __builtin_fmaf(r32, 0x1p-32f, t);          // RN(t + r): the product is exact
        return __builtin_fminf(__builtin_truncf(y), static_cast<float>(Levels<BITS>::top));
    } else {
        return __builtin_truncf(t + 0.5f);
    }
}

__device__ __forceinline__ float value_of(float level, const GroupScale& g) {
    return (level - g.offset) * g.step;
}

// Eight levels -> 8*BITS bits, element e at bits [e*BITS, e*BITS + BITS).
// The levels are small integers held in floats, so up to 24 bits of the stream
// are assembled exactly in binary32 (level * 2^shift added up: every partial sum
// is an integer below 2^24) and converted once, instead of one conversion and
// one shift-or per element.  Eight-bit levels go through v_cvt_pk_u8_f32, which
// converts and places a byte in one step.
template <int BITS>
__device__ __forceinline__ uint64_t pack_levels(const float (&q)[kChunk]) {
    if constexpr (BITS == 8) {
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            lo = __builtin_amdgcn_cvt_pk_u8_f32(q[e], e, lo);
            hi = __builtin_amdgcn_cvt_pk_u8_f32(q[4 + e], e, hi);
        }
        return (static_cast<uint64_t>(hi) << 32) | lo;
    } else if constexpr (BITS == 4 || BITS == 6) {  // two halves of 16 or 24 bits
        float lo = q[0], hi = q[4];
#pragma unroll
        for (int e = 1; e < 4; ++e) {
            lo = __builtin_fmaf(q[e], static_cast<float>(1 << (BITS * e)), lo);
            hi = __builtin_fmaf(q[4 + e], static_cast<float>(1 << (BITS * e)), hi);
        }
        return (static_cast<uint64_t>(static_cast<uint32_t>(hi)) << (4 * BITS)) | static_cast<uint32_t>(lo);
    } else {                                         // 2 or 3 bits: 16 or 24 bits in all
        float w = q[0];
#pragma unroll
        for (int e = 1; e < kChunk; ++e) w = __builtin_fmaf(q[e], static_cast<float>(1 << (BITS * e)), w);
        return static_cast<uint32_t>(w);
    }
}

// The inverse: eight levels as floats.
template <int BITS>
__device__ __forceinline__ void unpack_levels(uint64_t w, float (&q)[kChunk]) {
    if constexpr (BITS == 8) {
        const uint32_t lo = static_cast<uint32_t>(w), hi = static_cast<uint32_t>(w >> 32);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            q[e] = static_cast<float>((lo >> (8 * e)) & 0xffu);         // v_cvt_f32_ubyteN
            q[4 + e] = static_cast<float>((hi >> (8 * e)) & 0xffu);
        }
    } else if constexpr (BITS == 4) {
        const uint32_t even = static_cast<uint32_t>(w) & 0x0f0f0f0fu;          // elements 0, 2, 4, 6
        const uint32_t odd = (static_cast<uint32_t>(w) >> 4) & 0x0f0f0f0fu;    // elements 1, 3, 5, 7
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            q[2 * b] = static_cast<float>((even >> (8 * b)) & 0xffu);
            q[2 * b + 1] = static_cast<float>((odd >> (8 * b)) & 0xffu);
        }
    } else if constexpr (BITS == 2) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {                // byte b of this word holds element 4*b + s
            const uint32_t m = (static_cast<uint32_t>(w) >> (2 * s)) & 0x0303u;
            q[s] = static_cast<float>(m & 0xffu);
            q[4 + s] = static_cast<float>((m >> 8) & 0xffu);
        }
    } else if constexpr (BITS == 6) {
        const uint32_t lo = static_cast<uint32_t>(w) & 0xffffffu, hi = static_cast<uint32_t>(w >> 24);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            q[e] = static_cast<float>((lo >> (6 * e)) & 63u);
            q[4 + e] = static_cast<float>((hi >> (6 * e)) & 63u);
        }
    } else {
#pragma unroll
        for (int e = 0; e < kChunk; ++e)
            q[e] = static_cast<float>((static_cast<uint32_t>(w) >> (BITS * e)) & Levels<BITS>::top);
    }
}

// Three-bit codes: a chunk is 3 bytes, so four neighbouring lanes own 12 bytes =
// three aligned dwords.  Lane j of the quad (j < 3) assembles dword j from its own
// 24 bits and the next lane's (one DPP quad permute), which turns three byte
// stores per lane into one dword store for three lanes out of four.  `w` holds the
// lane's 24 code bits; `quad_base` points at the first byte of the quad's 12.
__device__ __forceinline__ void store_codes3_quad(uint8_t* quad_base, uint32_t w, int j, bool live) {
    const uint32_t next = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(
        0, static_cast<int>(w), 0xF9 /* quad_perm [1,2,3,3] */, 0xf, 0xf, false));
    const uint32_t word = (w >> (8 * j)) | (next << (24 - 8 * j));     // j = 0, 1, 2
    if (live && j < 3) reinterpret_cast<uint32_t*>(quad_base)[j] = word;
}

// The inverse: lanes 0..2 of the quad load one dword each, every lane rebuilds its
// own 24 bits from its dword and the previous lane's.
__device__ __forceinline__ uint32_t load_codes3_quad(const uint8_t* quad_base, int j) {
    const uint32_t cur = j < 3 ? reinterpret_cast<const uint32_t*>(quad_base)[j] : 0u;
    const uint32_t prev = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(
        0, static_cast<int>(cur), 0x90 /* quad_perm [0,0,1,2] */, 0xf, 0xf, false));
    const uint64_t both = (static_cast<uint64_t>(cur) << 32) | prev;   // lane j starts at bit 32 - 8j
    return static_cast<uint32_t>(both >> (32 - 8 * j)) & 0xffffffu;
}

// Codes of one chunk to / from the byte stream; chunk c of the call starts at
// byte c * BITS.
template <int BITS>
__device__ __forceinline__ void store_codes_at(uint8_t* p, uint64_t w) {
    if constexpr (BITS == 8) {
        *reinterpret_cast<uint2*>(p) = make_uint2(static_cast<uint32_t>(w), static_cast<uint32_t>(w >> 32));
    } else if constexpr (BITS == 4) {
        *reinterpret_cast<uint32_t*>(p) = static_cast<uint32_t>(w);
    } else if constexpr (BITS == 2) {
        *reinterpret_cast<uint16_t*>(p) = static_cast<uint16_t>(w);
    } else if constexpr (BITS == 6) {                // 6 bytes, 2-byte aligned
        uint16_t* h = reinterpret_cast<uint16_t*>(p);
        h[0] = static_cast<uint16_t>(w);
        h[1] = static_cast<uint16_t>(w >> 16);
        h[2] = static_cast<uint16_t>(w >> 32);
    } else {
        p[0] = static_cast<uint8_t>(w);
        p[1] = static_cast<uint8_t>(w >> 8);
        p[2] = static_cast<uint8_t>(w >> 16);
    }
}

template <int BITS>
__device__ __forceinline__ uint64_t load_codes_at(const uint8_t* p) {
    if constexpr (BITS == 8) {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        return (static_cast<uint64_t>(v.y) << 32) | v.x;
    } else if constexpr (BITS == 4) {
        return *reinterpret_cast<const uint32_t*>(p);
    } else if constexpr (BITS == 2) {
        return *reinterpret_cast<const uint16_t*>(p);
    } else if constexpr (BITS == 6) {
        const uint16_t* h = reinterpret_cast<const uint16_t*>(p);
        return static_cast<uint64_t>(h[0]) | (static_cast<uint64_t>(h[1]) << 16) |
               (static_cast<uint64_t>(h[2]) << 32);
    } else {
        return static_cast<uint32_t>(p[0]) | (static_cast<uint32_t>(p[1]) << 8) |
               (static_cast<uint32_t>(p[2]) << 16);
    }
}

// ---------------------------------------------------------------------------
// float32 in 16-byte units.
//
// A float32 chunk is 32 bytes; taken as one piece per lane, each of its two
// 16-byte accesses touches every cache line of the wavefront's span and uses half
// of it.  Instead a lane's eight elements are two *units* of four that lie a team
// width apart, so that consecutive lanes access consecutive 16 bytes, as the
// 16-bit types do (measured on the float32 stress shape with encode's traffic:
// 6.3 instead of 5.2 TB/s).  Four b-bit codes are b/2 bytes, whole bytes for every
// width but 3, which keeps the one-piece layout.
// ---------------------------------------------------------------------------
constexpr int kUnit = 4;           // elements of a 16-byte float32 unit

template <int DT, int BITS> struct UnitLayout {
    static constexpr bool value = DT == AQSGD_F32 && BITS != 3;
};

__device__ __forceinline__ Raw<AQSGD_F32> load_raw_units(const char* pa, const char* pb) {
    Raw<AQSGD_F32> r;
    r.lo = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(pa));
    r.hi = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(pb));
    return r;
}

__device__ __forceinline__ void store_raw_units(char* pa, char* pb, const Raw<AQSGD_F32>& r) {
    store16_through(pa, r.lo);
    store16_through(pb, r.hi);
}

// The two halves of pack_levels' word: levels 0..3 and 4..7, 4*BITS bits each.
template <int BITS>
__device__ __forceinline__ uint32_t low_unit_codes(uint64_t w) {
    return static_cast<uint32_t>(w) & static_cast<uint32_t>((uint64_t{1} << (4 * BITS)) - 1);
}
template <int BITS>
__device__ __forceinline__ uint32_t high_unit_codes(uint64_t w) {
    return static_cast<uint32_t>(w >> (4 * BITS));
}

// Codes of one unit to / from the byte stream; unit u of the call starts at byte
// u * BITS / 2.
template <int BITS>
__device__ __forceinline__ void store_unit_codes(uint8_t* p, uint32_t w) {
    static_assert(BITS == 2 || BITS == 4 || BITS == 6 || BITS == 8, "whole bytes per unit");
    if constexpr (BITS == 8) {
        *reinterpret_cast<uint32_t*>(p) = w;
    } else if constexpr (BITS == 4) {
        *reinterpret_cast<uint16_t*>(p) = static_cast<uint16_t>(w);
    } else if constexpr (BITS == 2) {
        p[0] = static_cast<uint8_t>(w);
    } else {                                         // 3 bytes, no alignment to rely on
        p[0] = static_cast<uint8_t>(w);
        p[1] = static_cast<uint8_t>(w >> 8);
        p[2] = static_cast<uint8_t>(w >> 16);
    }
}

template <int BITS>
__device__ __forceinline__ uint32_t load_unit_codes(const uint8_t* p) {
    static_assert(BITS == 2 || BITS == 4 || BITS == 6 || BITS == 8, "whole bytes per unit");
    if constexpr (BITS == 8) {
        return *reinterpret_cast<const uint32_t*>(p);
    } else if constexpr (BITS == 4) {
        return *reinterpret_cast<const uint16_t*>(p);
    } else if constexpr (BITS == 2) {
        return p[0];
    } else {
        return static_cast<uint32_t>(p[0]) | (static_cast<uint32_t>(p[1]) << 8) |
               (static_cast<uint32_t>(p[2]) << 16);
    }
}

// Rounding offsets (times 2^32) of two units whose first elements have flat indices
// ja and jb (multiples of 4): one Philox block each.
__device__ __forceinline__ void units_uniforms(uint64_t seed, uint64_t ja, uint64_t jb, float (&r)[kChunk]) {
    const uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
    const uint64_t blka = ja >> 2, blkb = jb >> 2;
    uint32_t w[4];
    philox4x32_10(static_cast<uint32_t>(blka), static_cast<uint32_t>(blka >> 32), k0, k1, w);
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = offset32_from_word(w[e]);
    philox4x32_10(static_cast<uint32_t>(blkb), static_cast<uint32_t>(blkb >> 32), k0, k1, w);
#pragma unroll
    for (int e = 0; e < 4; ++e) r[4 + e] = offset32_from_word(w[e]);
}

}  // namespace aqsgd

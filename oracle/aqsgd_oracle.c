/*
 * CPU oracle for the AQ-SGD stage-boundary codec.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, scalar C that follows the method
 * step by step so it can be read against the paper.  It shares no code with
 * the HIP library and must never be called from the product path; only the
 * tests, the smoke check and the CPU-baseline leg of the benchmark use it.
 *
 * What it computes
 *   - Sender and receiver sides of the forward message (Algorithm 2, the
 *     blocks for network a and for network b; Algorithm 1's update of m):
 *         delta   = a(xi) - m(xi)
 *         Delta m = Q(delta)
 *         m(xi)  <- m(xi) + Delta m          (identically on both machines)
 *   - The backward message Q(grad) and its reconstruction (Algorithm 1,
 *     the two comment lines in which machine b returns Q(grad)).
 *   - Q itself (Section 4.1): a vector is scaled into [-1, 1] and each entry
 *     becomes a b-bit integer on a uniform partition of that interval; with
 *     stochastic rounding as an option because Theorem 3.1 asks for an
 *     unbiased Q (the example in its footnote rounds at random).
 *
 * Readings taken where the paper leaves room (each is also listed in the
 * design notes of this repository):
 *   - the normaliser is the max-abs of a group of G consecutive elements;
 *   - the 2^b levels are equally spaced points on [-s, s], both ends included
 *     (spacing 2s/(2^b-1)), so the nearest-rounding error is <= s/(2^b-1);
 *   - nearest rounding resolves ties upwards (floor(x + 1/2)) so that both
 *     rounding modes are floor(x + r) with r = 1/2 or r ~ U[0,1);
 *   - m starts at zero, so the first visit of a sample is direct quantisation;
 *   - a group whose max-abs is below 2^-120 is sent as scale 0 / codes 0;
 *   - m is kept in the activation's own dtype; the sum m + Delta m is formed
 *     in binary32 and rounded to nearest-even once when stored;
 *   - random numbers: Philox4x32-10 (Salmon et al., SC'11), counter = index
 *     of the 4-element block within the call, key = the call's seed.
 *
 * Arithmetic: IEEE-754 binary32, round-to-nearest-even, one rounding per
 * written operation, no contraction into FMA, subnormals kept.  Build with
 *     gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math
 *
 * Parity pins (tests/test_oracle_*.py): half/bfloat conversions against
 * numpy/torch; Philox against the published known-answer vectors; the bit
 * stream against Python big-integer arithmetic; the level decision against
 * exact rational arithmetic; the hand-worked two-visit example; the paper's
 * invariants (first visit = direct quantisation, replica identity, error
 * bound, unbiasedness, contraction, message size); the uncompressed first
 * visit and the low-precision storage of m (end of this file) against their
 * own invariants and the appendix's ordering of errors; the sparsified
 * backward message against the definition of "k largest", the dense message
 * at keep = G and crafted ties; Algorithm 1's first-visit branch against
 * "uncompressed on both machines", the plain encoder on seen samples and
 * replica identity.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_BF16 = 2 };
enum { ORACLE_NEAREST = 0, ORACLE_STOCHASTIC = 1 };

/* ------------------------------------------------------------------ */
/* Storage formats, written from the IEEE-754 definitions.             */
/* ------------------------------------------------------------------ */
static uint32_t f32_bits(float x) { uint32_t u; memcpy(&u, &x, 4); return u; }
static float bits_f32(uint32_t u) { float x; memcpy(&x, &u, 4); return x; }

/* v / 2^shift rounded to the nearest integer, ties to the even one. */
static uint64_t rne_shift(uint64_t v, int shift)
{
    if (shift <= 0) return v << (-shift);
    if (shift > 62) return 0;
    uint64_t kept = v >> shift;
    uint64_t rest = v & ((1ull << shift) - 1);
    uint64_t half = 1ull << (shift - 1);
    if (rest > half || (rest == half && (kept & 1))) kept += 1;
    return kept;
}

float aqsgd_oracle_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    int exp = (h >> 10) & 0x1f;
    uint32_t man = h & 0x3ff;
    if (exp == 0) {                      /* zero or subnormal: man * 2^-24 */
        float mag = (float)man * 0x1p-24f;
        return bits_f32(sign | f32_bits(mag));
    }
    if (exp == 31)                       /* inf / nan */
        return bits_f32(sign | 0x7f800000u | (man << 13));
    return bits_f32(sign | ((uint32_t)(exp - 15 + 127) << 23) | (man << 13));
}

uint16_t aqsgd_oracle_float_to_half(float x)
{
    uint32_t u = f32_bits(x);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000);
    int bexp = (u >> 23) & 0xff;
    uint32_t frac = u & 0x7fffff;
    if (bexp == 0xff)                    /* inf / nan */
        return (uint16_t)(sign | 0x7c00 | (frac ? (0x200 | (frac >> 13)) : 0));
    if (bexp == 0) return sign;          /* |x| < 2^-126: far below half's range */
    int e = bexp - 127;                  /* |x| = sig * 2^(e-23), sig in [2^23, 2^24) */
    uint64_t sig = frac | 0x800000u;
    uint32_t mag;
    if (e >= -14) {
        /* normal half: 11 significant bits */
        uint64_t m = rne_shift(sig, 13);             /* in [2^10, 2^11] */
        mag = ((uint32_t)(e + 15) << 10) + (uint32_t)(m - 1024);
        if (mag >= 0x7c00) mag = 0x7c00;             /* overflow to infinity */
    } else {
        /* subnormal half: integer multiple of 2^-24 */
        mag = (uint32_t)rne_shift(sig, 13 + (-14 - e));  /* in [0, 2^10] */
    }
    return (uint16_t)(sign | mag);
}

float aqsgd_oracle_bf16_to_float(uint16_t b) { return bits_f32((uint32_t)b << 16); }

uint16_t aqsgd_oracle_float_to_bf16(float x)
{
    uint32_t u = f32_bits(x);
    uint32_t sign = u & 0x80000000u, mag = u & 0x7fffffffu;
    if (mag > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   /* nan */
    /* bfloat16 is binary32 cut to its top 16 bits; both formats are monotone
       in their magnitude bits, so rounding the integer rounds the value. */
    return (uint16_t)((sign >> 16) | (uint32_t)rne_shift(mag, 16));
}

static float load_elem(const void* p, int64_t idx, int dtype)
{
    switch (dtype) {
    case ORACLE_F16:  return aqsgd_oracle_half_to_float(((const uint16_t*)p)[idx]);
    case ORACLE_BF16: return aqsgd_oracle_bf16_to_float(((const uint16_t*)p)[idx]);
    default:          return ((const float*)p)[idx];
    }
}

static void store_elem(void* p, int64_t idx, int dtype, float v)
{
    switch (dtype) {
    case ORACLE_F16:  ((uint16_t*)p)[idx] = aqsgd_oracle_float_to_half(v); break;
    case ORACLE_BF16: ((uint16_t*)p)[idx] = aqsgd_oracle_float_to_bf16(v); break;
    default:          ((float*)p)[idx] = v; break;
    }
}

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random         */
/* numbers: as easy as 1, 2, 3", SC'11).                               */
/* ------------------------------------------------------------------ */
void aqsgd_oracle_philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2],
                                uint32_t out[4])
{
    uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
    uint32_t k0 = key_in[0], k1 = key_in[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;               /* key schedule between rounds */
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Uniform in [0,1) for element j of a call: 24 random bits, exact in binary32. */
float aqsgd_oracle_uniform(uint64_t seed, uint64_t j)
{
    uint64_t block = j / 4;
    uint32_t ctr[4] = { (uint32_t)block, (uint32_t)(block >> 32), 0u, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    aqsgd_oracle_philox4x32_10(ctr, key, w);
    return (float)(w[j % 4] >> 8) * 0x1p-24f;
}

/* ------------------------------------------------------------------ */
/* b-bit integers on the wire: element j owns stream bits              */
/* [j*b, j*b+b); stream bit k is bit (k mod 8) of byte k/8.            */
/* ------------------------------------------------------------------ */
void aqsgd_oracle_pack(const int32_t* q, int64_t count, int bits, uint8_t* bytes)
{
    memset(bytes, 0, (size_t)((count * bits + 7) / 8));
    for (int64_t j = 0; j < count; ++j)
        for (int k = 0; k < bits; ++k)
            if ((q[j] >> k) & 1) {
                int64_t pos = j * bits + k;
                bytes[pos / 8] |= (uint8_t)(1u << (pos % 8));
            }
}

void aqsgd_oracle_unpack(const uint8_t* bytes, int64_t count, int bits, int32_t* q)
{
    for (int64_t j = 0; j < count; ++j) {
        int32_t v = 0;
        for (int k = 0; k < bits; ++k) {
            int64_t pos = j * bits + k;
            if ((bytes[pos / 8] >> (pos % 8)) & 1) v |= (1 << k);
        }
        q[j] = v;
    }
}

/* ------------------------------------------------------------------ */
/* The quantiser Q on one group (Section 4.1).                         */
/*   d[0..G)  binary32 inputs                                          */
/*   r[0..G)  rounding offsets: 1/2 everywhere for nearest rounding,   */
/*            U[0,1) draws for stochastic rounding                     */
/* Out: level indices q in [0, 2^b-1], transmitted scale, Q(d).        */
/* ------------------------------------------------------------------ */
static float half_levels(int bits) { return (float)((1 << bits) - 1) / 2.0f; }  /* exact */

void aqsgd_oracle_quantize_group(const float* d, const float* r, int64_t G, int bits,
                                 int32_t* q, float* scale_out, float* dhat)
{
    const int L = (1 << bits) - 1;       /* index of the top level */
    const float hL = half_levels(bits);  /* 1.5, 3.5, 7.5, 31.5, 127.5: exact */

    float s = 0.0f;                      /* normaliser: max |d| over the group */
    for (int64_t e = 0; e < G; ++e) {
        float a = fabsf(d[e]);
        if (a > s) s = a;
    }
    if (s < 0x1p-120f) {                 /* nothing to send */
        for (int64_t e = 0; e < G; ++e) { q[e] = 0; dhat[e] = 0.0f; }
        *scale_out = 0.0f;
        return;
    }
    const float inv = hL / s;            /* maps [-s, s] onto [-hL, hL] */
    const float step = s / hL;           /* spacing of the levels */
    for (int64_t e = 0; e < G; ++e) {
        float t = d[e] * inv;            /* normalised, in level units */
        t = t + hL;                      /* levels sit at 0, 1, ..., L */
        float y = t + r[e];
        int32_t k = (int32_t)floorf(y);
        if (k < 0) k = 0;
        if (k > L) k = L;
        q[e] = k;
        dhat[e] = ((float)k - hL) * step;
    }
    *scale_out = s;
}

/* Q^-1 on one group, as the receiver computes it from (codes, scale). */
void aqsgd_oracle_dequantize_group(const int32_t* q, float scale, int64_t G, int bits,
                                   float* dhat)
{
    const float hL = half_levels(bits);
    if (scale == 0.0f) {
        for (int64_t e = 0; e < G; ++e) dhat[e] = 0.0f;
        return;
    }
    const float step = scale / hL;
    for (int64_t e = 0; e < G; ++e) dhat[e] = ((float)q[e] - hL) * step;
}

static void rounding_offsets(int rounding, uint64_t seed, int64_t j0, int64_t G, float* r)
{
    for (int64_t e = 0; e < G; ++e)
        r[e] = (rounding == ORACLE_STOCHASTIC)
                   ? aqsgd_oracle_uniform(seed, (uint64_t)(j0 + e)) : 0.5f;
}

static int check_shape(int dtype, int bits, int64_t group, int rounding,
                       int64_t batch, int64_t n_per)
{
    if (dtype < 0 || dtype > 2) return -1;
    if (!(bits == 2 || bits == 3 || bits == 4 || bits == 6 || bits == 8)) return -2;
    if (group <= 0 || n_per <= 0 || n_per % group) return -3;
    if ((group * bits) % 8) return -3;
    if (rounding != ORACLE_NEAREST && rounding != ORACLE_STOCHASTIC) return -4;
    if (batch < 0) return -5;
    return 0;
}

/* ------------------------------------------------------------------ */
/* Sender: Delta m = Q(a - m); m <- m + Delta m; emit Delta m.         */
/* act [batch, n_per]; ids[batch] select rows of m_buf [*, n_per].     */
/* Groups tile the call tensor contiguously: group g covers flat       */
/* elements [g*G, g*G+G), which never straddles two samples.           */
/* ------------------------------------------------------------------ */
int aqsgd_oracle_encode(int dtype, int bits, int64_t group, int rounding, uint64_t seed,
                        int64_t batch, int64_t n_per, const void* act,
                        const int64_t* ids, void* m_buf, uint8_t* codes, float* scales)
{
    int rc = check_shape(dtype, bits, group, rounding, batch, n_per);
    if (rc) return rc;
    const int64_t groups_per_sample = n_per / group;
    const int64_t n_groups = batch * groups_per_sample;
#pragma omp parallel
    {
        float* d = malloc(sizeof(float) * group);
        float* m_old = malloc(sizeof(float) * group);
        float* r = malloc(sizeof(float) * group);
        float* dhat = malloc(sizeof(float) * group);
        int32_t* q = malloc(sizeof(int32_t) * group);
#pragma omp for schedule(static)
        for (int64_t g = 0; g < n_groups; ++g) {
            const int64_t i = g / groups_per_sample;          /* sample in call */
            const int64_t within = (g % groups_per_sample) * group;
            const int64_t a0 = i * n_per + within;            /* = g * group */
            const int64_t m0 = ids[i] * n_per + within;       /* row of m(xi) */
            for (int64_t e = 0; e < group; ++e) {
                m_old[e] = load_elem(m_buf, m0 + e, dtype);
                d[e] = load_elem(act, a0 + e, dtype) - m_old[e];
            }
            rounding_offsets(rounding, seed, a0, group, r);
            aqsgd_oracle_quantize_group(d, r, group, bits, q, &scales[g], dhat);
            for (int64_t e = 0; e < group; ++e)
                store_elem(m_buf, m0 + e, dtype, m_old[e] + dhat[e]);
            aqsgd_oracle_pack(q, group, bits, codes + a0 * bits / 8);
        }
        free(d); free(m_old); free(r); free(dhat); free(q);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Uncompressed first visit (Algorithm 1's branch for a sample without  */
/* a previous message, which sets m(xi) to a(xi); Appendix D's warm-up   */
/* epoch): the row is the activation, bit for bit, on whichever machine  */
/* calls it.                                                            */
/* ------------------------------------------------------------------ */
int aqsgd_oracle_seed(int dtype, int64_t batch, int64_t n_per, const void* act,
                      const int64_t* ids, void* m_buf)
{
    if (dtype < 0 || dtype > 2 || batch < 0 || n_per <= 0) return -1;
    const size_t eb = dtype == ORACLE_F32 ? 4 : 2;
    for (int64_t i = 0; i < batch; ++i)
        for (int64_t e = 0; e < n_per; ++e)
            memcpy((char*)m_buf + ((size_t)ids[i] * n_per + e) * eb,
                   (const char*)act + ((size_t)i * n_per + e) * eb, eb);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Receiver: m <- m + Delta m on its own replica; the updated m is the */
/* activation the next stage consumes.                                 */
/* ------------------------------------------------------------------ */
int aqsgd_oracle_decode(int dtype, int bits, int64_t group, int64_t batch, int64_t n_per,
                        const uint8_t* codes, const float* scales, const int64_t* ids,
                        void* m_buf, void* out)
{
    int rc = check_shape(dtype, bits, group, ORACLE_NEAREST, batch, n_per);
    if (rc) return rc;
    const int64_t groups_per_sample = n_per / group;
    const int64_t n_groups = batch * groups_per_sample;
#pragma omp parallel
    {
        float* dhat = malloc(sizeof(float) * group);
        int32_t* q = malloc(sizeof(int32_t) * group);
#pragma omp for schedule(static)
        for (int64_t g = 0; g < n_groups; ++g) {
            const int64_t i = g / groups_per_sample;
            const int64_t within = (g % groups_per_sample) * group;
            const int64_t a0 = i * n_per + within;
            const int64_t m0 = ids[i] * n_per + within;
            aqsgd_oracle_unpack(codes + a0 * bits / 8, group, bits, q);
            aqsgd_oracle_dequantize_group(q, scales[g], group, bits, dhat);
            for (int64_t e = 0; e < group; ++e) {
                float m_new = load_elem(m_buf, m0 + e, dtype) + dhat[e];
                store_elem(m_buf, m0 + e, dtype, m_new);
                /* hand over exactly what was stored */
                store_elem(out, a0 + e, dtype, load_elem(m_buf, m0 + e, dtype));
            }
        }
        free(dhat); free(q);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Backward message: Q(grad) directly, no buffer.                      */
/* ------------------------------------------------------------------ */
int aqsgd_oracle_grad_quant(int dtype, int bits, int64_t group, int rounding, uint64_t seed,
                            int64_t batch, int64_t n_per, const void* grad,
                            uint8_t* codes, float* scales)
{
    int rc = check_shape(dtype, bits, group, rounding, batch, n_per);
    if (rc) return rc;
    const int64_t n_groups = batch * (n_per / group);
#pragma omp parallel
    {
        float* d = malloc(sizeof(float) * group);
        float* r = malloc(sizeof(float) * group);
        float* dhat = malloc(sizeof(float) * group);
        int32_t* q = malloc(sizeof(int32_t) * group);
#pragma omp for schedule(static)
        for (int64_t g = 0; g < n_groups; ++g) {
            const int64_t a0 = g * group;
            for (int64_t e = 0; e < group; ++e) d[e] = load_elem(grad, a0 + e, dtype);
            rounding_offsets(rounding, seed, a0, group, r);
            aqsgd_oracle_quantize_group(d, r, group, bits, q, &scales[g], dhat);
            aqsgd_oracle_pack(q, group, bits, codes + a0 * bits / 8);
        }
        free(d); free(r); free(dhat); free(q);
    }
    return 0;
}

int aqsgd_oracle_grad_dequant(int dtype, int bits, int64_t group, int64_t batch,
                              int64_t n_per, const uint8_t* codes, const float* scales,
                              void* out)
{
    int rc = check_shape(dtype, bits, group, ORACLE_NEAREST, batch, n_per);
    if (rc) return rc;
    const int64_t n_groups = batch * (n_per / group);
#pragma omp parallel
    {
        float* dhat = malloc(sizeof(float) * group);
        int32_t* q = malloc(sizeof(int32_t) * group);
#pragma omp for schedule(static)
        for (int64_t g = 0; g < n_groups; ++g) {
            const int64_t a0 = g * group;
            aqsgd_oracle_unpack(codes + a0 * bits / 8, group, bits, q);
            aqsgd_oracle_dequantize_group(q, scales[g], group, bits, dhat);
            for (int64_t e = 0; e < group; ++e) store_elem(out, a0 + e, dtype, dhat[e]);
        }
        free(dhat); free(q);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Previous messages kept at low precision (the "m z" runs of Appendix   */
/* H.5, in which m itself is quantised to z bits).  The appendix says    */
/* no more than that; reading:                                           */
/*   - m(xi) is stored as z-bit levels plus one binary32 max-abs scale   */
/*     per group (the message's group size), through the same Q with     */
/*     nearest rounding, so that both machines store the same bits;      */
/*   - both machines work from the stored value m^ = Q_z^-1(stored):     */
/*         sender:    Delta m = Q_b(a - m^)                              */
/*         both:      v = m^ + Delta m   (binary32);  store Q_z(v)       */
/*         receiver:  hands v (rounded to the activation dtype) on.      */
/*   All-zero storage decodes to m^ = 0: the first visit is direct       */
/*   quantisation, as with a full-precision m.                           */
/* ------------------------------------------------------------------ */
static int check_mbits(int m_bits, int64_t group)
{
    if (!(m_bits == 2 || m_bits == 8)) return -6;
    if ((group * m_bits) % 8) return -3;
    return 0;
}

/* m^ of one group from its stored levels and scale. */
static void stored_group(const uint8_t* m_codes, float m_scale, int64_t group, int m_bits,
                         int32_t* q, float* m_hat)
{
    aqsgd_oracle_unpack(m_codes, group, m_bits, q);
    aqsgd_oracle_dequantize_group(q, m_scale, group, m_bits, m_hat);
}

/* Q_z(v), nearest, written back as levels and scale. */
static void store_group(const float* v, int64_t group, int m_bits, float* half, int32_t* q,
                        float* scratch, uint8_t* m_codes, float* m_scale)
{
    for (int64_t e = 0; e < group; ++e) half[e] = 0.5f;
    aqsgd_oracle_quantize_group(v, half, group, m_bits, q, m_scale, scratch);
    aqsgd_oracle_pack(q, group, m_bits, m_codes);
}

int aqsgd_oracle_encode_lowbit(int dtype, int bits, int m_bits, int64_t group, int rounding,
                               uint64_t seed, int64_t batch, int64_t n_per, const void* act,
                               const int64_t* ids, uint8_t* m_codes, float* m_scales,
                               uint8_t* codes, float* scales)
{
    int rc = check_shape(dtype, bits, group, rounding, batch, n_per);
    if (!rc) rc = check_mbits(m_bits, group);
    if (rc) return rc;
    const int64_t groups_per_sample = n_per / group;
    const int64_t n_groups = batch * groups_per_sample;
#pragma omp parallel
    {
        float* m_hat = malloc(sizeof(float) * group);
        float* d = malloc(sizeof(float) * group);
        float* r = malloc(sizeof(float) * group);
        float* dhat = malloc(sizeof(float) * group);
        float* v = malloc(sizeof(float) * group);
        float* tmp = malloc(sizeof(float) * group);
        int32_t* q = malloc(sizeof(int32_t) * group);
#pragma omp for schedule(static)
        for (int64_t g = 0; g < n_groups; ++g) {
            const int64_t i = g / groups_per_sample;
            const int64_t gs = g % groups_per_sample;
            const int64_t a0 = i * n_per + gs * group;                    /* = g * group */
            uint8_t* mc = m_codes + (ids[i] * n_per + gs * group) * m_bits / 8;
            float* ms = m_scales + ids[i] * groups_per_sample + gs;
            stored_group(mc, *ms, group, m_bits, q, m_hat);
            for (int64_t e = 0; e < group; ++e) d[e] = load_elem(act, a0 + e, dtype) - m_hat[e];
            rounding_offsets(rounding, seed, a0, group, r);
            aqsgd_oracle_quantize_group(d, r, group, bits, q, &scales[g], dhat);
            aqsgd_oracle_pack(q, group, bits, codes + a0 * bits / 8);
            for (int64_t e = 0; e < group; ++e) v[e] = m_hat[e] + dhat[e];
            store_group(v, group, m_bits, r, q, tmp, mc, ms);
        }
        free(m_hat); free(d); free(r); free(dhat); free(v); free(tmp); free(q);
    }
    return 0;
}

int aqsgd_oracle_decode_lowbit(int dtype, int bits, int m_bits, int64_t group, int64_t batch,
                               int64_t n_per, const uint8_t* codes, const float* scales,
                               const int64_t* ids, uint8_t* m_codes, float* m_scales, void* out)
{
    int rc = check_shape(dtype, bits, group, ORACLE_NEAREST, batch, n_per);
    if (!rc) rc = check_mbits(m_bits, group);
    if (rc) return rc;
    const int64_t groups_per_sample = n_per / group;
    const int64_t n_groups = batch * groups_per_sample;
#pragma omp parallel
    {
        float* m_hat = malloc(sizeof(float) * group);
        float* dhat = malloc(sizeof(float) * group);
        float* v = malloc(sizeof(float) * group);
        float* half = malloc(sizeof(float) * group);
        float* tmp = malloc(sizeof(float) * group);
        int32_t* q = malloc(sizeof(int32_t) * group);
#pragma omp for schedule(static)
        for (int64_t g = 0; g < n_groups; ++g) {
            const int64_t i = g / groups_per_sample;
            const int64_t gs = g % groups_per_sample;
            const int64_t a0 = i * n_per + gs * group;
            uint8_t* mc = m_codes + (ids[i] * n_per + gs * group) * m_bits / 8;
            float* ms = m_scales + ids[i] * groups_per_sample + gs;
            stored_group(mc, *ms, group, m_bits, q, m_hat);
            aqsgd_oracle_unpack(codes + a0 * bits / 8, group, bits, q);
            aqsgd_oracle_dequantize_group(q, scales[g], group, bits, dhat);
            for (int64_t e = 0; e < group; ++e) {
                v[e] = m_hat[e] + dhat[e];
                store_elem(out, a0 + e, dtype, v[e]);
            }
            store_group(v, group, m_bits, half, q, tmp, mc, ms);
        }
        free(m_hat); free(dhat); free(v); free(half); free(tmp); free(q);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Sparsified backward message (the "bw8[0.2]" runs of Appendix H.6: the */
/* largest fifth of the gradient entries is kept, then quantised to      */
/* 8 bits).  The appendix says no more; reading: per group of G elements the */
/* `keep` entries of largest magnitude survive (equal magnitudes: the    */
/* lower index first); survivors are quantised by Q_b with the group's   */
/* max-abs scale (the largest entry always survives), everything else   */
/* reconstructs as +0.  On the wire, per call: a bitmap with one bit    */
/* per element (element j at bit j mod 8 of byte j/8), `keep` b-bit     */
/* levels per group in index order, one scale per group.                */
/* ------------------------------------------------------------------ */
typedef struct { float mag; int64_t idx; } oracle_ranked;

static int by_magnitude_then_index(const void* pa, const void* pb)
{
    const oracle_ranked* a = pa;
    const oracle_ranked* b = pb;
    if (a->mag > b->mag) return -1;
    if (a->mag < b->mag) return 1;
    return (a->idx > b->idx) - (a->idx < b->idx);
}

int aqsgd_oracle_grad_topk_quant(int dtype, int bits, int64_t group, int64_t keep, int rounding,
                                 uint64_t seed, int64_t n, const void* grad, uint8_t* bitmap,
                                 uint8_t* codes, float* scales)
{
    int rc = check_shape(dtype, bits, group, rounding, 1, n);
    if (rc) return rc;
    if (keep < 1 || keep > group || group % 8 || (keep * bits) % 8) return -7;
    const int64_t n_groups = n / group;
    memset(bitmap, 0, (size_t)(n / 8));
#pragma omp parallel
    {
        float* d = malloc(sizeof(float) * group);
        float* r = malloc(sizeof(float) * group);
        float* dhat = malloc(sizeof(float) * group);
        int32_t* q = malloc(sizeof(int32_t) * group);
        int32_t* kept_q = malloc(sizeof(int32_t) * keep);
        uint8_t* kept = malloc((size_t)group);
        oracle_ranked* order = malloc(sizeof(oracle_ranked) * group);
#pragma omp for schedule(static)
        for (int64_t g = 0; g < n_groups; ++g) {
            const int64_t a0 = g * group;
            for (int64_t e = 0; e < group; ++e) {
                d[e] = load_elem(grad, a0 + e, dtype);
                order[e].mag = fabsf(d[e]);
                order[e].idx = e;
                kept[e] = 0;
            }
            qsort(order, (size_t)group, sizeof(oracle_ranked), by_magnitude_then_index);
            for (int64_t k = 0; k < keep; ++k) kept[order[k].idx] = 1;
            rounding_offsets(rounding, seed, a0, group, r);
            aqsgd_oracle_quantize_group(d, r, group, bits, q, &scales[g], dhat);
            int64_t pos = 0;
            for (int64_t e = 0; e < group; ++e)
                if (kept[e]) {
                    bitmap[(a0 + e) / 8] |= (uint8_t)(1u << ((a0 + e) % 8));
                    kept_q[pos++] = q[e];
                }
            aqsgd_oracle_pack(kept_q, keep, bits, codes + g * keep * bits / 8);
        }
        free(d); free(r); free(dhat); free(q); free(kept_q); free(kept); free(order);
    }
    return 0;
}

int aqsgd_oracle_grad_topk_dequant(int dtype, int bits, int64_t group, int64_t keep, int64_t n,
                                   const uint8_t* bitmap, const uint8_t* codes, const float* scales,
                                   void* out)
{
    int rc = check_shape(dtype, bits, group, ORACLE_NEAREST, 1, n);
    if (rc) return rc;
    if (keep < 1 || keep > group || group % 8 || (keep * bits) % 8) return -7;
    const int64_t n_groups = n / group;
#pragma omp parallel
    {
        int32_t* kept_q = malloc(sizeof(int32_t) * keep);
        float* val = malloc(sizeof(float) * keep);
#pragma omp for schedule(static)
        for (int64_t g = 0; g < n_groups; ++g) {
            const int64_t a0 = g * group;
            aqsgd_oracle_unpack(codes + g * keep * bits / 8, keep, bits, kept_q);
            aqsgd_oracle_dequantize_group(kept_q, scales[g], keep, bits, val);
            int64_t pos = 0;
            for (int64_t e = 0; e < group; ++e) {
                const int on = (bitmap[(a0 + e) / 8] >> ((a0 + e) % 8)) & 1;
                store_elem(out, a0 + e, dtype, (on && pos < keep) ? val[pos++] : 0.0f);
            }
        }
        free(kept_q); free(val);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Algorithm 1 with its first-visit branch (a sample without a previous  */
/* message: the activation travels uncompressed and m(xi) <- a(xi);     */
/* otherwise the change is quantised).  seen[id] != 0 marks samples that have a   */
/* previous message.  Sender: first[i] = 1 tells the caller that row i  */
/* of act is the message of sample i and that the sample's slices of    */
/* codes / scales were not written.  Receiver: `full` holds those rows  */
/* (rows of samples that were seen before are not read).  Both sides    */
/* mark the call's samples as seen, so their flags stay identical.      */
/* ------------------------------------------------------------------ */
int aqsgd_oracle_encode_seen(int dtype, int bits, int64_t group, int rounding, uint64_t seed,
                             int64_t batch, int64_t n_per, const void* act, const int64_t* ids,
                             void* m_buf, uint8_t* seen, int32_t* first, uint8_t* codes,
                             float* scales)
{
    int rc = check_shape(dtype, bits, group, rounding, batch, n_per);
    if (rc) return rc;
    const int64_t groups_per_sample = n_per / group;
    float* d = malloc(sizeof(float) * group);
    float* m_old = malloc(sizeof(float) * group);
    float* r = malloc(sizeof(float) * group);
    float* dhat = malloc(sizeof(float) * group);
    int32_t* q = malloc(sizeof(int32_t) * group);
    for (int64_t i = 0; i < batch; ++i) {
        const int64_t id = ids[i];
        if (!seen[id]) {                              /* first visit: full precision */
            for (int64_t e = 0; e < n_per; ++e)
                store_elem(m_buf, id * n_per + e, dtype, load_elem(act, i * n_per + e, dtype));
            first[i] = 1;
            seen[id] = 1;
            continue;
        }
        first[i] = 0;
        for (int64_t gs = 0; gs < groups_per_sample; ++gs) {
            const int64_t a0 = i * n_per + gs * group;    /* flat index in the call */
            const int64_t m0 = id * n_per + gs * group;
            for (int64_t e = 0; e < group; ++e) {
                m_old[e] = load_elem(m_buf, m0 + e, dtype);
                d[e] = load_elem(act, a0 + e, dtype) - m_old[e];
            }
            rounding_offsets(rounding, seed, a0, group, r);
            aqsgd_oracle_quantize_group(d, r, group, bits, q, &scales[a0 / group], dhat);
            for (int64_t e = 0; e < group; ++e)
                store_elem(m_buf, m0 + e, dtype, m_old[e] + dhat[e]);
            aqsgd_oracle_pack(q, group, bits, codes + a0 * bits / 8);
        }
    }
    free(d); free(m_old); free(r); free(dhat); free(q);
    return 0;
}

int aqsgd_oracle_decode_seen(int dtype, int bits, int64_t group, int64_t batch, int64_t n_per,
                             const uint8_t* codes, const float* scales, const void* full,
                             const int64_t* ids, void* m_buf, uint8_t* seen, void* out)
{
    int rc = check_shape(dtype, bits, group, ORACLE_NEAREST, batch, n_per);
    if (rc) return rc;
    const int64_t groups_per_sample = n_per / group;
    float* dhat = malloc(sizeof(float) * group);
    int32_t* q = malloc(sizeof(int32_t) * group);
    for (int64_t i = 0; i < batch; ++i) {
        const int64_t id = ids[i];
        if (!seen[id]) {
            for (int64_t e = 0; e < n_per; ++e) {
                const float a = load_elem(full, i * n_per + e, dtype);
                store_elem(m_buf, id * n_per + e, dtype, a);
                store_elem(out, i * n_per + e, dtype, a);
            }
            seen[id] = 1;
            continue;
        }
        for (int64_t gs = 0; gs < groups_per_sample; ++gs) {
            const int64_t a0 = i * n_per + gs * group;
            const int64_t m0 = id * n_per + gs * group;
            aqsgd_oracle_unpack(codes + a0 * bits / 8, group, bits, q);
            aqsgd_oracle_dequantize_group(q, scales[a0 / group], group, bits, dhat);
            for (int64_t e = 0; e < group; ++e) {
                store_elem(m_buf, m0 + e, dtype, load_elem(m_buf, m0 + e, dtype) + dhat[e]);
                store_elem(out, a0 + e, dtype, load_elem(m_buf, m0 + e, dtype));
            }
        }
    }
    free(dhat); free(q);
    return 0;
}

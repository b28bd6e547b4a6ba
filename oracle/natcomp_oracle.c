/*
 * natcomp_oracle.c -- plain CPU oracle for natural compression C_nat, natural
 * dithering D_nat^{p,s}, their decoders and the n-worker decode-and-sum.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
 * of what the GPU library must compute.  It shares no code with the HIP path
 * and the product never calls it: only the tests, the smoke check and the
 * benchmark's cpu_baseline leg load it.
 *
 * Every routine is a scalar loop over elements in index order.  The only
 * concession to speed is an OpenMP "parallel for" over independent elements
 * (each element's result depends on its own index only), which changes no
 * arithmetic and no order of floating-point accumulation: all reductions
 * (norms, sums over workers) are sequential per output value.
 *
 * Sources, by routine:
 *   orc_nat_round        Sec. 2, Def. 1 and the binary32 derivation ("From 32 to 9 bits"):
 *                        P(exponent + 1) = m, P(mantissa dropped) = 1 - m.
 *   orc_nat_encode       the same rule element-wise; 1 sign + 8 exponent bits per entry.
 *   orc_nat_decode       sign and exponent kept, mantissa zero.
 *   orc_pnorm            Sec. 3, ||x||_p = (sum |x_i|^p)^(1/p), 1 <= p <= inf.
 *   orc_dither_level     Sec. 3, Def. 3 (general dithering) with the natural level set
 *                        {0, 2^(1-s), ..., 1/2, 1}.
 *   orc_dither_encode    y_i = |x_i| / ||x||_p, xi(y_i), sign(x_i); norm per caller segment.
 *   orc_dither_decode    ||x||_p * sign * level.
 *   orc_aggregate_*      Algorithm 1, the master's sum over workers of the decompressed updates.
 *   orc_sparse_*         Appendix "Sparsification - formal definition": S^q(x) = (d/q) xi o x with
 *                        exactly q kept coordinates, composed with C_nat (composition theorem);
 *                        how the q coordinates are drawn (a keyed permutation) is this build's choice.
 *   orc_philox4x32_10    Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
 *                        as 1, 2, 3" (SC'11), Philox-4x32 with 10 rounds.  The paper only
 *                        asks for a Bernoulli draw per element; the generator, its keying by
 *                        (seed, worker, index), how many elements share a call and the width
 *                        of the comparison are this build's choice.
 *
 * Parity status: every arithmetic rule here is pinned by tests against the
 * paper's worked examples, exact probabilities by exhaustive enumeration of
 * the random word, closed-form moments and brute force.  The byte/bit packing
 * of the code planes is a free choice the paper does not fix: "parity
 * unpinned" for the layout itself (it is checked only for self-consistency:
 * decode(encode) and GPU bytes == oracle bytes).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Random words                                                             */
/* ------------------------------------------------------------------------ */

/* One Philox-4x32 bijection with 10 rounds.  Round: with products
 * P0 = M0*c0 and P1 = M1*c2 (32x32 -> 64 bits),
 *   (c0, c1, c2, c3) <- (hi(P1)^c1^k0, lo(P1), hi(P0)^c3^k1, lo(P0)),
 * then the key is bumped by the Weyl constants. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)M0 * c0;
        uint64_t p1 = (uint64_t)M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Domains keep the streams of different operators apart. */
enum { ORC_DOMAIN_NAT = 0, ORC_DOMAIN_DITHER = 1, ORC_DOMAIN_MASTER = 3, ORC_DOMAIN_NORM = 4 };

/* The 32-bit uniform word of global element g: the counter is (g/4, worker,
 * domain), the key is the seed, and the element takes output word g mod 4.
 * It depends on nothing but (seed, worker, domain, g).  (Natural compression, the
 * master's compression and the compressed norms draw this way; the dithering
 * operators use orc_dither_word below.) */
uint32_t orc_random_word(uint64_t seed, uint32_t worker, uint32_t domain, uint64_t g)
{
    uint64_t q = g >> 2;
    uint32_t ctr[4] = { (uint32_t)q, (uint32_t)(q >> 32), worker, domain };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return out[g & 3];
}

/* The dithering operators (domain 1) draw from a denser layout: one Philox call per 8
 * consecutive elements, counter (g/8, worker, 1).  Elements 0..3 of the group share the
 * words (a, b) = (w0, w1), elements 4..7 the words (a, b) = (w2, w3), and within such a
 * half the four elements take a, b, a<<16 | b>>16 and b<<16 | a>>16.  Each of the four is a
 * rearrangement of 32 distinct bits of the call's output, hence uniform on [0, 2^32) by
 * itself; only the per-coordinate marginals enter the definition of the class B(omega)
 * (Def. 2: unbiasedness and the second-moment bound are sums over coordinates), so the
 * dependence between neighbours costs nothing there, and it is weak anyway: the top 23
 * bits that decide two different elements share at most 7 bits. */
uint32_t orc_dither_word_of_call(const uint32_t w[4], uint32_t j)
{
    uint32_t a = (j & 4) ? w[2] : w[0], b = (j & 4) ? w[3] : w[1];
    switch (j & 3) {
        case 0: return a;
        case 1: return b;
        case 2: return (a << 16) | (b >> 16);
        default: return (b << 16) | (a >> 16);
    }
}
uint32_t orc_dither_word(uint64_t seed, uint32_t worker, uint64_t g)
{
    uint64_t q = g >> 3;
    uint32_t ctr[4] = { (uint32_t)q, (uint32_t)(q >> 32), worker, ORC_DOMAIN_DITHER };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return orc_dither_word_of_call(out, (uint32_t)(g & 7));
}

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* ------------------------------------------------------------------------ */
/* Natural compression                                                      */
/* ------------------------------------------------------------------------ */

/* The rounding rule on one binary32 value with bits u = (sign, e, m) and one
 * uniform 32-bit word r.  t = (-1)^sign 2^(e-127) (1 + m/2^23); it goes to
 * exponent e+1 with probability m/2^23 and keeps exponent e (mantissa dropped)
 * otherwise.  r/2^32 < m/2^23  <=>  r < m * 2^9, an integer comparison.
 * m = 0 (zero or an exact power of two) never moves.  Returns the new 8-bit
 * exponent field; 255 (the Inf/NaN exponent) is an absorbing ceiling. */
uint32_t orc_nat_round(uint32_t u, uint32_t r)
{
    uint32_t e = (u >> 23) & 255u;
    uint64_t m = u & 0x7FFFFFu;
    uint32_t up = ((uint64_t)r < (m << 9)) ? 1u : 0u;
    uint32_t e_new = e + up;
    return e_new > 255u ? 255u : e_new;
}

/* Exhaustive count of "exponent + 1" outcomes over all 2^32 words r. */
uint64_t orc_nat_count_up(uint32_t u)
{
    uint32_t e = (u >> 23) & 255u;
    uint64_t count = 0;
#pragma omp parallel for reduction(+ : count)
    for (int64_t r = 0; r < ((int64_t)1 << 32); ++r)
        count += (orc_nat_round(u, (uint32_t)r) != e);
    return count;
}

/* x[0..d): exponent plane exp_out[i] = new exponent field of x[i];
 * sign plane: bit (i mod 8) of sign_out[i/8] = sign bit of x[i]; the unused
 * high bits of the last sign byte are zero.  Element i draws the word of
 * global index index_offset + i. */
static void nat_encode_domain(const float *x, uint64_t d, uint64_t seed, uint32_t worker, uint32_t domain,
                              uint64_t index_offset, uint8_t *exp_out, uint8_t *sign_out)
{
    uint64_t nsign = (d + 7) / 8;
    memset(sign_out, 0, nsign);
#pragma omp parallel for
    for (int64_t byte = 0; byte < (int64_t)nsign; ++byte) {
        uint8_t sb = 0;
        for (int bit = 0; bit < 8; ++bit) {
            uint64_t i = (uint64_t)byte * 8 + bit;
            if (i >= d) break;
            uint32_t u = f32_bits(x[i]);
            uint32_t r = orc_random_word(seed, worker, domain, index_offset + i);
            exp_out[i] = (uint8_t)orc_nat_round(u, r);
            sb |= (uint8_t)((u >> 31) << bit);
        }
        sign_out[byte] = sb;
    }
}

void orc_nat_encode(const float *x, uint64_t d, uint64_t seed, uint32_t worker,
                    uint64_t index_offset, uint8_t *exp_out, uint8_t *sign_out)
{
    nat_encode_domain(x, d, seed, worker, ORC_DOMAIN_NAT, index_offset, exp_out, sign_out);
}

/* The decoded value has the stored sign and exponent and a zero mantissa. */
static float nat_value(const uint8_t *exp, const uint8_t *sign, uint64_t i)
{
    uint32_t s = (sign[i >> 3] >> (i & 7)) & 1u;
    return bits_f32((s << 31) | ((uint32_t)exp[i] << 23));
}

void orc_nat_decode(const uint8_t *exp, const uint8_t *sign, uint64_t d, float *out)
{
#pragma omp parallel for
    for (int64_t i = 0; i < (int64_t)d; ++i)
        out[i] = nat_value(exp, sign, (uint64_t)i);
}

/* ------------------------------------------------------------------------ */
/* p-norm                                                                   */
/* ------------------------------------------------------------------------ */

/* ||x||_p over x[0..len), accumulated in double in index order.
 * p = 1, 2 or INFINITY. Returns -1 for any other p. */
double orc_pnorm(const float *x, uint64_t len, double p)
{
    double acc = 0.0;
    if (isinf(p)) {
        for (uint64_t i = 0; i < len; ++i) { double a = fabs((double)x[i]); if (a > acc) acc = a; }
        return acc;
    }
    if (p == 1.0) {
        for (uint64_t i = 0; i < len; ++i) acc += fabs((double)x[i]);
        return acc;
    }
    if (p == 2.0) {
        for (uint64_t i = 0; i < len; ++i) acc += (double)x[i] * (double)x[i];
        return sqrt(acc);
    }
    return -1.0;
}

/* Segment s covers [seg_begin(s), seg_begin(s+1)).  Three ways to describe the
 * segments: explicit offsets (num_segments+1 ascending values, first 0, last
 * d); a fixed bucket length (offsets NULL, bucket > 0); or the whole vector
 * (offsets NULL, bucket 0). */
static uint64_t seg_count(uint64_t d, const uint64_t *offsets, uint32_t num_segments, uint32_t bucket)
{
    if (offsets) return num_segments;
    if (bucket) return (d + bucket - 1) / bucket;
    return 1;
}
static uint64_t seg_begin(uint64_t s, uint64_t d, const uint64_t *offsets, uint32_t num_segments, uint32_t bucket)
{
    uint64_t n = seg_count(d, offsets, num_segments, bucket);
    if (s >= n) return d;
    if (offsets) return offsets[s];
    if (bucket) return s * (uint64_t)bucket;
    return 0;
}

uint64_t orc_segment_count(uint64_t d, const uint64_t *offsets, uint32_t num_segments, uint32_t bucket)
{
    return seg_count(d, offsets, num_segments, bucket);
}

/* norms64[s] = ||x_segment s||_p in double. */
void orc_pnorm_segments(const float *x, uint64_t d, const uint64_t *offsets, uint32_t num_segments,
                        uint32_t bucket, double p, double *norms64)
{
    int64_t n = (int64_t)seg_count(d, offsets, num_segments, bucket);
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t s = 0; s < n; ++s) {
        uint64_t b = seg_begin((uint64_t)s, d, offsets, num_segments, bucket);
        uint64_t e = seg_begin((uint64_t)s + 1, d, offsets, num_segments, bucket);
        norms64[s] = orc_pnorm(x + b, e - b, p);
    }
}

/* ------------------------------------------------------------------------ */
/* Natural dithering                                                        */
/* ------------------------------------------------------------------------ */

/* Levels l_s = 0 < l_{s-1} = 2^(1-s) < ... < l_1 = 1/2 < l_0 = 1.  Level code
 * c in {0..s}: c = 0 is the level 0 and c >= 1 is 2^(c-s).  y in [0,1] is
 * given by its binary32 bits yb (sign cleared); r is a uniform 32-bit word, of
 * which the top 23 bits r23 decide.  With l_low <= y <= l_high adjacent levels,
 * the result is l_high with probability (y - l_low) / (l_high - l_low):
 *   y = 2^-k (1 + m/2^23), k <= s-1: between 2^-k and 2^(1-k), P(high) = m/2^23,
 *     exactly: high iff r23 < m;
 *   y below the lowest level 2^(1-s): between 0 and 2^(1-s), P(high) = y 2^(s-1),
 *     taken to 23 bits: high iff r23 < T with T = y 2^(s+22) rounded to the nearest
 *     integer, ties to even (|T/2^23 - y 2^(s-1)| <= 2^-24; T = 2^23 means always).
 *     For s <= 126 this T is the mantissa field of fl(y/2 + 2^-s), one fused
 *     multiply-add: the same draw as in the geometric region, applied to a value that
 *     carries y's position between 0 and 2^(1-s) in its mantissa.  It is evaluated
 *     here in integers so that subnormal y and s = 127 need no special case.
 * y >= 1 (possible by one rounding of the normalisation) is level 1. */
uint32_t orc_dither_level(uint32_t yb, uint32_t s, uint32_t r)
{
    if (yb >= 0x3F800000u) return s;
    uint32_t r23 = r >> 9;
    uint32_t e_y = yb >> 23;
    uint32_t m_y = yb & 0x7FFFFFu;
    if (e_y + s >= 128u) {                   /* 2^-k <= y < 2^(1-k) with k = 127 - e_y <= s - 1 */
        uint32_t k = 127u - e_y;
        return s - k + (r23 < m_y ? 1u : 0u);
    }
    /* y = M 2^(E-150) with E = max(e_y, 1); y 2^(s+22) = M / 2^sh, sh = 128 - s - E >= 0 */
    uint64_t M = e_y ? (0x800000u | (uint64_t)m_y) : (uint64_t)m_y;
    uint32_t sh = 128u - s - (e_y ? e_y : 1u);
    uint64_t T;
    if (sh == 0) {
        T = M;
    } else if (sh > 25) {
        T = 0;                               /* M < 2^24: less than a quarter */
    } else {
        uint64_t q = M >> sh, rem = M & (((uint64_t)1 << sh) - 1), half = (uint64_t)1 << (sh - 1);
        T = q + ((rem > half || (rem == half && (q & 1))) ? 1u : 0u);
    }
    return ((uint64_t)r23 < T) ? 1u : 0u;
}

/* Exhaustive count, over all 2^32 words r, of outcomes equal to `code`. */
uint64_t orc_dither_count(uint32_t yb, uint32_t s, uint32_t code)
{
    uint64_t count = 0;
#pragma omp parallel for reduction(+ : count)
    for (int64_t r = 0; r < ((int64_t)1 << 32); ++r)
        count += (orc_dither_level(yb, s, (uint32_t)r) == code);
    return count;
}

/* The normalisation: y = fl(|x| * fl(1/norm)), two correctly rounded binary32
 * operations.  A norm below the smallest normal number (including 0) makes the
 * whole segment code to zero (Def. 3: D(0) = 0). */
float orc_dither_inv_norm(float norm)
{
    if (!(norm >= 1.17549435e-38f)) return 0.0f;
    volatile float inv = 1.0f / norm;
    return inv;
}
uint32_t orc_dither_y_bits(float x, float inv)
{
    volatile float y = fabsf(x) * inv;
    return f32_bits(y) & 0x7FFFFFFFu;
}

/* Bits per level code: 1 <= s <= 127. */
static uint32_t code_width(uint32_t s) { uint32_t b = 0; while ((1u << b) < s + 1) ++b; return b; }

/* Packed layout, by code width b = ceil(log2(s+1)):
 *   b <= 3: one fused nibble (sign << 3) | c per element, element i in byte i/2,
 *           low nibble for even i; no sign plane.
 *   b == 4: nibble plane with c (same nibble order) plus the sign plane of C_nat.
 *   b >= 5: one byte c per element plus the sign plane.
 * Planes are indexed by the element's position in x, not restarted per segment. */
uint64_t orc_dither_code_bytes(uint64_t d, uint32_t s)
{
    return code_width(s) <= 4 ? (d + 1) / 2 : d;
}
uint64_t orc_dither_sign_bytes(uint64_t d, uint32_t s)
{
    return code_width(s) <= 3 ? 0 : (d + 7) / 8;
}

static void put_code(uint8_t *code, uint8_t *sign, uint64_t i, uint32_t s, uint32_t c, uint32_t sg)
{
    uint32_t b = code_width(s);
    if (b <= 3) {
        uint32_t nib = (sg << 3) | c;
        code[i >> 1] |= (uint8_t)(nib << ((i & 1) * 4));
    } else if (b == 4) {
        code[i >> 1] |= (uint8_t)(c << ((i & 1) * 4));
        sign[i >> 3] |= (uint8_t)(sg << (i & 7));
    } else {
        code[i] = (uint8_t)c;
        sign[i >> 3] |= (uint8_t)(sg << (i & 7));
    }
}
static void get_code(const uint8_t *code, const uint8_t *sign, uint64_t i, uint32_t s, uint32_t *c, uint32_t *sg)
{
    uint32_t b = code_width(s);
    if (b <= 3) {
        uint32_t nib = (code[i >> 1] >> ((i & 1) * 4)) & 15u;
        *c = nib & 7u; *sg = nib >> 3;
    } else if (b == 4) {
        *c = (code[i >> 1] >> ((i & 1) * 4)) & 15u;
        *sg = (sign[i >> 3] >> (i & 7)) & 1u;
    } else {
        *c = code[i];
        *sg = (sign[i >> 3] >> (i & 7)) & 1u;
    }
}

/* norms[s] is the binary32 norm of segment s that the encoder normalises by
 * (the caller computes it: orc_pnorm_segments rounded to float, or the norm
 * another implementation produced).  Writes the packed planes. */
void orc_dither_encode(const float *x, uint64_t d, const uint64_t *offsets, uint32_t num_segments,
                       uint32_t bucket, uint32_t s, const float *norms, uint64_t seed, uint32_t worker,
                       uint64_t index_offset, uint8_t *code_out, uint8_t *sign_out)
{
    memset(code_out, 0, orc_dither_code_bytes(d, s));
    if (orc_dither_sign_bytes(d, s)) memset(sign_out, 0, orc_dither_sign_bytes(d, s));
    uint64_t n = seg_count(d, offsets, num_segments, bucket);
    /* sequential over elements: neighbouring elements share bytes */
    for (uint64_t sgm = 0; sgm < n; ++sgm) {
        uint64_t b = seg_begin(sgm, d, offsets, num_segments, bucket);
        uint64_t e = seg_begin(sgm + 1, d, offsets, num_segments, bucket);
        float inv = orc_dither_inv_norm(norms[sgm]);
        for (uint64_t i = b; i < e; ++i) {
            uint32_t yb = orc_dither_y_bits(x[i], inv);
            uint32_t r = orc_dither_word(seed, worker, index_offset + i);
            uint32_t c = orc_dither_level(yb, s, r);
            put_code(code_out, sign_out, i, s, c, f32_bits(x[i]) >> 31);
        }
    }
}

/* Level value times norm: c = 0 gives a signed zero, c >= 1 gives
 * fl(norm * 2^(c-s)) with the sign applied (exact unless it underflows). */
static float dither_value(float norm, uint32_t s, uint32_t c, uint32_t sg)
{
    float mag = 0.0f;
    if (c > 0) {
        volatile float v = norm * ldexpf(1.0f, (int)c - (int)s);
        mag = v;
    }
    return sg ? -mag : mag;
}

void orc_dither_decode(const float *norms, const uint8_t *code, const uint8_t *sign, uint64_t d,
                       const uint64_t *offsets, uint32_t num_segments, uint32_t bucket, uint32_t s,
                       float *out)
{
    uint64_t n = seg_count(d, offsets, num_segments, bucket);
    for (uint64_t sgm = 0; sgm < n; ++sgm) {
        uint64_t b = seg_begin(sgm, d, offsets, num_segments, bucket);
        uint64_t e = seg_begin(sgm + 1, d, offsets, num_segments, bucket);
        for (uint64_t i = b; i < e; ++i) {
            uint32_t c, sg;
            get_code(code, sign, i, s, &c, &sg);
            out[i] = dither_value(norms[sgm], s, c, sg);
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Sum over workers                                                         */
/* ------------------------------------------------------------------------ */

/* Worker w's planes start at exp + w*exp_stride and sign + w*sign_stride (bytes).
 * out64[i]  = sum over w of the decoded values, in double.
 * out32[i]  = the same sum taken left to right in binary32 (w = 0, 1, ...),
 *             starting from the first worker's value.
 * abs64[i]  = sum over w of |decoded value|, the scale a tolerance is relative to.
 * Any of the three outputs may be NULL. */
void orc_aggregate_nat(const uint8_t *exp, uint64_t exp_stride, const uint8_t *sign, uint64_t sign_stride,
                       uint32_t n, uint64_t d, double *out64, float *out32, double *abs64)
{
#pragma omp parallel for
    for (int64_t i = 0; i < (int64_t)d; ++i) {
        double acc64 = 0.0, acca = 0.0;
        volatile float acc32 = 0.0f;
        for (uint32_t w = 0; w < n; ++w) {
            float v = nat_value(exp + (uint64_t)w * exp_stride, sign + (uint64_t)w * sign_stride, (uint64_t)i);
            acc64 += (double)v;
            acca += fabs((double)v);
            acc32 = (w == 0) ? v : acc32 + v;
        }
        if (out64) out64[i] = acc64;
        if (out32) out32[i] = acc32;
        if (abs64) abs64[i] = acca;
    }
}

/* The same for dithering codes; worker w's norms start at norms + w*norm_stride (floats). */
void orc_aggregate_dither(const float *norms, uint64_t norm_stride, const uint8_t *code, uint64_t code_stride,
                          const uint8_t *sign, uint64_t sign_stride, uint32_t n, uint64_t d,
                          const uint64_t *offsets, uint32_t num_segments, uint32_t bucket, uint32_t s,
                          double *out64, float *out32, double *abs64)
{
    int64_t nseg = (int64_t)seg_count(d, offsets, num_segments, bucket);
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t sgm = 0; sgm < nseg; ++sgm) {
        uint64_t b = seg_begin((uint64_t)sgm, d, offsets, num_segments, bucket);
        uint64_t e = seg_begin((uint64_t)sgm + 1, d, offsets, num_segments, bucket);
        for (uint64_t i = b; i < e; ++i) {
            double acc64 = 0.0, acca = 0.0;
            volatile float acc32 = 0.0f;
            for (uint32_t w = 0; w < n; ++w) {
                uint32_t c, sg;
                get_code(code + (uint64_t)w * code_stride, sign ? sign + (uint64_t)w * sign_stride : NULL, i, s, &c, &sg);
                float v = dither_value(norms[(uint64_t)w * norm_stride + (uint64_t)sgm], s, c, sg);
                acc64 += (double)v;
                acca += fabs((double)v);
                acc32 = (w == 0) ? v : acc32 + v;
            }
            if (out64) out64[i] = acc64;
            if (out32) out32[i] = acc32;
            if (abs64) abs64[i] = acca;
        }
    }
}

/* Number of threads the "parallel for" loops above use (for reporting timings). */
#ifdef _OPENMP
#include <omp.h>
int orc_threads(void) { return omp_get_max_threads(); }
void orc_set_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int orc_threads(void) { return 1; }
void orc_set_threads(int n) { (void)n; }
#endif

/* ------------------------------------------------------------------------ */
/* Random sparsification composed with natural compression                  */
/* ------------------------------------------------------------------------ */

/* Random sparsification S^q (formal definition in the appendix on sparsification):
 * S^q(x) = (d/q) xi o x with xi uniform over the binary vectors with exactly q
 * ones; C_nat o S^q is then in B(9d/8q - 1) by the composition theorem.
 *
 * The paper does not say how xi is drawn.  Here the q kept coordinates are the
 * images pi(0), ..., pi(q-1) of a keyed pseudo-random permutation pi of [0, d):
 * a 4-round alternating Feistel network on b = ceil(log2 d) bits (at least 2)
 * whose round keys are the four words of one Philox call (counter
 * (0, 0, worker, 2), key = seed), with cycle walking (apply the network again
 * while the value is >= d; fewer than two applications on average), so pi is a
 * bijection of [0, d) and any j can be evaluated on its own. */
enum { ORC_DOMAIN_SPARSE = 2 };

static uint32_t feistel_round_fn(uint32_t r, uint32_t key)
{
    uint32_t t = r * 0x9E3779B1u + key;
    t ^= t >> 16; t *= 0x85EBCA6Bu;
    t ^= t >> 13; t *= 0xC2B2AE35u;
    t ^= t >> 16;
    return t;
}

/* Number of bits of the network: the smallest b >= 2 with 2^b >= d. */
static uint32_t network_bits(uint64_t d)
{
    uint32_t b = 2;
    while (b < 32 && ((uint64_t)1 << b) < d) ++b;
    return b;
}

/* pi(j) for 0 <= j < d <= 2^32.  The b-bit value is split into a high part A of
 * floor(b/2) bits and a low part B of the remaining bits; the four rounds are
 * A ^= F(B, k0), B ^= F(A, k1), A ^= F(B, k2), B ^= F(A, k3), each truncated to
 * the width of the part it changes (every round is its own inverse, so the
 * network is a bijection of [0, 2^b)). */
uint64_t orc_sparse_index(uint64_t d, uint64_t seed, uint32_t worker, uint64_t j)
{
    uint32_t ctr[4] = { 0, 0, worker, ORC_DOMAIN_SPARSE };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t rk[4];
    orc_philox4x32_10(ctr, key, rk);
    uint32_t b = network_bits(d);
    uint32_t bits_a = b / 2, bits_b = b - bits_a;
    uint32_t mask_a = (1u << bits_a) - 1u, mask_b = (1u << bits_b) - 1u;
    uint64_t v = j;
    do {
        uint32_t A = (uint32_t)(v >> bits_b) & mask_a, B = (uint32_t)v & mask_b;
        A ^= feistel_round_fn(B, rk[0]) & mask_a;
        B ^= feistel_round_fn(A, rk[1]) & mask_b;
        A ^= feistel_round_fn(B, rk[2]) & mask_a;
        B ^= feistel_round_fn(A, rk[3]) & mask_b;
        v = ((uint64_t)A << bits_b) | B;
    } while (v >= d);
    return v;
}

/* Worker's message: for j < k the kept index i = pi(j), and C_nat applied to
 * fl(scale * x[i]) (scale = d/k makes the operator unbiased) with the random
 * word of dense position i in the C_nat stream.  Exponent byte j and sign bit j
 * of the planes belong to idx_out[j]. */
void orc_sparse_nat_encode(const float *x, uint64_t d, uint64_t k, float scale, uint64_t seed,
                           uint32_t worker, uint32_t *idx_out, uint8_t *exp_out, uint8_t *sign_out)
{
    memset(sign_out, 0, (k + 7) / 8);
    for (uint64_t j = 0; j < k; ++j) {
        uint64_t i = orc_sparse_index(d, seed, worker, j);
        volatile float v = scale * x[i];
        uint32_t u = f32_bits(v);
        uint32_t r = orc_random_word(seed, worker, ORC_DOMAIN_NAT, i);
        idx_out[j] = (uint32_t)i;
        exp_out[j] = (uint8_t)orc_nat_round(u, r);
        sign_out[j >> 3] |= (uint8_t)((u >> 31) << (j & 7));
    }
}

/* Dense sum of n sparse messages: out starts at zero; workers are added in
 * the order w = 0, 1, ...; out32 in binary32, out64 in double, abs64 = sum of
 * magnitudes.  Strides are in elements of the respective arrays. */
void orc_sparse_nat_aggregate(const uint32_t *idx, uint64_t idx_stride, const uint8_t *exp, uint64_t exp_stride,
                              const uint8_t *sign, uint64_t sign_stride, uint32_t n, uint64_t k, uint64_t d,
                              float *out32, double *out64, double *abs64)
{
    for (uint64_t i = 0; i < d; ++i) {
        if (out32) out32[i] = 0.0f;
        if (out64) out64[i] = 0.0;
        if (abs64) abs64[i] = 0.0;
    }
    for (uint32_t w = 0; w < n; ++w) {
        for (uint64_t j = 0; j < k; ++j) {
            uint64_t i = idx[(uint64_t)w * idx_stride + j];
            float v = nat_value(exp + (uint64_t)w * exp_stride, sign + (uint64_t)w * sign_stride, j);
            if (out32) { volatile float t = out32[i] + v; out32[i] = t; }
            if (out64) out64[i] += (double)v;
            if (abs64) abs64[i] += fabs((double)v);
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Master-side compression                                                  */
/* ------------------------------------------------------------------------ */

/* Algorithm 1, master: Delta = sum over workers of the decompressed updates,
 * then g = C_M(Delta) with C_M = C_nat (bidirectional compression; the master's
 * draws come from their own stream, domain 3, keyed by `master` instead of a
 * worker id).  The sum is the binary32 left-to-right sum of orc_aggregate_nat.
 * `sum32` is caller scratch of d floats (it receives Delta). */
void orc_master_nat(const uint8_t *exp, uint64_t exp_stride, const uint8_t *sign, uint64_t sign_stride,
                    uint32_t n, uint64_t d, uint64_t seed, uint32_t master, uint64_t index_offset,
                    float *sum32, uint8_t *exp_out, uint8_t *sign_out)
{
    orc_aggregate_nat(exp, exp_stride, sign, sign_stride, n, d, NULL, sum32, NULL);
    nat_encode_domain(sum32, d, seed, master, ORC_DOMAIN_MASTER, index_offset, exp_out, sign_out);
}

/* ------------------------------------------------------------------------ */
/* Compressed norm                                                          */
/* ------------------------------------------------------------------------ */

/* General dithering sends C(||x||_p); with C = C_nat the norm is a power of two
 * (8 bits on the wire) and multiplying a level by it is an exponent addition
 * (Sec. 3).  norm s of a worker draws the word of index s in a stream of its own
 * (domain 4).  exp_out[s] = exponent byte, q_out[s] = the power of two it stands
 * for (norms are non-negative: no sign is kept). */
void orc_norm_compress(const float *norms, uint64_t count, uint64_t seed, uint32_t worker,
                       uint8_t *exp_out, float *q_out)
{
    for (uint64_t s = 0; s < count; ++s) {
        uint32_t u = f32_bits(norms[s]) & 0x7FFFFFFFu;
        uint32_t r = orc_random_word(seed, worker, ORC_DOMAIN_NORM, s);
        uint32_t e = orc_nat_round(u, r);
        exp_out[s] = (uint8_t)e;
        q_out[s] = bits_f32(e << 23);
    }
}

/* ------------------------------------------------------------------------ */
/* Standard dithering (comparison operator)                                 */
/* ------------------------------------------------------------------------ */

/* Def. 3 with the linear partition l_j = j/s (standard dithering, the operator
 * of QSGD and TernGrad) and the norm sent as it is.  Level code c in 0..s
 * stands for c/s.  y lies between floor(ys)/s and (floor(ys)+1)/s and goes to
 * the higher one with probability ys - floor(ys).  y is given as a binary32
 * number; t = fl(y s) is one rounded product, t - floor(t) is exact, and the
 * comparison with r/2^32 is the integer comparison r < floor(frac 2^32).
 * t >= s (y >= 1, or a NaN) is the top level. */
uint32_t orc_sta_level(float y, uint32_t s, uint32_t r)
{
    volatile float t = y * (float)s;
    if (!(t < (float)s)) return s;
    float fl = floorf(t);
    float frac = t - fl;
    uint64_t threshold = (uint64_t)(frac * 4294967296.0f);
    return (uint32_t)fl + (((uint64_t)r < threshold) ? 1u : 0u);
}

uint64_t orc_sta_count(float y, uint32_t s, uint32_t code)
{
    uint64_t count = 0;
#pragma omp parallel for reduction(+ : count)
    for (int64_t r = 0; r < ((int64_t)1 << 32); ++r)
        count += (orc_sta_level(y, s, (uint32_t)r) == code);
    return count;
}

/* Same segments, normalisation (y = fl(|x| fl(1/norm))), random stream and packed
 * layout as orc_dither_encode; 1 <= s <= 255. */
void orc_sta_encode(const float *x, uint64_t d, const uint64_t *offsets, uint32_t num_segments,
                    uint32_t bucket, uint32_t s, const float *norms, uint64_t seed, uint32_t worker,
                    uint64_t index_offset, uint8_t *code_out, uint8_t *sign_out)
{
    memset(code_out, 0, orc_dither_code_bytes(d, s));
    if (orc_dither_sign_bytes(d, s)) memset(sign_out, 0, orc_dither_sign_bytes(d, s));
    uint64_t n = seg_count(d, offsets, num_segments, bucket);
    for (uint64_t sgm = 0; sgm < n; ++sgm) {
        uint64_t b = seg_begin(sgm, d, offsets, num_segments, bucket);
        uint64_t e = seg_begin(sgm + 1, d, offsets, num_segments, bucket);
        float inv = orc_dither_inv_norm(norms[sgm]);
        for (uint64_t i = b; i < e; ++i) {
            volatile float y = fabsf(x[i]) * inv;
            uint32_t r = orc_dither_word(seed, worker, index_offset + i);
            put_code(code_out, sign_out, i, s, orc_sta_level(y, s, r), f32_bits(x[i]) >> 31);
        }
    }
}

/* sign * fl(norm * fl(c / s)), a signed zero for c = 0. */
void orc_sta_decode(const float *norms, const uint8_t *code, const uint8_t *sign, uint64_t d,
                    const uint64_t *offsets, uint32_t num_segments, uint32_t bucket, uint32_t s, float *out)
{
    uint64_t n = seg_count(d, offsets, num_segments, bucket);
    for (uint64_t sgm = 0; sgm < n; ++sgm) {
        uint64_t b = seg_begin(sgm, d, offsets, num_segments, bucket);
        uint64_t e = seg_begin(sgm + 1, d, offsets, num_segments, bucket);
        for (uint64_t i = b; i < e; ++i) {
            uint32_t c, sg;
            get_code(code, sign, i, s, &c, &sg);
            float mag = 0.0f;
            if (c > 0) {
                volatile float level = (float)c / (float)s;
                volatile float v = norms[sgm] * level;
                mag = v;
            }
            out[i] = sg ? -mag : mag;
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Clipped 8-bit format and integer aggregation                             */
/* ------------------------------------------------------------------------ */

/* The 8-bit representation of the in-network aggregation prototype
 * (experimental setup, "Implementation optimization"): one sign bit, one bit
 * that marks a zero, and 6 bits for the exponent of C_nat(x) clipped to the
 * range -50 .. 10, so that the aggregator can hold every value as a 64-bit
 * integer in units of 2^-50.  Byte layout chosen here: bit 7 = sign, bit 6 =
 * zero flag, bits 5..0 = clip(exponent, -50, 10) + 50 (0 when the flag is set).
 * Readings: "clip" clamps, so a value below 2^-50 becomes 2^-50 and a value
 * above 2^10 (Inf and NaN included) becomes 2^10, which biases the operator
 * outside the range exactly as the text accepts; C_nat(x) = 0 only for x = 0
 * (and for a subnormal x that rounds down to exponent field 0).  The draws
 * are those of orc_nat_encode (domain 0). */
void orc_clip_encode(const float *x, uint64_t d, uint64_t seed, uint32_t worker, uint64_t index_offset,
                     uint8_t *code_out)
{
#pragma omp parallel for
    for (int64_t ii = 0; ii < (int64_t)d; ++ii) {
        uint64_t i = (uint64_t)ii;
        uint32_t u = f32_bits(x[i]);
        uint32_t r = orc_random_word(seed, worker, ORC_DOMAIN_NAT, index_offset + i);
        int32_t e = (int32_t)orc_nat_round(u, r); /* exponent field of C_nat(x) */
        uint32_t byte;
        if (e == 0) {
            byte = 0x40u;
        } else {
            int32_t expo = e - 127;
            if (expo < -50) expo = -50;
            if (expo > 10) expo = 10;
            byte = (uint32_t)(expo + 50);
        }
        code_out[i] = (uint8_t)(byte | ((u >> 31) << 7));
    }
}

/* The value a byte stands for as an integer in units of 2^-50: 0 if the zero
 * flag is set, else +-2^field.  Fields 61..63 are never produced by the encoder;
 * they are taken literally (arithmetic modulo 2^64). */
static uint64_t clip_units(uint8_t byte)
{
    uint64_t mag = (byte & 0x40u) ? 0ull : (1ull << (byte & 63u));
    return (byte & 0x80u) ? (0ull - mag) : mag;
}

/* Decoded binary32 value: sign and 2^(field - 50), or a signed zero. */
void orc_clip_decode(const uint8_t *code, uint64_t d, float *out)
{
    for (uint64_t i = 0; i < d; ++i) {
        uint32_t sign = (uint32_t)(code[i] >> 7) << 31;
        uint32_t mag = (code[i] & 0x40u) ? 0u : (((uint32_t)(code[i] & 63u) - 50u + 127u) << 23);
        out[i] = bits_f32(sign | mag);
    }
}

/* Aggregator of the prototype (experimental setup; appendix on fast
 * aggregation): every value is restored as a 64-bit integer with one non-zero
 * bit, the n workers are added as integers (exact; two's complement, so the
 * order does not matter; n * 2^60 < 2^63 holds for n <= 7, beyond that the sum
 * is exact modulo 2^64), and the sum is compressed again with C_nat (Algorithm
 * 1, master side) from the master's stream (domain 3).  C_nat of an integer
 * S != 0 with 2^k <= |S| < 2^(k+1): exponent k + 1 with probability
 * (|S| - 2^k) / 2^k, else k.  Reading: the probability is compared in 32 bits,
 * r < floor(((|S| - 2^k) / 2^k) * 2^32), the same rule as orc_nat_round when |S|
 * has at most 24 significant bits; below that, at most 2^-32 of probability is
 * lost to truncation.  Outputs: sum_out[i] (may be NULL) in units of 2^-50; the
 * planes of orc_nat_encode for the compressed sum, exponent field k - 50 + 127
 * (+1), 0 for S = 0; sign bit set for S < 0. */
/* C_nat of one integer sum (two's complement in `total`) with the word r: the
 * exponent field of the result, 0 for a zero sum. */
uint32_t orc_clip_round(int64_t total_signed, uint32_t r)
{
    uint64_t total = (uint64_t)total_signed;
    uint64_t mag = (total >> 63) ? (0ull - total) : total;
    if (mag == 0) return 0;
    int k = 63;
    while (!((mag >> k) & 1ull)) --k;
    uint64_t rest = mag - (1ull << k);  /* < 2^k */
    /* floor(rest / 2^k * 2^32) */
    uint64_t threshold = k >= 32 ? (rest >> (k - 32)) : (rest << (32 - k));
    return (uint32_t)(k - 50 + 127) + (((uint64_t)r < threshold) ? 1u : 0u);
}

/* Exhaustive count of "exponent + 1" outcomes over all 2^32 words r. */
uint64_t orc_clip_count_up(int64_t total)
{
    uint32_t low = orc_clip_round(total, 0xFFFFFFFFu);
    uint64_t count = 0;
#pragma omp parallel for reduction(+ : count)
    for (int64_t r = 0; r < ((int64_t)1 << 32); ++r)
        count += (orc_clip_round(total, (uint32_t)r) != low);
    return count;
}

/* First global index g in [start, start + count) whose word is below `bound`,
 * or -1 (lets a test place a chosen sum on an element whose word it knows). */
int64_t orc_find_word_below(uint64_t seed, uint32_t worker, uint32_t domain, uint64_t start, uint64_t count,
                            uint32_t bound)
{
    for (uint64_t g = start; g < start + count; ++g)
        if (orc_random_word(seed, worker, domain, g) < bound) return (int64_t)g;
    return -1;
}

void orc_clip_aggregate(const uint8_t *code, uint64_t code_stride, uint32_t n, uint64_t d, uint64_t seed,
                        uint32_t master, uint64_t index_offset, int64_t *sum_out, uint8_t *exp_out,
                        uint8_t *sign_out)
{
    memset(sign_out, 0, (d + 7) / 8);
    for (uint64_t i = 0; i < d; ++i) {
        uint64_t total = 0;
        for (uint32_t w = 0; w < n; ++w) total += clip_units(code[(uint64_t)w * code_stride + i]);
        if (sum_out) sum_out[i] = (int64_t)total;
        uint32_t negative = (uint32_t)(total >> 63);
        uint32_t r = orc_random_word(seed, master, ORC_DOMAIN_MASTER, index_offset + i);
        exp_out[i] = (uint8_t)orc_clip_round((int64_t)total, r);
        sign_out[i >> 3] |= (uint8_t)(negative << (i & 7));
    }
}

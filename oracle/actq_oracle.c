/*
 * actq_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow CPU statement of what the activation-compression hot path of
 * ActNN (arXiv 2104.14129) computes: per-group min/range, stochastic rounding
 * to b-bit codes, a linear bit stream, dequantization, and the greedy bit
 * allocator, plus the exact contexts of ReLU and max-pooling layers.  It follows
 * the paper step by step (Sec. 4.1 for the quantizer, Sec. 4.2 Prob. (9) and
 * Sec. 4.3 for the allocator, the appendix sections "Activation Layers" and
 * "Pooling Layers" for the exact contexts) and shares no code,
 * header, table or constant with the GPU library.  Only tests, the smoke check
 * and the cpu_baseline leg of the benchmark may call it.
 *
 * Parity status: every function below is pinned by tests that do not depend on
 * this file (see tests/test_oracle_*.py), except the *optimality* of the greedy
 * allocator in general, which the paper itself calls a heuristic: that is
 * "parity unpinned".
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC.
 * -ffp-contract=off matters: the subtraction and the multiplication of the
 * scaling step are two separately rounded binary32 operations.
 * The loops over groups carry an OpenMP pragma; results do not depend on the
 * thread count because the noise is a pure function of (seed, tag, n, d).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_EINFEASIBLE (-2)

/* ------------------------------------------------------------------------- */
/* binary16 <-> binary32, written out by hand (this gcc has no _Float16).     */

/* Exact widening of an IEEE binary16 bit pattern. */
float orc_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    int exp = (h >> 10) & 0x1f;
    uint32_t man = h & 0x3ffu;
    float v;
    if (exp == 0) {
        v = ldexpf((float)man, -24); /* zero or subnormal: man * 2^-24 */
    } else if (exp == 31) {
        v = man ? NAN : INFINITY;
    } else {
        v = ldexpf((float)(man | 0x400u), exp - 25); /* 1.man * 2^(exp-15) */
    }
    return sign ? -v : v;
}

/* Round-to-nearest-even narrowing of a binary32 value to binary16 bits. */
uint16_t orc_float_to_half(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    float a = fabsf(f);
    if (isnan(f)) return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0f) return (uint16_t)(sign | 0x7c00u); /* rounds to infinity */
    if (a < 6.103515625e-05f) {
        /* below the smallest normal half: the result is an integer multiple of
         * 2^-24; nearbyintf rounds half-way cases to even. */
        float k = nearbyintf(ldexpf(a, 24));
        return (uint16_t)(sign | (uint16_t)k); /* k == 1024 lands on the smallest normal */
    }
    int e;
    float m = frexpf(a, &e);                 /* a = m * 2^e, m in [0.5, 1) */
    float k = nearbyintf(ldexpf(m, 11));     /* 11 significant bits, in [1024, 2048] */
    if (k == 2048.0f) { k = 1024.0f; e += 1; }
    /* a = (k/1024) * 2^(e-1): biased exponent e-1+15 */
    return (uint16_t)(sign | (uint16_t)((e + 14) << 10) | ((uint16_t)k & 0x3ffu));
}

static float load_elem(const void* x, int dtype, int64_t idx)
{
    if (dtype == 0) return ((const float*)x)[idx];
    return orc_half_to_float(((const uint16_t*)x)[idx]);
}

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of two        */
/* 32x32->64 multiplications; the key is bumped by the Weyl constants before   */
/* every round but the first.                                                  */

void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Uniform noise on a grid of 2^noise_bits points in [0,1) for feature d of
 * sample n.  24 bits: one output word per element, four elements per counter.
 * 16 bits: half a word per element, eight elements per counter. */
float orc_noise(uint64_t seed, uint64_t tag, uint32_t n, uint64_t d, int noise_bits)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t ctr[4], out[4];
    ctr[1] = n;
    ctr[2] = (uint32_t)tag;
    ctr[3] = (uint32_t)(tag >> 32);
    if (noise_bits == 24) {
        ctr[0] = (uint32_t)(d >> 2);
        orc_philox4x32_10(ctr, key, out);
        uint32_t r = out[d & 3];
        return (float)(r >> 8) * 5.9604644775390625e-08f; /* 2^-24, exact */
    }
    ctr[0] = (uint32_t)(d >> 3);
    orc_philox4x32_10(ctr, key, out);
    uint32_t word = out[(d >> 1) & 3];
    uint32_t r16 = (d & 1) ? (word >> 16) : (word & 0xffffu);
    return (float)r16 * 1.52587890625e-05f; /* 2^-16, exact */
}

/* ------------------------------------------------------------------------- */

/* Any whole number of bits from 1 to 8 (Sec. 4.3 lowers a width one bit at a time). */
static int width_ok(int b) { return b >= 1 && b <= 8; }

/* The bit stream is linear and LSB-first: bit k of the stream is bit (k mod 8) of byte
 * floor(k / 8), and the code of element j of a group occupies stream bits [j*b, j*b + b).
 * A code whose width does not divide 8 may straddle two bytes. */
static void put_code(uint8_t* dst, int64_t j, int b, unsigned code)
{
    for (int k = 0; k < b; ++k) {
        int64_t bit = j * b + k;
        if ((code >> k) & 1u) dst[bit / 8] |= (uint8_t)(1u << (bit % 8));
    }
}

static unsigned get_code(const uint8_t* src, int64_t j, int b)
{
    unsigned code = 0;
    for (int k = 0; k < b; ++k) {
        int64_t bit = j * b + k;
        code |= (unsigned)((src[bit / 8] >> (bit % 8)) & 1u) << k;
    }
    return code;
}

int orc_packed_bytes(int64_t N, int64_t D, int32_t G, const uint8_t* bits,
                     uint64_t* offsets, uint64_t* total)
{
    if (N <= 0 || D <= 0 || G <= 0 || (G % 8) != 0 || !bits) return ORC_EINVAL;
    uint64_t ng = (uint64_t)((D + G - 1) / G);
    uint64_t acc = 0;
    for (int64_t n = 0; n < N; ++n) {
        if (!width_ok(bits[n])) return ORC_EINVAL;
        if (offsets) offsets[n] = acc;
        acc += ng * (uint64_t)G * bits[n] / 8;
    }
    if (total) *total = acc;
    return ORC_OK;
}

/* Sec. 4.1: zero point Z = min and range R = max - min of one group. */
static void group_min_range(const void* x, int dtype, int64_t base, int64_t len,
                            float* mn_out, float* range_out)
{
    float mn = load_elem(x, dtype, base);
    float mx = mn;
    for (int64_t j = 1; j < len; ++j) {
        float v = load_elem(x, dtype, base + j);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    mn = mn + 0.0f; /* -0.0 becomes +0.0: one canonical stored zero point */
    *mn_out = mn;
    /* a range of zero is +0.0 whichever zeros the extremes were (the maximum of -0.0 and +0.0 is
     * either of them) */
    *range_out = (mx - mn) + 0.0f;
}

int orc_group_stats(const void* x, int dtype, int64_t N, int64_t D, int32_t G,
                    float* gmin, float* grange)
{
    if (!x || !gmin || !grange || N <= 0 || D <= 0 || G <= 0) return ORC_EINVAL;
    int64_t ng = (D + G - 1) / G;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N * ng; ++t) {
        int64_t n = t / ng, g = t % ng;
        int64_t len = (g * G + G <= D) ? G : D - g * G;
        group_min_range(x, dtype, n * D + g * G, len, &gmin[t], &grange[t]);
    }
    return ORC_OK;
}

/* Sec. 4.1: the factor B / R of the scaling step and the stored step R / B.  A group
 * whose range is zero, or so small that B / R overflows, is degenerate: both are 0,
 * every code is 0 and dequantization returns Z. */
static void group_scale(float B, float range, float* inv_out, float* scale_out)
{
    float inv = 0.0f, scale = 0.0f;
    if (range != 0.0f) {
        float cand = B / range;
        if (isfinite(cand)) {
            inv = cand;
            scale = range / B;
        }
    }
    *inv_out = inv;
    *scale_out = scale;
}

/* Sec. 4.1: u = B (h - Z) / R in [0, B]; the code is ceil(u) with probability
 * u - floor(u) and floor(u) otherwise.  Two realisations of that rule:
 *   24-bit noise: compare the noise with the fractional part, code = floor(u) + [noise < frac];
 *   16-bit noise: add the noise and floor, code = floor(u + noise), the sum being one binary32
 *                 addition rounded to nearest.  (In exact arithmetic floor(u + U) with U uniform
 *                 on [0,1) rounds up when U >= 1 - frac, i.e. with probability frac.  Here the
 *                 noise lies on a 2^-16 grid and the sum is rounded, so the probability of
 *                 rounding up over the 65,536 noise values is frac only to within 2^-16: that is
 *                 the bound the tests enumerate.)  With u <= 255 the sum of an integer u and the
 *                 noise is exact, so grid points keep their code, and u + noise <= B + 1 - 2^-16
 *                 is representable, so the code never exceeds B. */
static unsigned stochastic_code(float h, float mn, float inv, float B, float noise, int noise_bits)
{
    float centred = h - mn;
    float u = centred * inv;
    if (u > B) u = B; /* the two roundings above can overshoot B by an ulp */
    if (noise_bits == 16) {
        float shifted = u + noise;
        return (unsigned)floorf(shifted);
    }
    float fl = floorf(u);
    float frac = u - fl; /* exact */
    return (unsigned)fl + (noise < frac ? 1u : 0u);
}

/* Sec. 4.1: u = B (h - Z) / R scaled to [0, B], then stochastic rounding:
 * ceil(u) with probability u - floor(u), floor(u) otherwise. */
/* One group: `len` valid elements starting at element index `first` of buffer x, being
 * features d_start .. d_start+len-1 of sample n.  Writes G*b/8 bytes of bit stream (the
 * padding codes of a ragged group are 0) and the two header floats (Z, R / B). */
int orc_quantize_group(const void* x, int dtype, int64_t first, int64_t len, int32_t G, int b,
                       uint64_t seed, uint64_t tag, uint32_t n, uint64_t d_start,
                       int32_t noise_bits, uint8_t* dst, float* header2)
{
    if (!x || !dst || !header2 || len <= 0 || len > G || !width_ok(b)) return ORC_EINVAL;
    if (noise_bits != 24 && noise_bits != 16) return ORC_EINVAL;
    float B = (float)((1 << b) - 1);
    float mn, range;
    group_min_range(x, dtype, first, len, &mn, &range);
    float inv, scale;
    group_scale(B, range, &inv, &scale);
    header2[0] = mn;
    header2[1] = scale;
    memset(dst, 0, (size_t)G * b / 8);
    for (int64_t j = 0; j < len; ++j) {
        float h = load_elem(x, dtype, first + j);
        float noise = orc_noise(seed, tag, n, d_start + (uint64_t)j, noise_bits);
        unsigned code = stochastic_code(h, mn, inv, B, noise, noise_bits);
        put_code(dst, j, b, code);
    }
    return ORC_OK;
}

int orc_quantize_pack(const void* x, int dtype, int64_t N, int64_t D, int32_t G,
                      const uint8_t* bits, const uint64_t* offsets,
                      uint64_t seed, uint64_t tag, int32_t noise_bits,
                      uint8_t* packed, float* header)
{
    if (!x || !bits || !offsets || !packed || !header) return ORC_EINVAL;
    if (N <= 0 || D <= 0 || G <= 0 || (G % 8) != 0) return ORC_EINVAL;
    if (noise_bits != 24 && noise_bits != 16) return ORC_EINVAL;
    for (int64_t n = 0; n < N; ++n)
        if (!width_ok(bits[n])) return ORC_EINVAL;
    int64_t ng = (D + G - 1) / G;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N * ng; ++t) {
        int64_t n = t / ng, g = t % ng;
        int b = bits[n];
        int64_t len = (g * G + G <= D) ? G : D - g * G;
        uint8_t* dst = packed + offsets[n] + (uint64_t)g * G * b / 8;
        orc_quantize_group(x, dtype, n * D + g * G, len, G, b, seed, tag, (uint32_t)n,
                           (uint64_t)(g * G), noise_bits, dst, &header[2 * t]);
    }
    return ORC_OK;
}

/* One group of the backward pass: `len` values from G*b/8 bytes and (Z, scale). */
int orc_dequantize_group(const uint8_t* src, const float* header2, int b, int64_t len,
                         void* out, int out_dtype, int64_t first)
{
    if (!src || !header2 || !out || len <= 0 || !width_ok(b)) return ORC_EINVAL;
    float mn = header2[0], scale = header2[1];
    for (int64_t j = 0; j < len; ++j) {
        unsigned code = get_code(src, j, b);
        float v = fmaf((float)code, scale, mn);
        if (out_dtype == 0)
            ((float*)out)[first + j] = v;
        else
            ((uint16_t*)out)[first + j] = orc_float_to_half(v);
    }
    return ORC_OK;
}

/* Sec. 4.1: h^ = code * R / B + Z with scale = R / B stored in the header. */
int orc_unpack_dequantize(const uint8_t* packed, const float* header,
                          const uint8_t* bits, const uint64_t* offsets,
                          int64_t N, int64_t D, int32_t G, void* out, int out_dtype)
{
    if (!packed || !header || !bits || !offsets || !out) return ORC_EINVAL;
    if (N <= 0 || D <= 0 || G <= 0 || (G % 8) != 0) return ORC_EINVAL;
    for (int64_t n = 0; n < N; ++n)
        if (!width_ok(bits[n])) return ORC_EINVAL;
    int64_t ng = (D + G - 1) / G;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N * ng; ++t) {
        int64_t n = t / ng, g = t % ng;
        int b = bits[n];
        int64_t len = (g * G + G <= D) ? G : D - g * G;
        const uint8_t* src = packed + offsets[n] + (uint64_t)g * G * b / 8;
        orc_dequantize_group(src, &header[2 * t], b, len, out, out_dtype, n * D + g * G);
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Sec. 4.1, last paragraph: the per-group range and zero point stored in       */
/* bfloat16, 32 bits per group.  So that every element still scales into [0, B] */
/* the zero point is rounded DOWN to bfloat16 and the range, taken from that     */
/* rounded zero point, is rounded UP; the quantizer stays unbiased because it is */
/* unbiased for any (Z, R) that cover the group.                                 */

float orc_bf16_to_float(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* largest bfloat16 value <= f (f finite) */
uint16_t orc_bf16_floor(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t top = u >> 16;
    if ((u & 0xffffu) != 0 && (u >> 31)) top += 1; /* negative: truncation moved it up, step down */
    return (uint16_t)top;
}

/* smallest bfloat16 value >= f (f finite) */
uint16_t orc_bf16_ceil(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t top = u >> 16;
    if ((u & 0xffffu) != 0 && !(u >> 31)) top += 1; /* positive: truncation moved it down, step up */
    return (uint16_t)top;
}

static void group_min_max(const void* x, int dtype, int64_t base, int64_t len, float* mn_out, float* mx_out)
{
    float mn = load_elem(x, dtype, base), mx = mn;
    for (int64_t j = 1; j < len; ++j) {
        float v = load_elem(x, dtype, base + j);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    *mn_out = mn + 0.0f;
    *mx_out = mx;
}

int orc_quantize_group_bf16(const void* x, int dtype, int64_t first, int64_t len, int32_t G, int b,
                            uint64_t seed, uint64_t tag, uint32_t n, uint64_t d_start,
                            int32_t noise_bits, uint8_t* dst, uint16_t* header2)
{
    if (!x || !dst || !header2 || len <= 0 || len > G || !width_ok(b)) return ORC_EINVAL;
    if (noise_bits != 24 && noise_bits != 16) return ORC_EINVAL;
    float B = (float)((1 << b) - 1);
    float mn, mx;
    group_min_max(x, dtype, first, len, &mn, &mx);
    uint16_t zb = orc_bf16_floor(mn);
    float z = orc_bf16_to_float(zb);
    float span = mx - z;                       /* from the stored zero point */
    uint16_t rb = orc_bf16_ceil(span);
    float r = orc_bf16_to_float(rb);
    float inv, scale;
    if (!isfinite(r)) r = 0.0f;                /* rounding up overflowed: treat as degenerate */
    group_scale(B, r, &inv, &scale);
    if (inv == 0.0f) rb = 0;                   /* degenerate groups store R = 0 */
    header2[0] = zb;
    header2[1] = rb;
    memset(dst, 0, (size_t)G * b / 8);
    for (int64_t j = 0; j < len; ++j) {
        float h = load_elem(x, dtype, first + j);
        float noise = orc_noise(seed, tag, n, d_start + (uint64_t)j, noise_bits);
        unsigned code = stochastic_code(h, z, inv, B, noise, noise_bits);
        put_code(dst, j, b, code);
    }
    return ORC_OK;
}

int orc_quantize_pack_bf16(const void* x, int dtype, int64_t N, int64_t D, int32_t G,
                           const uint8_t* bits, const uint64_t* offsets,
                           uint64_t seed, uint64_t tag, int32_t noise_bits,
                           uint8_t* packed, uint16_t* header)
{
    if (!x || !bits || !offsets || !packed || !header) return ORC_EINVAL;
    if (N <= 0 || D <= 0 || G <= 0 || (G % 8) != 0) return ORC_EINVAL;
    if (noise_bits != 24 && noise_bits != 16) return ORC_EINVAL;
    for (int64_t n = 0; n < N; ++n)
        if (!width_ok(bits[n])) return ORC_EINVAL;
    int64_t ng = (D + G - 1) / G;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N * ng; ++t) {
        int64_t n = t / ng, g = t % ng;
        int b = bits[n];
        int64_t len = (g * G + G <= D) ? G : D - g * G;
        uint8_t* dst = packed + offsets[n] + (uint64_t)g * G * b / 8;
        orc_quantize_group_bf16(x, dtype, n * D + g * G, len, G, b, seed, tag, (uint32_t)n,
                                (uint64_t)(g * G), noise_bits, dst, &header[2 * t]);
    }
    return ORC_OK;
}

/* Sec. 4.1: h^ = code * R / B + Z from the bfloat16 header: the step R / B is one binary32
 * division, then one fused multiply-add. */
int orc_unpack_dequantize_bf16(const uint8_t* packed, const uint16_t* header,
                               const uint8_t* bits, const uint64_t* offsets,
                               int64_t N, int64_t D, int32_t G, void* out, int out_dtype)
{
    if (!packed || !header || !bits || !offsets || !out) return ORC_EINVAL;
    if (N <= 0 || D <= 0 || G <= 0 || (G % 8) != 0) return ORC_EINVAL;
    for (int64_t n = 0; n < N; ++n)
        if (!width_ok(bits[n])) return ORC_EINVAL;
    int64_t ng = (D + G - 1) / G;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N * ng; ++t) {
        int64_t n = t / ng, g = t % ng;
        int b = bits[n];
        int64_t len = (g * G + G <= D) ? G : D - g * G;
        const uint8_t* src = packed + offsets[n] + (uint64_t)g * G * b / 8;
        float hd[2];
        hd[0] = orc_bf16_to_float(header[2 * t + 0]);
        hd[1] = orc_bf16_to_float(header[2 * t + 1]) / (float)((1 << b) - 1);
        orc_dequantize_group(src, hd, b, len, out, out_dtype, n * D + g * G);
    }
    return ORC_OK;
}

/* Sec. 4.2, Eq. (8) and the sentence after Prob. (9): the sensitivity of sample n of a linear
 * layer is w_n = (G / 6) * ||grad_n||^2 * ||R_n||^2, with R_n the vector of its group ranges.
 * grad2 may be NULL (then ||grad_n||^2 = 1).  Accumulated in double. */
int orc_sample_sensitivity(const float* grange, int64_t N, int64_t ng, int32_t G,
                           const float* grad2, float* w_out)
{
    if (!grange || !w_out || N <= 0 || ng <= 0 || G <= 0) return ORC_EINVAL;
    for (int64_t n = 0; n < N; ++n) {
        double acc = 0.0;
        for (int64_t g = 0; g < ng; ++g) {
            double r = grange[n * ng + g];
            acc += r * r;
        }
        double w = (double)G / 6.0 * acc * (grad2 ? (double)grad2[n] : 1.0);
        w_out[n] = (float)w;
    }
    return ORC_OK;
}

/* Codes alone (no packing), for tests that look at the rounding itself. */
int orc_quantize_codes(const void* x, int dtype, int64_t N, int64_t D, int32_t G,
                       const uint8_t* bits, uint64_t seed, uint64_t tag,
                       int32_t noise_bits, uint8_t* codes)
{
    if (!x || !bits || !codes || N <= 0 || D <= 0 || G <= 0) return ORC_EINVAL;
    int64_t ng = (D + G - 1) / G;
    for (int64_t n = 0; n < N; ++n)
        if (!width_ok(bits[n])) return ORC_EINVAL;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N * ng; ++t) {
        int64_t n = t / ng, g = t % ng;
        float B = (float)((1 << bits[n]) - 1);
        int64_t len = (g * G + G <= D) ? G : D - g * G;
        float mn, range;
        group_min_range(x, dtype, n * D + g * G, len, &mn, &range);
        float inv, scale;
        group_scale(B, range, &inv, &scale);
        for (int64_t j = 0; j < len; ++j) {
            float h = load_elem(x, dtype, n * D + g * G + j);
            float noise = orc_noise(seed, tag, (uint32_t)n, (uint64_t)(g * G + j), noise_bits);
            codes[n * D + g * G + j] = (uint8_t)stochastic_code(h, mn, inv, B, noise, noise_bits);
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Sec. 4.3: start every item at the widest allowed width and keep applying the  */
/* cheapest move until the budget of Prob. (9) holds.  The allowed widths are a    */
/* set given as a mask (bit b set: b bits allowed); a move takes one item to the   */
/* next narrower allowed width.  With every width allowed this is the paper's      */
/* one-bit-at-a-time greedy.  The price of a move is the variance it adds,         */
/* w (1/B_new^2 - 1/B_old^2), per bit it frees, D (b_old - b_new).                 */
/* Plain repeated linear scan: no heap, no sort.                                  */

static int next_narrower(uint32_t widths, int b)
{
    for (int c = b - 1; c >= 1; --c)
        if ((widths >> c) & 1u) return c;
    return 0;
}

static double move_price(float w, int64_t D, int b_now, int b_next)
{
    double B_now = (double)((1 << b_now) - 1), B_next = (double)((1 << b_next) - 1);
    double c = (1.0 / (B_next * B_next) - 1.0 / (B_now * B_now)) / (double)(b_now - b_next);
    return ((double)w * c) / (double)D;
}

int orc_allocate_bits_ladder(const float* w, const int64_t* D, int64_t M,
                             int64_t budget_bits, uint32_t widths, uint8_t* bits_out)
{
    if (!w || !D || !bits_out || M <= 0 || budget_bits < 0) return ORC_EINVAL;
    if ((widths & ~0x1feu) != 0 || (widths & 0x1feu) == 0) return ORC_EINVAL;
    for (int64_t i = 0; i < M; ++i)
        if (!(w[i] >= 0.0f) || !isfinite(w[i]) || D[i] <= 0) return ORC_EINVAL;
    int widest = next_narrower(widths, 9);
    /* the sum of D * 8 stays far below 2^63 for any real tensor */
    int64_t used = 0;
    for (int64_t i = 0; i < M; ++i) {
        bits_out[i] = (uint8_t)widest;
        used += widest * D[i];
    }
    while (used > budget_bits) {
        int64_t best = -1;
        double best_price = 0.0;
        for (int64_t i = 0; i < M; ++i) {
            int nb = next_narrower(widths, bits_out[i]);
            if (nb == 0) continue;
            double price = move_price(w[i], D[i], bits_out[i], nb);
            if (best < 0 || price < best_price) { /* ties: the lowest index wins */
                best = i;
                best_price = price;
            }
        }
        if (best < 0) return ORC_EINFEASIBLE; /* everything already at the narrowest width */
        int nb = next_narrower(widths, bits_out[best]);
        used -= D[best] * (bits_out[best] - nb);
        bits_out[best] = (uint8_t)nb;
    }
    return ORC_OK;
}

/* The widths {1, 2, 4, 8}: a code never straddles a byte. */
int orc_allocate_bits(const float* w, const int64_t* D, int64_t M,
                      int64_t budget_bits, uint8_t* bits_out)
{
    return orc_allocate_bits_ladder(w, D, M, budget_bits, 0x116u, bits_out);
}

/* The objective of Prob. (9), sum_i w_i / B_i^2, in double precision. */
double orc_objective(const float* w, const uint8_t* bits, int64_t M)
{
    double acc = 0.0;
    for (int64_t i = 0; i < M; ++i) {
        double B = (double)((1 << bits[i]) - 1);
        acc += (double)w[i] / (B * B);
    }
    return acc;
}

/* ------------------------------------------------------------------------- */
/* Appendix, "Activation Layers": a ReLU layer's context is one bit per         */
/* element, f'(x) = [x > 0], with no approximation.  The bits form the same     */
/* LSB-first stream as 1-bit codes and are padded with zeros to a whole number  */
/* of 256-bit groups.  Forward: y = x where x > 0, +0 elsewhere (so NaN and     */
/* -0.0 give +0).  Backward: grad_x = grad_y where the bit is set, +0 elsewhere. */

static void store_elem(void* y, int dtype, int64_t idx, float v)
{
    if (dtype == 0)
        ((float*)y)[idx] = v;
    else
        ((uint16_t*)y)[idx] = orc_float_to_half(v);
}

int orc_relu_forward(const void* x, int dtype, int64_t n, void* y, uint8_t* mask)
{
    if (!x || !y || !mask || n <= 0 || (dtype != 0 && dtype != 1)) return ORC_EINVAL;
    memset(mask, 0, (size_t)((n + 255) / 256) * 32);
    for (int64_t i = 0; i < n; ++i) {
        float v = load_elem(x, dtype, i);
        int positive = v > 0.0f;
        store_elem(y, dtype, i, positive ? v : 0.0f);
        if (positive) put_code(mask, i, 1, 1u);
    }
    return ORC_OK;
}

int orc_relu_backward(const uint8_t* mask, const void* grad_y, int dtype, int64_t n, void* grad_x)
{
    if (!mask || !grad_y || !grad_x || n <= 0 || (dtype != 0 && dtype != 1)) return ORC_EINVAL;
    for (int64_t i = 0; i < n; ++i) {
        float g = load_elem(grad_y, dtype, i);
        store_elem(grad_x, dtype, i, get_code(mask, i, 1) ? g : 0.0f);
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Appendix, "Max Pooling": y = max over the window; the context is, for every  */
/* output location, the position k of the maximum inside the window,            */
/* 0 <= k < K = kh*kw, stored in 8 bits.  k counts window positions row by row  */
/* (k = a*kw + b for window row a, column b); padded positions never win; among */
/* equal values the first in that order wins.  The gradient of an input         */
/* location is the sum of the output gradients whose stored position points at  */
/* it; outputs are visited row by row and added in binary32.                    */

int orc_pool2d_output_size(int32_t H, int32_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                           int32_t ph, int32_t pw, int32_t dh, int32_t dw, int32_t* OH, int32_t* OW)
{
    if (H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0 ||
        dh <= 0 || dw <= 0 || kh * kw > 256 || 2 * ph > kh || 2 * pw > kw)
        return ORC_EINVAL;
    int64_t eh = (int64_t)dh * (kh - 1) + 1, ew = (int64_t)dw * (kw - 1) + 1;
    if (H + 2 * ph < eh || W + 2 * pw < ew) return ORC_EINVAL;
    *OH = (int32_t)((H + 2 * ph - eh) / sh + 1);
    *OW = (int32_t)((W + 2 * pw - ew) / sw + 1);
    return ORC_OK;
}

int orc_maxpool2d_forward(const void* x, int dtype, int64_t planes, int32_t H, int32_t W,
                          int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                          int32_t dh, int32_t dw, void* y, uint8_t* argmax)
{
    int32_t OH, OW;
    if (!x || !y || !argmax || planes <= 0 || (dtype != 0 && dtype != 1)) return ORC_EINVAL;
    if (orc_pool2d_output_size(H, W, kh, kw, sh, sw, ph, pw, dh, dw, &OH, &OW)) return ORC_EINVAL;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < planes; ++p)
        for (int32_t i = 0; i < OH; ++i)
            for (int32_t j = 0; j < OW; ++j) {
                int have = 0, best_k = 0;
                float best = 0.0f;
                for (int32_t a = 0; a < kh; ++a)
                    for (int32_t b = 0; b < kw; ++b) {
                        int64_t r = (int64_t)sh * i - ph + (int64_t)dh * a;
                        int64_t c = (int64_t)sw * j - pw + (int64_t)dw * b;
                        if (r < 0 || r >= H || c < 0 || c >= W) continue;
                        float v = load_elem(x, dtype, (p * H + r) * W + c);
                        if (!have || v > best) {
                            have = 1;
                            best = v;
                            best_k = a * kw + b;
                        }
                    }
                int64_t o = (p * OH + i) * OW + j;
                store_elem(y, dtype, o, best);
                argmax[o] = (uint8_t)best_k;
            }
    return ORC_OK;
}

int orc_maxpool2d_backward(const uint8_t* argmax, const void* grad_y, int dtype, int64_t planes,
                           int32_t H, int32_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                           int32_t ph, int32_t pw, int32_t dh, int32_t dw, void* grad_x)
{
    int32_t OH, OW;
    if (!argmax || !grad_y || !grad_x || planes <= 0 || (dtype != 0 && dtype != 1)) return ORC_EINVAL;
    if (orc_pool2d_output_size(H, W, kh, kw, sh, sw, ph, pw, dh, dw, &OH, &OW)) return ORC_EINVAL;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < planes; ++p) {
        float* acc = (float*)malloc(sizeof(float) * (size_t)H * (size_t)W); /* binary32 accumulators of one plane */
        if (!acc) {
            bad = 1;
            continue;
        }
        for (int64_t t = 0; t < (int64_t)H * W; ++t) acc[t] = 0.0f;
        for (int32_t i = 0; i < OH; ++i)
            for (int32_t j = 0; j < OW; ++j) {
                int64_t o = (p * OH + i) * OW + j;
                int k = argmax[o];
                int64_t r = (int64_t)sh * i - ph + (int64_t)dh * (k / kw);
                int64_t c = (int64_t)sw * j - pw + (int64_t)dw * (k % kw);
                if (k >= kh * kw || r < 0 || r >= H || c < 0 || c >= W) {
                    bad = 1; /* a position the forward pass cannot have produced */
                    continue;
                }
                acc[r * W + c] += load_elem(grad_y, dtype, o);
            }
        for (int64_t t = 0; t < (int64_t)H * W; ++t) store_elem(grad_x, dtype, p * H * W + t, acc[t]);
        free(acc);
    }
    return bad ? ORC_EINVAL : ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Sec. 4.1 (the comparison made there) and Sec. 6.1 (the per-tensor baseline): */
/* one range and one zero point for the whole tensor, i.e. a single group.      */
/* Z = min over all elements, R = max - min; everything else (scaling, rounding, */
/* the bit stream, the widths per sample) is as in the per-group quantizer.      */

int orc_tensor_stats(const void* x, int dtype, int64_t n, float* zr)
{
    if (!x || !zr || n <= 0 || (dtype != 0 && dtype != 1)) return ORC_EINVAL;
    float mn, range;
    group_min_range(x, dtype, 0, n, &mn, &range);
    zr[0] = mn;
    zr[1] = range;
    return ORC_OK;
}

int orc_quantize_pack_tensor(const void* x, int dtype, int64_t N, int64_t D, int32_t G,
                             const uint8_t* bits, const uint64_t* offsets, uint64_t seed, uint64_t tag,
                             int32_t noise_bits, const float* zr, uint8_t* packed)
{
    if (!x || !bits || !offsets || !packed || !zr) return ORC_EINVAL;
    if (N <= 0 || D <= 0 || G <= 0 || (G % 8) != 0) return ORC_EINVAL;
    if (noise_bits != 24 && noise_bits != 16) return ORC_EINVAL;
    for (int64_t n = 0; n < N; ++n)
        if (!width_ok(bits[n])) return ORC_EINVAL;
    int64_t ng = (D + G - 1) / G;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N * ng; ++t) {
        int64_t n = t / ng, g = t % ng;
        int b = bits[n];
        float B = (float)((1 << b) - 1);
        float inv, scale;
        group_scale(B, zr[1], &inv, &scale);
        int64_t len = (g * G + G <= D) ? G : D - g * G;
        uint8_t* dst = packed + offsets[n] + (uint64_t)g * G * b / 8;
        memset(dst, 0, (size_t)G * b / 8);
        for (int64_t j = 0; j < len; ++j) {
            float h = load_elem(x, dtype, n * D + g * G + j);
            float noise = orc_noise(seed, tag, (uint32_t)n, (uint64_t)(g * G + j), noise_bits);
            put_code(dst, j, b, stochastic_code(h, zr[0], inv, B, noise, noise_bits));
        }
    }
    return ORC_OK;
}

int orc_unpack_dequantize_tensor(const uint8_t* packed, const float* zr, const uint8_t* bits,
                                 const uint64_t* offsets, int64_t N, int64_t D, int32_t G,
                                 void* out, int out_dtype)
{
    if (!packed || !zr || !bits || !offsets || !out) return ORC_EINVAL;
    if (N <= 0 || D <= 0 || G <= 0 || (G % 8) != 0) return ORC_EINVAL;
    for (int64_t n = 0; n < N; ++n)
        if (!width_ok(bits[n])) return ORC_EINVAL;
    int64_t ng = (D + G - 1) / G;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N * ng; ++t) {
        int64_t n = t / ng, g = t % ng;
        int b = bits[n];
        float hd[2], inv;
        hd[0] = zr[0];
        group_scale((float)((1 << b) - 1), zr[1], &inv, &hd[1]); /* the step R / B of this width */
        int64_t len = (g * G + G <= D) ? G : D - g * G;
        const uint8_t* src = packed + offsets[n] + (uint64_t)g * G * b / 8;
        orc_dequantize_group(src, hd, b, len, out, out_dtype, n * D + g * G);
    }
    return ORC_OK;
}

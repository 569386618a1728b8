/*
 * mesa_ref.c -- CPU oracle for Mesa's activation-compression hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * tests, the smoke check and the benchmark's cpu_baseline leg compare the GPU
 * library against.  Nothing in the product path may call it, and it shares no
 * code, header, table or constant generator with the HIP sources.
 *
 * What it follows (Mesa, arXiv 2111.11124):
 *   Sec. 3.2 Eq. (3)   x_bar = clip(round((x - beta_h) * 255 / alpha_h), 0, 255)
 *   Sec. 3.2 Eq. (4)   stochastic rounding: ceil with probability frac(x)
 *   Sec. 3.2 Eq. (5)   x_hat = x_bar * alpha_h / 255 + beta_h
 *   Sec. 3.2 Eq. (6,7) running estimates of alpha (range) and beta (minimum)
 *   Sec. 3.1 Eq. (2)   layer gradients evaluated at the de-quantized x_hat (softmax, GELU,
 *                      LayerNorm, the Linear weight, and the two matrix products of attention)
 *   Sec. 3.2 / Fig. "bucketing": one (alpha, beta) pair per head or channel group
 *
 * Conventions
 *   - A tensor is viewed as (outer, groups, inner): element (o, g, i) sits at
 *     flat index (o*groups + g)*inner + i and uses alpha[g], beta[g].
 *   - Codes are stored signed: q = x_bar - 128, so Eq. (3)'s clip to [0, 255]
 *     is a clip of q to [-128, 127]; Eq. (5) adds the 128 back.
 *   - Everything that decides an integer code or a running parameter is done
 *     in IEEE binary32, one rounded operation per line (build with
 *     -ffp-contract=off); gradients are evaluated in binary64 from the
 *     binary32 x_hat and returned as doubles.
 *   - dt: 0 = binary32 storage, 1 = binary16 storage (raw uint16 bit patterns).
 *   - OpenMP (optional) splits the outermost independent index only.
 *
 * Pins: see tests/test_oracle_*.py.  The Philox generator is pinned to the
 * known-answer vectors of its publication's reference distribution; the
 * assignment of generator output bits to elements is this project's own
 * convention (the paper names no random source) -- that part is
 * "parity unpinned" beyond statistical tests.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* binary16 <-> binary32, written out bit by bit                             */
/* ------------------------------------------------------------------------ */

float mesa_ref_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    uint32_t expo = (h >> 10) & 0x1Fu;
    uint32_t mant = h & 0x3FFu;
    uint32_t bits;
    if (expo == 0) {
        if (mant == 0) {
            bits = sign;
        } else { /* subnormal half: value = mant * 2^-24, exact in binary32 */
            float v = (float)mant * 5.9604644775390625e-08f; /* 2^-24 */
            memcpy(&bits, &v, 4);
            bits |= sign;
        }
    } else if (expo == 31) {
        bits = sign | 0x7F800000u | (mant << 13);
    } else {
        bits = sign | ((expo + 112u) << 23) | (mant << 13);
    }
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

/* round-to-nearest, ties-to-even */
uint16_t mesa_ref_float_to_half(float f)
{
    uint32_t bits;
    memcpy(&bits, &f, 4);
    uint16_t sign = (uint16_t)((bits >> 16) & 0x8000u);
    uint32_t absb = bits & 0x7FFFFFFFu;
    if (absb >= 0x7F800000u) { /* inf / nan */
        return (uint16_t)(sign | 0x7C00u | ((absb > 0x7F800000u) ? 0x200u : 0u));
    }
    if (absb >= 0x477FF000u) { /* >= 65520 rounds to infinity */
        return (uint16_t)(sign | 0x7C00u);
    }
    if (absb < 0x33000001u) { /* <= 2^-25: rounds to zero (tie at 2^-25 goes to even = 0) */
        return sign;
    }
    int32_t e = (int32_t)(absb >> 23) - 127; /* unbiased exponent */
    uint32_t m = (absb & 0x7FFFFFu) | 0x800000u; /* 24-bit significand */
    int shift; /* number of low bits of m to drop */
    uint32_t base;
    if (e >= -14) { /* normal half */
        shift = 13;
        base = (uint32_t)(e + 15) << 10;
    } else { /* subnormal half: unit is 2^-24 */
        shift = 13 + (-14 - e);
        base = 0;
    }
    uint32_t kept = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (kept & 1u))) kept += 1u;
    /* for normals 'kept' carries the implicit bit at position 10: adding it to
       base - 0x400 lets a mantissa overflow bump the exponent naturally */
    uint32_t out = (e >= -14) ? (base - 0x400u + kept) : kept;
    return (uint16_t)(sign | out);
}

/* ------------------------------------------------------------------------ */
/* bfloat16 (the upper half of a binary32 word) <-> binary32                 */
/* ------------------------------------------------------------------------ */

float mesa_ref_bf16_to_float(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16; /* widening is exact */
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

/* round-to-nearest, ties-to-even on the 16 bits that are dropped */
uint16_t mesa_ref_float_to_bf16(float f)
{
    uint32_t bits;
    memcpy(&bits, &f, 4);
    if ((bits & 0x7FFFFFFFu) > 0x7F800000u) { /* nan: keep it a nan whatever the dropped bits were */
        return (uint16_t)((bits >> 16) | 0x0040u);
    }
    uint32_t kept = bits >> 16;
    uint32_t rem = bits & 0xFFFFu;
    if (rem > 0x8000u || (rem == 0x8000u && (kept & 1u))) kept += 1u; /* a carry out of the mantissa bumps the exponent; 0x7F7F + 1 is infinity */
    return (uint16_t)kept;
}

/* dt: 0 binary32, 1 binary16, 2 bfloat16 */
static float load_as_float(const void *p, int dt, int64_t idx)
{
    if (dt == 0) return ((const float *)p)[idx];
    if (dt == 2) return mesa_ref_bf16_to_float(((const uint16_t *)p)[idx]);
    return mesa_ref_half_to_float(((const uint16_t *)p)[idx]);
}

static double load_as_double(const void *p, int dt, int64_t idx)
{
    return (double)load_as_float(p, dt, idx);
}

/* ------------------------------------------------------------------------ */
/* Philox-4x32 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11)   */
/* ------------------------------------------------------------------------ */

#define MESA_REF_PHILOX_ROUNDS 10

void mesa_ref_philox4x32(const uint32_t ctr[4], const uint32_t key[2], int rounds, uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < rounds; ++r) {
        if (r > 0) { /* Weyl sequence on the key: golden ratio and sqrt(3)-1 */
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * Random fraction for stochastic rounding of flat element e.
 * Convention (the paper names no random source): elements are taken in blocks
 * of 8; block b = e / 8 uses counter (offset + b) as a 64-bit value in counter
 * words 0 and 1 (words 2, 3 zero) and the 64-bit seed as key words 0 and 1.
 * Element j = e % 8 takes 16 bits: word j/2, low half for even j, high half
 * for odd j; u = bits * 2^-16 lies in [0, 1).
 */
float mesa_ref_sr_uniform(uint64_t seed, uint64_t offset, uint64_t e)
{
    uint64_t c = offset + (e >> 3);
    uint32_t ctr[4] = { (uint32_t)c, (uint32_t)(c >> 32), 0u, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    mesa_ref_philox4x32(ctr, key, MESA_REF_PHILOX_ROUNDS, out);
    unsigned j = (unsigned)(e & 7u);
    uint32_t w = out[j >> 1];
    uint32_t bits16 = (j & 1u) ? (w >> 16) : (w & 0xFFFFu);
    return (float)bits16 * 1.52587890625e-05f; /* 2^-16, exact */
}

/* ------------------------------------------------------------------------ */
/* Eq. (6), (7): running estimates                                           */
/* ------------------------------------------------------------------------ */

/*
 * For each group: min and max over every element of the group in this call
 * (all samples and tokens: the parameters are shared across samples), then
 *   first call : alpha = max - min, beta = min               (Sec. 5.1)
 *   otherwise  : alpha = lambda*alpha + (1-lambda)*(max-min)  Eq. (6)
 *                beta  = lambda*beta  + (1-lambda)*min        Eq. (7)
 * each line one binary32 operation.
 */
int mesa_ref_update_running_params(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner,
                                   float *alpha, float *beta, float lambda, int first_call)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
    for (int64_t g = 0; g < groups; ++g) {
        float mn = INFINITY, mx = -INFINITY;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) reduction(min : mn) reduction(max : mx)
#endif
        for (int64_t o = 0; o < outer; ++o) {
            for (int64_t i = 0; i < inner; ++i) {
                float v = load_as_float(x, dt, (o * groups + g) * inner + i);
                if (v < mn) mn = v;
                if (v > mx) mx = v;
            }
        }
        float range = mx - mn;
        if (first_call) {
            alpha[g] = range;
            beta[g] = mn;
        } else {
            float a = lambda * alpha[g];
            float b = 1.0f - lambda;
            float c = b * range;
            alpha[g] = a + c;
            float e = lambda * beta[g];
            float f = b * mn;
            beta[g] = e + f;
        }
    }
    return 0;
}

/*
 * Symmetric range (the ablation of Sec. 5.2, asymmetric vs. symmetric quantization): one scale from
 * m = max |x| over the group and no free offset.  Reading taken here (the paper gives the scale factor
 * only): the clipping range is [-m, +m], i.e. Eq. (3)-(7) with the group's minimum replaced by -m and
 * its maximum by +m, so alpha moves towards 2m and beta towards -m; everything downstream (quantizer,
 * dequantizer, backward) is unchanged.
 */
int mesa_ref_update_running_params_sym(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner,
                                       float *alpha, float *beta, float lambda, int first_call)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
    for (int64_t g = 0; g < groups; ++g) {
        float m = 0.0f;
        for (int64_t o = 0; o < outer; ++o)
            for (int64_t i = 0; i < inner; ++i) {
                float v = fabsf(load_as_float(x, dt, (o * groups + g) * inner + i));
                if (v > m) m = v;
            }
        float mn = -m + 0.0f; /* -0.0 -> +0.0 */
        float range = m - mn;
        if (first_call) {
            alpha[g] = range;
            beta[g] = mn;
        } else {
            float a = lambda * alpha[g];
            float b = 1.0f - lambda;
            float c = b * range;
            alpha[g] = a + c;
            float e = lambda * beta[g];
            float f = b * mn;
            beta[g] = e + f;
        }
    }
    return 0;
}

/*
 * Scale-only symmetric quantization, the scheme the ablation of Sec. 5.2 compares Mesa with: the input is
 * quantized "by a scale factor only" -- no offset, zero is a code.  The paper prints the scale as
 * (2^b - 1) / max|X|; with signed b-bit codes that range would need b + 1 bits, so the reading taken here is
 * the usual signed one: 2^(b-1) - 1 = 127 steps on each side of zero,
 *   m      running estimate of max |x| over the group (Eq. (6) with max|x| in place of the range;
 *          first call: m = max|x|)
 *   r      = 127 / m   (0 when m <= 0)
 *   q      = clip(round(x * r), -127, 127)     round: nearest-even, or floor(v + u) as in Eq. (4)
 *   x_hat  = q * (m / 127)
 * binary32, each operation rounded on its own.
 */
int mesa_ref_update_running_scale_sym(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner,
                                      float *m, float lambda, int first_call)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
    for (int64_t g = 0; g < groups; ++g) {
        float mx = 0.0f;
        for (int64_t o = 0; o < outer; ++o)
            for (int64_t i = 0; i < inner; ++i) {
                float v = fabsf(load_as_float(x, dt, (o * groups + g) * inner + i));
                if (v > mx) mx = v;
            }
        if (first_call) {
            m[g] = mx;
        } else {
            float a = lambda * m[g];
            float b = 1.0f - lambda;
            float c = b * mx;
            m[g] = a + c;
        }
    }
    return 0;
}

int mesa_ref_quantize_sym(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner,
                          const float *m, int8_t *q, int mode, uint64_t seed, uint64_t offset)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t o = 0; o < outer; ++o) {
        for (int64_t g = 0; g < groups; ++g) {
            float r = (m[g] > 0.0f) ? 127.0f / m[g] : 0.0f;
            for (int64_t i = 0; i < inner; ++i) {
                int64_t e = (o * groups + g) * inner + i;
                float v = load_as_float(x, dt, e) * r;
                float w;
                if (mode == 0) {
                    w = rintf(v);
                } else {
                    float u = mesa_ref_sr_uniform(seed, offset, (uint64_t)e);
                    float s = v + u;
                    w = floorf(s);
                }
                if (w < -127.0f) w = -127.0f;
                if (w > 127.0f) w = 127.0f;
                q[e] = (int8_t)(int)w;
            }
        }
    }
    return 0;
}

int mesa_ref_dequantize_sym(const int8_t *q, int64_t outer, int64_t groups, int64_t inner,
                            const float *m, void *x_hat, int dt)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t o = 0; o < outer; ++o) {
        for (int64_t g = 0; g < groups; ++g) {
            float step = m[g] / 127.0f;
            for (int64_t i = 0; i < inner; ++i) {
                int64_t e = (o * groups + g) * inner + i;
                float xh = (float)(int)q[e] * step;
                if (dt == 0) ((float *)x_hat)[e] = xh;
                else if (dt == 2) ((uint16_t *)x_hat)[e] = mesa_ref_float_to_bf16(xh);
                else ((uint16_t *)x_hat)[e] = mesa_ref_float_to_half(xh);
            }
        }
    }
    return 0;
}

/*
 * Fixed offset (Sec. 6, evolution of alpha and beta in FFN layers: the offset of the second FFN layer's
 * input settles at the minimum of GELU, about -0.17, so it need not be estimated): beta_g = beta_fixed for every
 * group, and only the range is a running estimate, of max - beta_fixed:
 *   first call : alpha = max - beta_fixed
 *   otherwise  : alpha = lambda*alpha + (1-lambda)*(max - beta_fixed)
 * each line one binary32 operation.  Values below beta_fixed saturate at code 0 (Eq. 3's clip).
 */
int mesa_ref_update_running_params_fixed_beta(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner,
                                              float *alpha, float *beta, float lambda, int first_call, float beta_fixed)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
    for (int64_t g = 0; g < groups; ++g) {
        float mx = -INFINITY;
        for (int64_t o = 0; o < outer; ++o)
            for (int64_t i = 0; i < inner; ++i) {
                float v = load_as_float(x, dt, (o * groups + g) * inner + i);
                if (v > mx) mx = v;
            }
        mx = mx + 0.0f;
        float range = mx - beta_fixed;
        if (first_call) {
            alpha[g] = range;
        } else {
            float a = lambda * alpha[g];
            float b = 1.0f - lambda;
            float c = b * range;
            alpha[g] = a + c;
        }
        beta[g] = beta_fixed;
    }
    return 0;
}

/* raw per-group extrema, exposed for tests */
int mesa_ref_group_minmax(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner,
                          float *mn_out, float *mx_out)
{
    for (int64_t g = 0; g < groups; ++g) {
        float mn = INFINITY, mx = -INFINITY;
        for (int64_t o = 0; o < outer; ++o)
            for (int64_t i = 0; i < inner; ++i) {
                float v = load_as_float(x, dt, (o * groups + g) * inner + i);
                if (v < mn) mn = v;
                if (v > mx) mx = v;
            }
        mn_out[g] = mn;
        mx_out[g] = mx;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Eq. (3), (4): quantize                                                    */
/* ------------------------------------------------------------------------ */

/* mode 0: round to nearest, ties to even; mode 1: stochastic rounding, Eq. (4) */
int mesa_ref_quantize_headwise(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner,
                               const float *alpha, const float *beta, int8_t *q,
                               int mode, uint64_t seed, uint64_t offset)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t o = 0; o < outer; ++o) {
        for (int64_t g = 0; g < groups; ++g) {
            float a = alpha[g];
            float b = beta[g];
            float r = (a > 0.0f) ? 255.0f / a : 0.0f; /* constant group: every code is 0 */
            for (int64_t i = 0; i < inner; ++i) {
                int64_t e = (o * groups + g) * inner + i;
                float xv = load_as_float(x, dt, e);
                float t = xv - b;
                float v = t * r;
                float w;
                if (mode == 0) {
                    w = rintf(v); /* default rounding mode: nearest, ties to even */
                } else {
                    float u = mesa_ref_sr_uniform(seed, offset, (uint64_t)e);
                    float s = v + u;  /* floor(v + u) rounds up with probability frac(v) */
                    w = floorf(s);
                }
                if (w < 0.0f) w = 0.0f;
                if (w > 255.0f) w = 255.0f;
                q[e] = (int8_t)((int)w - 128);
            }
        }
    }
    return 0;
}

/*
 * Four-bit codes (Sec. 4.2 names lower bit widths as the step beyond the method's fixed 8 bits): Eq. (3)-(5) with
 * 2^b - 1 = 15 steps across the clipping range,
 *   x_bar = clip(round((x - beta) * (15 / alpha)), 0, 15),    x_hat = x_bar * (alpha / 15) + beta,
 * the same binary32 operation sequence and the same random fractions as the 8-bit quantizer.  Two codes share a
 * byte: element e sits in byte e / 2, in the low four bits when e is even, the high four when it is odd; with an odd
 * number of elements the last byte's high bits are zero.  q4 holds (numel + 1) / 2 bytes.
 */
int mesa_ref_quantize_headwise_b4(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner,
                                  const float *alpha, const float *beta, uint8_t *q4,
                                  int mode, uint64_t seed, uint64_t offset)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
    int64_t numel = outer * groups * inner;
    memset(q4, 0, (size_t)((numel + 1) / 2));
    for (int64_t e = 0; e < numel; ++e) {
        int64_t g = (e / inner) % groups;
        float a = alpha[g];
        float b = beta[g];
        float r = (a > 0.0f) ? 15.0f / a : 0.0f;
        float xv = load_as_float(x, dt, e);
        float t = xv - b;
        float v = t * r;
        float w;
        if (mode == 0) {
            w = rintf(v);
        } else {
            float u = mesa_ref_sr_uniform(seed, offset, (uint64_t)e);
            float s = v + u;
            w = floorf(s);
        }
        if (w < 0.0f) w = 0.0f;
        if (w > 15.0f) w = 15.0f;
        unsigned code = (unsigned)(int)w;
        q4[e / 2] = (uint8_t)(q4[e / 2] | (code << (4 * (e & 1))));
    }
    return 0;
}

static float dequant_one_b4(const uint8_t *q4, int64_t e, float step, float b)
{
    unsigned code = (q4[e / 2] >> (4 * (e & 1))) & 0xFu;
    float xh = (float)code * step;
    xh = xh + b;
    return xh;
}

int mesa_ref_dequantize_b4(const uint8_t *q4, int64_t outer, int64_t groups, int64_t inner,
                           const float *alpha, const float *beta, void *x_hat, int dt)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
    int64_t numel = outer * groups * inner;
    for (int64_t e = 0; e < numel; ++e) {
        int64_t g = (e / inner) % groups;
        float xh = dequant_one_b4(q4, e, alpha[g] / 15.0f, beta[g]);
        if (dt == 0) ((float *)x_hat)[e] = xh;
        else if (dt == 2) ((uint16_t *)x_hat)[e] = mesa_ref_float_to_bf16(xh);
        else ((uint16_t *)x_hat)[e] = mesa_ref_float_to_half(xh);
    }
    return 0;
}

/* GELU backward at the four-bit x_hat: the formula of mesa_ref_gelu_bwd_q, binary64, at the binary32 x_hat above */
int mesa_ref_gelu_bwd_q_b4(const uint8_t *q4, int64_t outer, int64_t groups, int64_t inner,
                           const float *alpha, const float *beta, const void *dy, int dt, double *dx)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
    int64_t numel = outer * groups * inner;
    for (int64_t e = 0; e < numel; ++e) {
        int64_t g = (e / inner) % groups;
        double xh = (double)dequant_one_b4(q4, e, alpha[g] / 15.0f, beta[g]);
        double cdf = 0.5 * (1.0 + erf(xh / sqrt(2.0)));
        double pdf = exp(-0.5 * xh * xh) / sqrt(2.0 * 3.14159265358979323846);
        dx[e] = load_as_double(dy, dt, e) * (cdf + xh * pdf);
    }
    return 0;
}

/*
 * Single-pass forward (a variant of the method, not the order the paper implies
 * in Sec. 5.1, where the first iteration's statistics initialise the
 * parameters it quantizes with): the codes are taken with the running
 * estimates AS THEY ARE ON ENTRY, Eq. (3)-(4); the same batch's extrema then
 * move the estimates by Eq. (6)-(7) for the next call.  One read of x on a
 * machine that fuses the two; here simply the two steps in that order.
 */
int mesa_ref_quantize_update_fused(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner,
                                   float *alpha, float *beta, float lambda, int8_t *q,
                                   int mode, uint64_t seed, uint64_t offset)
{
    int rc = mesa_ref_quantize_headwise(x, dt, outer, groups, inner, alpha, beta, q, mode, seed, offset);
    if (rc) return rc;
    return mesa_ref_update_running_params(x, dt, outer, groups, inner, alpha, beta, lambda, 0);
}

/*
 * A Mesa GELU layer's forward in one step (Sec. 3.1: the forward pass is computed exactly, the input
 * is what gets saved, compressed): y = gelu(x) = x * Phi(x) from the exact x, and the single-pass
 * forward above for the saved input (codes with the estimates as they are on entry, then Eq. (6)-(7)).
 */
int mesa_ref_gelu_fwd_q(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner,
                        float *alpha, float *beta, float lambda, double *y, int8_t *q,
                        int mode, uint64_t seed, uint64_t offset)
{
    int64_t n = outer * groups * inner;
    for (int64_t e = 0; e < n; ++e) {
        double v = load_as_double(x, dt, e);
        y[e] = 0.5 * v * (1.0 + erf(v / sqrt(2.0)));
    }
    return mesa_ref_quantize_update_fused(x, dt, outer, groups, inner, alpha, beta, lambda, q, mode, seed, offset);
}

/* ------------------------------------------------------------------------ */
/* Eq. (5): dequantize                                                       */
/* ------------------------------------------------------------------------ */

static float dequant_one(int8_t code, float step, float b)
{
    float xh = (float)((int)code + 128) * step;
    xh = xh + b;
    return xh;
}

int mesa_ref_dequantize(const int8_t *q, int64_t outer, int64_t groups, int64_t inner,
                        const float *alpha, const float *beta, void *x_hat, int dt)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t o = 0; o < outer; ++o) {
        for (int64_t g = 0; g < groups; ++g) {
            float step = alpha[g] / 255.0f;
            float b = beta[g];
            for (int64_t i = 0; i < inner; ++i) {
                int64_t e = (o * groups + g) * inner + i;
                float xh = dequant_one(q[e], step, b);
                if (dt == 0) ((float *)x_hat)[e] = xh;
                else if (dt == 2) ((uint16_t *)x_hat)[e] = mesa_ref_float_to_bf16(xh);
                else ((uint16_t *)x_hat)[e] = mesa_ref_float_to_half(xh);
            }
        }
    }
    return 0;
}

/*
 * Softmax forward over the last axis, the exact forward of a Mesa softmax layer (Sec. 3.1: the
 * forward pass is computed exactly; what the layer saves, compressed, is this output):
 *   y_j = exp(s_j - max_k s_k) / sum_k exp(s_k - max_k s_k)   per row of cols elements.
 */
int mesa_ref_softmax_fwd(const void *s, int dt, int64_t total_rows, int64_t cols, double *y)
{
    for (int64_t r = 0; r < total_rows; ++r) {
        double mx = -INFINITY, sum = 0.0;
        for (int64_t j = 0; j < cols; ++j) {
            double v = load_as_double(s, dt, r * cols + j);
            if (v > mx) mx = v;
        }
        for (int64_t j = 0; j < cols; ++j) {
            y[r * cols + j] = exp(load_as_double(s, dt, r * cols + j) - mx);
            sum += y[r * cols + j];
        }
        for (int64_t j = 0; j < cols; ++j) y[r * cols + j] /= sum;
    }
    return 0;
}

/*
 * LayerNorm forward over the last axis of an (M, D) matrix, the exact forward of a Mesa LayerNorm
 * layer (Sec. 3.1); what the layer saves is its input x, compressed, plus the two statistics:
 *   mean_m = sum_j x_mj / D,  var_m = sum_j (x_mj - mean_m)^2 / D,  rstd_m = 1 / sqrt(var_m + eps),
 *   y_mj = (x_mj - mean_m) * rstd_m * gamma_j + bias_j.
 */
int mesa_ref_layernorm_fwd(const void *x, int dt, int64_t M, int64_t D, const void *gamma, const void *bias,
                           double eps, double *y, double *mean, double *rstd)
{
    for (int64_t m = 0; m < M; ++m) {
        double mu = 0.0, var = 0.0;
        for (int64_t j = 0; j < D; ++j) mu += load_as_double(x, dt, m * D + j);
        mu /= (double)D;
        for (int64_t j = 0; j < D; ++j) {
            double d = load_as_double(x, dt, m * D + j) - mu;
            var += d * d;
        }
        var /= (double)D;
        double rs = 1.0 / sqrt(var + eps);
        mean[m] = mu;
        rstd[m] = rs;
        for (int64_t j = 0; j < D; ++j)
            y[m * D + j] = (load_as_double(x, dt, m * D + j) - mu) * rs * load_as_double(gamma, dt, j) + load_as_double(bias, dt, j);
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Eq. (2): layer gradients at x_hat                                         */
/* ------------------------------------------------------------------------ */

/*
 * Softmax.  The saved tensor is the softmax output y (the attention map,
 * shape (B, H, rows, cols), one parameter pair per head).  For one row,
 *   d = sum_j dy_j * y_hat_j,   dx_j = y_hat_j * (dy_j - d).
 */
int mesa_ref_softmax_bwd_q(const int8_t *yq, int64_t B, int64_t H, int64_t rows, int64_t cols,
                           const float *alpha, const float *beta, const void *dy, int dt, double *dx)
{
    if (B <= 0 || H <= 0 || rows <= 0 || cols <= 0) return 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t h = 0; h < H; ++h) {
            float step = alpha[h] / 255.0f;
            float off = beta[h];
            for (int64_t r = 0; r < rows; ++r) {
                int64_t base = ((b * H + h) * rows + r) * cols;
                double d = 0.0;
                for (int64_t j = 0; j < cols; ++j) {
                    double yh = (double)dequant_one(yq[base + j], step, off);
                    d += load_as_double(dy, dt, base + j) * yh;
                }
                for (int64_t j = 0; j < cols; ++j) {
                    double yh = (double)dequant_one(yq[base + j], step, off);
                    dx[base + j] = yh * (load_as_double(dy, dt, base + j) - d);
                }
            }
        }
    }
    return 0;
}

/*
 * GELU (exact, erf form).  The saved tensor is the GELU input x.
 *   gelu(x) = x * Phi(x),  gelu'(x) = Phi(x) + x * phi(x)
 *   Phi(x) = (1 + erf(x / sqrt 2)) / 2,  phi(x) = exp(-x^2 / 2) / sqrt(2 pi)
 */
int mesa_ref_gelu_bwd_q(const int8_t *xq, int64_t outer, int64_t groups, int64_t inner,
                        const float *alpha, const float *beta, const void *dy, int dt, double *dx)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t o = 0; o < outer; ++o) {
        for (int64_t g = 0; g < groups; ++g) {
            float step = alpha[g] / 255.0f;
            float off = beta[g];
            for (int64_t i = 0; i < inner; ++i) {
                int64_t e = (o * groups + g) * inner + i;
                double xh = (double)dequant_one(xq[e], step, off);
                double cdf = 0.5 * (1.0 + erf(xh / sqrt(2.0)));
                double pdf = exp(-0.5 * xh * xh) / sqrt(2.0 * 3.14159265358979323846);
                dx[e] = load_as_double(dy, dt, e) * (cdf + xh * pdf);
            }
        }
    }
    return 0;
}

/*
 * ReLU (one of the CNN layers Sec. 3.3 lists as covered, quantized group-wise like every other
 * activation).  The saved tensor is the ReLU input x:  relu'(x) = 1 for x > 0, else 0 (0 at x = 0).
 */
int mesa_ref_relu_bwd_q(const int8_t *xq, int64_t outer, int64_t groups, int64_t inner,
                        const float *alpha, const float *beta, const void *dy, int dt, double *dx)
{
    if (outer <= 0 || groups <= 0 || inner <= 0) return 0;
    for (int64_t o = 0; o < outer; ++o) {
        for (int64_t g = 0; g < groups; ++g) {
            float step = alpha[g] / 255.0f;
            float off = beta[g];
            for (int64_t i = 0; i < inner; ++i) {
                int64_t e = (o * groups + g) * inner + i;
                float xh = dequant_one(xq[e], step, off);
                dx[e] = xh > 0.0f ? load_as_double(dy, dt, e) : 0.0;
            }
        }
    }
    return 0;
}

/*
 * LayerNorm over the last axis of an (M, D) matrix, D split into G channel
 * groups of D/G columns.  Saved: codes of the input x plus the forward's own
 * per-row mean and reciprocal standard deviation (binary32).
 *   xn = (x_hat - mean) * rstd,  g = dy * gamma
 *   dx = rstd * (g - mean_j(g) - xn * mean_j(g * xn))
 *   dgamma_j = sum_rows dy * xn,  dbeta_j = sum_rows dy
 */
int mesa_ref_layernorm_bwd_q(const int8_t *xq, int64_t M, int64_t D, int64_t G,
                             const float *alpha, const float *beta,
                             const float *mean, const float *rstd, const void *gamma,
                             const void *dy, int dt, double *dx, double *dgamma, double *dbeta)
{
    if (M <= 0 || D <= 0 || G <= 0 || D % G != 0) return (M <= 0 || D <= 0) ? 0 : 1;
    int64_t per = D / G;
    for (int64_t j = 0; j < D; ++j) { dgamma[j] = 0.0; dbeta[j] = 0.0; }
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t m = 0; m < M; ++m) {
        double mu = (double)mean[m], rs = (double)rstd[m];
        double s1 = 0.0, s2 = 0.0;
        for (int64_t j = 0; j < D; ++j) {
            int64_t g = j / per;
            double xh = (double)dequant_one(xq[m * D + j], alpha[g] / 255.0f, beta[g]);
            double xn = (xh - mu) * rs;
            double gg = load_as_double(dy, dt, m * D + j) * load_as_double(gamma, dt, j);
            s1 += gg;
            s2 += gg * xn;
        }
        double c1 = s1 / (double)D, c2 = s2 / (double)D;
        for (int64_t j = 0; j < D; ++j) {
            int64_t g = j / per;
            double xh = (double)dequant_one(xq[m * D + j], alpha[g] / 255.0f, beta[g]);
            double xn = (xh - mu) * rs;
            double gg = load_as_double(dy, dt, m * D + j) * load_as_double(gamma, dt, j);
            dx[m * D + j] = rs * (gg - c1 - xn * c2);
        }
    }
    /* column sums: rows in order, serial, so the result does not depend on threads */
    for (int64_t m = 0; m < M; ++m) {
        double mu = (double)mean[m], rs = (double)rstd[m];
        for (int64_t j = 0; j < D; ++j) {
            int64_t g = j / per;
            double xh = (double)dequant_one(xq[m * D + j], alpha[g] / 255.0f, beta[g]);
            double xn = (xh - mu) * rs;
            double d = load_as_double(dy, dt, m * D + j);
            dgamma[j] += d * xn;
            dbeta[j] += d;
        }
    }
    return 0;
}

/*
 * Linear weight gradient.  y = x W^T with W of shape (N_out, K); saved: codes
 * of x (M, K), K split into G channel groups.
 *   dW[n, k] = sum_m dy[m, n] * x_hat[m, k],   db[n] = sum_m dy[m, n]
 */
static double dw_entry(const int8_t *xq, int64_t M, int64_t K, int64_t per,
                       const float *alpha, const float *beta, const void *dy, int64_t N_out, int dt,
                       int64_t n, int64_t k)
{
    int64_t g = k / per;
    float step = alpha[g] / 255.0f;
    float off = beta[g];
    double acc = 0.0;
    for (int64_t m = 0; m < M; ++m)
        acc += load_as_double(dy, dt, m * N_out + n) * (double)dequant_one(xq[m * K + k], step, off);
    return acc;
}

int mesa_ref_linear_dw_q(const int8_t *xq, int64_t M, int64_t K, int64_t G,
                         const float *alpha, const float *beta, const void *dy, int64_t N_out, int dt,
                         double *dW, double *db)
{
    if (M < 0 || K <= 0 || G <= 0 || N_out <= 0 || K % G != 0) return 1;
    int64_t per = K / G;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t n = 0; n < N_out; ++n) {
        for (int64_t k = 0; k < K; ++k)
            dW[n * K + k] = dw_entry(xq, M, K, per, alpha, beta, dy, N_out, dt, n, k);
        if (db) {
            double acc = 0.0;
            for (int64_t m = 0; m < M; ++m) acc += load_as_double(dy, dt, m * N_out + n);
            db[n] = acc;
        }
    }
    return 0;
}

/* the same definition at a list of (n, k) positions, for sizes where the full
   matrix is out of reach of a CPU */
int mesa_ref_linear_dw_q_entries(const int8_t *xq, int64_t M, int64_t K, int64_t G,
                                 const float *alpha, const float *beta, const void *dy, int64_t N_out, int dt,
                                 const int64_t *n_idx, const int64_t *k_idx, int64_t count, double *out)
{
    if (M < 0 || K <= 0 || G <= 0 || N_out <= 0 || K % G != 0) return 1;
    int64_t per = K / G;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t t = 0; t < count; ++t)
        out[t] = dw_entry(xq, M, K, per, alpha, beta, dy, N_out, dt, n_idx[t], k_idx[t]);
    return 0;
}

/*
 * Weight gradient of a two-dimensional convolution at the de-quantized input (Eq. (2) with G_l the gradient of a
 * convolution; Sec. 3.3 covers the convolutional layer with the group-wise scheme, the input's channels split into
 * G groups of C_in / G consecutive channels, one (alpha, beta) pair each).  Tensors are contiguous, channels-first:
 *   xq (B, C_in, H, W) codes,   dy (B, C_out, OH, OW),   dW (C_out, C_in, KH, KW),   db [C_out]
 *   OH = (H + 2*pad_h - dil_h*(KH-1) - 1) / stride_h + 1,  OW likewise
 *   dW[co, ci, kh, kw] = sum over b, oh, ow of dy[b, co, oh, ow] * x_hat[b, ci, oh*stride_h - pad_h + kh*dil_h,
 *                                                                             ow*stride_w - pad_w + kw*dil_w]
 * where a position outside the image contributes nothing: the forward pads with zeros, not with de-quantized codes.
 * geom: {B, C_in, H, W, C_out, KH, KW, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w}.
 */
static int conv_out_extent(int64_t in, int64_t k, int64_t stride, int64_t pad, int64_t dil, int64_t *out)
{
    int64_t span = in + 2 * pad - dil * (k - 1) - 1;
    if (in <= 0 || k <= 0 || stride <= 0 || pad < 0 || dil <= 0 || span < 0) return 1;
    *out = span / stride + 1;
    return 0;
}

static double conv_dw_entry(const int8_t *xq, const int64_t *geom, int64_t OH, int64_t OW, int64_t per,
                            const float *alpha, const float *beta, const void *dy, int dt,
                            int64_t co, int64_t ci, int64_t kh, int64_t kw)
{
    int64_t B = geom[0], Cin = geom[1], H = geom[2], W = geom[3], Cout = geom[4];
    int64_t sh = geom[7], sw = geom[8], ph = geom[9], pw = geom[10], dh = geom[11], dw = geom[12];
    float step = alpha[ci / per] / 255.0f;
    float off = beta[ci / per];
    double acc = 0.0;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t oh = 0; oh < OH; ++oh) {
            int64_t ih = oh * sh - ph + kh * dh;
            if (ih < 0 || ih >= H) continue;
            for (int64_t ow = 0; ow < OW; ++ow) {
                int64_t iw = ow * sw - pw + kw * dw;
                if (iw < 0 || iw >= W) continue;
                double g = load_as_double(dy, dt, ((b * Cout + co) * OH + oh) * OW + ow);
                acc += g * (double)dequant_one(xq[((b * Cin + ci) * H + ih) * W + iw], step, off);
            }
        }
    return acc;
}

int mesa_ref_conv2d_dw_q(const int8_t *xq, const int64_t *geom, int64_t G, const float *alpha, const float *beta,
                         const void *dy, int dt, double *dW, double *db)
{
    int64_t B = geom[0], Cin = geom[1], Cout = geom[4], KH = geom[5], KW = geom[6], OH, OW;
    if (B < 0 || Cin <= 0 || Cout <= 0 || G <= 0 || Cin % G != 0) return 1;
    if (conv_out_extent(geom[2], KH, geom[7], geom[9], geom[11], &OH)) return 1;
    if (conv_out_extent(geom[3], KW, geom[8], geom[10], geom[12], &OW)) return 1;
    int64_t per = Cin / G;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t co = 0; co < Cout; ++co) {
        for (int64_t ci = 0; ci < Cin; ++ci)
            for (int64_t kh = 0; kh < KH; ++kh)
                for (int64_t kw = 0; kw < KW; ++kw)
                    dW[((co * Cin + ci) * KH + kh) * KW + kw] =
                        conv_dw_entry(xq, geom, OH, OW, per, alpha, beta, dy, dt, co, ci, kh, kw);
        if (db) {
            double acc = 0.0;
            for (int64_t b = 0; b < B; ++b)
                for (int64_t p = 0; p < OH * OW; ++p) acc += load_as_double(dy, dt, (b * Cout + co) * OH * OW + p);
            db[co] = acc;
        }
    }
    return 0;
}

/* the same definition at a list of (co, ci, kh, kw) positions, idx[4*t .. 4*t+3], for sizes where the full
   gradient is out of reach of a CPU */
int mesa_ref_conv2d_dw_q_entries(const int8_t *xq, const int64_t *geom, int64_t G, const float *alpha, const float *beta,
                                 const void *dy, int dt, const int64_t *idx, int64_t count, double *out)
{
    int64_t B = geom[0], Cin = geom[1], Cout = geom[4], KH = geom[5], KW = geom[6], OH, OW;
    if (B < 0 || Cin <= 0 || Cout <= 0 || G <= 0 || Cin % G != 0) return 1;
    if (conv_out_extent(geom[2], KH, geom[7], geom[9], geom[11], &OH)) return 1;
    if (conv_out_extent(geom[3], KW, geom[8], geom[10], geom[12], &OW)) return 1;
    int64_t per = Cin / G;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t t = 0; t < count; ++t)
        out[t] = conv_dw_entry(xq, geom, OH, OW, per, alpha, beta, dy, dt, idx[4 * t], idx[4 * t + 1], idx[4 * t + 2], idx[4 * t + 3]);
    return 0;
}

/*
 * The two matrix products of self-attention, backward, at the de-quantized
 * operands (Eq. (2) with G_l the gradient of a matrix product; the operands
 * are saved head-wise, Sec. 3.2: one (alpha, beta) pair per head for each of
 * the four tensors).  All tensors are (B, H, N, .) contiguous.
 *
 *   O = A V,  A (N x N) the attention map, V (N x Dh):
 *       dA[i,j] = sum_d dO[i,d] * V_hat[j,d]        dV[j,d] = sum_i A_hat[i,j] * dO[i,d]
 */
int mesa_ref_attn_av_bwd_q(const int8_t *aq, const int8_t *vq, int64_t B, int64_t H, int64_t N, int64_t Dh,
                           const float *alpha_a, const float *beta_a, const float *alpha_v, const float *beta_v,
                           const void *dO, int dt, double *dA, double *dV)
{
    if (B <= 0 || H <= 0 || N <= 0 || Dh <= 0) return 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t bh = 0; bh < B * H; ++bh) {
        int64_t h = bh % H;
        float sa = alpha_a[h] / 255.0f, sv = alpha_v[h] / 255.0f;
        const int8_t *a = aq + bh * N * N;
        const int8_t *v = vq + bh * N * Dh;
        for (int64_t i = 0; i < N; ++i)
            for (int64_t j = 0; j < N; ++j) {
                double acc = 0.0;
                for (int64_t d = 0; d < Dh; ++d)
                    acc += load_as_double(dO, dt, (bh * N + i) * Dh + d) * (double)dequant_one(v[j * Dh + d], sv, beta_v[h]);
                dA[(bh * N + i) * N + j] = acc;
            }
        for (int64_t j = 0; j < N; ++j)
            for (int64_t d = 0; d < Dh; ++d) {
                double acc = 0.0;
                for (int64_t i = 0; i < N; ++i)
                    acc += (double)dequant_one(a[i * N + j], sa, beta_a[h]) * load_as_double(dO, dt, (bh * N + i) * Dh + d);
                dV[(bh * N + j) * Dh + d] = acc;
            }
    }
    return 0;
}

/*
 *   S = scale * Q K^T,  Q, K (N x Dh):
 *       dQ[i,d] = scale * sum_j dS[i,j] * K_hat[j,d]     dK[j,d] = scale * sum_i dS[i,j] * Q_hat[i,d]
 */
int mesa_ref_attn_qk_bwd_q(const int8_t *qq, const int8_t *kq, int64_t B, int64_t H, int64_t N, int64_t Dh,
                           const float *alpha_q, const float *beta_q, const float *alpha_k, const float *beta_k,
                           const void *dS, int dt, double scale, double *dQ, double *dK)
{
    if (B <= 0 || H <= 0 || N <= 0 || Dh <= 0) return 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t bh = 0; bh < B * H; ++bh) {
        int64_t h = bh % H;
        float sq = alpha_q[h] / 255.0f, sk = alpha_k[h] / 255.0f;
        const int8_t *q = qq + bh * N * Dh;
        const int8_t *k = kq + bh * N * Dh;
        for (int64_t i = 0; i < N; ++i)
            for (int64_t d = 0; d < Dh; ++d) {
                double acc = 0.0;
                for (int64_t j = 0; j < N; ++j)
                    acc += load_as_double(dS, dt, (bh * N + i) * N + j) * (double)dequant_one(k[j * Dh + d], sk, beta_k[h]);
                dQ[(bh * N + i) * Dh + d] = scale * acc;
            }
        for (int64_t j = 0; j < N; ++j)
            for (int64_t d = 0; d < Dh; ++d) {
                double acc = 0.0;
                for (int64_t i = 0; i < N; ++i)
                    acc += load_as_double(dS, dt, (bh * N + i) * N + j) * (double)dequant_one(q[i * Dh + d], sq, beta_q[h]);
                dK[(bh * N + j) * Dh + d] = scale * acc;
            }
    }
    return 0;
}

int mesa_ref_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

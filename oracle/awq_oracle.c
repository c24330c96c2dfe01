/*
 * awq_oracle.c -- plain CPU oracle for the W4A16 group-quantized linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct reference
 * that the GPU library is checked against.  It shares no code, header, table or
 * helper with the HIP path, and nothing in the product may call it.
 *
 * What it computes (AWQ, arXiv 2306.00978):
 *   - Sec. 3.2, Eq. 1-2: the group quantizer Q applied to w*s, where s is the
 *     per-input-channel activation-aware scale.  Eq. 1 prints a symmetric
 *     abs-max form; the build target fixes the asymmetric 16-level min/max
 *     form used here:  scale = (max-min)/15, zero = clamp(round(-min/scale)),
 *     q = clamp(round(w/scale)+zero, 0, 15), group = 128 consecutive input
 *     channels of one output row (Sec. 4.1 "group size of 128").
 *   - Sec. 3.2, Eq. 4: W x == (W diag(s)) (diag(s)^-1 x); the caller divides x.
 *   - Sec. 4.2 (dequantization fused into the linear's kernel): y = x * dequant(q)^T with
 *     dequant(q) = (q - zero) * scale, written out here as a plain loop.
 *   - Sec. 4.2 "SIMD-aware weight packing": the packed byte layout is a pure
 *     index permutation; pack/unpack below are written from the layout text
 *     in the public header of the library under test, with plain index arithmetic.
 *
 * Arithmetic: the quantizer decides integers, so both sides take those
 * decisions in IEEE binary32, one operation per statement, no FMA contraction
 * (build with -ffp-contract=off), round-to-nearest-even.  The matmul
 * accumulates in binary64.
 *
 * Pins (tests/test_oracle_*.py): code range, |w' - dequant| <= scale/2 for
 * unclipped elements, end-point codes, round-off mean 0.25 (Sec. 3.2,
 * observation 1), the Eq. 3 error-ratio law, exact-grid round trip, Eq. 4
 * equivalence in fp64, brute-force dot products, hand-placed pack offsets,
 * fp16 conversion against an independent implementation (numpy).
 * Parity unpinned: none of the functions below (the paper prints no worked
 * numeric example, so all pins are invariants / closed forms / brute force).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#define ORACLE_GROUP 128

/* ---------- binary16 <-> binary32, bit level ---------- */

float awq_oracle_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    int exp = (h >> 10) & 0x1f;
    uint32_t man = h & 0x3ffu;
    uint32_t bits;
    float f;
    if (exp == 0x1f) {                      /* inf / nan */
        bits = sign | 0x7f800000u | (man << 13);
    } else if (exp != 0) {                  /* normal */
        bits = sign | ((uint32_t)(exp + 112) << 23) | (man << 13);
    } else if (man == 0) {                  /* signed zero */
        bits = sign;
    } else {                                /* subnormal: man * 2^-24 */
        float v = (float)man * 5.9604644775390625e-08f;
        memcpy(&bits, &v, 4);
        bits |= sign;
    }
    memcpy(&f, &bits, 4);
    return f;
}

/* round-to-nearest-even binary32 -> binary16 */
uint16_t awq_oracle_f32_to_f16(float f)
{
    uint32_t bits;
    memcpy(&bits, &f, 4);
    uint16_t sign = (uint16_t)((bits >> 16) & 0x8000u);
    uint32_t a = bits & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);       /* nan */
    if (a >= 0x47800000u) {                                        /* >= 65536 or inf */
        return (uint16_t)(sign | 0x7c00u);
    }
    if (a >= 0x38800000u) {                                        /* normal half range */
        uint32_t m = a - 0x38000000u;      /* rebias exponent by 112 */
        uint32_t keep = m >> 13;
        uint32_t rest = m & 0x1fffu;
        if (rest > 0x1000u || (rest == 0x1000u && (keep & 1u))) keep += 1;
        /* a carry may walk into the exponent, up to 0x7c00 = inf: correct */
        return (uint16_t)(sign | keep);
    }
    if (a < 0x33000000u) return sign;                              /* < 2^-25 -> 0 */
    {
        /* subnormal half: value = m24 * 2^(e-150); target unit 2^-24 */
        int e = (int)(a >> 23);
        uint32_t m24 = (a & 0x7fffffu) | 0x800000u;
        int shift = 126 - e;               /* e in [102,112] -> shift in [14,24] */
        uint32_t keep = m24 >> shift;
        uint32_t rest = m24 & ((1u << shift) - 1u);
        uint32_t half = 1u << (shift - 1);
        if (rest > half || (rest == half && (keep & 1u))) keep += 1;
        return (uint16_t)(sign | keep);
    }
}

/* ---------- a0: per-input-channel activation statistic (Sec. 3.2, Eq. 5) ----------
 * s[k] = max(mean_t |X[t,k]|, floor)^alpha, accumulated in binary64.            */
int awq_oracle_act_scale(const uint16_t *X, int64_t T, int64_t K, double alpha,
                         double floor_, double *s)
{
    if (!X || !s || T <= 0 || K <= 0) return -1;
    for (int64_t k = 0; k < K; ++k) {
        double acc = 0.0;
        for (int64_t t = 0; t < T; ++t)
            acc += fabs((double)awq_oracle_f16_to_f32(X[t * K + k]));
        double mean = acc / (double)T;
        if (mean < floor_) mean = floor_;
        s[k] = pow(mean, alpha);
    }
    return 0;
}

/* x'[m,k] = fp16( fp32(x[m,k]) / s[k] ) : the inverse scale of Eq. 4 applied to
 * the activation by the caller (Sec. 3.2: the factor belongs to the producer of x). */
int awq_oracle_apply_inv_scale(const uint16_t *x, const float *s, int64_t M,
                               int64_t K, uint16_t *xs)
{
    if (!x || !s || !xs || M <= 0 || K <= 0) return -1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            float q = awq_oracle_f16_to_f32(x[m * K + k]) / s[k];
            xs[m * K + k] = awq_oracle_f32_to_f16(q);
        }
    return 0;
}

/* ---------- a1..a4: quantize one matrix ----------
 * W      [N,K] binary16, row-major (out-features x in-features)
 * s      [K] binary32 or NULL (= all ones, plain round-to-nearest)
 * codes  [N,K] one code per byte, 0..15
 * scales [N,G] binary16 bits, G = K/128
 * zeros  [N,G] one zero point per byte, 0..15                                   */
/* ---------- normalisation fused with the inverse scale (Sec. 4.2, kernel fusion: the
 * operators of a layer normalisation as one kernel; Sec. 3.2: the diag(s)^-1 factor of Eq. 4
 * belongs to the operator that produces x).  RMS form, as the Llama-2-shaped layers
 * of the workloads use it:
 *   xs[m,k] = fp16( x[m,k] / sqrt(mean_k x[m,k]^2 + eps) * gamma[k] / s[k] ),  binary64 inside.
 * gamma [K] binary16; s [K] binary32 or NULL (= ones).                                  */
int awq_oracle_rmsnorm_inv_scale(const uint16_t *x, const uint16_t *gamma, const float *s,
                                 int64_t M, int64_t K, double eps, uint16_t *xs)
{
    if (!x || !gamma || !xs || M <= 0 || K <= 0) return -1;
    for (int64_t m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double v = (double)awq_oracle_f16_to_f32(x[m * K + k]);
            ss += v * v;
        }
        double inv = 1.0 / sqrt(ss / (double)K + eps);
        for (int64_t k = 0; k < K; ++k) {
            double v = (double)awq_oracle_f16_to_f32(x[m * K + k]) * inv *
                       (double)awq_oracle_f16_to_f32(gamma[k]);
            if (s) v = v / (double)s[k];
            xs[m * K + k] = awq_oracle_f32_to_f16((float)v);
        }
    }
    return 0;
}

static float clampf(float v, float lo, float hi)
{
    if (v < lo) return lo;
    if (v > hi) return hi;
    return v;
}

int awq_oracle_quantize(const uint16_t *W, const float *s, int64_t N, int64_t K,
                        int group, uint8_t *codes, uint16_t *scales, uint8_t *zeros)
{
    if (!W || !codes || !scales || !zeros) return -1;
    if (group != ORACLE_GROUP || N <= 0 || K <= 0 || K % group) return -2;
    const int64_t G = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float wp[ORACLE_GROUP];
        for (int64_t g = 0; g < G; ++g) {
            const int64_t k0 = g * group;
            /* a1: fold the activation-aware scale (Eq. 2: Q(w*s)) */
            for (int j = 0; j < group; ++j) {
                float w = awq_oracle_f16_to_f32(W[n * K + k0 + j]);
                float sk = s ? s[k0 + j] : 1.0f;
                wp[j] = w * sk;
            }
            /* a2: range of the group */
            float mx = wp[0], mn = wp[0];
            for (int j = 1; j < group; ++j) {
                if (wp[j] > mx) mx = wp[j];
                if (wp[j] < mn) mn = wp[j];
            }
            /* a3: step size, stored as binary16; the codes use the stored value */
            float range = mx - mn;
            float sc32 = range / 15.0f;
            sc32 = clampf(sc32, 6.103515625e-05f /* 2^-14 */, 65504.0f);
            uint16_t sc_h = awq_oracle_f32_to_f16(sc32);
            float scale = awq_oracle_f16_to_f32(sc_h);
            float nmn = -mn;
            float zr = nmn / scale;
            float zero = clampf(rintf(zr), 0.0f, 15.0f);
            scales[n * G + g] = sc_h;
            zeros[n * G + g] = (uint8_t)zero;
            /* a4: codes */
            for (int j = 0; j < group; ++j) {
                float r = wp[j] / scale;
                float q = rintf(r);
                q = q + zero;
                q = clampf(q, 0.0f, 15.0f);
                codes[n * K + k0 + j] = (uint8_t)q;
            }
        }
    }
    return 0;
}

/* ---------- weight clipping (Sec. 3.2 names it in one sentence, as a second step that lowers
 * the squared quantization error).  The paper gives no more than that sentence; the reading
 * taken here: per quantization group, the range [min, max] of w*s is shrunk to
 * [r*min, r*max] for every r of a given grid, the group is quantized with that range (values
 * outside it saturate at code 0 or 15), and the r with the smallest sum of squared
 * differences between the dequantized and the scaled weights wins (first one on ties).
 * Quantization arithmetic as in awq_oracle_quantize (binary32, one rounding per operation);
 * an error is e = (q - zero) * scale - w*s in binary32, the sum of e*e is taken in binary64.
 * With activation rows xs = x/s [T,K] (optional) the error of a group is instead its
 * contribution to the layer output on those rows, sum_t (sum_k e[k] xs[t,k])^2 in binary64:
 * the counterpart of Eq. 4 for one group, weighting every weight error by the activation
 * it meets.  choice[n*G+g] (optional) receives the index of the winning r.              */
static void quantize_group_range(const float *wp, int group, float mx, float mn, uint16_t *sc_h_out,
                                 float *zero_out, uint8_t *codes /* may be NULL */, double *err,
                                 const uint16_t *xs /* may be NULL: rows of x/s, this group's columns */,
                                 int64_t T, int64_t row_stride)
{
    float diff[ORACLE_GROUP];
    float range = mx - mn;
    float sc32 = range / 15.0f;
    sc32 = clampf(sc32, 6.103515625e-05f, 65504.0f);
    uint16_t sc_h = awq_oracle_f32_to_f16(sc32);
    float scale = awq_oracle_f16_to_f32(sc_h);
    float nmn = -mn;
    float zr = nmn / scale;
    float zero = clampf(rintf(zr), 0.0f, 15.0f);
    double acc = 0.0;
    for (int j = 0; j < group; ++j) {
        float r = wp[j] / scale;
        float q = rintf(r);
        q = q + zero;
        q = clampf(q, 0.0f, 15.0f);
        if (codes) codes[j] = (uint8_t)q;
        float lv = q - zero;
        float dq = lv * scale;
        float e = dq - wp[j];
        diff[j] = e;
        acc += (double)e * (double)e;
    }
    if (xs) {
        /* the group's contribution to the layer output on the given rows:
         * sum_t ( sum_k e[k] * x'[t,k] )^2, in binary64 */
        acc = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double dot = 0.0;
            for (int j = 0; j < group; ++j)
                dot += (double)diff[j] * (double)awq_oracle_f16_to_f32(xs[t * row_stride + j]);
            acc += dot * dot;
        }
    }
    *sc_h_out = sc_h;
    *zero_out = zero;
    *err = acc;
}

int awq_oracle_quantize_clip(const uint16_t *W, const float *s, int64_t N, int64_t K, int group,
                             const float *ratios, int n_ratios, const uint16_t *xs, int64_t T,
                             uint8_t *codes, uint16_t *scales, uint8_t *zeros, uint8_t *choice)
{
    if (xs && T <= 0) return -4;
    if (!W || !codes || !scales || !zeros || !ratios) return -1;
    if (group != ORACLE_GROUP || N <= 0 || K <= 0 || K % group) return -2;
    if (n_ratios < 1 || n_ratios > 255) return -3;
    const int64_t G = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float wp[ORACLE_GROUP];
        for (int64_t g = 0; g < G; ++g) {
            const int64_t k0 = g * group;
            for (int j = 0; j < group; ++j) {
                float w = awq_oracle_f16_to_f32(W[n * K + k0 + j]);
                float sk = s ? s[k0 + j] : 1.0f;
                wp[j] = w * sk;
            }
            float mx = wp[0], mn = wp[0];
            for (int j = 1; j < group; ++j) {
                if (wp[j] > mx) mx = wp[j];
                if (wp[j] < mn) mn = wp[j];
            }
            int best = 0;
            double best_err = 0.0;
            for (int i = 0; i < n_ratios; ++i) {
                float mxr = mx * ratios[i];
                float mnr = mn * ratios[i];
                uint16_t sc_h;
                float zero;
                double err;
                quantize_group_range(wp, group, mxr, mnr, &sc_h, &zero, NULL, &err,
                                     xs ? xs + k0 : NULL, T, K);
                if (i == 0 || err < best_err) {
                    best = i;
                    best_err = err;
                }
            }
            {
                float mxr = mx * ratios[best];
                float mnr = mn * ratios[best];
                uint16_t sc_h;
                float zero;
                double err;
                quantize_group_range(wp, group, mxr, mnr, &sc_h, &zero, codes + n * K + k0, &err,
                                     NULL, 0, 0);
                scales[n * G + g] = sc_h;
                zeros[n * G + g] = (uint8_t)zero;
                if (choice) choice[n * G + g] = (uint8_t)best;
            }
        }
    }
    return 0;
}

/* ---------- a5: packed layout (written from the layout text) ----------
 * qweight: tiles of 16 rows x 128 columns, 1024 bytes each, tile index
 *          (n/16)*G + (k/128).  Inside a tile, 64 slots of 16 bytes; slot
 *          l = (n%16) + 16*c owns row n%16 and, in its 32-bit word j (0..3),
 *          the eight codes of columns 32*j + 8*c + e, e = 0..7.  Element e sits
 *          in nibble position P[e] of the little-endian word, P = {0,4,1,5,2,6,3,7}
 *          (so the nibbles, low to high, hold elements 0,2,4,6,1,3,5,7).
 * scales : [N/16][G][16] binary16  (row n%16 innermost)
 * zeros  : [N/16][G][8] bytes; byte b holds row 2b in its low nibble and row
 *          2b+1 in its high nibble.                                              */
static const int NIB_POS[8] = {0, 4, 1, 5, 2, 6, 3, 7};

int awq_oracle_pack(const uint8_t *codes, const uint16_t *scales, const uint8_t *zeros,
                    int64_t N, int64_t K, int group, uint8_t *qweight,
                    uint16_t *scales_p, uint8_t *zeros_p)
{
    if (!codes || !scales || !zeros || !qweight || !scales_p || !zeros_p) return -1;
    if (group != ORACLE_GROUP || N <= 0 || K <= 0 || K % group || N % 16) return -2;
    const int64_t G = K / group;
    memset(qweight, 0, (size_t)(N * K / 2));
    memset(zeros_p, 0, (size_t)(N * G / 2));
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t k = 0; k < K; ++k) {
            int64_t tile = (n / 16) * G + (k / 128);
            int kk = (int)(k % 128);
            int j = kk / 32;
            int c = (kk % 32) / 8;
            int e = kk % 8;
            int slot = (int)(n % 16) + 16 * c;
            int64_t word_byte = tile * 1024 + slot * 16 + j * 4;
            int bit = 4 * NIB_POS[e];
            uint8_t code = codes[n * K + k] & 0xf;
            qweight[word_byte + bit / 8] |= (uint8_t)(code << (bit % 8));
        }
        for (int64_t g = 0; g < G; ++g) {
            int64_t rb = n / 16;
            int r = (int)(n % 16);
            scales_p[(rb * G + g) * 16 + r] = scales[n * G + g];
            zeros_p[(rb * G + g) * 8 + r / 2] |= (uint8_t)((zeros[n * G + g] & 0xf) << (4 * (r % 2)));
        }
    }
    return 0;
}

int awq_oracle_unpack(const uint8_t *qweight, const uint16_t *scales_p,
                      const uint8_t *zeros_p, int64_t N, int64_t K, int group,
                      uint8_t *codes, uint16_t *scales, uint8_t *zeros)
{
    if (!codes || !scales || !zeros || !qweight || !scales_p || !zeros_p) return -1;
    if (group != ORACLE_GROUP || N <= 0 || K <= 0 || K % group || N % 16) return -2;
    const int64_t G = K / group;
    /* walk the packed bytes in storage order and scatter to [n,k] */
    for (int64_t tile = 0; tile < (N / 16) * G; ++tile) {
        int64_t rb = tile / G, g = tile % G;
        for (int slot = 0; slot < 64; ++slot) {
            int r = slot % 16, c = slot / 16;
            for (int j = 0; j < 4; ++j) {
                const uint8_t *wb = qweight + tile * 1024 + slot * 16 + j * 4;
                uint32_t word = (uint32_t)wb[0] | ((uint32_t)wb[1] << 8) |
                                ((uint32_t)wb[2] << 16) | ((uint32_t)wb[3] << 24);
                for (int e = 0; e < 8; ++e) {
                    int64_t n = rb * 16 + r;
                    int64_t k = g * 128 + 32 * j + 8 * c + e;
                    codes[n * K + k] = (uint8_t)((word >> (4 * NIB_POS[e])) & 0xf);
                }
            }
        }
        for (int r = 0; r < 16; ++r) {
            int64_t n = rb * 16 + r;
            scales[n * G + g] = scales_p[tile * 16 + r];
            zeros[n * G + g] = (uint8_t)((zeros_p[tile * 8 + r / 2] >> (4 * (r % 2))) & 0xf);
        }
    }
    return 0;
}

/* ---------- dequantize: Wdq[n,k] = (q - zero) * scale  (exact in binary32) ---------- */
int awq_oracle_dequant(const uint8_t *codes, const uint16_t *scales, const uint8_t *zeros,
                       int64_t N, int64_t K, int group, float *Wdq)
{
    if (!codes || !scales || !zeros || !Wdq) return -1;
    if (group <= 0 || N <= 0 || K <= 0 || K % group) return -2;
    const int64_t G = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            int64_t g = k / group;
            float d = (float)((int)codes[n * K + k] - (int)zeros[n * G + g]);
            Wdq[n * K + k] = d * awq_oracle_f16_to_f32(scales[n * G + g]);
        }
    return 0;
}

/* ---------- INT3-g128 variant (Sec. 5: "We focus on INT4/INT3 quantization"; Tab. 2 uses
 * INT3-g128).  The same asymmetric min/max quantizer with 8 levels:
 *   scale = fp16(clamp((max-min)/7, 2^-14, 65504)); zero = clamp(rint(-min/scale), 0, 7);
 *   q = clamp(rint(w'/scale) + zero, 0, 7).                                              */
int awq_oracle_quantize_w3(const uint16_t *W, const float *s, int64_t N, int64_t K,
                           int group, uint8_t *codes, uint16_t *scales, uint8_t *zeros)
{
    if (!W || !codes || !scales || !zeros) return -1;
    if (group != ORACLE_GROUP || N <= 0 || K <= 0 || K % group) return -2;
    const int64_t G = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float wp[ORACLE_GROUP];
        for (int64_t g = 0; g < G; ++g) {
            const int64_t k0 = g * group;
            for (int j = 0; j < group; ++j) {
                float w = awq_oracle_f16_to_f32(W[n * K + k0 + j]);
                float sk = s ? s[k0 + j] : 1.0f;
                wp[j] = w * sk;
            }
            float mx = wp[0], mn = wp[0];
            for (int j = 1; j < group; ++j) {
                if (wp[j] > mx) mx = wp[j];
                if (wp[j] < mn) mn = wp[j];
            }
            float range = mx - mn;
            float sc32 = range / 7.0f;
            sc32 = clampf(sc32, 6.103515625e-05f, 65504.0f);
            uint16_t sc_h = awq_oracle_f32_to_f16(sc32);
            float scale = awq_oracle_f16_to_f32(sc_h);
            float nmn = -mn;
            float zr = nmn / scale;
            float zero = clampf(rintf(zr), 0.0f, 7.0f);
            scales[n * G + g] = sc_h;
            zeros[n * G + g] = (uint8_t)zero;
            for (int j = 0; j < group; ++j) {
                float r = wp[j] / scale;
                float q = rintf(r);
                q = q + zero;
                q = clampf(q, 0.0f, 7.0f);
                codes[n * K + k0 + j] = (uint8_t)q;
            }
        }
    }
    return 0;
}

/* Packed layout of the 3-bit codes (written from the layout text):
 * qweight: tiles of 16 rows x 128 columns, 768 bytes each, tile index (n/16)*G + k/128.
 *          Inside a tile, 64 slots of 12 bytes = three little-endian 32-bit words; slot
 *          l = (n%16) + 16*c owns row n%16 and the 32 codes of columns 32*j + 8*c + e
 *          (j = 0..3, e = 0..7).  Code i = 8*j + e belongs to pair p = i/2, member h = i%2
 *          (h = 0: low 16-bit half of a word, h = 1: high half).  Pairs 0..14 sit in word p/5
 *          at bits [3f, 3f+3) of their half, f = p%5.  Pair 15 is spread over the spare top
 *          bit of the halves: bit b of its code is bit 15 (h = 0) or bit 31 (h = 1) of word b.
 * scales, zeros: as in the 4-bit layout (zero points 0..7 in nibbles).                  */
static void w3_position(int i, int bit, int *word, int *pos)
{
    int p = i / 2, h = i % 2;
    if (p < 15) {
        *word = p / 5;
        *pos = 16 * h + 3 * (p % 5) + bit;
    } else {
        *word = bit;
        *pos = 16 * h + 15;
    }
}

int awq_oracle_pack_w3(const uint8_t *codes, const uint16_t *scales, const uint8_t *zeros,
                       int64_t N, int64_t K, int group, uint8_t *qweight,
                       uint16_t *scales_p, uint8_t *zeros_p)
{
    if (!codes || !scales || !zeros || !qweight || !scales_p || !zeros_p) return -1;
    if (group != ORACLE_GROUP || N <= 0 || K <= 0 || K % group || N % 16) return -2;
    const int64_t G = K / group;
    memset(qweight, 0, (size_t)(N * K * 3 / 8));
    memset(zeros_p, 0, (size_t)(N * G / 2));
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t k = 0; k < K; ++k) {
            int64_t tile = (n / 16) * G + (k / 128);
            int kk = (int)(k % 128);
            int j = kk / 32, c = (kk % 32) / 8, e = kk % 8;
            int slot = (int)(n % 16) + 16 * c;
            uint8_t code = codes[n * K + k] & 0x7;
            for (int bit = 0; bit < 3; ++bit) {
                int word, pos;
                w3_position(8 * j + e, bit, &word, &pos);
                if ((code >> bit) & 1)
                    qweight[tile * 768 + slot * 12 + word * 4 + pos / 8] |= (uint8_t)(1u << (pos % 8));
            }
        }
        for (int64_t g = 0; g < G; ++g) {
            int64_t rb = n / 16;
            int r = (int)(n % 16);
            scales_p[(rb * G + g) * 16 + r] = scales[n * G + g];
            zeros_p[(rb * G + g) * 8 + r / 2] |= (uint8_t)((zeros[n * G + g] & 0xf) << (4 * (r % 2)));
        }
    }
    return 0;
}

int awq_oracle_unpack_w3(const uint8_t *qweight, const uint16_t *scales_p,
                         const uint8_t *zeros_p, int64_t N, int64_t K, int group,
                         uint8_t *codes, uint16_t *scales, uint8_t *zeros)
{
    if (!codes || !scales || !zeros || !qweight || !scales_p || !zeros_p) return -1;
    if (group != ORACLE_GROUP || N <= 0 || K <= 0 || K % group || N % 16) return -2;
    const int64_t G = K / group;
    for (int64_t tile = 0; tile < (N / 16) * G; ++tile) {
        int64_t rb = tile / G, g = tile % G;
        for (int slot = 0; slot < 64; ++slot) {
            int r = slot % 16, c = slot / 16;
            const uint8_t *sb = qweight + tile * 768 + slot * 12;
            for (int i = 0; i < 32; ++i) {
                uint8_t code = 0;
                for (int bit = 0; bit < 3; ++bit) {
                    int word, pos;
                    w3_position(i, bit, &word, &pos);
                    if ((sb[word * 4 + pos / 8] >> (pos % 8)) & 1) code |= (uint8_t)(1u << bit);
                }
                int64_t n = rb * 16 + r;
                int64_t k = g * 128 + 32 * (i / 8) + 8 * c + (i % 8);
                codes[n * K + k] = code;
            }
        }
        for (int r = 0; r < 16; ++r) {
            int64_t n = rb * 16 + r;
            scales[n * G + g] = scales_p[tile * 16 + r];
            zeros[n * G + g] = (uint8_t)((zeros_p[tile * 8 + r / 2] >> (4 * (r % 2))) & 0xf);
        }
    }
    return 0;
}

/* ---------- INT2-g64 variant (Sec. 5, the extreme low-bit table: INT2 with group size 64).
 * The same asymmetric min/max quantizer with 4 levels over groups of 64 input channels:
 *   scale = fp16(clamp((max-min)/3, 2^-14, 65504)); zero = clamp(rint(-min/scale), 0, 3);
 *   q = clamp(rint(w'/scale) + zero, 0, 3),  binary32, one rounding per operation.        */
#define ORACLE_GROUP_W2 64

int awq_oracle_quantize_w2(const uint16_t *W, const float *s, int64_t N, int64_t K,
                           int group, uint8_t *codes, uint16_t *scales, uint8_t *zeros)
{
    if (!W || !codes || !scales || !zeros) return -1;
    if (group != ORACLE_GROUP_W2 || N <= 0 || K <= 0 || K % group) return -2;
    const int64_t G = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        float wp[ORACLE_GROUP_W2];
        for (int64_t g = 0; g < G; ++g) {
            const int64_t k0 = g * group;
            for (int j = 0; j < group; ++j) {
                float w = awq_oracle_f16_to_f32(W[n * K + k0 + j]);
                float sk = s ? s[k0 + j] : 1.0f;
                wp[j] = w * sk;
            }
            float mx = wp[0], mn = wp[0];
            for (int j = 1; j < group; ++j) {
                if (wp[j] > mx) mx = wp[j];
                if (wp[j] < mn) mn = wp[j];
            }
            float range = mx - mn;
            float sc32 = range / 3.0f;
            sc32 = clampf(sc32, 6.103515625e-05f, 65504.0f);
            uint16_t sc_h = awq_oracle_f32_to_f16(sc32);
            float scale = awq_oracle_f16_to_f32(sc_h);
            float nmn = -mn;
            float zr = nmn / scale;
            float zero = clampf(rintf(zr), 0.0f, 3.0f);
            scales[n * G + g] = sc_h;
            zeros[n * G + g] = (uint8_t)zero;
            for (int j = 0; j < group; ++j) {
                float r = wp[j] / scale;
                float q = rintf(r);
                q = q + zero;
                q = clampf(q, 0.0f, 3.0f);
                codes[n * K + k0 + j] = (uint8_t)q;
            }
        }
    }
    return 0;
}

/* Packed layout of the 2-bit codes (written from the layout text).  K is a multiple of 256:
 * qweight: blocks of 16 rows x 256 columns (four groups of 64), 1024 bytes each, block index
 *          (n/16)*(K/256) + k/256.  Inside a block, 64 slots of 16 bytes = four little-endian
 *          32-bit words; slot l = (n%16) + 16*c owns row n%16 and the 64 codes of columns
 *          64*t + 32*j + 8*c + 2*i + h of the block (group t = 0..3, half of the group j = 0..1,
 *          i = 0..3, h = 0..1).  Word i holds the codes with that i: the code of (t, j, h) sits
 *          in field f = t + 4*j, bits [2f, 2f+2), of the low (h = 0) or high (h = 1) 16-bit
 *          half of the word.
 * scales : [N/16][K/256][16 rows][4 groups] binary16 (the group of the block innermost)
 * zeros  : [N/16][K/256][16 rows] bytes; the byte of a row holds the zero point of group t of
 *          the block at bits [2t, 2t+2).                                                   */
int awq_oracle_pack_w2(const uint8_t *codes, const uint16_t *scales, const uint8_t *zeros,
                       int64_t N, int64_t K, int group, uint8_t *qweight,
                       uint16_t *scales_p, uint8_t *zeros_p)
{
    if (!codes || !scales || !zeros || !qweight || !scales_p || !zeros_p) return -1;
    if (group != ORACLE_GROUP_W2 || N <= 0 || K <= 0 || K % 256 || N % 16) return -2;
    const int64_t G = K / group, B = K / 256;
    memset(qweight, 0, (size_t)(N * K / 4));
    memset(zeros_p, 0, (size_t)(N * G / 4));
    for (int64_t n = 0; n < N; ++n) {
        const int64_t rb = n / 16;
        const int r = (int)(n % 16);
        for (int64_t k = 0; k < K; ++k) {
            int64_t block = rb * B + k / 256;
            int kk = (int)(k % 256);
            int t = kk / 64, j = (kk % 64) / 32, c = (kk % 32) / 8, e = kk % 8;
            int slot = r + 16 * c;
            int i = e / 2, h = e % 2, f = t + 4 * j;
            int pos = 16 * h + 2 * f;
            uint8_t code = codes[n * K + k] & 0x3;
            qweight[block * 1024 + slot * 16 + i * 4 + pos / 8] |= (uint8_t)(code << (pos % 8));
        }
        for (int64_t g = 0; g < G; ++g) {
            int64_t block = rb * B + g / 4;
            int t = (int)(g % 4);
            scales_p[(block * 16 + r) * 4 + t] = scales[n * G + g];
            zeros_p[block * 16 + r] |= (uint8_t)((zeros[n * G + g] & 0x3) << (2 * t));
        }
    }
    return 0;
}

int awq_oracle_unpack_w2(const uint8_t *qweight, const uint16_t *scales_p,
                         const uint8_t *zeros_p, int64_t N, int64_t K, int group,
                         uint8_t *codes, uint16_t *scales, uint8_t *zeros)
{
    if (!codes || !scales || !zeros || !qweight || !scales_p || !zeros_p) return -1;
    if (group != ORACLE_GROUP_W2 || N <= 0 || K <= 0 || K % 256 || N % 16) return -2;
    const int64_t G = K / group, B = K / 256;
    /* walk the packed bytes in storage order and scatter to [n,k] */
    for (int64_t block = 0; block < (N / 16) * B; ++block) {
        int64_t rb = block / B, b = block % B;
        for (int slot = 0; slot < 64; ++slot) {
            int r = slot % 16, c = slot / 16;
            int64_t n = rb * 16 + r;
            for (int i = 0; i < 4; ++i) {
                const uint8_t *wb = qweight + block * 1024 + slot * 16 + i * 4;
                uint32_t word = (uint32_t)wb[0] | ((uint32_t)wb[1] << 8) |
                                ((uint32_t)wb[2] << 16) | ((uint32_t)wb[3] << 24);
                for (int h = 0; h < 2; ++h)
                    for (int f = 0; f < 8; ++f) {
                        int t = f % 4, j = f / 4;
                        int64_t k = b * 256 + 64 * t + 32 * j + 8 * c + 2 * i + h;
                        codes[n * K + k] = (uint8_t)((word >> (16 * h + 2 * f)) & 0x3);
                    }
            }
        }
        for (int r = 0; r < 16; ++r) {
            int64_t n = rb * 16 + r;
            for (int t = 0; t < 4; ++t) {
                scales[n * G + 4 * b + t] = scales_p[(block * 16 + r) * 4 + t];
                zeros[n * G + 4 * b + t] = (uint8_t)((zeros_p[block * 16 + r] >> (2 * t)) & 0x3);
            }
        }
    }
    return 0;
}

/* ---------- a6/a7: y[m,n] = sum_k x[m,k] * Wdq[n,k] ----------
 * x [M,K] binary16; Wdq [N,K] binary32; y [M,N] binary64.
 * acc32 != 0 switches to sequential binary32 accumulation (reported variant). */
int awq_oracle_matmul(const uint16_t *x, const float *Wdq, int64_t M, int64_t N,
                      int64_t K, int acc32, double *y)
{
    if (!x || !Wdq || !y || M <= 0 || N <= 0 || K <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) {
            if (acc32) {
                float acc = 0.0f;
                for (int64_t k = 0; k < K; ++k) {
                    float p = awq_oracle_f16_to_f32(x[m * K + k]) * Wdq[n * K + k];
                    acc = acc + p;
                }
                y[m * N + n] = (double)acc;
            } else {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k)
                    acc += (double)awq_oracle_f16_to_f32(x[m * K + k]) * (double)Wdq[n * K + k];
                y[m * N + n] = acc;
            }
        }
    return 0;
}

/* The acceptance metric of the build target, per element:
 * err[m,n] = |y_gpu - y_ref| / (||x[m,:]||_2 * max|Wdq| + 1e-6)                */
int awq_oracle_norm_error(const uint16_t *y_gpu, const double *y_ref, const uint16_t *x,
                          const float *Wdq, int64_t M, int64_t N, int64_t K, double *err)
{
    if (!y_gpu || !y_ref || !x || !Wdq || !err) return -1;
    double wmax = 0.0;
    for (int64_t i = 0; i < N * K; ++i) {
        double a = fabs((double)Wdq[i]);
        if (a > wmax) wmax = a;
    }
    for (int64_t m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double v = (double)awq_oracle_f16_to_f32(x[m * K + k]);
            ss += v * v;
        }
        double den = sqrt(ss) * wmax + 1e-6;
        for (int64_t n = 0; n < N; ++n) {
            double d = (double)awq_oracle_f16_to_f32(y_gpu[m * N + n]) - y_ref[m * N + n];
            err[m * N + n] = fabs(d) / den;
        }
    }
    return 0;
}

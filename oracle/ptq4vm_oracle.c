/*
 * CPU oracle for the PTQ4VM quantized-linear path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct loops written from the paper's definitions.
 * It shares no code with the HIP library and must never be called from the
 * product path: only tests, the smoke check and the benchmark's CPU-baseline leg
 * use it.  Build: gcc -O2 -fopenmp -ffp-contract=off -fno-fast-math (no FMA
 * contraction, IEEE semantics), see oracle/ptq4vm_oracle.py.
 *
 * What each function follows:
 *   oracle_fold_smoothing   SmoothQuant identity Y = (W diag(s)) (diag(s)^-1 X), Sec. 2.4
 *                           Eq. (smooth); symmetric per-output-channel weight quantizer,
 *                           Sec. 2.3 (the Delta_W / W-hat pair of equations), b = 8.
 *   oracle_quantize_pts     Per-Token Static quantization, Sec. 5.1: one static step per
 *                           token position, symmetric (zero offset omitted as in the PTS
 *                           equation), round-to-nearest + clip of Sec. 2.3; activation
 *                           smoothing then quantization in the order of App. B.1.
 *   oracle_int8_gemm        the integer product W-bar . X-bar of the PTS equation, Sec. 5.1.
 *   oracle_dequant          diag(Delta_W) (W-bar X-bar) diag(Delta_X) of the PTS equation
 *                           (+ bias), evaluated in double, rounded once to fp16.
 *   oracle_f16_linear       the unquantized FP16 linear the paper's latency table compares to.
 *
 *   oracle_quantize_dynamic per-token dynamic quantization, the comparison scheme of Sec. 4 and of the
 *                           latency table of Sec. 6.4: the step of a token row is computed online
 *                           from that row (after smoothing), s_r = max_k|v| / 127.
 *   oracle_fold_smoothing_bits / oracle_quantize_pts_bits
 *                           the same quantizers at b bits (Sec. 2.3: clip to +-(2^(b-1) - 1)); b = 4
 *                           is the W4A4 setting of the paper's latency table.
 *   oracle_pack_int4 / oracle_unpack_int4
 *                           two adjacent 4-bit codes per byte, the even index in the low nibble
 *                           (App. B.1 "Quantization").
 *   oracle_pack_e2m3 / oracle_unpack_e2m3
 *                           the same 4-bit codes (-7..7) written as 6-bit floating-point numbers
 *                           (1 sign, 2 exponent, 3 mantissa bits, exponent bias 1: the "E2M3" element
 *                           of the OCP microscaling formats), which hold every integer of that range
 *                           exactly; a storage container of the boundary, not a step of the paper's
 *                           method (the paper packs two's-complement nibbles, App. B.1).
 *   oracle_quantize_pts_offset / oracle_weight_rowsum / oracle_dequant_offset
 *                           PTS with the per-token zero offset that Sec. 5.1 mentions and then
 *                           omits; the offset form is the activation quantizer of Sec. 2.3
 *                           (clip(round(X / Delta) + eps, 0, 2^b - 1)) with the code range shifted
 *                           by 128 so that codes are int8: q = clip(rint(v) + z, -128, 127),
 *                           x-hat = s (q - z), and sum_k (q - z) w = acc - z * rowsum(w).
 *
 * Readings where the paper is silent (all stated again in the design notes):
 *   - rounding is round-half-to-even; clip range is [-127, 127] for weights and activations;
 *   - the integer decision of the activation quantizer is taken in fp32 in this exact order:
 *     v = f32(x) * inv_m[k];  v = v * inv_s[t];  q = rint(v);  clamp;  with
 *     inv_m[k] = 1/m[k] and inv_s[t] = 1/s_tok[t] correctly rounded fp32 divisions;
 *   - the weight decision: wf = f32(w) * m[k];  s_w = max_k|wf| / 127 (1 if the row is zero);
 *     q = rint(wf / s_w);  clamp;  all fp32, IEEE division;
 *   - NaN quantizes to 0, +-Inf to +-127;
 *   - storage is token-major: X[B*L, K], W[N, K], Y[B*L, N]; row r has token position r mod L.
 *
 * Layout: every matrix is dense row-major with leading dimension = its width.
 * fp16 values are passed as raw uint16_t bit patterns.
 */
#include <stdint.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- IEEE binary16 <-> binary32/64, written out bit by bit ---- */

static float half_bits_to_float(uint16_t h) {
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1Fu;
    uint32_t man = h & 0x3FFu;
    uint32_t bits;
    if (exp == 0) {
        if (man == 0) {
            bits = sign;
        } else { /* subnormal: value = man * 2^-24, normalise */
            int e = -1;
            do { man <<= 1; e++; } while ((man & 0x400u) == 0);
            man &= 0x3FFu;
            bits = sign | (uint32_t)(127 - 15 - e) << 23 | (man << 13);
        }
    } else if (exp == 31) {
        bits = sign | 0x7F800000u | (man << 13);
    } else {
        bits = sign | (exp + (127 - 15)) << 23 | (man << 13);
    }
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

/* double -> binary16, round-half-to-even, single rounding step. */
static uint16_t double_to_half_bits(double d) {
    uint64_t u;
    memcpy(&u, &d, 8);
    uint16_t sign = (uint16_t)((u >> 48) & 0x8000u);
    int64_t exp = (int64_t)((u >> 52) & 0x7FF);
    uint64_t man = u & 0xFFFFFFFFFFFFFull;
    if (exp == 0x7FF) { /* Inf / NaN */
        return (uint16_t)(sign | 0x7C00u | (man ? 0x200u : 0u));
    }
    if (exp == 0) { /* double zero / subnormal: far below half's range */
        return sign;
    }
    int64_t e = exp - 1023;              /* unbiased exponent, value = 1.man * 2^e */
    uint64_t sig = man | (1ull << 52);   /* 53-bit significand */
    int shift;                           /* bits of sig to drop */
    int64_t hexp;                        /* biased half exponent of the kept leading bit */
    if (e >= -14) {                      /* normal half (before rounding) */
        shift = 42;                      /* keep 11 bits */
        hexp = e + 15;
    } else {                             /* subnormal half: unit is 2^-24 */
        int64_t extra = -14 - e;         /* additional right shift */
        if (extra > 12) return sign;     /* < 2^-26: rounds to zero (2^-25 tie -> even = 0 handled below) */
        shift = 42 + (int)extra;
        hexp = 0;
    }
    uint64_t kept = sig >> shift;
    uint64_t rem = sig & ((1ull << shift) - 1);
    uint64_t half = 1ull << (shift - 1);
    if (rem > half || (rem == half && (kept & 1))) kept++;
    uint32_t out;
    if (hexp == 0) {
        out = (uint32_t)kept;            /* carries into exponent field naturally at 0x400 */
    } else {
        /* kept in [0x400, 0x800]; adding (hexp-1)<<10 lets a mantissa carry bump the exponent */
        out = (uint32_t)(((uint64_t)(hexp - 1) << 10) + kept);
    }
    if (out >= 0x7C00u) out = 0x7C00u;   /* overflow -> Inf */
    return (uint16_t)(sign | out);
}

/* exported for the conversion pins */
float oracle_half_to_float(uint16_t h) { return half_bits_to_float(h); }
uint16_t oracle_double_to_half(double d) { return double_to_half_bits(d); }

int oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- a0: fold the smoothing vector into the weight, then quantize per output channel ---- */
void oracle_fold_smoothing(const uint16_t *w_f16, const float *m, int8_t *wq, float *s_w,
                           float *inv_m, int64_t N, int64_t K) {
    for (int64_t k = 0; k < K; k++) inv_m[k] = 1.0f / m[k];
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < N; o++) {
        float amax = 0.0f;
        for (int64_t k = 0; k < K; k++) {
            float wf = half_bits_to_float(w_f16[o * K + k]) * m[k];
            float a = fabsf(wf);
            if (a > amax) amax = a;
        }
        float step = (amax == 0.0f) ? 1.0f : amax / 127.0f;
        s_w[o] = step;
        for (int64_t k = 0; k < K; k++) {
            float wf = half_bits_to_float(w_f16[o * K + k]) * m[k];
            float q = rintf(wf / step);
            if (q != q) q = 0.0f;
            if (q > 127.0f) q = 127.0f;
            if (q < -127.0f) q = -127.0f;
            wq[o * K + k] = (int8_t)q;
        }
    }
}

/* ---- a1: per-token static activation quantizer (smoothing multiply fused in front) ---- */
void oracle_quantize_pts(const uint16_t *x_f16, const float *inv_m /* NULL => all ones */,
                         const float *s_tok, int8_t *xq, int64_t B, int64_t L, int64_t K) {
    int64_t M = B * L;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; r++) {
        float inv_s = 1.0f / s_tok[r % L];
        for (int64_t k = 0; k < K; k++) {
            float v = half_bits_to_float(x_f16[r * K + k]);
            if (inv_m) v = v * inv_m[k];
            v = v * inv_s;
            float q = rintf(v);
            if (q != q) q = 0.0f;
            if (q > 127.0f) q = 127.0f;
            if (q < -127.0f) q = -127.0f;
            xq[r * K + k] = (int8_t)q;
        }
    }
}

/* ---- a2: integer GEMM acc[r,o] = sum_k Xq[r,k] * Wq[o,k].
 * Returns the number of outputs whose exact (int64) sum does not fit int32. ---- */
int64_t oracle_int8_gemm(const int8_t *xq, const int8_t *wq, int32_t *acc, int64_t M, int64_t K,
                         int64_t N) {
    int64_t overflow = 0;
#pragma omp parallel for schedule(static) reduction(+ : overflow)
    for (int64_t r = 0; r < M; r++) {
        for (int64_t o = 0; o < N; o++) {
            int64_t wide = 0;
            for (int64_t k = 0; k < K; k++) wide += (int64_t)xq[r * K + k] * (int64_t)wq[o * K + k];
            if (wide > INT32_MAX || wide < INT32_MIN) overflow++;
            acc[r * N + o] = (int32_t)wide;
        }
    }
    return overflow;
}

/* ---- a3: dequantize: Y[r,o] = fp16( acc * s_tok[r mod L] * s_w[o] + bias[o] ) in double.
 * y64_out (nullable) receives the unrounded double value for tolerance checks. ---- */
void oracle_dequant(const int32_t *acc, const float *s_tok, const float *s_w,
                    const uint16_t *bias_f16 /* nullable */, uint16_t *y_f16, double *y64_out,
                    int64_t B, int64_t L, int64_t N) {
    int64_t M = B * L;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; r++) {
        double st = (double)s_tok[r % L];
        for (int64_t o = 0; o < N; o++) {
            double y = (double)acc[r * N + o] * st * (double)s_w[o];
            if (bias_f16) y += (double)half_bits_to_float(bias_f16[o]);
            if (y64_out) y64_out[r * N + o] = y;
            y_f16[r * N + o] = double_to_half_bits(y);
        }
    }
}

/* ---- a4: unquantized comparison linear, fp16 inputs, double accumulation ---- */
void oracle_f16_linear(const uint16_t *x_f16, const uint16_t *w_f16, const uint16_t *bias_f16,
                       uint16_t *y_f16, double *y64_out, double *abs_sum_out, int64_t M, int64_t K,
                       int64_t N) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; r++) {
        for (int64_t o = 0; o < N; o++) {
            double s = 0.0, a = 0.0;
            for (int64_t k = 0; k < K; k++) {
                double p = (double)half_bits_to_float(x_f16[r * K + k]) *
                           (double)half_bits_to_float(w_f16[o * K + k]);
                s += p;
                a += fabs(p);
            }
            if (bias_f16) {
                double b = (double)half_bits_to_float(bias_f16[o]);
                s += b;
                a += fabs(b);
            }
            if (y64_out) y64_out[r * N + o] = s;
            if (abs_sum_out) abs_sum_out[r * N + o] = a;
            y_f16[r * N + o] = double_to_half_bits(s);
        }
    }
}


/* ---- per-token dynamic activation quantizer (Sec. 4; the "Per-token dynamic" rows of the latency
 * table, Sec. 6.4).  Every row gets its own step from its own smoothed values:
 *   v[k] = f32(x[r,k]) * inv_m[k];  s_r = max_k |v[k]| / 127 (1 if the row is all zero; NaNs do not
 *   take part in the maximum);  q = clip(rint(v * (1 / s_r)), -127, 127), all in fp32. ---- */
void oracle_quantize_dynamic(const uint16_t *x_f16, const float *inv_m /* NULL => all ones */,
                             int8_t *xq, float *s_row, int64_t M, int64_t K) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; r++) {
        float amax = 0.0f;
        for (int64_t k = 0; k < K; k++) {
            float v = half_bits_to_float(x_f16[r * K + k]);
            if (inv_m) v = v * inv_m[k];
            float a = fabsf(v);
            if (a > amax) amax = a;
        }
        float step = (amax == 0.0f) ? 1.0f : amax / 127.0f;
        float inv_s = 1.0f / step;
        s_row[r] = step;
        for (int64_t k = 0; k < K; k++) {
            float v = half_bits_to_float(x_f16[r * K + k]);
            if (inv_m) v = v * inv_m[k];
            v = v * inv_s;
            float q = rintf(v);
            if (q != q) q = 0.0f;
            if (q > 127.0f) q = 127.0f;
            if (q < -127.0f) q = -127.0f;
            xq[r * K + k] = (int8_t)q;
        }
    }
}

/* ---- b-bit forms of a0 and a1 (Sec. 2.3: codes clipped to +-qmax, qmax = 2^(b-1) - 1).  Codes are
 * returned one per int8; packing is a separate step. ---- */
void oracle_fold_smoothing_bits(const uint16_t *w_f16, const float *m, int8_t *wq, float *s_w,
                                float *inv_m, int64_t N, int64_t K, int qmax) {
    const float fq = (float)qmax;
    for (int64_t k = 0; k < K; k++) inv_m[k] = 1.0f / m[k];
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < N; o++) {
        float amax = 0.0f;
        for (int64_t k = 0; k < K; k++) {
            float a = fabsf(half_bits_to_float(w_f16[o * K + k]) * m[k]);
            if (a > amax) amax = a;
        }
        float step = (amax == 0.0f) ? 1.0f : amax / fq;
        s_w[o] = step;
        for (int64_t k = 0; k < K; k++) {
            float wf = half_bits_to_float(w_f16[o * K + k]) * m[k];
            float q = rintf(wf / step);
            if (q != q) q = 0.0f;
            if (q > fq) q = fq;
            if (q < -fq) q = -fq;
            wq[o * K + k] = (int8_t)q;
        }
    }
}

void oracle_quantize_pts_bits(const uint16_t *x_f16, const float *inv_m, const float *s_tok,
                              int8_t *xq, int64_t B, int64_t L, int64_t K, int qmax) {
    const float fq = (float)qmax;
    int64_t M = B * L;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; r++) {
        float inv_s = 1.0f / s_tok[r % L];
        for (int64_t k = 0; k < K; k++) {
            float v = half_bits_to_float(x_f16[r * K + k]);
            if (inv_m) v = v * inv_m[k];
            v = v * inv_s;
            float q = rintf(v);
            if (q != q) q = 0.0f;
            if (q > fq) q = fq;
            if (q < -fq) q = -fq;
            xq[r * K + k] = (int8_t)q;
        }
    }
}

/* ---- INT4 packing (App. B.1): byte j of a row holds codes 2j (low nibble) and 2j + 1 (high
 * nibble), each in two's complement.  K must be even. ---- */
void oracle_pack_int4(const int8_t *codes, uint8_t *packed, int64_t rows, int64_t K) {
    for (int64_t r = 0; r < rows; r++)
        for (int64_t j = 0; j < K / 2; j++) {
            int lo = codes[r * K + 2 * j], hi = codes[r * K + 2 * j + 1];
            packed[r * (K / 2) + j] = (uint8_t)(((hi & 15) << 4) | (lo & 15));
        }
}

void oracle_unpack_int4(const uint8_t *packed, int8_t *codes, int64_t rows, int64_t K) {
    for (int64_t r = 0; r < rows; r++)
        for (int64_t j = 0; j < K / 2; j++) {
            int b = packed[r * (K / 2) + j];
            int lo = b & 15, hi = b >> 4;
            codes[r * K + 2 * j] = (int8_t)(lo >= 8 ? lo - 16 : lo);
            codes[r * K + 2 * j + 1] = (int8_t)(hi >= 8 ? hi - 16 : hi);
        }
}

/* ---- E2M3 container of 4-bit codes.  A 6-bit pattern s e1 e0 m2 m1 m0 stands for
 *   (-1)^s * 2^(e - 1) * (1 + m / 8)   for e = 1, 2, 3,        (-1)^s * (m / 8)   for e = 0,
 * so the integers 0..7 are the patterns with values 0, 1, 2, 3, 4, 5, 6, 7 and a clear sign bit, and
 * their negatives have the sign bit set (zero is always written with a clear sign bit).
 * A row of K codes is padded with zeros to a multiple of 128 and written in blocks of 96 bytes, one per
 * 128 codes.  Inside a block, group g = 0..3 holds codes 32 g .. 32 g + 31 as a 192-bit little-endian
 * string, code j of the group at bits [6 j, 6 j + 6); the first 16 bytes of group g sit at block offset
 * 16 g, its last 8 bytes at block offset 64 + 8 g.
 * The matrix is stored block-major: plane b holds block b of every row, row r at byte 96 r of the plane,
 * planes back to back (plane pitch 96 rows): packed[b][r][96]. ---- */
static double e2m3_value(int pattern) {
    int s = (pattern >> 5) & 1, e = (pattern >> 3) & 3, m = pattern & 7;
    double mag = e == 0 ? m / 8.0 : ldexp(1.0 + m / 8.0, e - 1);
    return s ? -mag : mag;
}

static int e2m3_pattern_of(int code) { /* the pattern whose value is `code`; -1 if there is none */
    for (int pattern = 0; pattern < 64; pattern++)
        if (e2m3_value(pattern) == (double)code && !(code == 0 && pattern != 0)) return pattern;
    return -1;
}

int64_t oracle_e2m3_blocks(int64_t K) { return (K + 127) / 128; }

/* returns 0, or -1 if a code has no E2M3 pattern (|code| > 7) */
int oracle_pack_e2m3(const int8_t *codes, uint8_t *packed, int64_t rows, int64_t K) {
    const int64_t plane = rows * 96;
    memset(packed, 0, (size_t)(oracle_e2m3_blocks(K) * plane));
    for (int64_t r = 0; r < rows; r++)
        for (int64_t k = 0; k < K; k++) {
            const int pattern = e2m3_pattern_of(codes[r * K + k]);
            if (pattern < 0) return -1;
            const int64_t block = k / 128, g = (k % 128) / 32, j = k % 32;
            for (int b = 0; b < 6; b++) {
                if (!((pattern >> b) & 1)) continue;
                const int64_t bit = 6 * j + b;           /* position in the group's 192-bit string */
                const int64_t byte = bit / 8;            /* 0..23 */
                const int64_t off = byte < 16 ? 16 * g + byte : 64 + 8 * g + (byte - 16);
                packed[block * plane + r * 96 + off] |= (uint8_t)(1u << (bit % 8));
            }
        }
    return 0;
}

/* returns 0, or -1 if a pattern's value is not an integer (codes of padding positions are skipped) */
int oracle_unpack_e2m3(const uint8_t *packed, int8_t *codes, int64_t rows, int64_t K) {
    const int64_t plane = rows * 96;
    for (int64_t r = 0; r < rows; r++)
        for (int64_t k = 0; k < K; k++) {
            const int64_t block = k / 128, g = (k % 128) / 32, j = k % 32;
            int pattern = 0;
            for (int b = 0; b < 6; b++) {
                const int64_t bit = 6 * j + b, byte = bit / 8;
                const int64_t off = byte < 16 ? 16 * g + byte : 64 + 8 * g + (byte - 16);
                if ((packed[block * plane + r * 96 + off] >> (bit % 8)) & 1) pattern |= 1 << b;
            }
            const double v = e2m3_value(pattern);
            if (v != floor(v)) return -1;
            codes[r * K + k] = (int8_t)v;
        }
    return 0;
}

/* ---- PTS with a per-token zero offset (Sec. 5.1 names it, the PTS equation omits it; Sec. 2.3
 * gives the offset quantizer).  z_tok[t] is the int8-range offset of token position t:
 *   q = clip(rint((f32(x) * inv_m[k]) * (1 / s_tok[t])) + z_tok[t], -128, 127),  x-hat = s_tok[t] (q - z_tok[t]). ---- */
void oracle_quantize_pts_offset(const uint16_t *x_f16, const float *inv_m, const float *s_tok,
                                const int32_t *z_tok, int8_t *xq, int64_t B, int64_t L, int64_t K) {
    int64_t M = B * L;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; r++) {
        float inv_s = 1.0f / s_tok[r % L];
        int64_t z = z_tok[r % L];
        for (int64_t k = 0; k < K; k++) {
            float v = half_bits_to_float(x_f16[r * K + k]);
            if (inv_m) v = v * inv_m[k];
            v = v * inv_s;
            float q = rintf(v);
            if (q != q) q = 0.0f;
            if (q > 1.0e6f) q = 1.0e6f;   /* keep the integer sum below in range; the clip follows */
            if (q < -1.0e6f) q = -1.0e6f;
            int64_t c = (int64_t)q + z;
            if (c > 127) c = 127;
            if (c < -128) c = -128;
            xq[r * K + k] = (int8_t)c;
        }
    }
}

/* rowsum[o] = sum_k wq[o,k]: what the offset multiplies in  sum_k (q - z) w = sum_k q w - z rowsum. */
void oracle_weight_rowsum(const int8_t *wq, int32_t *rowsum, int64_t N, int64_t K) {
    for (int64_t o = 0; o < N; o++) {
        int64_t s = 0;
        for (int64_t k = 0; k < K; k++) s += wq[o * K + k];
        rowsum[o] = (int32_t)s;
    }
}

/* Y[r,o] = fp16( (acc - z_tok[r mod L] * rowsum[o]) * s_tok[r mod L] * s_w[o] + bias[o] ), in double. */
void oracle_dequant_offset(const int32_t *acc, const float *s_tok, const int32_t *z_tok,
                           const int32_t *rowsum, const float *s_w, const uint16_t *bias_f16,
                           uint16_t *y_f16, double *y64_out, int64_t B, int64_t L, int64_t N) {
    int64_t M = B * L;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; r++) {
        double st = (double)s_tok[r % L];
        int64_t z = z_tok[r % L];
        for (int64_t o = 0; o < N; o++) {
            int64_t corrected = (int64_t)acc[r * N + o] - z * (int64_t)rowsum[o];
            double y = (double)corrected * st * (double)s_w[o];
            if (bias_f16) y += (double)half_bits_to_float(bias_f16[o]);
            if (y64_out) y64_out[r * N + o] = y;
            y_f16[r * N + o] = double_to_half_bits(y);
        }
    }
}

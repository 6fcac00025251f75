/*
 * mx_oracle.c -- CPU oracle for the MXFP4 quantized linear layer of TetraJet
 * (arxiv 2502.20853).  TEST INFRASTRUCTURE ONLY: see mx_oracle.h.
 *
 * Every step is written the way the paper states it, one element at a time.
 * Precision: S is a power of two, so the scaled value y = x / S of an FP32 input
 * is exact in FP64 (2^-149 * 2^-127 is far inside its range); every comparison
 * that picks a code is evaluated exactly in FP64 on that exact y.  The EMA
 * update is FP32.  Matrix products are FP64.
 *
 * Build: gcc -O2 -std=c11 -fopenmp -ffp-contract=off -fPIC -shared mx_oracle.c -lm
 */
#include "mx_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- E2M1 ---- */

/* Sec. 3.1: E2M1 has 2 exponent bits and 1 mantissa bit, Q_p = 6.  With
 * exponent bias 1 the eight magnitudes are: subnormal 0, 0.5; then
 * (1 + m/2) * 2^(e-1) for e = 1, 2, 3. */
static const double E2M1_MAG[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};

double orc_e2m1_value(int code)
{
    double m = E2M1_MAG[code & 7];
    return (code & 8) ? -m : m;
}

/* index (0..7) of an E2M1 magnitude */
static int mag_index(double m)
{
    for (int t = 0; t < 8; ++t)
        if (E2M1_MAG[t] == m) return t;
    return 7;
}

/* Two consecutive E2M1 magnitudes with m1 <= a <= m2 (Sec. 3.2).  If a is at
 * or beyond the largest magnitude the bracket collapses to m1 = m2 = 6. */
static void bracket(double a, double* m1, double* m2)
{
    int i = 0;
    for (int t = 0; t < 8; ++t)
        if (E2M1_MAG[t] <= a) i = t;
    *m1 = E2M1_MAG[i];
    *m2 = (i < 7) ? E2M1_MAG[i + 1] : E2M1_MAG[7];
}

/* -------------------------------------------------------------- Philox ---- */

static void mulhilo32(uint32_t a, uint32_t b, uint32_t* hi, uint32_t* lo)
{
    uint64_t p = (uint64_t)a * (uint64_t)b;
    *hi = (uint32_t)(p >> 32);
    *lo = (uint32_t)p;
}

void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;   /* round multipliers   */
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;   /* key schedule (Weyl) */
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint32_t hi0, lo0, hi1, lo1;
        mulhilo32(M0, c0, &hi0, &lo0);
        mulhilo32(M1, c2, &hi1, &lo1);
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

uint32_t orc_sr_bits(uint64_t seed, uint32_t tensor_id, uint64_t e)
{
    uint64_t blk = e >> 3;
    uint32_t ctr[4] = {(uint32_t)blk, (uint32_t)(blk >> 32), tensor_id, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t w[4];
    orc_philox4x32_10(ctr, key, w);
    unsigned j = (unsigned)(e & 7u);
    return (w[j >> 1] >> (16u * (j & 1u))) & 0xFFFFu;
}

/* ------------------------------------------------------- shared exponent -- */

int orc_shared_exponent(float M, int scale_mode)
{
    double Mt = (M > 0.0f) ? (double)M : 1e-8;   /* epsilon for the all-zero group */
    int guess;
    (void)frexp(Mt, &guess);                     /* only a starting point */
    int s;
    if (scale_mode == ORC_SCALE_TRUNCFREE) {
        /* s = ceil(log2(2*Mt/(Qp-Qn))) = ceil(log2(Mt/6)): the smallest
         * integer s with Mt <= 6 * 2^s.  ldexp and the comparison are exact. */
        s = guess;
        while (ldexp(6.0, s) < Mt) ++s;
        while (ldexp(6.0, s - 1) >= Mt) --s;
    } else {
        /* floor(log2 Mt): the largest integer e with 2^e <= Mt; s = e - E_max. */
        int e = guess;
        while (ldexp(1.0, e) > Mt) --e;
        while (ldexp(1.0, e + 1) <= Mt) ++e;
        s = e - 2;
    }
    if (s > 127) s = 127;
    if (s < -127) s = -127;
    return s;
}

/* x / S with S = 2^s: exact in FP64. */
static double scale_to_group(float x, int s, int scale_mode)
{
    double y = ldexp((double)x, -s);
    if (scale_mode == ORC_SCALE_FLOOR) {
        /* Eq. 2's scale can leave |y| > Q_p; such values saturate at +-Q_p (Sec. 3.2) */
        if (y > 6.0) y = 6.0;
        if (y < -6.0) y = -6.0;
    }
    return y;
}

/* -------------------------------------------------------------- rounding -- */

static int round_rtn_d(double y)
{
    int sign = signbit(y) ? 8 : 0;
    double yd = y, m1, m2, q1, q2;
    bracket(fabs(yd), &m1, &m2);
    if (!sign) { q1 = m1;  q2 = m2;  }           /* q1 < q2 in signed terms */
    else       { q1 = -m2; q2 = -m1; }
    double pick = (fabs(yd - q1) < fabs(yd - q2)) ? q1 : q2;
    return sign | mag_index(fabs(pick));
}

int orc_round_rtn(float y) { return round_rtn_d((double)y); }

static int round_sr_d(double y, uint32_t r16)
{
    /* round_S: xi ~ U(-D/2, D/2), D = q2 - q1; q1 iff y + xi < (q1+q2)/2, so
     * P(q2) = (y - q1)/D and P(q1) = (q2 - y)/D.  On the magnitude a = |y| both
     * signs read: the larger magnitude m2 is taken with probability
     * p = (a - m1)/(m2 - m1).  The uniform variate is r16/65536. */
    int sign = signbit(y) ? 8 : 0;
    double a = fabs(y), m1, m2;
    bracket(a, &m1, &m2);
    double p = (m2 > m1) ? (a - m1) / (m2 - m1) : 0.0;
    int up = ((double)r16 < 65536.0 * p);
    return sign | mag_index(up ? m2 : m1);
}

int orc_round_sr(float y, uint32_t r16) { return round_sr_d((double)y, r16); }

/* Q-EMA's choice (Algorithm 1).  The candidate pair (q1, q2) is read as the BRACKETING pair of
 * y = w/S, q1 <= y <= q2, the pair Sec. 3.2 names with the same symbols.  Algorithm 1's wording
 * (the two values nearest to y) and Sec. 5's (the two values of smallest error) name a different
 * pair wherever E2M1's spacing changes: for |y| in (2, 2.25) the two nearest values are 1.5 and 2
 * while the bracket is (2, 3), and for |y| in (4, 4.5) they are 3 and 4 while the bracket is (4, 6).
 * The bracket is taken because the threshold that y can oscillate across is the midpoint of the two
 * values either side of it (Sec. 4.1), because a choice outside the bracket would move the weight
 * past a representable value that lies between it and the result, and because only the bracket
 * makes Q-EMA with W_EMA = W identical to round_D on every input. */
static int round_ema_d(double y, double z)
{
    int sign = signbit(y) ? 8 : 0;
    double yd = y, zd = z, m1, m2, q1, q2;
    bracket(fabs(yd), &m1, &m2);
    if (m1 == fabs(yd)) return sign | mag_index(m1);   /* y is an E2M1 value */
    if (!sign) { q1 = m1;  q2 = m2;  }
    else       { q1 = -m2; q2 = -m1; }
    double pick = (fabs(zd - q1) < fabs(zd - q2)) ? q1 : q2;
    return sign | mag_index(fabs(pick));
}

int orc_round_ema(float y, float z) { return round_ema_d((double)y, (double)z); }

/* ------------------------------------------------------------ quantizers -- */

static float group_amax(const float* x, int64_t stride)
{
    float M = 0.0f;
    for (int i = 0; i < 32; ++i) {
        float a = fabsf(x[i * stride]);
        if (a > M) M = a;
    }
    return M;
}

static void put_code(uint8_t* codes, int64_t idx, int code)
{
    uint8_t* b = &codes[idx >> 1];
    if (idx & 1) *b = (uint8_t)((*b & 0x0F) | (code << 4));
    else         *b = (uint8_t)((*b & 0xF0) | code);
}

static int get_code(const uint8_t* codes, int64_t idx)
{
    uint8_t b = codes[idx >> 1];
    return (idx & 1) ? (b >> 4) : (b & 0x0F);
}

void orc_quantize(const float* src, int64_t rows, int64_t cols, int64_t ld,
                  uint8_t* codes, uint8_t* scales,
                  int round, int scale_mode,
                  uint64_t seed, uint32_t tensor_id, uint64_t index_base)
{
    int64_t groups = cols / 32;
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t g = 0; g < groups; ++g) {
            const float* x = src + r * ld + 32 * g;
            float M = group_amax(x, 1);
            int s = orc_shared_exponent(M, scale_mode);
            scales[r * groups + g] = (uint8_t)(s + 127);
            for (int i = 0; i < 32; ++i) {
                int64_t c = 32 * g + i;
                double y = scale_to_group(x[i], s, scale_mode);
                int code;
                if (round == ORC_ROUND_SR) {
                    uint64_t e = index_base + (uint64_t)r * (uint64_t)cols + (uint64_t)c;
                    code = round_sr_d(y, orc_sr_bits(seed, tensor_id, e));
                } else {
                    code = round_rtn_d(y);
                }
                put_code(codes + r * (cols / 2), c, code);
            }
        }
    }
}

/* ------------------------------------------------------------------ GELU -- */

/* The activation between the two linear layers of a transformer MLP (Sec. 7.1 quantizes all linear
 * layers of the MLP module): GELU(x) = x * Phi(x), Phi the standard normal distribution function,
 * Phi(x) = erfc(-x / sqrt(2)) / 2.  FP64. */
void orc_gelu(const double* x, int64_t n, double* out)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        out[i] = x[i] * (0.5 * erfc(-x[i] / sqrt(2.0)));
}

/* ----------------------------------------- E3M0 elements (Table 7's ablation) -- */

/* The format ablation (Table 7 and its paragraph) names E3M0 as the other possible FP4 format and
 * says no more.  Reading, built the way Sec. 3.1's E2M1 is: sign bit, 3 exponent bits, no mantissa
 * bit, exponent bias 2^(3-1) - 1 = 3, no Inf/NaN codes.  Exponent field 0 is the subnormal range,
 * which without a mantissa bit holds only 0; field E >= 1 is 2^(E-3).  Q_p = -Q_n = 16, and the
 * E_max of Eq. 2 (the exponent of the largest value) is 4. */
static const double E3M0_MAG[8] = {0.0, 0.25, 0.5, 1.0, 2.0, 4.0, 8.0, 16.0};

double orc_e3m0_value(int code)
{
    double m = E3M0_MAG[code & 7];
    return (code & 8) ? -m : m;
}

/* Sec. 3.2 with Q_p - Q_n = 32 and E_max = 4. */
int orc_shared_exponent_e3m0(float M, int scale_mode)
{
    double Mt = (M > 0.0f) ? (double)M : 1e-8;
    int guess, s;
    (void)frexp(Mt, &guess);
    if (scale_mode == ORC_SCALE_TRUNCFREE) {
        /* s = ceil(log2(2*Mt/32)): the smallest integer s with Mt <= 16 * 2^s */
        s = guess;
        while (ldexp(16.0, s) < Mt) ++s;
        while (ldexp(16.0, s - 1) >= Mt) --s;
    } else {
        /* s = floor(log2 Mt) - E_max */
        int e = guess;
        while (ldexp(1.0, e) > Mt) --e;
        while (ldexp(1.0, e + 1) <= Mt) ++e;
        s = e - 4;
    }
    if (s > 127) s = 127;
    if (s < -127) s = -127;
    return s;
}

/* two consecutive E3M0 magnitudes with m1 <= a <= m2; m1 = m2 = 16 at or beyond the largest */
static void bracket_e3m0(double a, double* m1, double* m2)
{
    int i = 0;
    for (int t = 0; t < 8; ++t)
        if (E3M0_MAG[t] <= a) i = t;
    *m1 = E3M0_MAG[i];
    *m2 = (i < 7) ? E3M0_MAG[i + 1] : E3M0_MAG[7];
}

static int mag_index_e3m0(double m)
{
    for (int t = 0; t < 8; ++t)
        if (E3M0_MAG[t] == m) return t;
    return 7;
}

/* round_D of Sec. 3.2 on the E3M0 grid: q1 iff strictly nearer, else q2 */
static int round_rtn_e3m0_d(double y)
{
    int sign = signbit(y) ? 8 : 0;
    double m1, m2, q1, q2;
    bracket_e3m0(fabs(y), &m1, &m2);
    if (!sign) { q1 = m1;  q2 = m2;  }
    else       { q1 = -m2; q2 = -m1; }
    double pick = (fabs(y - q1) < fabs(y - q2)) ? q1 : q2;
    return sign | mag_index_e3m0(fabs(pick));
}

/* round_S of Sec. 3.2 on the E3M0 grid, with the same use of the 16 random bits as for E2M1 */
static int round_sr_e3m0_d(double y, uint32_t r16)
{
    int sign = signbit(y) ? 8 : 0;
    double a = fabs(y), m1, m2;
    bracket_e3m0(a, &m1, &m2);
    double p = (m2 > m1) ? (a - m1) / (m2 - m1) : 0.0;
    int up = ((double)r16 < 65536.0 * p);
    return sign | mag_index_e3m0(up ? m2 : m1);
}

int orc_round_rtn_e3m0(float y) { return round_rtn_e3m0_d((double)y); }
int orc_round_sr_e3m0(float y, uint32_t r16) { return round_sr_e3m0_d((double)y, r16); }

void orc_quantize_e3m0(const float* src, int64_t rows, int64_t cols, int64_t ld,
                  uint8_t* codes, uint8_t* scales,
                  int round, int scale_mode,
                  uint64_t seed, uint32_t tensor_id, uint64_t index_base)
{
    int64_t groups = cols / 32;
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t g = 0; g < groups; ++g) {
            const float* x = src + r * ld + 32 * g;
            float M = group_amax(x, 1);
            int s = orc_shared_exponent_e3m0(M, scale_mode);
            scales[r * groups + g] = (uint8_t)(s + 127);
            for (int i = 0; i < 32; ++i) {
                int64_t c = 32 * g + i;
                double y = ldexp((double)x[i], -s);                 /* exact */
                if (scale_mode == ORC_SCALE_FLOOR) {                /* Eq. 2's scale leaves |y| up to 32: truncated to Q_p */
                    if (y > 16.0) y = 16.0;
                    if (y < -16.0) y = -16.0;
                }
                int code;
                if (round == ORC_ROUND_SR) {
                    uint64_t e = index_base + (uint64_t)r * (uint64_t)cols + (uint64_t)c;
                    code = round_sr_e3m0_d(y, orc_sr_bits(seed, tensor_id, e));
                } else {
                    code = round_rtn_e3m0_d(y);
                }
                put_code(codes + r * (cols / 2), c, code);
            }
        }
    }
}

void orc_dequantize_e3m0(const uint8_t* codes, const uint8_t* scales,
                    int64_t rows, int64_t cols, double* out)
{
    int64_t groups = cols / 32;
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            int s = (int)scales[r * groups + c / 32] - 127;
            out[r * cols + c] = ldexp(orc_e3m0_value(get_code(codes + r * (cols / 2), c)), s);
        }
}

void orc_dequantize(const uint8_t* codes, const uint8_t* scales,
                    int64_t rows, int64_t cols, double* out)
{
    int64_t groups = cols / 32;
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            int s = (int)scales[r * groups + c / 32] - 127;
            out[r * cols + c] = ldexp(orc_e2m1_value(get_code(codes + r * (cols / 2), c)), s);
        }
}

void orc_quantize_transposed(const float* src, int64_t rows, int64_t cols, int64_t ld,
                  uint8_t* codes_t, uint8_t* scales_t,
                  int round_t, uint32_t tensor_id_t, int pre_quant,
                  uint8_t* codes_row, uint8_t* scales_row,
                  int round_row, uint32_t tensor_id_row,
                  const uint8_t* row_codes_in, const uint8_t* row_scales_in,
                  int scale_mode, uint64_t seed, uint64_t index_base)
{
    /* 1. the 1x32 quantizer (forward operand), if asked for or needed */
    uint8_t* tmp_codes = NULL;
    uint8_t* tmp_scales = NULL;
    const uint8_t* rc = row_codes_in;
    const uint8_t* rs = row_scales_in;
    int need_row = (codes_row != NULL) || (pre_quant && rc == NULL);
    if (need_row) {
        uint8_t* oc = codes_row;
        uint8_t* os = scales_row;
        if (oc == NULL) {
            oc = tmp_codes = (uint8_t*)malloc((size_t)(rows * (cols / 2)));
            os = tmp_scales = (uint8_t*)malloc((size_t)(rows * (cols / 32)));
        }
        if (rc != NULL) {            /* caller supplied the row result: pass it on */
            memcpy(oc, rc, (size_t)(rows * (cols / 2)));
            memcpy(os, rs, (size_t)(rows * (cols / 32)));
        } else {
            orc_quantize(src, rows, cols, ld, oc, os, round_row, scale_mode,
                         seed, tensor_id_row, index_base);
            rc = oc; rs = os;
        }
    }

    /* 2. the matrix the 32x1 quantizer sees: src, or dequant(Q_row(src)) */
    float* V = (float*)malloc((size_t)(rows * cols) * sizeof(float));
    if (pre_quant) {
        double* dq = (double*)malloc((size_t)(rows * cols) * sizeof(double));
        orc_dequantize(rc, rs, rows, cols, dq);
        for (int64_t t = 0; t < rows * cols; ++t) V[t] = (float)dq[t];   /* exact */
        free(dq);
    } else {
        for (int64_t i = 0; i < rows; ++i)
            for (int64_t c = 0; c < cols; ++c) V[i * cols + c] = src[i * ld + c];
    }

    /* 3. 32x1 groups: 32 consecutive rows of one column; result stored transposed */
    int64_t groups = rows / 32;
    #pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < cols; ++c) {
        for (int64_t g = 0; g < groups; ++g) {
            const float* x = V + (32 * g) * cols + c;
            float M = group_amax(x, cols);
            int s = orc_shared_exponent(M, scale_mode);
            scales_t[c * groups + g] = (uint8_t)(s + 127);
            for (int t = 0; t < 32; ++t) {
                int64_t i = 32 * g + t;
                double y = scale_to_group(x[t * cols], s, scale_mode);
                int code;
                if (round_t == ORC_ROUND_SR) {
                    uint64_t e = index_base + (uint64_t)i * (uint64_t)cols + (uint64_t)c;
                    code = round_sr_d(y, orc_sr_bits(seed, tensor_id_t, e));
                } else {
                    code = round_rtn_d(y);
                }
                put_code(codes_t + c * (rows / 2), i, code);
            }
        }
    }
    free(V);
    free(tmp_codes);
    free(tmp_scales);
}

void orc_ema_weight_quant(const float* w, float* w_ema, float beta, int update_ema,
                  int64_t rows, int64_t cols, int64_t ld,
                  uint8_t* codes, uint8_t* scales, int scale_mode)
{
    int64_t groups = cols / 32;
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t g = 0; g < groups; ++g) {
            const float* x = w + r * ld + 32 * g;
            float* ema = w_ema + r * ld + 32 * g;
            /* Eq. 8: W_EMA <- beta * W_EMA + (1 - beta) * W, in FP32 */
            for (int i = 0; i < 32; ++i) {
                if (update_ema == 1) {
                    float one_minus_beta = 1.0f - beta;
                    float t = one_minus_beta * x[i];
                    ema[i] = fmaf(beta, ema[i], t);
                } else if (update_ema == 2) {
                    ema[i] = x[i];
                }
            }
            /* Algorithm 1: the scale comes from the weight block itself */
            float M = group_amax(x, 1);
            int s = orc_shared_exponent(M, scale_mode);
            scales[r * groups + g] = (uint8_t)(s + 127);
            for (int i = 0; i < 32; ++i) {
                double y = scale_to_group(x[i], s, scale_mode);
                double z = ldexp((double)ema[i], -s);
                put_code(codes + r * (cols / 2), 32 * g + i, round_ema_d(y, z));
            }
        }
    }
}

/* ------------------------------------------------------------------ GEMM -- */

void orc_gemm_f64(const uint8_t* a_codes, const uint8_t* a_scales,
                  const uint8_t* b_codes, const uint8_t* b_scales,
                  int64_t m, int64_t n, int64_t k, double* c)
{
    double* A = (double*)malloc((size_t)(m * k) * sizeof(double));
    double* B = (double*)malloc((size_t)(n * k) * sizeof(double));
    orc_dequantize(a_codes, a_scales, m, k, A);
    orc_dequantize(b_codes, b_scales, n, k, B);
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int64_t t = 0; t < k; ++t) acc += A[i * k + t] * B[j * k + t];
            c[i * n + j] = acc;
        }
    free(A);
    free(B);
}

void orc_gemm_f64_sampled(const uint8_t* a_codes, const uint8_t* a_scales,
                  const uint8_t* b_codes, const uint8_t* b_scales,
                  int64_t m, int64_t n, int64_t k,
                  const int64_t* ii, const int64_t* jj, int64_t nsamp,
                  double* out, double* abs_out)
{
    (void)m; (void)n;
    int64_t groups = k / 32;
    #pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < nsamp; ++t) {
        const uint8_t* ac = a_codes + ii[t] * (k / 2);
        const uint8_t* bc = b_codes + jj[t] * (k / 2);
        const uint8_t* as = a_scales + ii[t] * groups;
        const uint8_t* bs = b_scales + jj[t] * groups;
        double acc = 0.0, aacc = 0.0;
        for (int64_t d = 0; d < k; ++d) {
            double a = ldexp(orc_e2m1_value(get_code(ac, d)), (int)as[d / 32] - 127);
            double b = ldexp(orc_e2m1_value(get_code(bc, d)), (int)bs[d / 32] - 127);
            acc += a * b;
            aacc += fabs(a * b);
        }
        out[t] = acc;
        if (abs_out) abs_out[t] = aacc;
    }
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- Q-Ramping: oscillation detection (Sec. 6.1) and amplification factor (Algorithm 2) ---- */

void orc_oscillation_accumulate(const float* w, int64_t rows, int64_t cols, int64_t ld,
                  const uint8_t* codes, const uint8_t* scales,
                  float* w_prev, float* wq_prev, float* dist_w, float* dist_q, int init)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            const int64_t i = r * cols + c;
            const uint8_t byte = codes[r * (cols / 2) + c / 2];
            const int code = (c & 1) ? (byte >> 4) : (byte & 15);
            const int s = (int)scales[r * (cols / 32) + c / 32] - 127;
            /* the quantized weight the forward pass uses: P * 2^s, exact in FP32 */
            const float wq = (float)ldexp(orc_e2m1_value(code), s);
            const float wc = w[r * ld + c];
            if (init) {
                dist_w[i] = 0.0f;
                dist_q[i] = 0.0f;
            } else {
                const float dw = fabsf(wc - w_prev[i]);
                const float dq = fabsf(wq - wq_prev[i]);
                dist_w[i] = dist_w[i] + dw;
                dist_q[i] = dist_q[i] + dq;
            }
            w_prev[i] = wc;
            wq_prev[i] = wq;
        }
}

void orc_ramping_factor(const float* dist_w, const float* dist_q, int64_t count,
                  float k1, int k2, int n_max, int32_t* factor)
{
    for (int64_t i = 0; i < count; ++i) {
        float ratio;
        if (dist_w[i] == 0.0f) ratio = dist_q[i] == 0.0f ? 0.0f : INFINITY;
        else                   ratio = dist_q[i] / dist_w[i];
        const float steps = floorf(ratio / k1);               /* floor(R_w / k1) */
        /* k2 * steps + 1, capped: compare in floating point first so that +infinity is capped too */
        int32_t n = n_max;
        if (steps < (float)n_max) {
            const int64_t v = (int64_t)k2 * (int64_t)steps + 1;
            n = v < (int64_t)n_max ? (int32_t)v : n_max;
        }
        factor[i] = n;
    }
}

/* ----------------------------------------------------------- diagnostics -- */

/* distance from y to the nearest of the 14 rounding thresholds (midpoints of neighbouring signed
 * E2M1 values) */
static double nearest_threshold_distance(double y)
{
    double best = INFINITY;
    for (int t = 0; t < 7; ++t) {
        const double thr = 0.5 * (E2M1_MAG[t] + E2M1_MAG[t + 1]);
        const double dp = fabs(y - thr), dn = fabs(y + thr);
        if (dp < best) best = dp;
        if (dn < best) best = dn;
    }
    return best;
}

/* MaxDist of Sec. 4.2 for the E2M1 value with magnitude index t (the same for both signs): the
 * cell of the value reaches from the midpoint towards the neighbour below to the midpoint towards
 * the neighbour above; the cell of 0 is [-0.25, 0.25]; the cell of 6 ends at 6. */
static double cell_max_distance(int t)
{
    if (t == 7) return E2M1_MAG[7] - 0.5 * (E2M1_MAG[6] + E2M1_MAG[7]);
    const double hi = 0.5 * (E2M1_MAG[t] + E2M1_MAG[t + 1]);
    const double lo = (t == 0) ? -hi : 0.5 * (E2M1_MAG[t - 1] + E2M1_MAG[t]);
    return 0.5 * (hi - lo);
}

void orc_quant_confidence(const float* w, int64_t rows, int64_t cols, int64_t ld, int scale_mode,
                  float* conf, uint64_t* hist, int bins)
{
    int64_t groups = cols / 32;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t g = 0; g < groups; ++g) {
            const float* x = w + r * ld + 32 * g;
            const int s = orc_shared_exponent(group_amax(x, 1), scale_mode);
            for (int i = 0; i < 32; ++i) {
                const double y = scale_to_group(x[i], s, scale_mode);
                const int code = round_rtn_d(y);
                const float num = (float)nearest_threshold_distance(y);   /* exact */
                const float den = (float)cell_max_distance(code & 7);     /* exact */
                const float c = num / den;
                if (conf) conf[r * cols + 32 * g + i] = c;
                if (hist) {
                    int b = (int)floorf(c * (float)bins);
                    if (b > bins - 1) b = bins - 1;
                    hist[b] += 1;
                }
            }
        }
}

/* Column sums of a matrix, out[c] = sum over r of x[r][c], rows in index order, FP64.  For the
 * gradient dY of a linear layer's output (Sec. 3.3) this is the gradient of the layer's bias; the
 * layer's products themselves carry no bias. */
void orc_column_sums(const float* x, int64_t rows, int64_t cols, int64_t ld, double* out)
{
    for (int64_t c = 0; c < cols; ++c) {
        double s = 0.0;
        for (int64_t r = 0; r < rows; ++r) s += (double)x[r * ld + c];
        out[c] = s;
    }
}

double orc_rate_of_change_term(const float* x, int64_t rows, int64_t cols, int64_t ld, float* x_prev)
{
    double diff2 = 0.0, prev2 = 0.0;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            const double cur = (double)x[r * ld + c];
            const double old = (double)x_prev[r * cols + c];
            diff2 += (cur - old) * (cur - old);
            prev2 += old * old;
            x_prev[r * cols + c] = x[r * ld + c];
        }
    if (prev2 == 0.0) return diff2 == 0.0 ? 0.0 : INFINITY;
    return sqrt(diff2) / sqrt(prev2);
}

/* --------------------------------------------------- Q-Ramping's optimizer -- */

void orc_ramping_adamw_step(double* w, const double* grad, int64_t count,
                  double* m, double* v, double* g_acc,
                  const int32_t* factor, int32_t* acc_steps, int32_t* updates,
                  double lr, double beta1, double beta2, double eps, double weight_decay)
{
    for (int64_t i = 0; i < count; ++i) {
        const int32_t n_w = factor ? factor[i] : 1;
        g_acc[i] += grad[i];
        acc_steps[i] += 1;
        if (acc_steps[i] < n_w) continue;              /* this element's batch is not full yet */
        const double g = g_acc[i] / (double)acc_steps[i];
        const double lr_w = (double)n_w * lr;
        updates[i] += 1;
        const double u = (double)updates[i];
        w[i] = w[i] * (1.0 - lr_w * weight_decay);
        m[i] = beta1 * m[i] + (1.0 - beta1) * g;
        v[i] = beta2 * v[i] + (1.0 - beta2) * g * g;
        const double bc1 = 1.0 - pow(beta1, u);
        const double bc2 = 1.0 - pow(beta2, u);
        w[i] = w[i] - (lr_w / bc1) * m[i] / (sqrt(v[i]) / sqrt(bc2) + eps);
        g_acc[i] = 0.0;
        acc_steps[i] = 0;
    }
}

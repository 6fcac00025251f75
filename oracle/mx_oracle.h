/*
 * mx_oracle.h -- CPU oracle for the MXFP4 quantized linear layer of TetraJet
 * (arxiv 2502.20853).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow,
 * step-by-step implementation of what the paper defines, written so that a
 * reader can check it against the paper by eye.  Only the tests, the smoke
 * check and the benchmark's "cpu_baseline" leg may call it.  It shares no
 * code, table or constant generator with the HIP path.
 *
 * Parity status: every function below is pinned by tests that do not run the
 * function's own formula a second time (worked values printed in the paper,
 * closed forms, invariants, brute force).  The one exception is the Philox
 * stream, whose constants the paper does not give: it is pinned against the
 * published Philox4x32-10 known-answer vectors and a second big-integer
 * implementation in the tests.
 *
 * Notation follows the paper: a group is 32 consecutive elements along the
 * contraction dimension, S = 2^s its shared scale, P_i the E2M1 element,
 * Q_p = 6, Q_n = -6, M the group's largest absolute value.
 *
 * Packed layout used everywhere (Sec. 3.1 "stored as ({P_i}, S)"; nibble order
 * is this build's choice): for a row-major [rows x cols] matrix quantized
 * along its columns,
 *     codes [r][j] = code(r, 2j) | code(r, 2j+1) << 4      (cols/2 bytes per row)
 *     scales[r][g] = s + 127   for group g = cols [32g, 32g+32)  (cols/32 bytes)
 * An E2M1 code is sign<<3 | exponent<<1 | mantissa; magnitudes of codes 0..7
 * are 0, 0.5, 1, 1.5, 2, 3, 4, 6.
 */
#ifndef MX_ORACLE_H
#define MX_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_ROUND_RTN = 0, ORC_ROUND_SR = 1 };
enum { ORC_SCALE_TRUNCFREE = 0, ORC_SCALE_FLOOR = 1 };

/* Value of one E2M1 code (0..15).  Sec. 3.1: E2M1 with Q_p = 6. */
double orc_e2m1_value(int code);

/* Philox4x32 with 10 rounds (Salmon et al., SC'11).  ctr and out are 4 words,
 * key is 2 words. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* The 16 random bits that decide the stochastic rounding of the element with
 * global index e of tensor tensor_id under seed.  One Philox call, with
 * counter (e>>3 low, e>>3 high, tensor_id, 0) and key (seed low, seed high),
 * serves 8 consecutive elements: element e uses 16-bit field (e & 7), fields
 * numbered from the low half of word 0. */
uint32_t orc_sr_bits(uint64_t seed, uint32_t tensor_id, uint64_t e);

/* Shared exponent s of a group whose largest absolute value is M.
 * TRUNCFREE: s = ceil(log2(2*Mt/(Q_p-Q_n))) (Sec. 3.2, truncation-free scaling);
 * FLOOR:     s = floor(log2 Mt) - E_max, E_max = 2 (Eq. 2);
 * Mt = M if M > 0 else 1e-8; the result is clamped to |s| <= 127 (Sec. 3.1). */
int orc_shared_exponent(float M, int scale_mode);

/* round_D of Sec. 3.2 applied to the scaled value y (|y| <= 6): returns the
 * E2M1 code; the sign bit of the code is the sign bit of y. */
int orc_round_rtn(float y);

/* round_S of Sec. 3.2 with the 16 random bits r16 (0..65535): with a = |y|,
 * m1 <= a <= m2 the bracketing magnitudes and p = (a-m1)/(m2-m1), the larger
 * magnitude is taken iff r16 < 65536*p. */
int orc_round_sr(float y, uint32_t r16);

/* Q-EMA decision (Algorithm 1) for one element: y = w/S proposes the bracket
 * (q1, q2), z = w_ema/S picks the nearer (q1 iff strictly nearer).  If y is
 * itself an E2M1 value the result is y. */
int orc_round_ema(float y, float z);

/* GELU(x) = x * Phi(x) (exact form), FP64, element-wise: the activation between the two linear layers of
 * the MLP module, used by the check of the product with the fused activation and next-layer quantizer. */
void orc_gelu(const double* x, int64_t n, double* out);

/* E3M0 elements, the other FP4 format of the format ablation (Table 7): sign, 3 exponent bits, no
 * mantissa bit, bias 3; magnitudes 0, 0.25, 0.5, 1, 2, 4, 8, 16 (Q_p = 16, E_max = 4).  The functions
 * below are the E3M0 counterparts of orc_e2m1_value, orc_shared_exponent, orc_round_rtn,
 * orc_round_sr, orc_quantize and orc_dequantize: Sec. 3.2 with these constants. */
double orc_e3m0_value(int code);
int orc_shared_exponent_e3m0(float M, int scale_mode);
int orc_round_rtn_e3m0(float y);
int orc_round_sr_e3m0(float y, uint32_t r16);
void orc_quantize_e3m0(const float* src, int64_t rows, int64_t cols, int64_t ld,
                  uint8_t* codes, uint8_t* scales,
                  int round, int scale_mode,
                  uint64_t seed, uint32_t tensor_id, uint64_t index_base);
void orc_dequantize_e3m0(const uint8_t* codes, const uint8_t* scales,
                    int64_t rows, int64_t cols, double* out);

/* Quantize src[rows x cols] (row stride ld elements) in 1x32 groups along the
 * columns.  Element (r, c) has global index index_base + r*cols + c. */
void orc_quantize(const float* src, int64_t rows, int64_t cols, int64_t ld,
                  uint8_t* codes, uint8_t* scales,
                  int round, int scale_mode,
                  uint64_t seed, uint32_t tensor_id, uint64_t index_base);

/* Quantize src[rows x cols] in 32x1 groups (32 consecutive rows of one
 * column) and store the result transposed: codes_t[cols x rows/2],
 * scales_t[cols x rows/32].
 * pre_quant = 1: the quantizer's input is dequant(Q_row(src)) (double
 *   quantization, Sec. 3.3), where Q_row is the 1x32 quantizer with rounding
 *   round_row / tensor_id_row, or the given (row_codes_in, row_scales_in) when
 *   those are non-NULL.
 * codes_row/scales_row, when non-NULL, receive the 1x32 result as well.
 * Element (i, c) keeps its source index index_base + i*cols + c in both
 * quantizers. */
void orc_quantize_transposed(const float* src, int64_t rows, int64_t cols, int64_t ld,
                  uint8_t* codes_t, uint8_t* scales_t,
                  int round_t, uint32_t tensor_id_t, int pre_quant,
                  uint8_t* codes_row, uint8_t* scales_row,
                  int round_row, uint32_t tensor_id_row,
                  const uint8_t* row_codes_in, const uint8_t* row_scales_in,
                  int scale_mode, uint64_t seed, uint64_t index_base);

/* Q-EMA (Eq. 8 and Algorithm 1).  update_ema: 0 leave w_ema, 1 set
 * w_ema = beta*w_ema + (1-beta)*w first, 2 set w_ema = w first.  Then quantize
 * w in 1x32 groups with the scale of w and the rounding of orc_round_ema. */
void orc_ema_weight_quant(const float* w, float* w_ema, float beta, int update_ema,
                  int64_t rows, int64_t cols, int64_t ld,
                  uint8_t* codes, uint8_t* scales, int scale_mode);

/* Oscillation detection of Q-Ramping (Sec. 6.1 / "Identifying Oscillating Weights"): per weight
 * element, the lengths of the trajectories of the master weight w and of its quantized value
 * w_Q = P * 2^s over a window of steps,
 *     dist_W = sum_t |w^t - w^(t-1)|,   dist_Q = sum_t |w_Q^t - w_Q^(t-1)|.
 * One call is one step t.  init != 0 opens a window: the previous values are set to the current
 * ones and both sums to 0.  All arithmetic is FP32, one rounding per operation (difference, then
 * add), in the order written.  w_prev, wq_prev, dist_w, dist_q are dense [rows x cols]. */
void orc_oscillation_accumulate(const float* w, int64_t rows, int64_t cols, int64_t ld,
                  const uint8_t* codes, const uint8_t* scales,
                  float* w_prev, float* wq_prev, float* dist_w, float* dist_q, int init);

/* Amplification factor of Algorithm 2 (Q-Ramping): R_w = dist_Q / dist_W (FP32 division),
 * N_w = min(k2 * floor(R_w / k1) + 1, n_max); LR_w = N_w * LR, BS_w = N_w * BS.
 * dist_W = 0: R_w is taken as 0 when dist_Q = 0 too and as +infinity otherwise (the paper does not
 * say).  k1 > 0, k2 >= 0, n_max >= 1. */
void orc_ramping_factor(const float* dist_w, const float* dist_q, int64_t count,
                  float k1, int k2, int n_max, int32_t* factor);

/* One optimizer step of Q-Ramping's customised AdamW (Algorithm 2, "update w according to LR_w and
 * BS_w"; Sec. 6.2: the batch size of an oscillating weight is N_w times the global one, realised by
 * accumulating its gradient, and its learning rate grows in proportion).  Per element, FP64:
 *     g_acc += grad;  acc_steps += 1;
 *     if acc_steps >= N_w:                       (N_w = factor, 1 everywhere if factor is NULL)
 *         g = g_acc / acc_steps;  lr_w = N_w * lr;  u = ++updates;
 *         w = w * (1 - lr_w * weight_decay)                              (decoupled decay)
 *         m = beta1 * m + (1 - beta1) * g;   v = beta2 * v + (1 - beta2) * g * g;
 *         w = w - (lr_w / (1 - beta1^u)) * m / (sqrt(v) / sqrt(1 - beta2^u) + eps);
 *         g_acc = 0;  acc_steps = 0;
 * so that an element with factor N follows exactly AdamW at learning rate N * lr on the means of N
 * consecutive gradients, its bias correction counting its own updates.  The paper gives no formula
 * for the update; this is the reading taken. */
void orc_ramping_adamw_step(double* w, const double* grad, int64_t count,
                  double* m, double* v, double* g_acc,
                  const int32_t* factor, int32_t* acc_steps, int32_t* updates,
                  double lr, double beta1, double beta2, double eps, double weight_decay);

/* Quantization confidence (Sec. 4.2): for a weight element w of a 1x32 group with scale S,
 * on the latent value y = w / S,
 *     QuantConf = min_i |y - thrd_i| / MaxDist(y_FP4),
 * where the thresholds are the 14 midpoints between neighbouring signed E2M1 values, y_FP4 is the
 * deterministic rounding of y, and MaxDist(v) is the largest distance to the nearest threshold a
 * latent value rounded to v can have: half the width of v's cell for a cell between two thresholds,
 * the whole width for the two outermost cells [5, 6] and [-6, -5].  (The ratio is the same in the
 * unscaled domain: S multiplies numerator and denominator alike.)  Numerator and denominator are
 * exact in FP32; the quotient is one FP32 division.  conf is dense [rows x cols].
 * hist, if not NULL, holds `bins` counters and is ADDED to: element with confidence c counts in bin
 * min(bins - 1, floor(c * bins)), the product taken in FP32. */
void orc_quant_confidence(const float* w, int64_t rows, int64_t cols, int64_t ld, int scale_mode,
                  float* conf, uint64_t* hist, int bins);

/* One term of the rate of change of a tensor (Sec. 4.1):
 *     r(X) = (1/T0) sum_{t=1..T0} ||X^t - X^(t-1)||_F / ||X^(t-1)||_F.
 * Returns ||x - x_prev||_F / ||x_prev||_F in FP64 (differences of FP32 values are exact in FP64;
 * the sums of squares run in FP64 in index order), then sets x_prev = x.  x_prev is dense
 * [rows x cols].  A zero ||x_prev|| gives 0 if the difference is zero too, +infinity otherwise. */
void orc_column_sums(const float* x, int64_t rows, int64_t cols, int64_t ld, double* out);
double orc_rate_of_change_term(const float* x, int64_t rows, int64_t cols, int64_t ld, float* x_prev);

/* X_i = P_i * 2^s (Sec. 3.1), exact in double. */
void orc_dequantize(const uint8_t* codes, const uint8_t* scales,
                  int64_t rows, int64_t cols, double* out);

/* C[m x n] = A[m x k] * B[n x k]^T on the dequantized operands, FP64
 * (Sec. 3.3: the three products all take this form once the second operand is
 * stored along its contraction dimension). */
void orc_gemm_f64(const uint8_t* a_codes, const uint8_t* a_scales,
                  const uint8_t* b_codes, const uint8_t* b_scales,
                  int64_t m, int64_t n, int64_t k, double* c);

/* Same product, only at the nsamp entries (ii[t], jj[t]); also returns
 * sum_k |A||B| per entry in abs_out (may be NULL). */
void orc_gemm_f64_sampled(const uint8_t* a_codes, const uint8_t* a_scales,
                  const uint8_t* b_codes, const uint8_t* b_scales,
                  int64_t m, int64_t n, int64_t k,
                  const int64_t* ii, const int64_t* jj, int64_t nsamp,
                  double* out, double* abs_out);

/* Threads the parallel loops use. */
int orc_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif

/*
 * mxfp4.h -- C ABI of the MI355X (gfx950) implementation of the MXFP4 quantized
 * linear layer of TetraJet (arxiv 2502.20853): the six quantizers and three
 * matrix products of Eqs. 3-5 (Sec. 3.3) and the EMA weight quantizer
 * (Sec. 5, Algorithm 1).
 *
 * Conventions
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *    never allocates, frees or synchronises; all work is enqueued on the HIP
 *    stream passed as `stream` (a hipStream_t cast to void*, NULL = default
 *    stream).  Outputs are valid once that stream has reached the call.
 *  - Every function returns MX_OK or a negative MX_ERR_* code.  Arguments are
 *    validated on the host before anything is launched, so a call that returns
 *    an error other than MX_ERR_HIP has touched no memory.  MX_ERR_HIP means
 *    the HIP runtime refused a launch; mx_last_hip_error() gives its code.
 *  - Matrices are row-major; `ld` is the row stride in elements.
 *  - Packed MXFP4 layout (Sec. 3.1: a group of 32 elements shares S = 2^s, each
 *    element is an E2M1 value P_i, stored as ({P_i}, S)).  For a [rows x cols]
 *    matrix grouped 1x32 along its columns:
 *        codes [r][j] = code(r, 2j) | code(r, 2j+1) << 4     rows x cols/2  bytes
 *        scales[r][g] = s + 127 for columns [32g, 32g+32)    rows x cols/32 bytes
 *    both dense (no padding).  An E2M1 code is sign<<3 | exponent<<1 | mantissa
 *    (magnitudes 0, .5, 1, 1.5, 2, 3, 4, 6); its sign bit is the sign bit of
 *    the source element, also when the magnitude rounds to zero.  |s| <= 127,
 *    so a scale byte of 255 is never produced.
 *  - Inputs must be finite.  NaN/Inf give unspecified codes but never an
 *    out-of-bounds access.  With pre_quant, |x| must stay below 2^126 so that
 *    the dequantized intermediate is finite in FP32.
 *  - Stochastic rounding draws 16 bits per element from Philox4x32-10 with key
 *    (seed low, seed high) and counter (e>>3 low, e>>3 high, tensor_id, 0),
 *    e = index_base + row*cols + col being the element's index in the SOURCE
 *    tensor as passed (before any transposition); element e takes the 16-bit
 *    field (e & 7), counted from the low half of output word 0.  The larger
 *    magnitude of the bracketing E2M1 pair is taken iff field < 65536 * p,
 *    p = (|y| - m1) / (m2 - m1)  (round_S of Sec. 3.2).  index_base must be a
 *    multiple of 8 when stochastic rounding is used.
 */
#ifndef MXFP4_H
#define MXFP4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MX_OK = 0,
    MX_ERR_NULL = -1,       /* a required pointer is NULL, or an optional pair is half set */
    MX_ERR_SHAPE = -2,      /* non-positive size, contraction/group dimension not a multiple of 32, ld < cols, size out of range */
    MX_ERR_DTYPE = -3,      /* unknown dtype code */
    MX_ERR_MODE = -4,       /* unknown rounding / scale / update mode, beta outside [0,1) */
    MX_ERR_ALIGN = -5,      /* pointer, ld or index_base violates the stated alignment */
    MX_ERR_WORKSPACE = -6,  /* workspace missing or smaller than mx_linear_workspace_bytes() */
    MX_ERR_HIP = -7         /* HIP launch failure, see mx_last_hip_error() */
};

enum { MX_DTYPE_F32 = 0, MX_DTYPE_BF16 = 1 };
enum { MX_ROUND_RTN = 0, MX_ROUND_SR = 1 };          /* round_D / round_S of Sec. 3.2 */
enum { MX_SCALE_TRUNCFREE = 0, MX_SCALE_FLOOR = 1 }; /* truncation-free scaling of Sec. 3.2 / Eq. 2 */
enum { MX_GEMM_FWD = 0, MX_GEMM_BWD_DX = 1, MX_GEMM_BWD_DW = 2 };

/*
 * Quantizers Q(1), Q(3) of Eqs. 3-4 (and Q(2) on W[C x D]): 1x32 groups along
 * the columns of src[rows x cols].  Sec. 3.1 Eq. 1, Sec. 3.2.
 *   src      device, dtype F32 or BF16, 16-byte aligned, ld % 8 == 0 (BF16) or ld % 4 == 0 (F32)
 *   codes    device out, rows*cols/2 bytes, 4-byte aligned
 *   scales   device out, rows*cols/32 bytes
 *   cols % 32 == 0, ld >= cols; rows*cols < 2^35.
 */
int mx_quantize(const void* src, int dtype, int64_t rows, int64_t cols, int64_t ld,
                uint8_t* codes, uint8_t* scales,
                int round, int scale_mode,
                uint64_t seed, uint32_t tensor_id, uint64_t index_base,
                void* stream);

/*
 * Quantizers Q(2)/Q(4), Q(5), Q(6) of Eqs. 3-5: 32x1 groups (32 consecutive
 * rows of one column of src[rows x cols]), result stored transposed so that it
 * is contiguous along the contraction dimension of the product that consumes
 * it ("Block Format", Sec. 3.3):
 *        codes_t[cols x rows/2], scales_t[cols x rows/32]
 *   pre_quant   0: quantize src itself;
 *               1: quantize dequant(Q_row(src)) -- the "double quantization" of
 *                  Sec. 3.3, Q(6)(Q(1)(X)) and Q(4)(Q(2)(W)).  Q_row is the 1x32
 *                  quantizer with (round_row, tensor_id_row).
 *   codes_row, scales_row   optional (both NULL or both set): also store the
 *               1x32 result Q_row(src), computed in the same pass.
 *   row_codes_in, row_scales_in   optional (both NULL or both set), only with
 *               pre_quant = 1: take Q_row(src) as given (e.g. the output of
 *               mx_ema_weight_quant) instead of computing it; src is then
 *               unused and may be NULL, and codes_row/scales_row must be NULL.
 *   rows % 32 == 0, cols % 32 == 0, ld >= cols; src alignment as mx_quantize;
 *   codes_t, codes_row and row_codes_in 16-byte aligned; rows*cols < 2^35.
 */
int mx_quantize_transposed(const void* src, int dtype, int64_t rows, int64_t cols, int64_t ld,
                uint8_t* codes_t, uint8_t* scales_t,
                int round_t, uint32_t tensor_id_t,
                int pre_quant,
                uint8_t* codes_row, uint8_t* scales_row,
                int round_row, uint32_t tensor_id_row,
                const uint8_t* row_codes_in, const uint8_t* row_scales_in,
                int scale_mode, uint64_t seed, uint64_t index_base,
                void* stream);

/*
 * Several mx_quantize_transposed requests in one launch (Sec. 3.3 runs two of them back to back in
 * the forward pass: the activation and the weight).  One kernel serves the whole batch, so the small
 * tensor costs no launch of its own and its workgroups fill the last, partly empty round of the
 * large one's.  Results are those of the separate calls, byte for byte.
 *   jobs    HOST array of `count` requests, 1 <= count <= MX_TRANSPOSED_BATCH_MAX; every field has the
 *           meaning, layout and alignment of the argument of the same name of mx_quantize_transposed
 *   round_t, round_row, scale_mode   shared by all jobs
 *   seed_dev   NULL, or a DEVICE pointer (8-byte aligned, else MX_ERR_ALIGN) to a 64-bit word that the
 *           kernel reads when it runs and uses in place of `seed`.  A launch recorded into a HIP graph
 *           keeps its arguments, so a host-side seed would repeat the same draws on every replay;
 *           with seed_dev the caller changes the word between replays (by a kernel or a copy on the
 *           same stream) and every replay rounds with fresh numbers.  The word is only read.
 *   col_sums   NULL, or DEVICE out, FP32 [cols]: the column sums of the source, sum over r of src[r][c],
 *           taken from the values the quantizer has loaded anyway (for dY this is the gradient of the
 *           layer's bias, which otherwise costs its own pass over dY).  FP32 sums, every addition
 *           rounded to nearest even, in one fixed order, so that a call repeats bit for bit: rows in
 *           blocks of 256, a block in tiles of 32 rows; in a tile, four consecutive rows left to right,
 *           g_i = ((x[4i] + x[4i+1]) + x[4i+2]) + x[4i+3], then ((g0+g1) + (g2+g3)) + ((g4+g5) + (g6+g7));
 *           the tiles of a block in index order; the blocks as eight contiguous runs of ceil(blocks/8),
 *           each run in index order starting from 0, and the eight runs in index order.  Needs a source
 *           (MX_ERR_MODE with row_codes_in), 4-byte alignment, and
 *   col_sum_workspace   DEVICE scratch of mx_column_sum_workspace_bytes(rows, cols) bytes
 *           (MX_ERR_WORKSPACE if NULL); a second, small kernel on the same stream finishes the sums.
 * All jobs must read the same kind of source: all F32, all BF16 (else MX_ERR_DTYPE), or all from
 * row_codes_in (else MX_ERR_MODE).  Any error of a single job is returned as that call would return
 * it, and nothing is launched.
 */
#define MX_TRANSPOSED_BATCH_MAX 4
typedef struct mx_transposed_job {
    const void* src;
    int dtype;
    int64_t rows, cols, ld;
    uint8_t* codes_t;
    uint8_t* scales_t;
    uint32_t tensor_id_t;
    int pre_quant;
    uint8_t* codes_row;
    uint8_t* scales_row;
    uint32_t tensor_id_row;
    const uint8_t* row_codes_in;
    const uint8_t* row_scales_in;
    uint64_t seed;
    uint64_t index_base;
    const uint64_t* seed_dev;
    float* col_sums;
    float* col_sum_workspace;
} mx_transposed_job;
int mx_quantize_transposed_batch(const mx_transposed_job* jobs, int count,
                int round_t, int round_row, int scale_mode, void* stream);
size_t mx_column_sum_workspace_bytes(int64_t rows, int64_t cols);

/*
 * The three products (Sec. 3.3, Eqs. 3-5), FP32 accumulation on the
 * block-scaled FP4 matrix cores.  X[N x D], W[C x D], Y[N x C].  Every operand
 * is packed along the product's contraction dimension, which must be a
 * multiple of 32 and at most 2^24; the other two dimensions are arbitrary
 * (>= 1, below 2^31, with fewer than 2^30 output tiles of 256 x 128).
 * Operand code pointers must be 16-byte aligned and the contraction dimension
 * a multiple of 32; out dtype F32 or BF16 (round to nearest even), ld >= row
 * length.  workspace: device, 256-byte aligned, at least
 * mx_linear_workspace_bytes(which, N, C, D) bytes (may be NULL when that is 0).
 *
 *   mx_linear_fwd     Y  = Q1(X) . Q2(W)^T        (Eq. 3)  xq[N x D/2] xs[N x D/32], wq[C x D/2] ws[C x D/32]
 *   mx_linear_bwd_dx  dX = Q3(dY) . Q4(...)       (Eq. 4)  dyq[N x C/2] dys[N x C/32], wtq[D x C/2] wts[D x C/32]
 *   mx_linear_bwd_dw  dW = Q5(dY^T) . Q6(...)     (Eq. 5)  dytq[C x N/2] dyts[C x N/32], xtq[D x N/2] xts[D x N/32]
 */
int mx_linear_fwd(const uint8_t* xq, const uint8_t* xs, const uint8_t* wq, const uint8_t* ws,
                  int64_t N, int64_t C, int64_t D,
                  void* y, int y_dtype, int64_t ldy,
                  void* workspace, size_t workspace_bytes, void* stream);
/* mx_linear_fwd with a bias row added in the product's output stage, before the one rounding to
 * y_dtype: Y = Q1(X) . Q2(W)^T + 1 . bias^T (Eq. 3 gives the product; the bias is the linear layer's
 * own, kept outside the quantized operands).  Saves the separate pass over Y that adding it afterwards
 * costs (read + write of N x C elements).
 *   bias   device, FP32, C values, 16-byte aligned (else MX_ERR_ALIGN); NULL is MX_ERR_NULL.
 *   C      must be a multiple of 4 (else MX_ERR_SHAPE).  Everything else as mx_linear_fwd. */
int mx_linear_fwd_bias(const uint8_t* xq, const uint8_t* xs, const uint8_t* wq, const uint8_t* ws,
                  int64_t N, int64_t C, int64_t D, const float* bias,
                  void* y, int y_dtype, int64_t ldy,
                  void* workspace, size_t workspace_bytes, void* stream);
/* The forward product of the first layer of a transformer MLP with the element-wise neighbour and the NEXT
 * layer's forward quantizer in its output stage (Sec. 7.1 quantizes all linear layers of the MLP module; fc1
 * feeds fc2 through GELU only).  One launch gives
 *     P      = Q1(X) . Q2(W)^T + 1 . bias^T                 (Eq. 3 of this layer), stored to y as y_dtype: the
 *              pre-activation, which the backward pass of the activation needs;
 *     aq, as = Q(1) of the next layer (Eq. 3 there: 1x32 groups along the C columns, round_D, scale_mode)
 *              applied to A = GELU(P), GELU(x) = x * Phi(x) with the exact normal distribution function,
 *              evaluated in FP32 on the FP32 value of P (before its rounding to y_dtype).
 * aq [N x C/2], as [N x C/32] are what mx_linear_fwd of the next layer takes as xq, xs; its Q(6) comes from
 * mx_quantize_transposed with row_codes_in = aq, row_scales_in = as (double quantization, Sec. 3.3).  This
 * removes the activation kernel's pass over P and the read of A by the next layer's quantizer.
 * Accuracy: P as mx_linear_fwd_bias; the value that is quantized differs from the exact GELU of the exact
 * product by at most 1.13 |P - P_exact| + 2^-18 |A| + 2^-120 (FP32 erfc, which underflows for |A| near 1e-38),
 * so a code or scale byte may differ from those of the exact A only where A lies within that distance of a
 * rounding threshold or a scale boundary.
 *   bias    device, FP32, C values, 16-byte aligned; required (pass zeros for a layer without bias)
 *   aq, as  device out; aq 16-byte aligned
 *   C % 32 == 0; D % 128 == 0 and D >= 512 and no K split (the sizes the main kernel takes without a K split;
 *   every MLP of the ViT configurations), else MX_ERR_SHAPE.  No workspace.  Everything else as
 *   mx_linear_fwd_bias. */
int mx_linear_fwd_gelu_quant(const uint8_t* xq, const uint8_t* xs, const uint8_t* wq, const uint8_t* ws,
                  int64_t N, int64_t C, int64_t D, const float* bias,
                  void* y, int y_dtype, int64_t ldy,
                  uint8_t* aq, uint8_t* as, int scale_mode, void* stream);
int mx_linear_bwd_dx(const uint8_t* dyq, const uint8_t* dys, const uint8_t* wtq, const uint8_t* wts,
                  int64_t N, int64_t C, int64_t D,
                  void* dx, int dx_dtype, int64_t lddx,
                  void* workspace, size_t workspace_bytes, void* stream);
int mx_linear_bwd_dw(const uint8_t* dytq, const uint8_t* dyts, const uint8_t* xtq, const uint8_t* xts,
                  int64_t N, int64_t C, int64_t D,
                  void* dw, int dw_dtype, int64_t lddw,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * mx_linear_bwd_dw for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving or training loops that own no allocator, harnesses
 * that forbid hipMalloc.  Same product, same kernels and the same result bit for bit as
 * mx_linear_bwd_dw with a workspace; the FP32 partial sums of the K split go to a device array of
 * MX_NOALLOC_MAX_WORKSPACE_BYTES that is part of the library's code object (each GPU the library
 * runs on holds its own copy until the process ends).  The call allocates and frees nothing and
 * calls no allocating routine; its first call on a device looks the array's address up once.
 *   Arguments, layouts, alignment and errors as mx_linear_bwd_dw.  Sizes whose K split needs more
 *   than MX_NOALLOC_MAX_WORKSPACE_BYTES (mx_linear_workspace_bytes(MX_GEMM_BWD_DW, N, C, D)) are
 *   rejected with MX_ERR_WORKSPACE and nothing is launched; every layer of the ViT-T/S/B/L
 *   configurations fits.
 *   All calls on one GPU share that GPU's array: calls that may overlap in time (different streams,
 *   different host threads) race on it and must be serialised by the caller.  The array keeps the
 *   previous call's partial sums; the kernels overwrite what they read, so nothing is cleared.
 */
#define MX_NOALLOC_MAX_WORKSPACE_BYTES (64u << 20)
int mx_linear_bwd_dw_noalloc(const uint8_t* dytq, const uint8_t* dyts, const uint8_t* xtq, const uint8_t* xts,
                  int64_t N, int64_t C, int64_t D,
                  void* dw, int dw_dtype, int64_t lddw, void* stream);

/*
 * Q-EMA (Sec. 5 Eq. 8, Algorithm 1): 1x32 quantizer of the weight w[rows x cols]
 * whose scale comes from w and whose choice between the two E2M1 neighbours of
 * w/S is the one nearer to w_ema/S (q1 iff strictly nearer).  A w/S that is
 * itself an E2M1 value is kept.  The two neighbours are the bracketing pair
 * q1 <= w/S <= q2 of Sec. 3.2; where E2M1's spacing changes, |w/S| in (2, 2.25)
 * or (4, 4.5), this is not the pair of the two nearest values (1.5, 2 resp.
 * 3, 4), and the bracket is the reading taken: the result never lies beyond a
 * representable value from w/S, and w_ema = w gives mx_quantize's RTN result.
 *   w        device, F32 or BF16, row stride ld
 *   w_ema    device, FP32, in/out, same shape and the same row stride ld
 *   update_ema  0: use w_ema as is; 1: w_ema <- beta*w_ema + (1-beta)*w (FP32,
 *               (1-beta)*w rounded, then one fused multiply-add), then quantize;
 *               2: w_ema <- w, then quantize
 *   0 <= beta < 1.  Shapes and alignment as mx_quantize; w_ema 16-byte aligned.
 */
int mx_ema_weight_quant(const void* w, int dtype, float* w_ema, float beta, int update_ema,
                  int64_t rows, int64_t cols, int64_t ld,
                  uint8_t* codes, uint8_t* scales, int scale_mode, void* stream);

/* ---- format variant of the ablations: E3M0 elements ---- */

/*
 * mx_quantize with E3M0 elements, the other 4-bit element format of the paper's format ablation
 * (Table 7 and its paragraph, which name the format and no more).  Reading, built the way Sec. 3.1's
 * E2M1 is: code = sign << 3 | exponent field E, three exponent bits, no mantissa bit, bias 3, no
 * Inf/NaN codes; magnitude 0 for E = 0 and 2^(E-3) for E = 1..7, i.e. 0, 0.25, 0.5, 1, 2, 4, 8, 16;
 * Q_p = -Q_n = 16, E_max = 4.  Everything else is Sec. 3.2 with these constants: truncation-free scale
 * s = ceil(log2(2M / (Q_p - Q_n))) = ceil(log2(M / 16)) (8 < M/S <= 16), Eq. 2's scale s = floor(log2 M) - 4
 * with truncation to +-16 (the group maximum then always lands on +-16), epsilon = 1e-8 for an all-zero
 * group (s = -30 resp. -31), |s| <= 127; round_D / round_S between the two neighbouring E3M0 values with
 * the tie rule, the 16-bit draw and the Philox indexing of mx_quantize.  Packed layout as for E2M1.
 * Only this 1x32 quantizer and the test aid below exist for E3M0: the matrix cores have no such operand
 * type, so no product takes these codes.  Arguments and errors as mx_quantize.
 */
int mx_quantize_e3m0(const void* src, int dtype, int64_t rows, int64_t cols, int64_t ld,
                uint8_t* codes, uint8_t* scales,
                int round, int scale_mode,
                uint64_t seed, uint32_t tensor_id, uint64_t index_base,
                void* stream);
/* out[rows x cols] (FP32, dense) = P * 2^s for E3M0 codes.  Test aid. */
int mx_dequantize_e3m0(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t cols,
                  float* out, void* stream);

/* ---- next step beyond the layer: Q-Ramping's oscillation detection ---- */

/*
 * One step of the trajectory lengths of Sec. 6.1 ("Identifying Oscillating Weights"), per weight
 * element of w[rows x cols]:
 *     dist_W += |w - w_prev|,     dist_Q += |w_Q - w_Q,prev|,     w_Q = P * 2^s,
 * FP32 with one rounding per operation, then w_prev <- w and the previous quantized weight <- the
 * current one.  codes/scales are this step's 1x32 quantization of w (mx_quantize or
 * mx_ema_weight_quant).
 *   w                     device, F32 or BF16, row stride ld (alignment as mx_quantize)
 *   w_prev, dist_w, dist_q   device in/out, FP32, dense [rows x cols], 16-byte aligned
 *   codes_prev, scales_prev  device in/out, packed like codes/scales: the previous step's w_Q
 *   init   1 opens a detection window: the sums are zeroed and nothing is added (the previous
 *          values are not read); 0 accumulates one step.
 */
int mx_oscillation_accumulate(const void* w, int dtype, int64_t rows, int64_t cols, int64_t ld,
                  const uint8_t* codes, const uint8_t* scales,
                  float* w_prev, uint8_t* codes_prev, uint8_t* scales_prev,
                  float* dist_w, float* dist_q, int init, void* stream);

/*
 * Amplification factor of Algorithm 2 (Q-Ramping) per element: with the oscillation ratio
 * R_w = dist_Q / dist_W (Sec. 6.1),  N_w = min(k2 * floor(R_w / k1) + 1, n_max); the per-element
 * learning rate and batch size are N_w times the global ones.  The paper's defaults are k1 = 16,
 * k2 = 5.  dist_W = 0 (not covered by the paper): N_w = 1 if dist_Q = 0 too, else n_max.
 *   dist_w, dist_q   device, FP32, count elements;  factor  device out, int32, count elements
 *   k1 > 0, k2 >= 0, n_max >= 1, else MX_ERR_MODE.
 */
int mx_ramping_factor(const float* dist_w, const float* dist_q, int64_t count,
                  float k1, int k2, int n_max, int32_t* factor, void* stream);

/*
 * One optimizer step of Q-Ramping's customised AdamW (Algorithm 2, "update w according to LR_w and
 * BS_w"; Sec. 6.2) on `count` weight elements.  An element with amplification factor N_w accumulates
 * its gradient over N_w steps (N_w times the batch size) and then takes one AdamW update at N_w
 * times the learning rate.  Per element:
 *     g_acc += grad;  acc_steps += 1;
 *     if acc_steps >= N_w:
 *         g = g_acc / acc_steps;  lr_w = N_w * lr;  u = ++updates;
 *         w = w * (1 - lr_w * weight_decay);
 *         m = beta1 * m + (1 - beta1) * g;   v = beta2 * v + (1 - beta2) * g * g;
 *         w = w - (lr_w / (1 - beta1^u)) * m / (sqrt(v) / sqrt(1 - beta2^u) + eps);
 *         g_acc = 0;  acc_steps = 0;
 * (the paper prints no formula for the update: this is AdamW with decoupled decay, the bias
 * correction counting the element's own updates, so that factor 1 is exactly AdamW).  FP32.
 *   w, m, v      device in/out, FP32, count elements (the master weight and AdamW's two moments)
 *   grad         device, F32 or BF16, count elements (e.g. the dW of mx_linear_bwd_dw)
 *   updates      device in/out, int32: updates each element has made; all zero at the start
 *   factor       device, int32: N_w >= 1 per element (mx_ramping_factor's output), or NULL for 1
 *                everywhere (plain AdamW; g_acc and acc_steps are then not used and may be NULL)
 *   g_acc, acc_steps   device in/out, FP32 / int32: the gradient sum an element holds and the number
 *                of steps in it; all zero at the start
 *   count % 4 == 0; every array 16-byte aligned (grad in BF16: 8).
 *   lr >= 0, 0 < beta1, beta2 < 1, eps >= 0, weight_decay >= 0, else MX_ERR_MODE.
 */
int mx_ramping_adamw_step(float* w, const void* grad, int grad_dtype, int64_t count,
                  float* m, float* v, int32_t* updates,
                  const int32_t* factor, float* g_acc, int32_t* acc_steps,
                  float lr, float beta1, float beta2, float eps, float weight_decay, void* stream);

/* ---- oscillation diagnostics (Sec. 4) ---- */

/*
 * Quantization confidence of Sec. 4.2 for every element of w[rows x cols], on the latent value
 * y = w / S of its 1x32 group (S as mx_quantize computes it for scale_mode):
 *     QuantConf = min_i |y - thrd_i| / MaxDist(y_FP4)   in [0, 1],
 * thresholds = the midpoints of neighbouring E2M1 values; MaxDist = half the width of the rounding
 * cell of y_FP4 (the whole width for the outermost cells [5, 6] and [-6, -5]).  0 on a threshold,
 * 1 at the point of the cell furthest from its thresholds.
 *   w      device, F32 or BF16, row stride ld (alignment as mx_quantize)
 *   conf   device out, FP32, dense [rows x cols], 16-byte aligned; or NULL
 *   hist   device in/out, `bins` 64-bit counters, ADDED to (clear them to open a histogram); or
 *          NULL.  An element with confidence c counts in bin min(bins - 1, floor(c * bins)), the
 *          product in FP32.  1 <= bins <= 1024, else MX_ERR_MODE.
 * conf and hist may not both be NULL.
 */
int mx_quant_confidence(const void* w, int dtype, int64_t rows, int64_t cols, int64_t ld, int scale_mode,
                  float* conf, uint64_t* hist, int bins, void* stream);

/*
 * One term of the rate of change of a tensor (Sec. 4.1),
 *     r(X) = (1/T0) sum_{t=1..T0} ||X^t - X^(t-1)||_F / ||X^(t-1)||_F:
 * with x = X^t and x_prev = X^(t-1), computes the term in FP64 (sums of squares in a fixed order:
 * results repeat bit for bit), then x_prev <- x.
 *   x        device, F32 or BF16, [rows x cols], row stride ld; cols % 8 == 0
 *   x_prev   device in/out, FP32, dense [rows x cols], 16-byte aligned
 *   init     1 opens a window: x_prev <- x, result <- {0, 0, 0}; 0 adds one term
 *   workspace   device scratch of mx_rate_of_change_workspace_bytes() bytes (MX_ERR_WORKSPACE if
 *            smaller), not kept between calls
 *   result   device in/out, 3 doubles: [0] this call's term, [1] the sum of the terms since the
 *            window opened, [2] their number; r(X) = result[1] / result[2].
 * ||x_prev|| = 0 gives a term of 0 if x = x_prev, +infinity otherwise.
 */
size_t mx_rate_of_change_workspace_bytes(void);
int mx_rate_of_change_step(const void* x, int dtype, int64_t rows, int64_t cols, int64_t ld,
                  float* x_prev, int init, void* workspace, size_t workspace_bytes,
                  double* result, void* stream);

/* ---- helpers (not part of the path) ---- */

/* Bytes of workspace the product `which` (MX_GEMM_*) needs for these sizes. */
size_t mx_linear_workspace_bytes(int which, int64_t N, int64_t C, int64_t D);

/* out[rows x cols] (FP32, dense) = P * 2^s.  Test aid. */
int mx_dequantize(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t cols,
                  float* out, void* stream);

/* Plain device-to-device copy kernel of `bytes` bytes (a multiple of 16; 16-byte aligned
 * pointers): a dispatch with known HBM traffic, used to scale profiler byte counters. */
int mx_calibration_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Register-resident loop of the products' matrix instruction (V_MFMA_SCALE_F32_32X32X64_F8F6F4, FP4 x
 * FP4, group scales 2^0): a dispatch with a known number of flops and no memory traffic inside its
 * loop, used to measure the rate the matrix cores sustain on GIVEN operand bytes (the rate depends on
 * the bytes: constant bytes run faster than random or real quantized ones, at the same instruction
 * stream).  A reported calibration figure, never a roofline peak.
 *   operands    device, MX_CALIBRATION_MFMA_OPERAND_BYTES bytes, 16-byte aligned: packed FP4 codes, every
 *               lane of the 8 waves of a workgroup reads 12 x 16 bytes of it once (all workgroups the same)
 *   workgroups  workgroups of 8 waves to launch (one per compute unit fills the chip: two waves per SIMD)
 *   iterations  loop count; each wave issues 16 MFMAs (8 independent accumulator tiles x two 64-K slices) per
 *               iteration: flops = workgroups * 8 * iterations * 16 * 2 * 32 * 32 * 64
 *   sink        device out, FP32, workgroups * 512 values (keeps the accumulators alive; contents unspecified)
 */
#define MX_CALIBRATION_MFMA_OPERAND_BYTES 98304
int mx_calibration_mfma(const uint8_t* operands, int workgroups, int iterations, float* sink, void* stream);

/* Raw hipError_t of the last launch that made a call return MX_ERR_HIP (0 if none). */
int mx_last_hip_error(void);

/* Static version string. */
const char* mx_version(void);

#ifdef __cplusplus
}
#endif
#endif

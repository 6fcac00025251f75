// C ABI of the library (declared in include/mxfp4.h): argument validation on
// the host, then launches.  No allocation, no synchronisation.
#include "../../include/mxfp4.h"
#include "mx_launch.hpp"

#include <atomic>

namespace {

std::atomic<int> g_last_hip_error{0};

int hip_status(hipError_t e)
{
    if (e == hipSuccess) return MX_OK;
    g_last_hip_error.store((int)e);
    return MX_ERR_HIP;
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

constexpr int64_t MAX_ELEMS = (int64_t)0xFFFF0000LL * 8;   // 8-element chunks are indexed with 32 bits

// shared checks of the 1x32 quantizer entry points
int check_rows_call(const void* src, int dtype, int64_t rows, int64_t cols, int64_t ld,
                    const uint8_t* codes, const uint8_t* scales, int scale_mode)
{
    if (!src || !codes || !scales) return MX_ERR_NULL;
    if (dtype != MX_DTYPE_F32 && dtype != MX_DTYPE_BF16) return MX_ERR_DTYPE;
    if (scale_mode != MX_SCALE_TRUNCFREE && scale_mode != MX_SCALE_FLOOR) return MX_ERR_MODE;
    if (rows <= 0 || cols <= 0 || (cols % 32) != 0 || ld < cols) return MX_ERR_SHAPE;
    if (rows > MAX_ELEMS / cols) return MX_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(codes, 4)) return MX_ERR_ALIGN;
    if (ld % (dtype == MX_DTYPE_BF16 ? 8 : 4) != 0) return MX_ERR_ALIGN;
    return MX_OK;
}

int check_gemm_call(const uint8_t* aq, const uint8_t* as, const uint8_t* bq, const uint8_t* bs,
                    int64_t m, int64_t n, int64_t k, const void* out, int out_dtype, int64_t ldo)
{
    if (!aq || !as || !bq || !bs || !out) return MX_ERR_NULL;
    if (out_dtype != MX_DTYPE_F32 && out_dtype != MX_DTYPE_BF16) return MX_ERR_DTYPE;
    if (m <= 0 || n <= 0 || k <= 0 || (k % 32) != 0 || ldo < n) return MX_ERR_SHAPE;
    // the kernels index with 32 bits: tile counts, and byte offsets of up to 256 packed rows
    if (m > 0x7FFFFFFFLL || n > 0x7FFFFFFFLL || k > (1LL << 24)) return MX_ERR_SHAPE;
    if (((m + 255) / 256) * ((n + 127) / 128) > 0x3FFFFFFFLL) return MX_ERR_SHAPE;
    if (!aligned(aq, 16) || !aligned(bq, 16) || !aligned(as, 4) || !aligned(bs, 4)) return MX_ERR_ALIGN;
    if (!aligned(out, out_dtype == MX_DTYPE_BF16 ? 8 : 16)) return MX_ERR_ALIGN;
    return MX_OK;
}

int run_gemm(const uint8_t* aq, const uint8_t* as, const uint8_t* bq, const uint8_t* bs,
             int64_t m, int64_t n, int64_t k, void* out, int out_dtype, int64_t ldo,
             void* workspace, size_t workspace_bytes, void* stream, const float* bias = nullptr)
{
    int rc = check_gemm_call(aq, as, bq, bs, m, n, k, out, out_dtype, ldo);
    if (rc != MX_OK) return rc;
    if (bias) {
        if ((n % 4) != 0) return MX_ERR_SHAPE;               // the kernels read the bias four columns at a time
        if (!aligned(bias, 16)) return MX_ERR_ALIGN;
    }
    int split = mxl::gemm_split_k(m, n, k);
    size_t need = split > 1 ? (size_t)split * (size_t)m * (size_t)n * sizeof(float) : 0;
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return MX_ERR_WORKSPACE;
        if (!aligned(workspace, 256)) return MX_ERR_ALIGN;
    }
    mxl::GemmParams p{};
    p.a_codes = aq; p.a_scales = as; p.b_codes = bq; p.b_scales = bs;
    p.m = m; p.n = n; p.k = k;
    p.c = out; p.c_bf16 = out_dtype == MX_DTYPE_BF16; p.ldc = ldo;
    p.workspace = workspace; p.split_k = split; p.bias = bias;
    return hip_status(mxl::launch_gemm(p, static_cast<hipStream_t>(stream)));
}

// ---- scratch memory of mx_linear_bwd_dw_noalloc: a device array that is part of the code object,
//      so it exists on every GPU the library is loaded on, from load to process end ----
static __device__ __align__(256) unsigned char scratch[MX_NOALLOC_MAX_WORKSPACE_BYTES];

constexpr int MAX_DEVICES = 64;
std::atomic<void*> g_scratch_ptr[MAX_DEVICES];

// Device address of `scratch` on the current device.  In host code the array's name is only a handle
// for the runtime: the address a kernel may use comes from hipGetSymbolAddress, once per device (each
// GPU holds its own copy at its own address).  Two threads racing here store the same value.
int scratch_of_current_device(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_status(e);
    if (dev < 0 || dev >= MAX_DEVICES) return hip_status(hipErrorInvalidDevice);
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_status(e);
        if (p == nullptr) return hip_status(hipErrorInvalidSymbol);
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return MX_OK;
}

}  // namespace

extern "C" {

int mx_quantize(const void* src, int dtype, int64_t rows, int64_t cols, int64_t ld,
                uint8_t* codes, uint8_t* scales, int round, int scale_mode,
                uint64_t seed, uint32_t tensor_id, uint64_t index_base, void* stream)
{
    int rc = check_rows_call(src, dtype, rows, cols, ld, codes, scales, scale_mode);
    if (rc != MX_OK) return rc;
    if (round != MX_ROUND_RTN && round != MX_ROUND_SR) return MX_ERR_MODE;
    if (round == MX_ROUND_SR && (index_base & 7u) != 0) return MX_ERR_ALIGN;
    mxl::QuantRowsParams p{};
    p.src = src; p.bf16 = dtype == MX_DTYPE_BF16; p.rows = rows; p.cols = cols; p.ld = ld;
    p.codes = codes; p.scales = scales; p.sr = round == MX_ROUND_SR;
    p.floor_mode = scale_mode == MX_SCALE_FLOOR;
    p.seed = seed; p.tensor_id = tensor_id; p.index_base = index_base;
    return hip_status(mxl::launch_quantize_rows(p, static_cast<hipStream_t>(stream)));
}

int mx_quantize_e3m0(const void* src, int dtype, int64_t rows, int64_t cols, int64_t ld,
                uint8_t* codes, uint8_t* scales, int round, int scale_mode,
                uint64_t seed, uint32_t tensor_id, uint64_t index_base, void* stream)
{
    int rc = check_rows_call(src, dtype, rows, cols, ld, codes, scales, scale_mode);
    if (rc != MX_OK) return rc;
    if (round != MX_ROUND_RTN && round != MX_ROUND_SR) return MX_ERR_MODE;
    if (round == MX_ROUND_SR && (index_base & 7u) != 0) return MX_ERR_ALIGN;
    mxl::QuantRowsParams p{};
    p.src = src; p.bf16 = dtype == MX_DTYPE_BF16; p.rows = rows; p.cols = cols; p.ld = ld;
    p.codes = codes; p.scales = scales; p.sr = round == MX_ROUND_SR;
    p.floor_mode = scale_mode == MX_SCALE_FLOOR;
    p.seed = seed; p.tensor_id = tensor_id; p.index_base = index_base;
    return hip_status(mxl::launch_quantize_rows_e3m0(p, static_cast<hipStream_t>(stream)));
}

int mx_dequantize_e3m0(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t cols,
                  float* out, void* stream)
{
    if (!codes || !scales || !out) return MX_ERR_NULL;
    if (rows <= 0 || cols <= 0 || (cols % 32) != 0) return MX_ERR_SHAPE;
    if (rows > MAX_ELEMS / cols) return MX_ERR_SHAPE;
    return hip_status(mxl::launch_dequantize_e3m0(codes, scales, rows, cols, out, static_cast<hipStream_t>(stream)));
}

// Checks one transposed-quantizer request and fills the launcher's parameters.
static int make_transposed_job(const void* src, int dtype, int64_t rows, int64_t cols, int64_t ld,
                uint8_t* codes_t, uint8_t* scales_t, int round_t, uint32_t tensor_id_t,
                int pre_quant, uint8_t* codes_row, uint8_t* scales_row,
                int round_row, uint32_t tensor_id_row,
                const uint8_t* row_codes_in, const uint8_t* row_scales_in,
                int scale_mode, uint64_t seed, uint64_t index_base, mxl::QuantTileParams& p)
{
    if (!codes_t || !scales_t) return MX_ERR_NULL;
    if ((codes_row == nullptr) != (scales_row == nullptr)) return MX_ERR_NULL;
    if ((row_codes_in == nullptr) != (row_scales_in == nullptr)) return MX_ERR_NULL;
    const bool given = row_codes_in != nullptr;
    if (!given && !src) return MX_ERR_NULL;
    if (pre_quant != 0 && pre_quant != 1) return MX_ERR_MODE;
    if (given && (pre_quant != 1 || codes_row != nullptr)) return MX_ERR_MODE;
    if (round_t != MX_ROUND_RTN && round_t != MX_ROUND_SR) return MX_ERR_MODE;
    if (round_row != MX_ROUND_RTN && round_row != MX_ROUND_SR) return MX_ERR_MODE;
    if (scale_mode != MX_SCALE_TRUNCFREE && scale_mode != MX_SCALE_FLOOR) return MX_ERR_MODE;
    if (!given && dtype != MX_DTYPE_F32 && dtype != MX_DTYPE_BF16) return MX_ERR_DTYPE;
    if (rows <= 0 || cols <= 0 || (rows % 32) != 0 || (cols % 32) != 0) return MX_ERR_SHAPE;
    if (!given && ld < cols) return MX_ERR_SHAPE;
    if (rows > MAX_ELEMS / cols || rows > 65535LL * 128) return MX_ERR_SHAPE;
    if (!aligned(codes_t, 16)) return MX_ERR_ALIGN;
    if (codes_row && !aligned(codes_row, 16)) return MX_ERR_ALIGN;
    if (given && !aligned(row_codes_in, 16)) return MX_ERR_ALIGN;
    if (!given) {
        if (!aligned(src, 16)) return MX_ERR_ALIGN;
        if (ld % (dtype == MX_DTYPE_BF16 ? 8 : 4) != 0) return MX_ERR_ALIGN;
    }
    const bool any_sr = round_t == MX_ROUND_SR || (!given && round_row == MX_ROUND_SR && (pre_quant || codes_row));
    if (any_sr && (index_base & 7u) != 0) return MX_ERR_ALIGN;
    p = mxl::QuantTileParams{};
    p.src = src; p.bf16 = !given && dtype == MX_DTYPE_BF16; p.rows = rows; p.cols = cols; p.ld = ld;
    p.codes_t = codes_t; p.scales_t = scales_t; p.sr_t = round_t == MX_ROUND_SR; p.tensor_id_t = tensor_id_t;
    p.pre_quant = pre_quant == 1; p.codes_row = codes_row; p.scales_row = scales_row;
    p.sr_row = round_row == MX_ROUND_SR; p.tensor_id_row = tensor_id_row;
    p.row_codes_in = row_codes_in; p.row_scales_in = row_scales_in;
    p.floor_mode = scale_mode == MX_SCALE_FLOOR; p.seed = seed; p.index_base = index_base;
    return MX_OK;
}

int mx_quantize_transposed(const void* src, int dtype, int64_t rows, int64_t cols, int64_t ld,
                uint8_t* codes_t, uint8_t* scales_t, int round_t, uint32_t tensor_id_t,
                int pre_quant, uint8_t* codes_row, uint8_t* scales_row,
                int round_row, uint32_t tensor_id_row,
                const uint8_t* row_codes_in, const uint8_t* row_scales_in,
                int scale_mode, uint64_t seed, uint64_t index_base, void* stream)
{
    mxl::QuantTileParams p;
    int rc = make_transposed_job(src, dtype, rows, cols, ld, codes_t, scales_t, round_t, tensor_id_t, pre_quant,
                                 codes_row, scales_row, round_row, tensor_id_row, row_codes_in, row_scales_in,
                                 scale_mode, seed, index_base, p);
    if (rc != MX_OK) return rc;
    return hip_status(mxl::launch_quantize_tile(p, static_cast<hipStream_t>(stream)));
}

int mx_quantize_transposed_batch(const mx_transposed_job* jobs, int count,
                int round_t, int round_row, int scale_mode, void* stream)
{
    if (!jobs) return MX_ERR_NULL;
    if (count < 1 || count > MX_TRANSPOSED_BATCH_MAX) return MX_ERR_SHAPE;
    mxl::QuantTileParams p[MX_TRANSPOSED_BATCH_MAX];
    for (int j = 0; j < count; ++j) {
        const mx_transposed_job& q = jobs[j];
        int rc = make_transposed_job(q.src, q.dtype, q.rows, q.cols, q.ld, q.codes_t, q.scales_t, round_t, q.tensor_id_t,
                                     q.pre_quant, q.codes_row, q.scales_row, round_row, q.tensor_id_row,
                                     q.row_codes_in, q.row_scales_in, scale_mode, q.seed, q.index_base, p[j]);
        if (rc != MX_OK) return rc;
        if (q.seed_dev && !aligned(q.seed_dev, 8)) return MX_ERR_ALIGN;
        p[j].seed_dev = q.seed_dev;
        if (q.col_sums) {
            if (!q.src) return MX_ERR_MODE;                           // sums are those of a source tensor
            if (!q.col_sum_workspace) return MX_ERR_WORKSPACE;
            if (!aligned(q.col_sums, 4) || !aligned(q.col_sum_workspace, 4)) return MX_ERR_ALIGN;
            p[j].col_sums = q.col_sums; p[j].col_sum_workspace = q.col_sum_workspace;
        }
        // one kernel serves the launch: the jobs must read the same kind of source
        if ((p[j].row_codes_in != nullptr) != (p[0].row_codes_in != nullptr)) return MX_ERR_MODE;
        if (p[j].bf16 != p[0].bf16) return MX_ERR_DTYPE;
    }
    return hip_status(mxl::launch_quantize_tile_batch(p, count, static_cast<hipStream_t>(stream)));
}

size_t mx_column_sum_workspace_bytes(int64_t rows, int64_t cols)
{
    if (rows <= 0 || cols <= 0) return 0;
    return mxl::column_sum_workspace_bytes(rows, cols);
}

int mx_linear_fwd(const uint8_t* xq, const uint8_t* xs, const uint8_t* wq, const uint8_t* ws,
                  int64_t N, int64_t C, int64_t D, void* y, int y_dtype, int64_t ldy,
                  void* workspace, size_t workspace_bytes, void* stream)
{
    if (N <= 0 || C <= 0 || D <= 0) return (!xq || !xs || !wq || !ws || !y) ? MX_ERR_NULL : MX_ERR_SHAPE;
    return run_gemm(xq, xs, wq, ws, N, C, D, y, y_dtype, ldy, workspace, workspace_bytes, stream);
}

int mx_linear_fwd_bias(const uint8_t* xq, const uint8_t* xs, const uint8_t* wq, const uint8_t* ws,
                  int64_t N, int64_t C, int64_t D, const float* bias, void* y, int y_dtype, int64_t ldy,
                  void* workspace, size_t workspace_bytes, void* stream)
{
    if (!bias) return MX_ERR_NULL;
    if (N <= 0 || C <= 0 || D <= 0) return (!xq || !xs || !wq || !ws || !y) ? MX_ERR_NULL : MX_ERR_SHAPE;
    return run_gemm(xq, xs, wq, ws, N, C, D, y, y_dtype, ldy, workspace, workspace_bytes, stream, bias);
}

int mx_linear_fwd_gelu_quant(const uint8_t* xq, const uint8_t* xs, const uint8_t* wq, const uint8_t* ws,
                  int64_t N, int64_t C, int64_t D, const float* bias, void* y, int y_dtype, int64_t ldy,
                  uint8_t* aq, uint8_t* as, int scale_mode, void* stream)
{
    if (!bias || !aq || !as) return MX_ERR_NULL;
    if (N <= 0 || C <= 0 || D <= 0) return (!xq || !xs || !wq || !ws || !y) ? MX_ERR_NULL : MX_ERR_SHAPE;
    int rc = check_gemm_call(xq, xs, wq, ws, N, C, D, y, y_dtype, ldy);
    if (rc != MX_OK) return rc;
    if (scale_mode != MX_SCALE_TRUNCFREE && scale_mode != MX_SCALE_FLOOR) return MX_ERR_MODE;
    if ((C % 32) != 0 || !mxl::gemm_takes_fused_quantizer(N, C, D)) return MX_ERR_SHAPE;
    if (!aligned(bias, 16) || !aligned(aq, 16)) return MX_ERR_ALIGN;
    mxl::GemmParams p{};
    p.a_codes = xq; p.a_scales = xs; p.b_codes = wq; p.b_scales = ws;
    p.m = N; p.n = C; p.k = D;
    p.c = y; p.c_bf16 = y_dtype == MX_DTYPE_BF16; p.ldc = ldy;
    p.workspace = nullptr; p.split_k = 1; p.bias = bias;
    p.q_codes = aq; p.q_scales = as; p.q_floor = scale_mode == MX_SCALE_FLOOR;
    return hip_status(mxl::launch_gemm(p, static_cast<hipStream_t>(stream)));
}

int mx_linear_bwd_dx(const uint8_t* dyq, const uint8_t* dys, const uint8_t* wtq, const uint8_t* wts,
                  int64_t N, int64_t C, int64_t D, void* dx, int dx_dtype, int64_t lddx,
                  void* workspace, size_t workspace_bytes, void* stream)
{
    if (N <= 0 || C <= 0 || D <= 0) return (!dyq || !dys || !wtq || !wts || !dx) ? MX_ERR_NULL : MX_ERR_SHAPE;
    return run_gemm(dyq, dys, wtq, wts, N, D, C, dx, dx_dtype, lddx, workspace, workspace_bytes, stream);
}

int mx_linear_bwd_dw(const uint8_t* dytq, const uint8_t* dyts, const uint8_t* xtq, const uint8_t* xts,
                  int64_t N, int64_t C, int64_t D, void* dw, int dw_dtype, int64_t lddw,
                  void* workspace, size_t workspace_bytes, void* stream)
{
    if (N <= 0 || C <= 0 || D <= 0) return (!dytq || !dyts || !xtq || !xts || !dw) ? MX_ERR_NULL : MX_ERR_SHAPE;
    return run_gemm(dytq, dyts, xtq, xts, C, D, N, dw, dw_dtype, lddw, workspace, workspace_bytes, stream);
}

int mx_linear_bwd_dw_noalloc(const uint8_t* dytq, const uint8_t* dyts, const uint8_t* xtq, const uint8_t* xts,
                  int64_t N, int64_t C, int64_t D, void* dw, int dw_dtype, int64_t lddw, void* stream)
{
    if (N <= 0 || C <= 0 || D <= 0) return (!dytq || !dyts || !xtq || !xts || !dw) ? MX_ERR_NULL : MX_ERR_SHAPE;
    // every argument check of the product first: an invalid call returns before the scratch is looked up
    int rc = check_gemm_call(dytq, dyts, xtq, xts, C, D, N, dw, dw_dtype, lddw);
    if (rc != MX_OK) return rc;
    const int split = mxl::gemm_split_k(C, D, N);
    const size_t need = split > 1 ? (size_t)split * (size_t)C * (size_t)D * sizeof(float) : 0;
    if (need > (size_t)MX_NOALLOC_MAX_WORKSPACE_BYTES) return MX_ERR_WORKSPACE;
    void* ws = nullptr;
    if (need > 0) {
        rc = scratch_of_current_device(&ws);
        if (rc != MX_OK) return rc;
    }
    // The K-split partials are written in full before the reduction reads them: nothing has to start at zero.
    return run_gemm(dytq, dyts, xtq, xts, C, D, N, dw, dw_dtype, lddw, ws, need, stream);
}

int mx_ema_weight_quant(const void* w, int dtype, float* w_ema, float beta, int update_ema,
                  int64_t rows, int64_t cols, int64_t ld,
                  uint8_t* codes, uint8_t* scales, int scale_mode, void* stream)
{
    int rc = check_rows_call(w, dtype, rows, cols, ld, codes, scales, scale_mode);
    if (rc != MX_OK) return rc;
    if (!w_ema) return MX_ERR_NULL;
    if (update_ema < 0 || update_ema > 2) return MX_ERR_MODE;
    if (!(beta >= 0.0f && beta < 1.0f)) return MX_ERR_MODE;
    if (!aligned(w_ema, 16) || (ld % 4) != 0) return MX_ERR_ALIGN;
    mxl::QuantRowsParams p{};
    p.src = w; p.bf16 = dtype == MX_DTYPE_BF16; p.rows = rows; p.cols = cols; p.ld = ld;
    p.codes = codes; p.scales = scales; p.sr = false; p.floor_mode = scale_mode == MX_SCALE_FLOOR;
    return hip_status(mxl::launch_ema_quantize(p, w_ema, beta, update_ema, static_cast<hipStream_t>(stream)));
}

size_t mx_linear_workspace_bytes(int which, int64_t N, int64_t C, int64_t D)
{
    if (N <= 0 || C <= 0 || D <= 0) return 0;
    int64_t m, n, k;
    switch (which) {
        case MX_GEMM_FWD:    m = N; n = C; k = D; break;
        case MX_GEMM_BWD_DX: m = N; n = D; k = C; break;
        case MX_GEMM_BWD_DW: m = C; n = D; k = N; break;
        default: return 0;
    }
    int split = mxl::gemm_split_k(m, n, k);
    return split > 1 ? (size_t)split * (size_t)m * (size_t)n * sizeof(float) : 0;
}

int mx_oscillation_accumulate(const void* w, int dtype, int64_t rows, int64_t cols, int64_t ld,
                  const uint8_t* codes, const uint8_t* scales,
                  float* w_prev, uint8_t* codes_prev, uint8_t* scales_prev,
                  float* dist_w, float* dist_q, int init, void* stream)
{
    if (!w_prev || !codes_prev || !scales_prev || !dist_w || !dist_q) return MX_ERR_NULL;
    int rc = check_rows_call(w, dtype, rows, cols, ld, codes, scales, MX_SCALE_TRUNCFREE);
    if (rc != MX_OK) return rc;
    if (init != 0 && init != 1) return MX_ERR_MODE;
    if (!aligned(w_prev, 16) || !aligned(dist_w, 16) || !aligned(dist_q, 16) || !aligned(codes_prev, 4)) return MX_ERR_ALIGN;
    mxl::OscillationParams p{};
    p.w = w; p.bf16 = dtype == MX_DTYPE_BF16; p.rows = rows; p.cols = cols; p.ld = ld;
    p.codes = codes; p.scales = scales; p.w_prev = w_prev; p.codes_prev = codes_prev; p.scales_prev = scales_prev;
    p.dist_w = dist_w; p.dist_q = dist_q; p.init = init;
    return hip_status(mxl::launch_oscillation(p, static_cast<hipStream_t>(stream)));
}

int mx_ramping_factor(const float* dist_w, const float* dist_q, int64_t count,
                  float k1, int k2, int n_max, int32_t* factor, void* stream)
{
    if (!dist_w || !dist_q || !factor) return MX_ERR_NULL;
    if (count <= 0 || count > ((int64_t)1 << 40)) return MX_ERR_SHAPE;
    if (!(k1 > 0.0f) || k2 < 0 || n_max < 1) return MX_ERR_MODE;
    return hip_status(mxl::launch_ramping_factor(dist_w, dist_q, count, k1, k2, n_max, factor, static_cast<hipStream_t>(stream)));
}

int mx_ramping_adamw_step(float* w, const void* grad, int grad_dtype, int64_t count,
                  float* m, float* v, int32_t* updates,
                  const int32_t* factor, float* g_acc, int32_t* acc_steps,
                  float lr, float beta1, float beta2, float eps, float weight_decay, void* stream)
{
    if (!w || !grad || !m || !v || !updates) return MX_ERR_NULL;
    if (factor && (!g_acc || !acc_steps)) return MX_ERR_NULL;
    if (grad_dtype != MX_DTYPE_F32 && grad_dtype != MX_DTYPE_BF16) return MX_ERR_DTYPE;
    if (count <= 0 || (count % 4) != 0 || count > ((int64_t)1 << 40)) return MX_ERR_SHAPE;
    // betas in (0, 1) so that 1 - beta^u > 0 for every u >= 1; written so that NaN fails
    if (!(lr >= 0.0f) || !(beta1 > 0.0f && beta1 < 1.0f) || !(beta2 > 0.0f && beta2 < 1.0f) ||
        !(eps >= 0.0f) || !(weight_decay >= 0.0f)) return MX_ERR_MODE;
    if (!aligned(w, 16) || !aligned(m, 16) || !aligned(v, 16) || !aligned(updates, 16) ||
        !aligned(grad, grad_dtype == MX_DTYPE_BF16 ? 8 : 16)) return MX_ERR_ALIGN;
    if (factor && (!aligned(factor, 16) || !aligned(g_acc, 16) || !aligned(acc_steps, 16))) return MX_ERR_ALIGN;
    mxl::RampingAdamwParams p{};
    p.w = w; p.grad = grad; p.grad_bf16 = grad_dtype == MX_DTYPE_BF16; p.count = count; p.m = m; p.v = v;
    p.updates = updates; p.factor = factor; p.g_acc = factor ? g_acc : nullptr; p.acc_steps = factor ? acc_steps : nullptr;
    p.lr = lr; p.beta1 = beta1; p.beta2 = beta2; p.eps = eps; p.weight_decay = weight_decay;
    return hip_status(mxl::launch_ramping_adamw(p, static_cast<hipStream_t>(stream)));
}

int mx_quant_confidence(const void* w, int dtype, int64_t rows, int64_t cols, int64_t ld, int scale_mode,
                  float* conf, uint64_t* hist, int bins, void* stream)
{
    if (!w || (!conf && !hist)) return MX_ERR_NULL;
    if (dtype != MX_DTYPE_F32 && dtype != MX_DTYPE_BF16) return MX_ERR_DTYPE;
    if (scale_mode != MX_SCALE_TRUNCFREE && scale_mode != MX_SCALE_FLOOR) return MX_ERR_MODE;
    if (rows <= 0 || cols <= 0 || (cols % 32) != 0 || ld < cols) return MX_ERR_SHAPE;
    if (rows > MAX_ELEMS / cols) return MX_ERR_SHAPE;
    if (hist && (bins < 1 || bins > mxl::CONFIDENCE_MAX_BINS)) return MX_ERR_MODE;
    if (!aligned(w, 16) || (conf && !aligned(conf, 16)) || (hist && !aligned(hist, 8))) return MX_ERR_ALIGN;
    if (ld % (dtype == MX_DTYPE_BF16 ? 8 : 4) != 0) return MX_ERR_ALIGN;
    mxl::ConfidenceParams p{};
    p.w = w; p.bf16 = dtype == MX_DTYPE_BF16; p.rows = rows; p.cols = cols; p.ld = ld;
    p.floor_mode = scale_mode == MX_SCALE_FLOOR; p.conf = conf; p.hist = hist; p.bins = bins;
    return hip_status(mxl::launch_confidence(p, static_cast<hipStream_t>(stream)));
}

size_t mx_rate_of_change_workspace_bytes(void) { return mxl::rate_workspace_bytes(); }

int mx_rate_of_change_step(const void* x, int dtype, int64_t rows, int64_t cols, int64_t ld,
                  float* x_prev, int init, void* workspace, size_t workspace_bytes,
                  double* result, void* stream)
{
    if (!x || !x_prev || !result) return MX_ERR_NULL;
    if (dtype != MX_DTYPE_F32 && dtype != MX_DTYPE_BF16) return MX_ERR_DTYPE;
    if (init != 0 && init != 1) return MX_ERR_MODE;
    if (rows <= 0 || cols <= 0 || (cols % 8) != 0 || ld < cols) return MX_ERR_SHAPE;
    if (rows > MAX_ELEMS / cols) return MX_ERR_SHAPE;
    if (!workspace || workspace_bytes < mxl::rate_workspace_bytes()) return MX_ERR_WORKSPACE;
    if (!aligned(x, 16) || !aligned(x_prev, 16) || !aligned(workspace, 8) || !aligned(result, 8)) return MX_ERR_ALIGN;
    if (ld % (dtype == MX_DTYPE_BF16 ? 8 : 4) != 0) return MX_ERR_ALIGN;
    mxl::RateParams p{};
    p.x = x; p.bf16 = dtype == MX_DTYPE_BF16; p.rows = rows; p.cols = cols; p.ld = ld;
    p.x_prev = x_prev; p.init = init; p.partial = static_cast<double*>(workspace); p.result = result;
    return hip_status(mxl::launch_rate_of_change(p, static_cast<hipStream_t>(stream)));
}

int mx_dequantize(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t cols,
                  float* out, void* stream)
{
    if (!codes || !scales || !out) return MX_ERR_NULL;
    if (rows <= 0 || cols <= 0 || (cols % 32) != 0) return MX_ERR_SHAPE;
    if (rows > MAX_ELEMS / cols) return MX_ERR_SHAPE;
    return hip_status(mxl::launch_dequantize(codes, scales, rows, cols, out, static_cast<hipStream_t>(stream)));
}

int mx_calibration_copy(void* dst, const void* src, size_t bytes, void* stream)
{
    if (!dst || !src) return MX_ERR_NULL;
    if (bytes == 0 || (bytes & 15u) != 0) return MX_ERR_SHAPE;
    if (!aligned(dst, 16) || !aligned(src, 16)) return MX_ERR_ALIGN;
    return hip_status(mxl::launch_calibration_copy(dst, src, bytes, static_cast<hipStream_t>(stream)));
}

int mx_calibration_mfma(const uint8_t* operands, int workgroups, int iterations, float* sink, void* stream)
{
    if (!operands || !sink) return MX_ERR_NULL;
    if (workgroups < 1 || workgroups > 65536 || iterations < 1 || iterations > (1 << 24)) return MX_ERR_SHAPE;
    if (!aligned(operands, 16) || !aligned(sink, 4)) return MX_ERR_ALIGN;
    return hip_status(mxl::launch_calibration_mfma(operands, workgroups, iterations, sink, static_cast<hipStream_t>(stream)));
}

int mx_last_hip_error(void) { return g_last_hip_error.load(); }

const char* mx_version(void) { return "mxfp4-gfx950 0.1"; }

}  // extern "C"

// Host-side launch interface between the C ABI (mx_api.hip) and the kernels.
// All arguments have been validated by the caller.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mxl {

struct QuantRowsParams {
    const void* src;
    bool bf16;
    int64_t rows, cols, ld;
    uint8_t* codes;
    uint8_t* scales;
    bool sr;
    bool floor_mode;
    uint64_t seed;
    uint32_t tensor_id;
    uint64_t index_base;
};

struct QuantTileParams {
    const void* src;
    bool bf16;
    int64_t rows, cols, ld;
    uint8_t* codes_t;
    uint8_t* scales_t;
    bool sr_t;
    uint32_t tensor_id_t;
    bool pre_quant;
    uint8_t* codes_row;
    uint8_t* scales_row;
    bool sr_row;
    uint32_t tensor_id_row;
    const uint8_t* row_codes_in;
    const uint8_t* row_scales_in;
    bool floor_mode;
    uint64_t seed;
    uint64_t index_base;
    const uint64_t* seed_dev = nullptr;   // device word that replaces `seed` when set
    float* col_sums = nullptr;            // [cols] column sums of the source (needs a source), with
    float* col_sum_workspace = nullptr;   // column_sum_workspace_bytes(rows, cols) of scratch
};

// C[m x n] = A[m x k] . B[n x k]^T, operands packed MXFP4 along k.
struct GemmParams {
    const uint8_t* a_codes;
    const uint8_t* a_scales;
    const uint8_t* b_codes;
    const uint8_t* b_scales;
    int64_t m, n, k;
    void* c;
    bool c_bf16;
    int64_t ldc;
    void* workspace;
    int split_k;     // >= 1; > 1 needs workspace of split_k * m * n floats
    const float* bias = nullptr;   // n values added to every output row (needs n % 4 == 0), or null
    // fused GELU + 1x32 round_D quantizer of the output (needs bias, k % 128 == 0, k >= 512, no K split,
    // n % 32 == 0): codes [m x n/2], scale bytes [m x n/32]; gemm_takes_fused_quantizer() tells
    uint8_t* q_codes = nullptr;
    uint8_t* q_scales = nullptr;
    bool q_floor = false;
};
// Whether launch_gemm runs these sizes on the kernel that carries the fused output quantizer.
bool gemm_takes_fused_quantizer(int64_t m, int64_t n, int64_t k);

hipError_t launch_quantize_rows(const QuantRowsParams& p, hipStream_t st);
hipError_t launch_quantize_rows_e3m0(const QuantRowsParams& p, hipStream_t st);      // E3M0 elements (Table 7)
hipError_t launch_dequantize_e3m0(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t cols,
                                  float* out, hipStream_t st);
hipError_t launch_ema_quantize(const QuantRowsParams& p, float* ema, float beta, int update_ema, hipStream_t st);
hipError_t launch_quantize_tile(const QuantTileParams& p, hipStream_t st);
size_t column_sum_workspace_bytes(int64_t rows, int64_t cols);
// Up to 4 tensors in one launch; they must share source kind, roundings and scale rule.
hipError_t launch_quantize_tile_batch(const QuantTileParams* jobs, int count, hipStream_t st);
hipError_t launch_dequantize(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t cols,
                             float* out, hipStream_t st);

struct OscillationParams {
    const void* w;
    bool bf16;
    int64_t rows, cols, ld;
    const uint8_t* codes;
    const uint8_t* scales;
    float* w_prev;
    uint8_t* codes_prev;
    uint8_t* scales_prev;
    float* dist_w;
    float* dist_q;
    int init;
};
hipError_t launch_oscillation(const OscillationParams& p, hipStream_t st);
hipError_t launch_ramping_factor(const float* dist_w, const float* dist_q, int64_t count, float k1, int k2,
                                 int n_max, int32_t* factor, hipStream_t st);

struct ConfidenceParams {
    const void* w;
    bool bf16;
    int64_t rows, cols, ld;
    int floor_mode;
    float* conf;            // may be null
    uint64_t* hist;         // may be null
    int bins;
};
constexpr int CONFIDENCE_MAX_BINS = 1024;
hipError_t launch_confidence(const ConfidenceParams& p, hipStream_t st);

struct RateParams {
    const void* x;
    bool bf16;
    int64_t rows, cols, ld;
    float* x_prev;
    int init;
    double* partial;        // rate_workspace_bytes() of scratch
    double* result;         // 3 doubles
};
size_t rate_workspace_bytes();
hipError_t launch_rate_of_change(const RateParams& p, hipStream_t st);

struct RampingAdamwParams {
    float* w;
    const void* grad;
    bool grad_bf16;
    int64_t count;          // multiple of 4
    float* m;
    float* v;
    float* g_acc;           // null iff factor is null
    const int32_t* factor;  // null: plain AdamW
    int32_t* acc_steps;     // null iff factor is null
    int32_t* updates;
    float lr, beta1, beta2, eps, weight_decay;
};
hipError_t launch_ramping_adamw(const RampingAdamwParams& p, hipStream_t st);

hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t st);

// Register-resident MFMA loop (calibration of the matrix pipe's sustained rate on given operand bytes).
size_t calibration_mfma_operand_bytes();
hipError_t launch_calibration_mfma(const uint8_t* operands, int workgroups, int iterations, float* sink, hipStream_t st);

// Number of K-splits the product will use for these sizes (1 = none).
int gemm_split_k(int64_t m, int64_t n, int64_t k);
hipError_t launch_gemm(const GemmParams& p, hipStream_t st);

}  // namespace mxl

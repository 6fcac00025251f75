// MXFP4 quantizer kernels for gfx950: streaming, no matrix cores (the fused
// tile kernel is bound by the vector ALUs, the others by memory and launch).
//
//  quantize_rows_kernel   1x32 groups along the columns (Q1, Q2, Q3 of Eqs. 3-4)
//  quantize_tile_kernel   32x1 groups stored transposed (Q4, Q5, Q6 of Eqs. 4-5),
//                         optionally fused with the 1x32 quantizer of the same
//                         source (one read of the tensor) and with double
//                         quantization (Sec. 3.3)
//  ema_quantize_kernel    Q-EMA (Eq. 8, Algorithm 1)
//  oscillation_kernel     trajectory lengths dist_W, dist_Q of Q-Ramping (Sec. 6.1)
//  ramping_factor_kernel  amplification factor N_w of Algorithm 2
//  confidence_kernel      quantization confidence per element and its histogram (Sec. 4.2)
//  rate_partial_kernel,   one term of the rate of change of a tensor (Sec. 4.1): FP64 sums of
//  rate_finish_kernel     squares, reduced in a fixed order
//  dequantize_kernel      test aid
//
// Work split: one lane owns 8 consecutive elements of a row (one 16-byte bf16
// load, one Philox call for its 8 rounding decisions, one 4-byte store of 8
// codes); 4 neighbouring lanes form a 1x32 group and reduce |x| with DPP.
#include "mx_device.hpp"
#include "mx_launch.hpp"


using namespace mxd;

namespace {

constexpr int ROWS_UNROLL = 4;       // 8-element chunks per lane in quantize_rows_kernel
constexpr int ROWS_THREADS = 256;

struct RowsArgs {
    const void* src;
    uint8_t* codes;
    uint8_t* scales;
    float* ema;            // Q-EMA only
    int64_t ld;            // elements
    uint32_t cpr;          // 8-element chunks per row (cols / 8)
    uint32_t total;        // rows * cpr
    int contiguous;        // ld == cols
    int floor_mode;
    uint32_t k0, k1, tensor_id;
    uint64_t base_blk;     // index_base >> 3
    float beta;
    int update_ema;
};

// Encode 8 elements of one group (inv = 2^-s) and pack them low nibble first.  The FP32
// rounding mode must be set for the rounding in use (see rtn_code / sr_code).
template <bool SR, bool FLOOR>
__device__ __forceinline__ uint32_t encode8(const F8& x, int e, const U8& add)
{
    uint32_t packed = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        uint32_t c = SR ? sr_code<FLOOR>(x.v[t], e, add.w[t]) : rtn_code<FLOOR>(x.v[t], e);
        packed |= c << (4 * t);
    }
    return packed;
}

template <bool SR>
__device__ __forceinline__ void set_round_mode_for()
{
    if (SR) f32_round_toward_plus_inf();
    else    f32_round_toward_minus_inf();
}

// The 1x32 quantizer with E3M0 elements (format ablation, Table 7): same work split as
// quantize_rows_kernel, the element codec one bit higher in the FP32 layout.
template <typename SrcT, bool SR, bool FLOOR>
__global__ __launch_bounds__(ROWS_THREADS) void quantize_rows_e3m0_kernel(RowsArgs a)
{
    set_round_mode_for<SR>();
    const SrcT* src = static_cast<const SrcT*>(a.src);
    for (uint32_t q = blockIdx.x * ROWS_THREADS + threadIdx.x; q < a.total; q += gridDim.x * ROWS_THREADS) {
        // a.total is a multiple of 4 and a quad starts at a multiple of 4: the four lanes of a group stay together
        int64_t off;
        if (a.contiguous) {
            off = (int64_t)q * 8;
        } else {
            uint32_t r = q / a.cpr;
            off = (int64_t)r * a.ld + (int64_t)(q - r * a.cpr) * 8;
        }
        const F8 x = load8(src + off);
        const uint32_t byte = scale_byte_e3m0(quad_max(amax_bits8(x)), FLOOR);
        const int e = grid_exponent_e3m0(byte);
        U8 rnd;
        if (SR) rnd = sr_addends_e3m0(a.base_blk + q, a.tensor_id, a.k0, a.k1);
        uint32_t packed = 0;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            uint32_t c = SR ? sr_code_e3m0<FLOOR>(x.v[t], e, rnd.w[t]) : rtn_code_e3m0<FLOOR>(x.v[t], e);
            packed |= c << (4 * t);
        }
        reinterpret_cast<uint32_t*>(a.codes)[q] = packed;
        if ((threadIdx.x & 3) == 0) a.scales[q >> 2] = (uint8_t)byte;
    }
}

template <typename SrcT, bool SR, bool FLOOR>
__global__ __launch_bounds__(ROWS_THREADS) void quantize_rows_kernel(RowsArgs a)
{
    set_round_mode_for<SR>();
    const SrcT* src = static_cast<const SrcT*>(a.src);
    const uint32_t q0 = blockIdx.x * (ROWS_THREADS * ROWS_UNROLL) + threadIdx.x;
    F8 x[ROWS_UNROLL];
    bool ok[ROWS_UNROLL];
#pragma unroll
    for (int u = 0; u < ROWS_UNROLL; ++u) {
        uint32_t q = q0 + u * ROWS_THREADS;
        ok[u] = q < a.total && q >= q0;
        if (ok[u]) {
            int64_t off;
            if (a.contiguous) {
                off = (int64_t)q * 8;
            } else {
                uint32_t r = q / a.cpr;
                off = (int64_t)r * a.ld + (int64_t)(q - r * a.cpr) * 8;
            }
            x[u] = load8(src + off);
        } else {
            x[u] = zero8();
        }
    }
#pragma unroll
    for (int u = 0; u < ROWS_UNROLL; ++u) {
        uint32_t q = q0 + u * ROWS_THREADS;
        uint32_t m = quad_max(amax_bits8(x[u]));
        uint32_t byte = scale_byte(m, FLOOR);
        U8 rnd;
        if (SR) rnd = sr_addends(a.base_blk + q, a.tensor_id, a.k0, a.k1);
        uint32_t packed = encode8<SR, FLOOR>(x[u], grid_exponent(byte), rnd);
        if (ok[u]) {
            reinterpret_cast<uint32_t*>(a.codes)[q] = packed;
            if ((threadIdx.x & 3) == 0) a.scales[q >> 2] = (uint8_t)byte;
        }
    }
}

template <typename SrcT>
__global__ __launch_bounds__(ROWS_THREADS) void ema_quantize_kernel(RowsArgs a)
{
    const SrcT* src = static_cast<const SrcT*>(a.src);
    const uint32_t q = blockIdx.x * ROWS_THREADS + threadIdx.x;
    const bool ok = q < a.total;
    F8 w = zero8(), e = zero8();
    int64_t off = 0;
    if (ok) {
        if (a.contiguous) {
            off = (int64_t)q * 8;
        } else {
            uint32_t r = q / a.cpr;
            off = (int64_t)r * a.ld + (int64_t)(q - r * a.cpr) * 8;
        }
        w = load8(src + off);
        if (a.update_ema != 2) e = load8(a.ema + off);
    }
    if (a.update_ema == 1) {
        const float omb = __fsub_rn(1.0f, a.beta);
#pragma unroll
        for (int t = 0; t < 8; ++t) e.v[t] = __fmaf_rn(a.beta, e.v[t], __fmul_rn(omb, w.v[t]));
    } else if (a.update_ema == 2) {
        e = w;
    }
    uint32_t m = quad_max(amax_bits8(w));
    uint32_t byte = scale_byte(m, a.floor_mode);
    float inv = inv_scale(byte);
    uint32_t packed = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t)
        packed |= round_ema(w.v[t] * inv, e.v[t] * inv, a.floor_mode,
                            (__float_as_uint(w.v[t]) & 0x7FFFFFFFu) == 0u) << (4 * t);
    if (ok) {
        if (a.update_ema != 0) {
            float4* p = reinterpret_cast<float4*>(a.ema + off);
            p[0] = make_float4(e.v[0], e.v[1], e.v[2], e.v[3]);
            p[1] = make_float4(e.v[4], e.v[5], e.v[6], e.v[7]);
        }
        reinterpret_cast<uint32_t*>(a.codes)[q] = packed;
        if ((threadIdx.x & 3) == 0) a.scales[q >> 2] = (uint8_t)byte;
    }
}

// ---------------------------------------------------------------------------
// Transposed / fused quantizer.
//
// A workgroup of 8 waves owns a 256 x 128 macro tile of the source (256 x 64 for small tensors
// and for the tiles of a sparsely filled last round); wave w owns rows [32w, 32w+32) of it and
// walks over its 32 x 64 tiles.  The grid is one-dimensional over the macro tiles in row-major order.
// Inside a tile, lane l holds rows 4*(l/8)+j (j = 0..3) x columns 8*(l%8)+t (t = 0..7):
//   - each load instruction reads 8 full rows of 64 elements,
//   - a 1x32 row group is 4 neighbouring lanes (DPP quad reduction),
//   - a 32x1 column group is 4 registers x 8 lanes (l/8 = 0..7) of one column.
// The 32 elements of a lane stay in registers through both quantizers.  Codes and scale
// bytes are collected in LDS ([256 rows][128 B] row codes, [256 columns][128 B] transposed
// codes) and written out at the end as whole 128-byte lines, 16 bytes per lane.
// ---------------------------------------------------------------------------
constexpr int TILE_THREADS = 512;
constexpr int ST_PITCH = 144;                       // bytes per staged row / column of codes (128 + pad)
constexpr int ST_ROW_OFF = 0;                       // row codes      [256][ST_PITCH]
constexpr int ST_COL_OFF = 256 * ST_PITCH;          // transposed     [256][ST_PITCH]
constexpr int ST_SROW_OFF = 2 * 256 * ST_PITCH;     // row scales     [256][8]
constexpr int ST_SCOL_OFF = ST_SROW_OFF + 256 * 8;  // transposed scales [256][8]
constexpr int ST_BYTES = ST_SCOL_OFF + 256 * 8;     // 77824: two workgroups per CU
constexpr int ST_CSUM_OFF = ST_BYTES;               // COLSUM instances: column sums per wave, [8][128] floats
constexpr int ST_BYTES_CSUM = ST_BYTES + 8 * 128 * 4; // 81920: still two workgroups per CU

struct TileArgs {
    const void* src;
    const uint8_t* row_codes_in;
    const uint8_t* row_scales_in;
    uint8_t* codes_t;
    uint8_t* scales_t;
    uint8_t* codes_row;
    uint8_t* scales_row;
    int64_t ld;
    uint32_t rows, cols;
    int pre_quant;
    // 1-D grid over macro tiles in row-major order: the first n_wide workgroups own 256 x 128 tiles
    // (two 32 x 64 tiles per wave), the rest own the two 256 x 64 halves of the tiles after those
    uint32_t n_wide;
    uint32_t wide_per_row; // 256 x 128 tiles per block of 256 rows = ceil(cols / 128)
    uint32_t k0, k1, tensor_id_t, tensor_id_row;
    uint64_t index_base;
    const uint32_t* seed_dev;  // when set: the two key words are read from here instead of k0, k1
    float* col_sum_partials;   // COLSUM instances: [ceil(rows / 256)][cols] sums of the source over 256-row blocks, or null
};

__device__ __forceinline__ uint32_t xor_lane_max(uint32_t v, int mask)
{
    uint32_t o = (uint32_t)__shfl_xor((int)v, mask, 64);
    return v > o ? v : o;
}

// Copies one staged result of a macro tile to memory: `lines` staged lines (rows of row codes, or
// columns of transposed codes), each `pieces` 16-byte pieces of codes (ST_PITCH apart in LDS,
// `code_pitch` bytes apart in memory) and `pieces` scale bytes (8 apart in LDS, `scale_pitch` apart
// in memory); pieces <= 8.  A lane keeps its piece and steps over the lines, so the loop has no
// index arithmetic beyond two additions; when a line's scale bytes form an aligned 8- or 4-byte
// word they leave as one store.
__device__ __forceinline__ void write_staged(const uint8_t* codes_st, const uint8_t* scales_st,
                                             uint32_t lines, uint32_t pieces,
                                             uint8_t* codes, size_t code_pitch,
                                             uint8_t* scales, size_t scale_pitch, uint32_t tid)
{
    if ((pieces & (pieces - 1u)) == 0u) {
        const uint32_t sh = (uint32_t)__builtin_ctz(pieces);
        const uint32_t lstep = (uint32_t)TILE_THREADS >> sh;
        uint32_t l = tid >> sh;
        const uint32_t pc = tid & (pieces - 1u);
        const uint8_t* s = codes_st + l * ST_PITCH + pc * 16;
        uint8_t* d = codes + (size_t)l * code_pitch + pc * 16;
        const size_t dstep = (size_t)lstep * code_pitch;
        for (; l < lines; l += lstep, s += lstep * ST_PITCH, d += dstep)
            *reinterpret_cast<uint4*>(d) = *reinterpret_cast<const uint4*>(s);
    } else {
        for (uint32_t q = tid; q < lines * pieces; q += TILE_THREADS) {
            const uint32_t l = q / pieces, pc = q - l * pieces;
            *reinterpret_cast<uint4*>(codes + (size_t)l * code_pitch + pc * 16) =
                *reinterpret_cast<const uint4*>(codes_st + l * ST_PITCH + pc * 16);
        }
    }
    const bool word_ok = ((reinterpret_cast<uintptr_t>(scales) | scale_pitch) & (pieces - 1u)) == 0u;
    if (pieces == 8u && word_ok) {
        for (uint32_t l = tid; l < lines; l += TILE_THREADS)
            *reinterpret_cast<uint2*>(scales + (size_t)l * scale_pitch) = *reinterpret_cast<const uint2*>(scales_st + l * 8);
    } else if (pieces == 4u && word_ok) {
        for (uint32_t l = tid; l < lines; l += TILE_THREADS)
            *reinterpret_cast<uint32_t*>(scales + (size_t)l * scale_pitch) = *reinterpret_cast<const uint32_t*>(scales_st + l * 8);
    } else {
        for (uint32_t q = tid; q < lines * 8u; q += TILE_THREADS) {
            const uint32_t l = q >> 3, pc = q & 7u;
            if (pc < pieces) scales[(size_t)l * scale_pitch + pc] = scales_st[l * 8 + pc];
        }
    }
}

// Sum of v over the 8 lanes that share lane % 8 (the 8 row groups of a wave tile), in a fixed order,
// returned in all of them: the partner 8 lanes away inside a row of 16 (DPP rotate), then the rows of
// 16 and the halves of the wave (lane-swap instructions; a swap of a register with its copy leaves
// the two partners' values side by side).
__device__ __forceinline__ float sum_over_row_groups(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xF, 0xF, true));   // row_ror:8
    const auto p16 = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(p16[0]) + __uint_as_float(p16[1]);
    const auto p32 = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(p32[0]) + __uint_as_float(p32[1]);
}

// Up to TILE_BATCH_MAX tensors per launch (e.g. the activation and the weight of a layer: one launch,
// and the small tensor's workgroups fill the last round of the large one's).  first[j] is the first
// workgroup of job j (0xFFFFFFFF for unused slots); all jobs share the template parameters.
constexpr int TILE_BATCH_MAX = 4;
struct TileBatch {
    TileArgs job[TILE_BATCH_MAX];
    uint32_t first[TILE_BATCH_MAX];
};

// SRC: 0 = FP32 source, 1 = bf16 source, 2 = packed row result given
// COLSUM: also the column sums of the source (a bias gradient is that of dY), per 256-row block; a
// separate instance, so that the plain quantizer's code does not change with this feature.
template <int SRC, bool ROW_SR, bool T_SR, bool FLOOR, bool COLSUM = false>
__global__ __launch_bounds__(TILE_THREADS, 4) void quantize_tile_kernel(TileBatch batch)
{
    uint32_t job = 0;
#pragma unroll
    for (int i = 1; i < TILE_BATCH_MAX; ++i) job += blockIdx.x >= batch.first[i] ? 1u : 0u;
    const TileArgs a = batch.job[job];
    const uint32_t block = blockIdx.x - batch.first[job];
    // Philox key: the seed argument, or the 64-bit word in device memory that the caller names (a
    // captured graph then draws new numbers on every replay).  Kept in scalar registers either way.
    uint32_t k0 = a.k0, k1 = a.k1;
    if ((ROW_SR || T_SR) && a.seed_dev) {
        k0 = __builtin_amdgcn_readfirstlane(a.seed_dev[0]);
        k1 = __builtin_amdgcn_readfirstlane(a.seed_dev[1]);
    }
    __shared__ __attribute__((aligned(16))) uint8_t st[COLSUM ? ST_BYTES_CSUM : ST_BYTES];
    // FP32 sources need the rounding mode of each rule (switched per phase when they differ).
    // bf16 and packed sources scale exactly wherever a round_D threshold is near (8 significant
    // bits), so there the mode of round_S, if any, serves the whole kernel.
    constexpr bool SWITCH_MODES = (SRC == 0) && (ROW_SR != T_SR);
    if (!SWITCH_MODES) set_round_mode_for<(ROW_SR || T_SR)>();
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int cc = lane & 7, rg = lane >> 3;
    const int wr = wave;                                  // wave position inside the macro tile
    // macro tile of this workgroup (uniform): a wide one, or one half of a wide one
    const bool wide = block < a.n_wide;
    const uint32_t narrow = wide ? 0u : block - a.n_wide;
    // Workgroup ids go round the 8 XCDs, each with its own L2.  A macro tile writes 4 scale bytes per row
    // and 8 per column: a 32-byte sector of a scale array is completed by up to 8 tiles side by side, or 4
    // on top of each other.  Each XCD therefore takes a contiguous range of the row-major tile order, so
    // that the tiles which share sectors meet in one L2 and the sectors leave it whole.
    const uint32_t xcd_class = block & 7u, per_xcd = a.n_wide >> 3, rem_xcd = a.n_wide & 7u;
    const uint32_t wide_index = wide ? xcd_class * per_xcd + min(xcd_class, rem_xcd) + (block >> 3)
                                     : a.n_wide + (narrow >> 1);
    const uint32_t row_block = wide_index / a.wide_per_row;
    const int tiles_per_wave = wide ? 2 : 1;
    const uint32_t macro_rows = 256u, macro_cols = 64u * tiles_per_wave;
    const uint32_t mrow0 = row_block * macro_rows;        // macro tile origin
    const uint32_t mcol0 = (wide_index - row_block * a.wide_per_row) * 128u + (wide ? 0u : (narrow & 1u) * 64u);
    if (mcol0 >= a.cols) return;                          // second half of a tile that is only 64 columns wide
    const bool wave_has_rows = mrow0 + wr * 32 < a.rows;
    const uint32_t lrow0 = wr * 32 + 4 * rg;              // first of this lane's 4 rows inside the macro tile
    const uint32_t row0 = mrow0 + lrow0;
    const bool want_row = a.codes_row != nullptr;
    const uint32_t half_rows = a.rows >> 1, grp_rows = a.rows >> 5;
    const uint32_t half_cols = a.cols >> 1, grp_cols = a.cols >> 5;

    // bf16 sources with a deterministic row quantizer: the raw 16 bytes per row of the wave's next tile are
    // fetched while the current tile is being encoded (16 registers), so that only the first load of a
    // workgroup is waited for: -8 to -10 % on those passes.  The instances with a stochastic row quantizer
    // have no registers to spare under the 128 that two workgroups per compute unit allow (3 spilled,
    // +2-5 %); issuing their fetch later in the tile, where registers are free, hides too little of the
    // latency to pay for the instructions it adds (measured: no change in the sum of those passes).
    constexpr bool PREFETCH = (SRC == 1) && !ROW_SR;
    bf16x8_raw raw[4];
    auto fetch_raw = [&](int ci) {
        const uint32_t col = mcol0 + ci * 64 + cc * 8;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            raw[j] = bf16x8_raw{0u, 0u, 0u, 0u};
            if (col < a.cols) raw[j] = load8_raw(static_cast<const uint16_t*>(a.src) + (int64_t)(row0 + j) * a.ld + col);
        }
    };
    if (PREFETCH && wave_has_rows) fetch_raw(0);
    for (int ci = 0; ci < tiles_per_wave && wave_has_rows; ++ci) {
        const uint32_t tcol0 = ci * 64;
        const uint32_t lcol0 = tcol0 + cc * 8;            // first of this lane's 8 columns inside the macro tile
        const uint32_t c = mcol0 + lcol0;
        if (mcol0 + tcol0 >= a.cols) break;               // uniform over the wave
        const bool ok = c < a.cols;
        F8 x[4];
        // ---- load -----------------------------------------------------------
        if (SRC == 2) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                x[j] = zero8();
                if (ok) {
                    uint32_t r = row0 + j;
                    uint32_t pk = *reinterpret_cast<const uint32_t*>(a.row_codes_in + (size_t)r * half_cols + (c >> 1));
                    uint32_t byte = a.row_scales_in[(size_t)r * grp_cols + (c >> 5)];
#pragma unroll
                    for (int t = 0; t < 8; ++t) x[j].v[t] = dequant((pk >> (4 * t)) & 15u, byte);
                }
            }
        } else {
            if (PREFETCH) {
#pragma unroll
                for (int j = 0; j < 4; ++j) x[j] = expand8(raw[j]);
                if (ci + 1 < tiles_per_wave && mcol0 + tcol0 + 64 < a.cols) fetch_raw(ci + 1);
            } else if (mcol0 + tcol0 + 64 <= a.cols) {    // whole tile inside the matrix (uniform): no masking, no zero fill
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int64_t off = (int64_t)(row0 + j) * a.ld + c;
                    if (SRC == 1) x[j] = load8(static_cast<const uint16_t*>(a.src) + off);
                    else          x[j] = load8(static_cast<const float*>(a.src) + off);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    x[j] = zero8();
                    if (ok) {
                        int64_t off = (int64_t)(row0 + j) * a.ld + c;
                        if (SRC == 1) x[j] = load8(static_cast<const uint16_t*>(a.src) + off);
                        else          x[j] = load8(static_cast<const float*>(a.src) + off);
                    }
                }
            }
            // ---- column sums of the source over this wave's 32 rows -------------
            if (COLSUM && a.col_sum_partials != nullptr) {
                f32_round_to_nearest_even();
                float cs[8];
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    cs[t] = sum_over_row_groups(((x[0].v[t] + x[1].v[t]) + x[2].v[t]) + x[3].v[t]);
                if (rg == 0) {
                    float* dst = reinterpret_cast<float*>(st + ST_CSUM_OFF) + wr * 128 + lcol0;
#pragma unroll
                    for (int t = 0; t < 8; ++t) dst[t] = cs[t];
                }
                if (!SWITCH_MODES) set_round_mode_for<(ROW_SR || T_SR)>();
            }
            // ---- 1x32 quantizer of the same elements ---------------------------
            if (want_row || a.pre_quant) {
                if (SWITCH_MODES) set_round_mode_for<ROW_SR>();
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    uint32_t r = row0 + j;
                    uint32_t byte = scale_byte(quad_max(amax_bits8(x[j])), FLOOR);
                    const int e = grid_exponent(byte);
                    U8 rnd;
                    if (ROW_SR) rnd = sr_addends((a.index_base + (uint64_t)r * a.cols + c) >> 3, a.tensor_id_row, k0, k1);
                    uint32_t pk = 0;
                    if (a.pre_quant) {
                        // keep sign in the value: the next quantizer takes |x| and the sign from it
#pragma unroll
                        for (int t = 0; t < 8; ++t) {
                            uint32_t gb;
                            if (ROW_SR) {
                                uint32_t code = sr_code_keep<FLOOR>(x[j].v[t], e, rnd.w[t], gb);
                                pk |= code << (4 * t);
                                float mag = __builtin_ldexpf(__uint_as_float(gb), (int)byte - 1);  // m * 2^s, exact
                                x[j].v[t] = __builtin_copysignf(mag, x[j].v[t]);
                            } else {
                                pk |= rtn_code_keep<FLOOR>(x[j].v[t], e, gb) << (4 * t);           // gb carries the sign
                                x[j].v[t] = __builtin_ldexpf(__uint_as_float(gb), (int)byte - 1);  // +-m * 2^s, exact
                            }
                        }
                    } else {
                        pk = encode8<ROW_SR, FLOOR>(x[j], e, rnd);
                    }
                    if (want_row) {
                        *reinterpret_cast<uint32_t*>(st + ST_ROW_OFF + (lrow0 + j) * ST_PITCH + (lcol0 >> 1)) = pk;
                        if ((cc & 3) == 0) st[ST_SROW_OFF + (lrow0 + j) * 8 + (lcol0 >> 5)] = (uint8_t)byte;
                    }
                }
            }
        }
        // ---- 32x1 quantizer: group = this lane's 4 rows x the 8 lanes sharing cc --
        uint32_t sb[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            uint32_t m = absmax3_bits(x[0].v[t], x[1].v[t], 0u);
            m = absmax3_bits(x[2].v[t], x[3].v[t], m);
            m = xor_lane_max(m, 8);
            m = xor_lane_max(m, 16);
            m = xor_lane_max(m, 32);
            sb[t] = scale_byte(m, FLOOR);
        }
        if (SWITCH_MODES) set_round_mode_for<T_SR>();
        uint32_t colpk[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) colpk[t] = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            U8 rnd;
            if (T_SR) rnd = sr_addends((a.index_base + (uint64_t)(row0 + j) * a.cols + c) >> 3, a.tensor_id_t, k0, k1);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                int e = grid_exponent(sb[t]);
                uint32_t code = T_SR ? sr_code<FLOOR>(x[j].v[t], e, rnd.w[t]) : rtn_code<FLOOR>(x[j].v[t], e);
                colpk[t] |= code << (4 * j);
            }
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            *reinterpret_cast<uint16_t*>(st + ST_COL_OFF + (lcol0 + t) * ST_PITCH + (lrow0 >> 1)) = (uint16_t)colpk[t];
            if (rg == 0) st[ST_SCOL_OFF + (lcol0 + t) * 8 + wr] = (uint8_t)sb[t];
        }
    }
    __syncthreads();

    // ---- write the staged macro tile out: 16 bytes per lane, whole 128-byte lines ----
    const uint32_t ncols_here = min(macro_cols, a.cols - mcol0);    // multiples of 32
    const uint32_t nrows_here = min(macro_rows, a.rows - mrow0);    // multiples of 32
    if (want_row)
        write_staged(st + ST_ROW_OFF, st + ST_SROW_OFF, nrows_here, ncols_here >> 5,
                     a.codes_row + (size_t)mrow0 * half_cols + (mcol0 >> 1), half_cols,
                     a.scales_row + (size_t)mrow0 * grp_cols + (mcol0 >> 5), grp_cols, tid);
    write_staged(st + ST_COL_OFF, st + ST_SCOL_OFF, ncols_here, nrows_here >> 5,
                 a.codes_t + (size_t)mcol0 * half_rows + (mrow0 >> 1), half_rows,
                 a.scales_t + (size_t)mcol0 * grp_rows + (mrow0 >> 5), grp_rows, tid);
    if (COLSUM && a.col_sum_partials != nullptr && (uint32_t)tid < ncols_here) {
        // the waves that had rows, in order; one value per column of this 256-row block.  Round to
        // nearest like the per-wave sums (no quantizer arithmetic follows, the mode is not restored).
        f32_round_to_nearest_even();
        const float* cs = reinterpret_cast<const float*>(st + ST_CSUM_OFF) + tid;
        float s = cs[0];
        for (uint32_t w = 1; w < (nrows_here >> 5); ++w) s += cs[w * 128];
        a.col_sum_partials[(size_t)row_block * a.cols + mcol0 + tid] = s;
    }
}

// Sums the per-block column sums in a fixed order: a workgroup owns 32 columns; each of its 8 parts
// (32 lanes) adds up a contiguous eighth of the blocks in index order (independent loads, 128 bytes
// per row of 32 lanes), then the eight parts are added in order.
__global__ __launch_bounds__(256) void column_sum_finish_kernel(const float* partials, uint32_t blocks, uint32_t cols, float* out)
{
    __shared__ float part[8][32];
    const uint32_t lc = threadIdx.x & 31u, p = threadIdx.x >> 5;
    const uint32_t c = blockIdx.x * 32u + lc;
    const uint32_t per = (blocks + 7u) / 8u;
    float s = 0.f;
    if (c < cols) {
        const uint32_t b0 = min(blocks, p * per), b1 = min(blocks, b0 + per);
        for (uint32_t b = b0; b < b1; ++b) s += partials[(size_t)b * cols + c];
    }
    part[p][lc] = s;
    __syncthreads();
    if (p == 0 && c < cols) {
        float t = part[0][lc];
#pragma unroll
        for (int q = 1; q < 8; ++q) t += part[q][lc];
        out[c] = t;
    }
}

// ---------------------------------------------------------------------------
// Q-Ramping's oscillation detection (Sec. 6.1): one step of
//     dist_W += |w - w_prev|,   dist_Q += |w_Q - w_Q,prev|,   w_Q = P * 2^s,
// per weight element, FP32, one rounding per operation.  The previous quantized weight is kept
// packed (codes_prev / scales_prev), not as FP32: 0.53 instead of 4 bytes per element of state.
// One lane owns 8 consecutive elements, as in the quantizers.
// ---------------------------------------------------------------------------
struct OscArgs {
    const void* w;
    const uint8_t* codes;
    const uint8_t* scales;
    float* w_prev;
    uint8_t* codes_prev;
    uint8_t* scales_prev;
    float* dist_w;
    float* dist_q;
    int64_t ld;
    uint32_t cpr;          // 8-element chunks per row
    uint32_t total;        // rows * cpr
    int init;
};

template <typename SrcT>
__global__ __launch_bounds__(ROWS_THREADS) void oscillation_kernel(OscArgs a)
{
    const uint32_t q = blockIdx.x * ROWS_THREADS + threadIdx.x;
    if (q >= a.total) return;
    const uint32_t r = q / a.cpr, ch = q - r * a.cpr;
    const F8 w = load8(static_cast<const SrcT*>(a.w) + (int64_t)r * a.ld + (int64_t)ch * 8);
    const size_t dense = (size_t)q * 8;                   // state arrays are dense [rows][cols]
    const uint32_t pk = reinterpret_cast<const uint32_t*>(a.codes)[q];
    const uint32_t byte = a.scales[(size_t)q >> 2];       // cols/32 groups per row = cpr/4
    float4* wp = reinterpret_cast<float4*>(a.w_prev + dense);
    if (!a.init) {
        const uint32_t pk0 = reinterpret_cast<const uint32_t*>(a.codes_prev)[q];
        const uint32_t byte0 = a.scales_prev[(size_t)q >> 2];
        const float4 p0 = wp[0], p1 = wp[1];
        const float prev[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
        float4* dwp = reinterpret_cast<float4*>(a.dist_w + dense);
        float4* dqp = reinterpret_cast<float4*>(a.dist_q + dense);
        const float4 a0 = dwp[0], a1 = dwp[1], b0 = dqp[0], b1 = dqp[1];
        float dw[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
        float dq[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const float wq = dequant((pk >> (4 * t)) & 15u, byte);
            const float wq0 = dequant((pk0 >> (4 * t)) & 15u, byte0);
            dw[t] = __fadd_rn(dw[t], __builtin_fabsf(__fsub_rn(w.v[t], prev[t])));
            dq[t] = __fadd_rn(dq[t], __builtin_fabsf(__fsub_rn(wq, wq0)));
        }
        dwp[0] = make_float4(dw[0], dw[1], dw[2], dw[3]);
        dwp[1] = make_float4(dw[4], dw[5], dw[6], dw[7]);
        dqp[0] = make_float4(dq[0], dq[1], dq[2], dq[3]);
        dqp[1] = make_float4(dq[4], dq[5], dq[6], dq[7]);
    } else {
        const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
        reinterpret_cast<float4*>(a.dist_w + dense)[0] = z;
        reinterpret_cast<float4*>(a.dist_w + dense)[1] = z;
        reinterpret_cast<float4*>(a.dist_q + dense)[0] = z;
        reinterpret_cast<float4*>(a.dist_q + dense)[1] = z;
    }
    wp[0] = make_float4(w.v[0], w.v[1], w.v[2], w.v[3]);
    wp[1] = make_float4(w.v[4], w.v[5], w.v[6], w.v[7]);
    reinterpret_cast<uint32_t*>(a.codes_prev)[q] = pk;
    if ((ch & 3) == 0) a.scales_prev[(size_t)q >> 2] = (uint8_t)byte;
}

// Amplification factor of Algorithm 2 (Q-Ramping): N_w = min(k2 * floor(R_w / k1) + 1, n_max),
// R_w = dist_Q / dist_W with IEEE FP32 divisions; dist_W = 0 gives R_w = 0 if dist_Q = 0, else +inf.
__global__ void ramping_factor_kernel(const float* dist_w, const float* dist_q, int64_t count,
                                      float k1, int k2, int n_max, int32_t* factor)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    const float dw = dist_w[i], dq = dist_q[i];
    float ratio;
    if (dw == 0.0f) ratio = dq == 0.0f ? 0.0f : __builtin_inff();
    else            ratio = __fdiv_rn(dq, dw);
    const float steps = floorf(__fdiv_rn(ratio, k1));
    int32_t n = n_max;
    if (steps < (float)n_max) {
        const int64_t v = (int64_t)k2 * (int64_t)steps + 1;
        n = v < (int64_t)n_max ? (int32_t)v : n_max;
    }
    factor[i] = n;
}

// ---------------------------------------------------------------------------
// Quantization confidence (Sec. 4.2) on the latent value y = w / S of a 1x32 group:
//     conf = min_i |y - thrd_i| / MaxDist(y_FP4).
// The thresholds are the midpoints of neighbouring E2M1 values; the cell of an E2M1 value reaches
// from the threshold below to the threshold above it (the cell of 0 is [-0.25, 0.25], the cell of
// 6 is [5, 6]), and MaxDist is half the cell's width, for the outermost cell the whole width.
// The sign plays no part: everything is taken on a = |y|.  y is exact (a power-of-two scaling),
// each distance is one FP32 subtraction, the quotient one IEEE division.
// ---------------------------------------------------------------------------
struct ConfArgs {
    const void* w;
    float* conf;                       // may be null
    unsigned long long* hist;          // may be null
    int64_t ld;
    uint32_t cpr, total;
    int bins;
    int floor_mode;
};

__device__ __forceinline__ float confidence_of(float a)
{
    // lower threshold, upper threshold, MaxDist of the cell that holds a
    float lo, hi, den;
    if (a < 0.25f)      { lo = -0.25f; hi = 0.25f; den = 0.25f; }
    else if (a < 0.75f) { lo = 0.25f;  hi = 0.75f; den = 0.25f; }
    else if (a < 1.25f) { lo = 0.75f;  hi = 1.25f; den = 0.25f; }
    else if (a < 1.75f) { lo = 1.25f;  hi = 1.75f; den = 0.25f; }
    else if (a < 2.5f)  { lo = 1.75f;  hi = 2.5f;  den = 0.375f; }
    else if (a < 3.5f)  { lo = 2.5f;   hi = 3.5f;  den = 0.5f; }
    else if (a < 5.0f)  { lo = 3.5f;   hi = 5.0f;  den = 0.75f; }
    else                { lo = 5.0f;   hi = __builtin_inff(); den = 1.0f; }
    const float below = __fsub_rn(a, lo), above = __fsub_rn(hi, a);
    return __fdiv_rn(below < above ? below : above, den);
}

constexpr int CONF_MAX_BINS = mxl::CONFIDENCE_MAX_BINS;

template <typename SrcT>
__global__ __launch_bounds__(ROWS_THREADS) void confidence_kernel(ConfArgs a)
{
    __shared__ uint32_t lh[CONF_MAX_BINS];
    if (a.hist) {
        for (int b = threadIdx.x; b < a.bins; b += ROWS_THREADS) lh[b] = 0u;
        __syncthreads();
    }
    // a.total is a multiple of 4 and a quad of lanes (one 1x32 group) starts at a multiple of 4:
    // the lanes of a group pass or fail the loop test together
    for (uint32_t q = blockIdx.x * ROWS_THREADS + threadIdx.x; q < a.total; q += gridDim.x * ROWS_THREADS) {
        const uint32_t r = q / a.cpr, ch = q - r * a.cpr;
        const F8 w = load8(static_cast<const SrcT*>(a.w) + (int64_t)r * a.ld + (int64_t)ch * 8);
        const uint32_t byte = scale_byte(quad_max(amax_bits8(w)), a.floor_mode);
        const float inv = inv_scale(byte);
        float c[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            float y = __builtin_fabsf(__fmul_rn(w.v[t], inv));
            y = y > 6.0f ? 6.0f : y;                       // Eq. 2's scale truncates to Q_p
            c[t] = confidence_of(y);
        }
        if (a.conf) {
            float4* out = reinterpret_cast<float4*>(a.conf + (size_t)q * 8);
            out[0] = make_float4(c[0], c[1], c[2], c[3]);
            out[1] = make_float4(c[4], c[5], c[6], c[7]);
        }
        if (a.hist) {
            const float nb = (float)a.bins;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                int b = (int)floorf(__fmul_rn(c[t], nb));
                b = b > a.bins - 1 ? a.bins - 1 : b;
                atomicAdd(&lh[b], 1u);
            }
        }
    }
    if (a.hist) {
        __syncthreads();
        for (int b = threadIdx.x; b < a.bins; b += ROWS_THREADS)
            if (lh[b]) atomicAdd(&a.hist[b], (unsigned long long)lh[b]);
    }
}

// ---------------------------------------------------------------------------
// One term of the rate of change (Sec. 4.1): ||x - x_prev||_F / ||x_prev||_F, then x_prev = x.
// Differences of FP32 values and their squares' sums are taken in FP64.  The order of the sums is
// fixed by the launch shape (RATE_BLOCKS x ROWS_THREADS lanes, grid-stride over 8-element chunks,
// then a tree within the block, then the blocks in index order), so a call repeats bit for bit.
// ---------------------------------------------------------------------------
constexpr int RATE_BLOCKS = 1024;

struct RateArgs {
    const void* x;
    float* x_prev;
    double* partial;                   // [RATE_BLOCKS][2]
    int64_t ld;
    uint32_t cpr, total;
    int init;
};

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}

template <typename SrcT>
__global__ __launch_bounds__(ROWS_THREADS) void rate_partial_kernel(RateArgs a)
{
    __shared__ double red[2][ROWS_THREADS / 64];
    double diff2 = 0.0, prev2 = 0.0;
    for (uint32_t q = blockIdx.x * ROWS_THREADS + threadIdx.x; q < a.total; q += RATE_BLOCKS * ROWS_THREADS) {
        const uint32_t r = q / a.cpr, ch = q - r * a.cpr;
        const F8 x = load8(static_cast<const SrcT*>(a.x) + (int64_t)r * a.ld + (int64_t)ch * 8);
        float4* pp = reinterpret_cast<float4*>(a.x_prev + (size_t)q * 8);
        if (!a.init) {
            const float4 p0 = pp[0], p1 = pp[1];
            const float old[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const double o = (double)old[t], d = (double)x.v[t] - o;
                diff2 = fma(d, d, diff2);
                prev2 = fma(o, o, prev2);
            }
        }
        pp[0] = make_float4(x.v[0], x.v[1], x.v[2], x.v[3]);
        pp[1] = make_float4(x.v[4], x.v[5], x.v[6], x.v[7]);
    }
    diff2 = wave_sum(diff2);
    prev2 = wave_sum(prev2);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { red[0][wave] = diff2; red[1][wave] = prev2; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double d = 0.0, p = 0.0;
        for (int i = 0; i < ROWS_THREADS / 64; ++i) { d += red[0][i]; p += red[1][i]; }
        a.partial[2 * blockIdx.x] = d;
        a.partial[2 * blockIdx.x + 1] = p;
    }
}

// result[0] = this step's term, result[1] = sum of the terms since the window opened,
// result[2] = their number.  One workgroup.
__global__ __launch_bounds__(ROWS_THREADS) void rate_finish_kernel(const double* partial, int init, double* result)
{
    __shared__ double red[2][ROWS_THREADS / 64];
    double d = 0.0, p = 0.0;
    for (int b = threadIdx.x; b < RATE_BLOCKS; b += ROWS_THREADS) { d += partial[2 * b]; p += partial[2 * b + 1]; }
    d = wave_sum(d);
    p = wave_sum(p);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { red[0][wave] = d; red[1][wave] = p; }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (init) {
            result[0] = 0.0; result[1] = 0.0; result[2] = 0.0;
        } else {
            double dd = 0.0, pp = 0.0;
            for (int i = 0; i < ROWS_THREADS / 64; ++i) { dd += red[0][i]; pp += red[1][i]; }
            double term;
            if (pp == 0.0) term = dd == 0.0 ? 0.0 : (double)__builtin_inff();
            else           term = sqrt(dd) / sqrt(pp);
            result[0] = term;
            result[1] = result[1] + term;
            result[2] = result[2] + 1.0;
        }
    }
}

__global__ void dequantize_kernel(const uint8_t* codes, const uint8_t* scales, int64_t total_bytes,
                                  int64_t cols, float* out)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;     // one code byte = 2 elements
    if (i >= total_bytes) return;
    int64_t half = cols >> 1;
    int64_t r = i / half, j = i - r * half;
    uint32_t byte = scales[r * (cols >> 5) + (j >> 4)];
    uint32_t b = codes[i];
    out[2 * i] = dequant(b & 15u, byte);
    out[2 * i + 1] = dequant(b >> 4, byte);
}

__global__ void dequantize_e3m0_kernel(const uint8_t* codes, const uint8_t* scales, int64_t total, int64_t cols, float* out)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;       // index of a code byte
    if (i >= total) return;
    int64_t half = cols >> 1;
    int64_t r = i / half, j = i - r * half;
    uint32_t byte = scales[r * (cols >> 5) + (j >> 4)];
    uint32_t b = codes[i];
    out[2 * i] = dequant_e3m0(b & 15u, byte);
    out[2 * i + 1] = dequant_e3m0(b >> 4, byte);
}

__global__ __launch_bounds__(256) void calibration_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

}  // namespace

// ------------------------------------------------------------------ launchers

namespace mxl {

hipError_t launch_quantize_rows(const QuantRowsParams& p, hipStream_t st)
{
    RowsArgs a{};
    a.src = p.src; a.codes = p.codes; a.scales = p.scales; a.ema = nullptr;
    a.ld = p.ld; a.cpr = (uint32_t)(p.cols / 8); a.total = (uint32_t)(p.rows * (p.cols / 8));
    a.contiguous = p.ld == p.cols; a.floor_mode = p.floor_mode;
    a.k0 = (uint32_t)p.seed; a.k1 = (uint32_t)(p.seed >> 32); a.tensor_id = p.tensor_id;
    a.base_blk = p.index_base >> 3;
    const uint32_t per_block = ROWS_THREADS * ROWS_UNROLL;
    dim3 grid((a.total + per_block - 1) / per_block), block(ROWS_THREADS);
#define MX_ROWS_LAUNCH(T, SR, FL) hipLaunchKernelGGL((quantize_rows_kernel<T, SR, FL>), grid, block, 0, st, a)
    const int variant = (p.bf16 ? 4 : 0) | (p.sr ? 2 : 0) | (p.floor_mode ? 1 : 0);
    switch (variant) {
        case 0: MX_ROWS_LAUNCH(float, false, false); break;
        case 1: MX_ROWS_LAUNCH(float, false, true); break;
        case 2: MX_ROWS_LAUNCH(float, true, false); break;
        case 3: MX_ROWS_LAUNCH(float, true, true); break;
        case 4: MX_ROWS_LAUNCH(uint16_t, false, false); break;
        case 5: MX_ROWS_LAUNCH(uint16_t, false, true); break;
        case 6: MX_ROWS_LAUNCH(uint16_t, true, false); break;
        default: MX_ROWS_LAUNCH(uint16_t, true, true); break;
    }
#undef MX_ROWS_LAUNCH
    return hipGetLastError();
}

hipError_t launch_quantize_rows_e3m0(const QuantRowsParams& p, hipStream_t st)
{
    RowsArgs a{};
    a.src = p.src; a.codes = p.codes; a.scales = p.scales; a.ema = nullptr;
    a.ld = p.ld; a.cpr = (uint32_t)(p.cols / 8); a.total = (uint32_t)(p.rows * (p.cols / 8));
    a.contiguous = p.ld == p.cols; a.floor_mode = p.floor_mode;
    a.k0 = (uint32_t)p.seed; a.k1 = (uint32_t)(p.seed >> 32); a.tensor_id = p.tensor_id;
    a.base_blk = p.index_base >> 3;
    uint32_t blocks = (a.total + ROWS_THREADS - 1) / ROWS_THREADS;
    dim3 grid(blocks < 8192u ? blocks : 8192u), block(ROWS_THREADS);
#define MX_ROWS_LAUNCH(T, SR, FL) hipLaunchKernelGGL((quantize_rows_e3m0_kernel<T, SR, FL>), grid, block, 0, st, a)
    const int variant = (p.bf16 ? 4 : 0) | (p.sr ? 2 : 0) | (p.floor_mode ? 1 : 0);
    switch (variant) {
        case 0: MX_ROWS_LAUNCH(float, false, false); break;
        case 1: MX_ROWS_LAUNCH(float, false, true); break;
        case 2: MX_ROWS_LAUNCH(float, true, false); break;
        case 3: MX_ROWS_LAUNCH(float, true, true); break;
        case 4: MX_ROWS_LAUNCH(uint16_t, false, false); break;
        case 5: MX_ROWS_LAUNCH(uint16_t, false, true); break;
        case 6: MX_ROWS_LAUNCH(uint16_t, true, false); break;
        default: MX_ROWS_LAUNCH(uint16_t, true, true); break;
    }
#undef MX_ROWS_LAUNCH
    return hipGetLastError();
}

hipError_t launch_dequantize_e3m0(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t cols,
                                  float* out, hipStream_t st)
{
    int64_t total = rows * (cols / 2);
    dim3 grid((unsigned)((total + 255) / 256)), block(256);
    hipLaunchKernelGGL(dequantize_e3m0_kernel, grid, block, 0, st, codes, scales, total, cols, out);
    return hipGetLastError();
}

hipError_t launch_ema_quantize(const QuantRowsParams& p, float* ema, float beta, int update_ema, hipStream_t st)
{
    RowsArgs a{};
    a.src = p.src; a.codes = p.codes; a.scales = p.scales; a.ema = ema;
    a.ld = p.ld; a.cpr = (uint32_t)(p.cols / 8); a.total = (uint32_t)(p.rows * (p.cols / 8));
    a.contiguous = p.ld == p.cols; a.floor_mode = p.floor_mode;
    a.beta = beta; a.update_ema = update_ema;
    dim3 grid((a.total + ROWS_THREADS - 1) / ROWS_THREADS), block(ROWS_THREADS);
    if (p.bf16) hipLaunchKernelGGL((ema_quantize_kernel<uint16_t>), grid, block, 0, st, a);
    else        hipLaunchKernelGGL((ema_quantize_kernel<float>), grid, block, 0, st, a);
    return hipGetLastError();
}

template <int SRC, bool FL, bool CS>
static void launch_tile_flags(const TileBatch& a, bool row_sr, bool t_sr, dim3 grid, hipStream_t st)
{
    dim3 block(TILE_THREADS);
    if (row_sr) {
        if (t_sr) hipLaunchKernelGGL((quantize_tile_kernel<SRC, true, true, FL, CS>), grid, block, 0, st, a);
        else      hipLaunchKernelGGL((quantize_tile_kernel<SRC, true, false, FL, CS>), grid, block, 0, st, a);
    } else {
        if (t_sr) hipLaunchKernelGGL((quantize_tile_kernel<SRC, false, true, FL, CS>), grid, block, 0, st, a);
        else      hipLaunchKernelGGL((quantize_tile_kernel<SRC, false, false, FL, CS>), grid, block, 0, st, a);
    }
}

template <int SRC, bool FL>
static void launch_tile_src(const TileBatch& a, bool row_sr, bool t_sr, bool col_sums, dim3 grid, hipStream_t st)
{
    if (SRC != 2 && col_sums) launch_tile_flags<SRC, FL, (SRC != 2)>(a, row_sr, t_sr, grid, st);
    else                      launch_tile_flags<SRC, FL, false>(a, row_sr, t_sr, grid, st);
}

// Fills the kernel arguments of one tensor; returns its number of workgroups.
static uint32_t make_tile_args(const QuantTileParams& p, TileArgs& a)
{
    a = TileArgs{};
    a.src = p.src; a.row_codes_in = p.row_codes_in; a.row_scales_in = p.row_scales_in;
    a.codes_t = p.codes_t; a.scales_t = p.scales_t; a.codes_row = p.codes_row; a.scales_row = p.scales_row;
    a.ld = p.ld; a.rows = (uint32_t)p.rows; a.cols = (uint32_t)p.cols;
    a.pre_quant = p.pre_quant;
    a.k0 = (uint32_t)p.seed; a.k1 = (uint32_t)(p.seed >> 32);
    a.seed_dev = reinterpret_cast<const uint32_t*>(p.seed_dev);
    a.col_sum_partials = p.col_sums ? p.col_sum_workspace : nullptr;
    a.tensor_id_t = p.tensor_id_t; a.tensor_id_row = p.tensor_id_row; a.index_base = p.index_base;
    // Macro tile of a workgroup (8 waves): 256 rows x 128 columns (whole 128-byte lines of the
    // transposed codes, 64-byte pieces of the row codes; measured a few percent faster than
    // 256 x 256), 256 x 64 for small tensors such as weights, where latency counts.
    // Two workgroups fit a compute unit (LDS), so 512 run at a time and a launch proceeds in rounds
    // of 512 equal tiles.  When the last round would be less than half full, its tiles are issued as
    // their 256 x 64 halves: twice the workgroups, half the time, and the round ends earlier.
    const uint32_t wide_per_row = (uint32_t)((p.cols + 127) / 128);
    const uint32_t n_tiles = (uint32_t)((p.rows + 255) / 256) * wide_per_row;
    const int64_t tiles32 = (p.rows / 32) * ((p.cols + 63) / 64);
    uint32_t n_wide = 0;
    if (tiles32 >= 8192) {
        const uint32_t rem = n_tiles % 512u;
        n_wide = (rem > 0u && rem <= 256u) ? n_tiles - rem : n_tiles;
    }
    a.n_wide = n_wide; a.wide_per_row = wide_per_row;
    return n_wide + 2u * (n_tiles - n_wide);
}

hipError_t launch_quantize_tile_batch(const QuantTileParams* jobs, int count, hipStream_t st)
{
    if (count < 1 || count > TILE_BATCH_MAX) return hipErrorInvalidValue;
    const QuantTileParams& p = jobs[0];
    const bool row_sr = p.row_codes_in ? false : p.sr_row;
    TileBatch b{};
    uint32_t blocks = 0;
    bool col_sums = false;
    for (int j = 0; j < TILE_BATCH_MAX; ++j) {
        b.first[j] = 0xFFFFFFFFu;
        if (j >= count) continue;
        const QuantTileParams& q = jobs[j];
        // one kernel instance serves the launch: source kind, roundings and scale rule are shared
        if ((q.row_codes_in != nullptr) != (p.row_codes_in != nullptr) || q.bf16 != p.bf16 || q.sr_t != p.sr_t ||
            (q.row_codes_in ? false : q.sr_row) != row_sr || q.floor_mode != p.floor_mode)
            return hipErrorInvalidValue;
        b.first[j] = blocks;
        blocks += make_tile_args(q, b.job[j]);
        col_sums = col_sums || q.col_sums != nullptr;
    }
    dim3 grid(blocks);
    if (p.floor_mode) {
        if (p.row_codes_in)  launch_tile_src<2, true>(b, row_sr, p.sr_t, col_sums, grid, st);
        else if (p.bf16)     launch_tile_src<1, true>(b, row_sr, p.sr_t, col_sums, grid, st);
        else                 launch_tile_src<0, true>(b, row_sr, p.sr_t, col_sums, grid, st);
    } else {
        if (p.row_codes_in)  launch_tile_src<2, false>(b, row_sr, p.sr_t, col_sums, grid, st);
        else if (p.bf16)     launch_tile_src<1, false>(b, row_sr, p.sr_t, col_sums, grid, st);
        else                 launch_tile_src<0, false>(b, row_sr, p.sr_t, col_sums, grid, st);
    }
    hipError_t e = hipGetLastError();
    for (int j = 0; j < count && e == hipSuccess; ++j) {
        const QuantTileParams& q = jobs[j];
        if (!q.col_sums) continue;
        hipLaunchKernelGGL(column_sum_finish_kernel, dim3((unsigned)((q.cols + 31) / 32)), dim3(256), 0, st,
                           q.col_sum_workspace, (uint32_t)((q.rows + 255) / 256), (uint32_t)q.cols, q.col_sums);
        e = hipGetLastError();
    }
    return e;
}

size_t column_sum_workspace_bytes(int64_t rows, int64_t cols)
{
    return (size_t)((rows + 255) / 256) * (size_t)cols * sizeof(float);
}

hipError_t launch_quantize_tile(const QuantTileParams& p, hipStream_t st)
{
    return launch_quantize_tile_batch(&p, 1, st);
}

hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t st)
{
    size_t n = bytes / 16;
    size_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(calibration_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                       static_cast<const uint4*>(src), static_cast<uint4*>(dst), n);
    return hipGetLastError();
}

hipError_t launch_oscillation(const OscillationParams& p, hipStream_t st)
{
    OscArgs a{};
    a.w = p.w; a.codes = p.codes; a.scales = p.scales; a.w_prev = p.w_prev;
    a.codes_prev = p.codes_prev; a.scales_prev = p.scales_prev; a.dist_w = p.dist_w; a.dist_q = p.dist_q;
    a.ld = p.ld; a.cpr = (uint32_t)(p.cols / 8); a.total = (uint32_t)(p.rows * (p.cols / 8)); a.init = p.init;
    dim3 grid((a.total + ROWS_THREADS - 1) / ROWS_THREADS), block(ROWS_THREADS);
    if (p.bf16) hipLaunchKernelGGL(oscillation_kernel<uint16_t>, grid, block, 0, st, a);
    else        hipLaunchKernelGGL(oscillation_kernel<float>, grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_confidence(const ConfidenceParams& p, hipStream_t st)
{
    ConfArgs a{};
    a.w = p.w; a.conf = p.conf; a.hist = reinterpret_cast<unsigned long long*>(p.hist); a.ld = p.ld;
    a.cpr = (uint32_t)(p.cols / 8); a.total = (uint32_t)(p.rows * (p.cols / 8));
    a.bins = p.hist ? p.bins : 0; a.floor_mode = p.floor_mode;
    // at most one workgroup per compute unit: each one flushes its histogram to memory once
    uint32_t blocks = (a.total + ROWS_THREADS - 1) / ROWS_THREADS;
    dim3 grid(blocks < 256u ? blocks : 256u), block(ROWS_THREADS);
    if (p.bf16) hipLaunchKernelGGL(confidence_kernel<uint16_t>, grid, block, 0, st, a);
    else        hipLaunchKernelGGL(confidence_kernel<float>, grid, block, 0, st, a);
    return hipGetLastError();
}

size_t rate_workspace_bytes() { return (size_t)RATE_BLOCKS * 2 * sizeof(double); }

hipError_t launch_rate_of_change(const RateParams& p, hipStream_t st)
{
    RateArgs a{};
    a.x = p.x; a.x_prev = p.x_prev; a.partial = p.partial; a.ld = p.ld;
    a.cpr = (uint32_t)(p.cols / 8); a.total = (uint32_t)(p.rows * (p.cols / 8)); a.init = p.init;
    dim3 grid(RATE_BLOCKS), block(ROWS_THREADS);
    if (p.bf16) hipLaunchKernelGGL(rate_partial_kernel<uint16_t>, grid, block, 0, st, a);
    else        hipLaunchKernelGGL(rate_partial_kernel<float>, grid, block, 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rate_finish_kernel, dim3(1), block, 0, st, p.partial, p.init, p.result);
    return hipGetLastError();
}

hipError_t launch_ramping_factor(const float* dist_w, const float* dist_q, int64_t count, float k1, int k2,
                                 int n_max, int32_t* factor, hipStream_t st)
{
    dim3 grid((unsigned)((count + 255) / 256)), block(256);
    hipLaunchKernelGGL(ramping_factor_kernel, grid, block, 0, st, dist_w, dist_q, count, k1, k2, n_max, factor);
    return hipGetLastError();
}

hipError_t launch_dequantize(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t cols,
                             float* out, hipStream_t st)
{
    int64_t total = rows * (cols / 2);
    dim3 grid((unsigned)((total + 255) / 256)), block(256);
    hipLaunchKernelGGL(dequantize_kernel, grid, block, 0, st, codes, scales, total, cols, out);
    return hipGetLastError();
}

}  // namespace mxl

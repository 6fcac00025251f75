// C[m x n] = A[m x k] . B[n x k]^T on packed MXFP4 operands, FP32 accumulation on gfx950's
// block-scaled FP4 matrix cores.  All three products of the layer (Eqs. 3-5, Sec. 3.3) have
// this form because every operand is stored along its own contraction dimension.
//
// Three kernels, chosen by the launcher at the end of the file:
//   mx_gemm_pingpong_kernel  the main path (K a multiple of 128, at least 4 K steps per K split;
//       every ViT-B/L product): V_MFMA_SCALE_F32_32X32X64_F8F6F4, one persistent workgroup of
//       8 waves per compute unit, tile 256 x 256, operands global -> LDS by DMA loads, two wave
//       groups alternating between their MFMA burst and their LDS/DMA work.  Described in full
//       above the kernel.
//   mx_gemm_dma_kernel       K a multiple of 128 but fewer than 4 K steps per split: same MFMA and
//       LDS layout, 4 waves, tile 256 x 128, one tile per workgroup.
//   mx_gemm_kernel           any K that is a multiple of 32 (e.g. 192): V_MFMA_SCALE_F32_16X16X128_F8F6F4,
//       register-staged loads, zero-filled K tail.
// A K-split product (dW: K = tokens, small output) writes FP32 partials to the caller's workspace
// and splitk_reduce*_kernel adds them in a fixed order.
//
// Common to all three:
//   - K step 128 = 64 bytes of codes and 4 scale bytes per row;
//   - an MFMA consumes, per lane, 32 consecutive K elements (16 bytes, exactly one MX group) of
//     one row and that group's E8M0 scale byte (16x16x128: row lane % 16, K block lane / 16;
//     32x32x64: row lane % 32, K block lane / 32);
//   - code tiles sit in LDS row-major with the 16-byte chunk index XOR-swizzled by (row >> 2) & 3,
//     so that both the 16-byte writes (4 lanes per row) and the MFMA operand reads (one chunk of
//     16 or 32 rows) are bank-conflict free;
//   - the MFMA's first operand is the B (n) side, so that a lane ends up with runs of four
//     consecutive n of one m and stores 8 or 16 contiguous bytes.
#include "mx_device.hpp"
#include "mx_launch.hpp"

#include <type_traits>

// Timing hooks for instrumented builds of this file (a build that defines them before including it);
// they expand to nothing in the library.
#ifndef MX_PROBE
#define MX_PROBE_INIT
#define MX_PROBE(id)
#endif

namespace {

// compile-time loop: the MFMA's op_sel (which scale byte) must be an immediate
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

struct GemmArgs {
    const uint8_t* a_codes;
    const uint8_t* a_scales;
    const uint8_t* b_codes;
    const uint8_t* b_scales;
    uint32_t m, n, k;        // k in elements
    uint32_t k_per_split;    // multiple of 128
    void* c;                 // final output, or FP32 partials [split][m][n] when split_k > 1
    int64_t ldc;
    int c_bf16;
    int split_k;
    uint32_t tiles_m, tiles_n;
    int stagger;             // start delay of every other workgroup of an XCD, in s_sleep(32) units
    const float* bias;       // n values added to every row of a final output (n % 4 == 0), or null
    uint8_t* q_codes;        // fused GELU + 1x32 quantizer of the output rows (main kernel only): packed codes
    uint8_t* q_scales;       //   [m x n/2] and scale bytes [m x n/32] of Q(GELU(product + bias)), or null
    int q_floor;             //   its scale rule: 0 truncation-free, 1 Eq. 2
};

constexpr int KSTEP_BYTES = 64;     // 128 FP4 elements

__device__ __forceinline__ uint32_t lds_code_offset(uint32_t row, uint32_t chunk)
{
    return row * KSTEP_BYTES + ((chunk ^ ((row >> 2) & 3u)) << 4);
}

__device__ __forceinline__ uint32_t lds_scale_offset(uint32_t row, uint32_t kb, uint32_t tile_rows)
{
    // [kb][row tile / 4][row % 16][row tile % 4]
    uint32_t tile = row >> 4;
    return kb * tile_rows + (tile >> 2) * 64 + (row & 15u) * 4 + (tile & 3u);
}

// FP32 -> bf16, round to nearest even, with gfx950's packed convert instruction.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi)
{
    f32x2_t v = {lo, hi};
    bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return *reinterpret_cast<uint32_t*>(&b);
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    return (uint16_t)f32x2_to_bf16x2(f, 0.f);
}

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64)
void mx_gemm_kernel(GemmArgs g)
{
    constexpr int WAVES_N = BN / WN;
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int A_CHUNKS = BM * 4 / NT, B_CHUNKS = BN * 4 / NT;
    static_assert(BM * 4 % NT == 0 && BN * 4 % NT == 0, "tile/thread mismatch");
    static_assert(TM % 4 == 0 && TN % 4 == 0, "scale packing needs 4 tiles per dword");
    static_assert(BM + BN <= NT * 2, "scale loader covers at most 2 rows per thread");

    __shared__ __attribute__((aligned(16))) uint8_t lds_a[2][BM * KSTEP_BYTES];
    __shared__ __attribute__((aligned(16))) uint8_t lds_b[2][BN * KSTEP_BYTES];
    __shared__ __attribute__((aligned(16))) uint8_t lds_sa[2][BM * 4];
    __shared__ __attribute__((aligned(16))) uint8_t lds_sb[2][BN * 4];

    // ---- which tile: give each XCD (workgroup id % 8) a contiguous range of tiles,
    //      consecutive tiles sharing the same A row panel ----
    const uint32_t nblk = g.tiles_m * g.tiles_n;
    uint32_t bid = blockIdx.x;
    {
        uint32_t per = nblk / 8, rem = nblk % 8;
        uint32_t xcd = bid % 8, idx = bid / 8;
        bid = xcd * per + (xcd < rem ? xcd : rem) + idx;   // bijection on [0, nblk)
    }
    const uint32_t tm = bid / g.tiles_n, tn = bid % g.tiles_n;
    const uint32_t m0 = tm * BM, n0 = tn * BN;
    const uint32_t kbeg = blockIdx.z * g.k_per_split;
    const uint32_t kend = min(g.k, kbeg + g.k_per_split);
    const uint32_t nk = (kend - kbeg + 127) / 128;
    const uint32_t kbytes = g.k >> 1, kgroups = g.k >> 5;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // ---- global -> register staging ----
    v4i ra[A_CHUNKS], rb[B_CHUNKS];
    uint32_t rs[2];                         // scale dwords (rows tid and tid + NT)

    auto gload = [&](uint32_t kt) {
        const uint32_t k0 = kbeg + kt * 128;
#pragma unroll
        for (int u = 0; u < A_CHUNKS; ++u) {
            uint32_t q = tid + u * NT, row = q >> 2, ch = q & 3;
            bool ok = (m0 + row < g.m) && (k0 + ch * 32 < kend);
            ra[u] = ok ? *reinterpret_cast<const v4i*>(g.a_codes + (size_t)(m0 + row) * kbytes + (k0 >> 1) + ch * 16)
                       : v4i{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < B_CHUNKS; ++u) {
            uint32_t q = tid + u * NT, row = q >> 2, ch = q & 3;
            bool ok = (n0 + row < g.n) && (k0 + ch * 32 < kend);
            rb[u] = ok ? *reinterpret_cast<const v4i*>(g.b_codes + (size_t)(n0 + row) * kbytes + (k0 >> 1) + ch * 16)
                       : v4i{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            int row = tid + u * NT;
            rs[u] = 0x7F7F7F7Fu;            // scale 2^0 for rows / groups outside the matrix (their codes are 0)
            if (row < BM + BN) {
                bool is_a = row < BM;
                uint32_t r = is_a ? m0 + row : n0 + (row - BM);
                uint32_t lim = is_a ? g.m : g.n;
                const uint8_t* sp = (is_a ? g.a_scales : g.b_scales) + (size_t)r * kgroups + (k0 >> 5);
                if (r < lim) {
                    if (k0 + 128 <= kend && (kgroups & 3u) == 0) {
                        rs[u] = *reinterpret_cast<const uint32_t*>(sp);
                    } else {
                        uint32_t v = 0;
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            uint32_t s = (k0 + b * 32 < kend) ? sp[b] : 0x7Fu;
                            v |= s << (8 * b);
                        }
                        rs[u] = v;
                    }
                }
            }
        }
    };

    auto lstore = [&](int buf) {
#pragma unroll
        for (int u = 0; u < A_CHUNKS; ++u) {
            uint32_t q = tid + u * NT;
            *reinterpret_cast<v4i*>(&lds_a[buf][lds_code_offset(q >> 2, q & 3)]) = ra[u];
        }
#pragma unroll
        for (int u = 0; u < B_CHUNKS; ++u) {
            uint32_t q = tid + u * NT;
            *reinterpret_cast<v4i*>(&lds_b[buf][lds_code_offset(q >> 2, q & 3)]) = rb[u];
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            int row = tid + u * NT;
            if (row < BM + BN) {
                bool is_a = row < BM;
                uint32_t r = is_a ? row : row - BM;
                uint8_t* dst = is_a ? lds_sa[buf] : lds_sb[buf];
                uint32_t tr = is_a ? BM : BN;
#pragma unroll
                for (int b = 0; b < 4; ++b) dst[lds_scale_offset(r, b, tr)] = (uint8_t)(rs[u] >> (8 * b));
            }
        }
    };

    v4f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    const uint32_t lrow = lane & 15, lkb = lane >> 4;

    auto compute = [&](int buf) {
        v4i fa[TM], fb[TN];
        uint32_t sa[TM / 4], sb[TN / 4];
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[i] = *reinterpret_cast<const v4i*>(&lds_a[buf][lds_code_offset(wm * WM + i * 16 + lrow, lkb)]);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[j] = *reinterpret_cast<const v4i*>(&lds_b[buf][lds_code_offset(wn * WN + j * 16 + lrow, lkb)]);
#pragma unroll
        for (int i = 0; i < TM / 4; ++i)
            sa[i] = *reinterpret_cast<const uint32_t*>(&lds_sa[buf][lkb * BM + ((wm * WM) / 64 + i) * 64 + lrow * 4]);
#pragma unroll
        for (int j = 0; j < TN / 4; ++j)
            sb[j] = *reinterpret_cast<const uint32_t*>(&lds_sb[buf][lkb * BN + ((wn * WN) / 64 + j) * 64 + lrow * 4]);
        static_for<0, TM>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            v8i xa = v8i{fa[i].x, fa[i].y, fa[i].z, fa[i].w, 0, 0, 0, 0};
            static_for<0, TN>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                v8i xb = v8i{fb[j].x, fb[j].y, fb[j].z, fb[j].w, 0, 0, 0, 0};
                // first operand = n side (B rows), second = m side (A rows)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                    xb, xa, acc[i][j], 4, 4, j & 3, (int)sb[j >> 2], i & 3, (int)sa[i >> 2]);
            });
        });
    };

    if (nk > 0) {
        gload(0);
        lstore(0);
    }
    __syncthreads();
    for (uint32_t kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) gload(kt + 1);
        compute(cur);
        if (more) lstore(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds C[m = .. + lane%16][n = .. + 4*(lane/16) + 0..3] ----
    float* cf = static_cast<float*>(g.c);
    uint16_t* ch = static_cast<uint16_t*>(g.c);
    int64_t ldc = g.ldc;
    if (g.split_k > 1) {
        cf += (size_t)blockIdx.z * g.m * g.n;
        ldc = g.n;
    }
    const bool as_bf16 = g.c_bf16 && g.split_k == 1;
    const bool vec_ok = (ldc & 3) == 0;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const uint32_t mm = m0 + wm * WM + i * 16 + lrow;
        if (mm >= g.m) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const uint32_t nn = n0 + wn * WN + j * 16 + lkb * 4;
            if (nn >= g.n) continue;
            v4f v = acc[i][j];
            if (g.bias) v += *reinterpret_cast<const v4f*>(g.bias + nn);      // nn + 3 < n: n is a multiple of 4
            size_t off = (size_t)mm * ldc + nn;
            if (nn + 3 < g.n && vec_ok) {
                if (as_bf16) {
                    uint2 pk;
                    pk.x = f32x2_to_bf16x2(v.x, v.y);
                    pk.y = f32x2_to_bf16x2(v.z, v.w);
                    *reinterpret_cast<uint2*>(ch + off) = pk;
                } else {
                    *reinterpret_cast<float4*>(cf + off) = make_float4(v.x, v.y, v.z, v.w);
                }
            } else {
                float e[4] = {v.x, v.y, v.z, v.w};
                for (int r = 0; r < 4; ++r)
                    if (nn + r < g.n) {
                        if (as_bf16) ch[off + r] = f32_to_bf16_rne(e[r]);
                        else         cf[off + r] = e[r];
                    }
            }
        }
    }
}

// Sum the split-K partials in a fixed order and write the final output.
__global__ void splitk_reduce_kernel(const float* part, int split, uint32_t m, uint32_t n,
                                     void* c, int64_t ldc, int c_bf16, const float* bias)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)m * n;
    if (idx >= total) return;
    float s = 0.f;
    for (int z = 0; z < split; ++z) s += part[(size_t)z * total + idx];
    uint32_t r = (uint32_t)(idx / n), col = (uint32_t)(idx - (size_t)r * n);
    if (bias) s += bias[col];
    if (c_bf16) static_cast<uint16_t*>(c)[(size_t)r * ldc + col] = f32_to_bf16_rne(s);
    else        static_cast<float*>(c)[(size_t)r * ldc + col] = s;
}

// The same for n % 4 == 0 and 16-byte aligned rows of the output: four columns per thread, the
// partial loads of a thread issued back to back (same summation order per element).
__global__ void splitk_reduce4_kernel(const float* part, int split, uint32_t m, uint32_t n,
                                      void* c, int64_t ldc, int c_bf16, const float* bias)
{
    const size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x;       // index of a group of 4 columns
    const size_t total = (size_t)m * n;
    if (q * 4 >= total) return;
    const float4* p4 = reinterpret_cast<const float4*>(part) + q;
    const size_t zstride = total / 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    int z = 0;
    for (; z + 4 <= split; z += 4) {
        const float4 a = p4[(size_t)z * zstride], b = p4[(size_t)(z + 1) * zstride];
        const float4 d = p4[(size_t)(z + 2) * zstride], e = p4[(size_t)(z + 3) * zstride];
        s.x = (((s.x + a.x) + b.x) + d.x) + e.x;
        s.y = (((s.y + a.y) + b.y) + d.y) + e.y;
        s.z = (((s.z + a.z) + b.z) + d.z) + e.z;
        s.w = (((s.w + a.w) + b.w) + d.w) + e.w;
    }
    for (; z < split; ++z) {
        const float4 a = p4[(size_t)z * zstride];
        s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
    }
    const size_t idx = q * 4;
    const uint32_t r = (uint32_t)(idx / n), col = (uint32_t)(idx - (size_t)r * n);
    if (bias) {
        const float4 bv = *reinterpret_cast<const float4*>(bias + col);
        s.x += bv.x; s.y += bv.y; s.z += bv.z; s.w += bv.w;
    }
    if (c_bf16) {
        uint2 o;
        o.x = f32x2_to_bf16x2(s.x, s.y);
        o.y = f32x2_to_bf16x2(s.z, s.w);
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(c) + (size_t)r * ldc + col) = o;
    } else {
        *reinterpret_cast<float4*>(static_cast<float*>(c) + (size_t)r * ldc + col) = s;
    }
}

constexpr int G_BM = 256, G_BN = 256, G_WM = 128, G_WN = 64;

// ---------------------------------------------------------------------------
// Fast path (K a multiple of 128): V_MFMA_SCALE_F32_32X32X64_F8F6F4, operands
// streamed global -> LDS by the DMA form of the load instructions.
//
//   workgroup 256 threads = 4 waves stacked along m; tile 256 (m) x 128 (n); wave
//   tile 64 x 128 = 2 x 4 MFMA tiles of 32 x 32 (128 accumulator registers).
//   Two workgroups fit on a CU (LDS 78 KB, <= 256 VGPRs): while one is waiting for
//   its first loads, sitting at a barrier or storing its output, the other one
//   keeps the matrix cores busy.
//   One 32x32x64 MFMA takes, per lane, the 32 K elements (16 bytes) of row
//   lane % 32, K block lane / 32, and that group's scale byte.
//   A stage (K step of 128) holds A codes [256][64 B], B codes [128][64 B],
//   A scales [256][4 B], B scales [128][4 B]; three stages.  A DMA load of 16 bytes
//   per lane lands at lds_base + 16 * lane, so lane i of the load that covers 16
//   rows fetches row i / 4, 16-byte chunk (i % 4) ^ ((row >> 2) & 3): the tile sits
//   in LDS row-major with XOR-swizzled chunks and the MFMA operand reads (32 rows
//   of one chunk per half wave) are bank-conflict free.
//   Rows past the matrix edge read the last valid row instead (their products
//   land in output rows/columns that are never stored).
//   Per K step: wait for this wave's loads of the stage, barrier, issue the loads
//   of stage +2, 12 operand reads + 16 MFMAs.
//   Epilogue: accumulators go through a per-wave LDS strip so that every global
//   store is 16 bytes per lane and whole 256/512-byte row segments per wave.
// ---------------------------------------------------------------------------
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int D_BM = 256, D_BN = 128, D_STAGES = 3, D_NT = 256, D_WAVES = 4;
constexpr int D_A_OFF = 0;
constexpr int D_B_OFF = D_BM * 64;                          // 16384
constexpr int D_SA_OFF = (D_BM + D_BN) * 64;                // 24576
constexpr int D_SB_OFF = D_SA_OFF + D_BM * 4;               // 25600
constexpr int D_STAGE_BYTES = D_SB_OFF + D_BN * 4;          // 26112
constexpr int D_LDS_BYTES = D_STAGES * D_STAGE_BYTES;       // 78336: two workgroups per CU
constexpr int D_LOADS_PER_STAGE = 8;                        // per wave: 4 A + 2 B code loads, 2 scale loads
constexpr int D_EP_PITCH_F32 = 528, D_EP_PITCH_BF16 = 264;  // bytes per 128-column strip row, padded
constexpr int D_EP_BYTES = 32 * D_EP_PITCH_F32;             // per wave
static_assert(D_WAVES * D_EP_BYTES <= D_LDS_BYTES, "epilogue strips must fit in the stage buffers");

#define MX_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define MX_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// Bias of four consecutive output columns starting at `col` (a multiple of 4), zero when there is no
// bias or the columns lie beyond n.
__device__ __forceinline__ v4f bias_of_columns(const GemmArgs& g, uint32_t col)
{
    if (g.bias != nullptr && col < g.n) return *reinterpret_cast<const v4f*>(g.bias + col);
    return v4f{0.f, 0.f, 0.f, 0.f};
}

// Accumulators -> per-wave LDS strip (32 rows x 128 columns) -> global, so that every
// store is 16 bytes per lane and a wave writes whole row segments.  The LDS region must
// no longer be in use by any wave of the workgroup.  The wave owns output rows
// [mrow0, mrow0 + 64) and columns [nbase, nbase + 128).
__device__ __forceinline__ void gemm_epilogue_32x32(const GemmArgs& g, uint8_t* ep, v16f (&acc)[2][4],
                                                    uint32_t mrow0, uint32_t nbase, int lane, uint32_t zsplit)
{
    const uint32_t lrow = lane & 31, lhalf = lane >> 5;
    float* cf = static_cast<float*>(g.c);
    uint16_t* ch = static_cast<uint16_t*>(g.c);
    int64_t ldc = g.ldc;
    if (g.split_k > 1) {
        cf += (size_t)zsplit * g.m * g.n;
        ldc = g.n;
    }
    const bool as_bf16 = g.c_bf16 && g.split_k == 1;
    if (as_bf16) {
        const bool vec_ok = (ldc & 7) == 0 && (reinterpret_cast<uintptr_t>(ch) & 15) == 0;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const v4f bv = bias_of_columns(g, nbase + 32 * j + 8 * q + 4 * lhalf);
                    uint2 pk;
                    pk.x = f32x2_to_bf16x2(acc[i][j][4 * q] + bv.x, acc[i][j][4 * q + 1] + bv.y);
                    pk.y = f32x2_to_bf16x2(acc[i][j][4 * q + 2] + bv.z, acc[i][j][4 * q + 3] + bv.w);
                    *reinterpret_cast<uint2*>(ep + lrow * D_EP_PITCH_BF16 + (32 * j + 8 * q + 4 * lhalf) * 2) = pk;
                }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const uint32_t row = it * 4 + (lane >> 4), col = (lane & 15) * 8;
                const uint32_t mm = mrow0 + i * 32 + row, nn = nbase + col;
                uint4 v = *reinterpret_cast<const uint4*>(ep + row * D_EP_PITCH_BF16 + col * 2);
                if (mm < g.m && nn < g.n) {
                    uint16_t* dst = ch + (size_t)mm * ldc + nn;
                    if (nn + 8 <= g.n && vec_ok) {
                        *reinterpret_cast<uint4*>(dst) = v;
                    } else {
                        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
                        for (int e = 0; e < 8; ++e)
                            if (nn + e < g.n) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                    }
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    } else {
        const bool vec_ok = (ldc & 3) == 0 && (reinterpret_cast<uintptr_t>(cf) & 15) == 0;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const v4f bv = bias_of_columns(g, nbase + 32 * j + 8 * q + 4 * lhalf);
                    *reinterpret_cast<float4*>(ep + lrow * D_EP_PITCH_F32 + (32 * j + 8 * q + 4 * lhalf) * 4) =
                        make_float4(acc[i][j][4 * q] + bv.x, acc[i][j][4 * q + 1] + bv.y, acc[i][j][4 * q + 2] + bv.z,
                                    acc[i][j][4 * q + 3] + bv.w);
                }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int it = 0; it < 16; ++it) {
                const uint32_t row = it * 2 + (lane >> 5), col = (lane & 31) * 4;
                const uint32_t mm = mrow0 + i * 32 + row, nn = nbase + col;
                float4 v = *reinterpret_cast<const float4*>(ep + row * D_EP_PITCH_F32 + col * 4);
                if (mm < g.m && nn < g.n) {
                    float* dst = cf + (size_t)mm * ldc + nn;
                    if (nn + 4 <= g.n && vec_ok) {
                        *reinterpret_cast<float4*>(dst) = v;
                    } else {
                        const float w[4] = {v.x, v.y, v.z, v.w};
                        for (int e = 0; e < 4; ++e)
                            if (nn + e < g.n) dst[e] = w[e];
                    }
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    }
}

// Workgroup -> (K split, tile).  The grid is one-dimensional over split * tiles.  Workgroup
// ids go round-robin over the 8 XCDs, each with its own L2, so id % 8 = XCD gets a
// contiguous range of the logical order (split, m tile, n tile): the workgroups that share
// an A row panel or a B panel of one K range run on the same XCD at about the same time.
__device__ __forceinline__ void decode_tile(const GemmArgs& g, uint32_t& zsplit, uint32_t& tm, uint32_t& tn)
{
    const uint32_t tiles = g.tiles_m * g.tiles_n, nblk = tiles * (uint32_t)g.split_k;
    uint32_t bid = blockIdx.x;
    uint32_t per = nblk / 8, rem = nblk % 8;
    uint32_t xcd = bid % 8, idx = bid / 8;
    bid = xcd * per + (xcd < rem ? xcd : rem) + idx;       // bijection on [0, nblk)
    zsplit = bid / tiles;
    uint32_t t = bid - zsplit * tiles;
    tm = t / g.tiles_n;
    tn = t - tm * g.tiles_n;
}

template <int N>
__device__ __forceinline__ void wait_vmcnt_then_barrier()
{
    // the memory clobber keeps LDS accesses on their side of the barrier
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

__global__ __launch_bounds__(D_NT, 2) void mx_gemm_dma_kernel(GemmArgs g)
{
    __shared__ __attribute__((aligned(1024))) uint8_t lds[D_LDS_BYTES];

    uint32_t zsplit, tm, tn;
    decode_tile(g, zsplit, tm, tn);
    const uint32_t m0 = tm * D_BM, n0 = tn * D_BN;
    const uint32_t kbeg = zsplit * g.k_per_split;
    const uint32_t kend = min(g.k, kbeg + g.k_per_split);
    const int nk = (int)((kend - kbeg) >> 7);
    const uint32_t kbytes = g.k >> 1, kgroups = g.k >> 5;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t lrow = lane & 31, lhalf = lane >> 5;
    const uint32_t swz = (lrow >> 2) & 3;

    // ---- DMA sources (per lane): wave w loads A rows [64w, 64w+64) and B rows [32w, 32w+32) ----
    const uint8_t* a_src[4];
    const uint8_t* b_src[2];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        uint32_t row = (4 * wave + u) * 16 + (lane >> 2);
        uint32_t ch = (lane & 3) ^ ((row >> 2) & 3);
        a_src[u] = g.a_codes + (size_t)min(m0 + row, g.m - 1) * kbytes + (kbeg >> 1) + ch * 16;
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        uint32_t row = (2 * wave + u) * 16 + (lane >> 2);
        uint32_t ch = (lane & 3) ^ ((row >> 2) & 3);
        b_src[u] = g.b_codes + (size_t)min(n0 + row, g.n - 1) * kbytes + (kbeg >> 1) + ch * 16;
    }
    const uint8_t* sa_src = g.a_scales + (size_t)min(m0 + wave * 64 + lane, g.m - 1) * kgroups + (kbeg >> 5);
    const uint8_t* sb_src = g.b_scales + (size_t)min(n0 + wave * 32 + lrow, g.n - 1) * kgroups + (kbeg >> 5);

    auto issue = [&](int buf, int kt) {
        uint8_t* base = lds + buf * D_STAGE_BYTES;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            __builtin_amdgcn_global_load_lds(MX_GPTR(a_src[u] + kt * 64), MX_LPTR(base + D_A_OFF + (4 * wave + u) * 1024), 16, 0, 0);
#pragma unroll
        for (int u = 0; u < 2; ++u)
            __builtin_amdgcn_global_load_lds(MX_GPTR(b_src[u] + kt * 64), MX_LPTR(base + D_B_OFF + (2 * wave + u) * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds(MX_GPTR(sa_src + kt * 4), MX_LPTR(base + D_SA_OFF + wave * 256), 4, 0, 0);
        if (lane < 32)      // 32 B rows per wave: the upper half wave sits this load out
            __builtin_amdgcn_global_load_lds(MX_GPTR(sb_src + kt * 4), MX_LPTR(base + D_SB_OFF + wave * 128), 4, 0, 0);
    };

    v16f acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Operand registers of one 64-K slice (one MFMA per accumulator tile) and the
    // scale dwords of one K step, already shifted so that op_sel 0 / 2 picks the byte.
    struct Frag { v4i a[2]; v4i b[4]; };
    struct Scales { uint32_t a[2]; uint32_t b[4]; };
    auto read_frag = [&](int buf, int kk, Frag& f) {
        const uint8_t* base = lds + buf * D_STAGE_BYTES;
        const uint32_t coff = ((2 * kk + lhalf) ^ swz) << 4;
#pragma unroll
        for (int i = 0; i < 2; ++i)
            f.a[i] = *reinterpret_cast<const v4i*>(base + D_A_OFF + (wave * 64 + i * 32 + lrow) * 64 + coff);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            f.b[j] = *reinterpret_cast<const v4i*>(base + D_B_OFF + (j * 32 + lrow) * 64 + coff);
    };
    auto read_scales = [&](int buf, Scales& sc) {
        const uint8_t* base = lds + buf * D_STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < 2; ++i)
            sc.a[i] = *reinterpret_cast<const uint32_t*>(base + D_SA_OFF + (wave * 64 + i * 32 + lrow) * 4);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            sc.b[j] = *reinterpret_cast<const uint32_t*>(base + D_SB_OFF + (j * 32 + lrow) * 4);
    };
    auto shift_scales = [&](Scales& sc) {
#pragma unroll
        for (int i = 0; i < 2; ++i) sc.a[i] >>= 8 * lhalf;
#pragma unroll
        for (int j = 0; j < 4; ++j) sc.b[j] >>= 8 * lhalf;
    };
    auto mma = [&](const Frag& f, const Scales& sc, auto kc) {
        constexpr int kk = decltype(kc)::value;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            v8i xa = v8i{f.a[i].x, f.a[i].y, f.a[i].z, f.a[i].w, 0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v8i xb = v8i{f.b[j].x, f.b[j].y, f.b[j].z, f.b[j].w, 0, 0, 0, 0};
                // first operand = n side, second = m side: a lane ends up with one m and runs of 4 n
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                    xb, xa, acc[i][j], 4, 4, 2 * kk, (int)sc.b[j], 2 * kk, (int)sc.a[i]);
            }
        }
    };

    // ---- main loop, software-pipelined by half K steps: the LDS reads of the next 64-K
    //      slice are issued before the 8 MFMAs of the current one ----
    // Three stages, two in flight: at the barrier in the middle of step kt every wave's reads of
    // stage kt have returned (lgkmcnt(0) before the barrier), so that buffer takes stage kt+3
    // while stage kt+2 is still on its way and stage kt+1 has just landed.
    if (nk > 0) issue(0, 0);
    if (nk > 1) issue(1, 1);
    if (nk > 2) issue(2, 2);
    if (nk > 2)      wait_vmcnt_then_barrier<2 * D_LOADS_PER_STAGE>();
    else if (nk > 1) wait_vmcnt_then_barrier<1 * D_LOADS_PER_STAGE>();
    else             wait_vmcnt_then_barrier<0>();
    Frag f0, f1;
    Scales sc, scn;
    read_scales(0, sc);
    read_frag(0, 0, f0);
    shift_scales(sc);
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt % D_STAGES;
        read_frag(cur, 1, f1);
        mma(f0, sc, std::integral_constant<int, 0>{});
        if (kt + 1 < nk) {
            // stage kt+1 must have landed; stage kt+2, if any, may stay in flight
            if (kt + 2 < nk) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(D_LOADS_PER_STAGE) : "memory");
            else             asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            if (kt + 3 < nk) issue(cur, kt + 3);
            const int nxt = (kt + 1) % D_STAGES;
            read_scales(nxt, scn);
            read_frag(nxt, 0, f0);
        }
        mma(f1, sc, std::integral_constant<int, 1>{});
        if (kt + 1 < nk) {
            shift_scales(scn);
            sc = scn;
        }
    }
    wait_vmcnt_then_barrier<0>();          // every wave is done reading the stage buffers

    gemm_epilogue_32x32(g, lds + wave * D_EP_BYTES, acc, m0 + wave * 64, n0, lane, zsplit);
}


// ---------------------------------------------------------------------------
// Helpers of the main path (K range of at least 512 per split; mx_gemm_pingpong_kernel below).
// ---------------------------------------------------------------------------

// No instruction is scheduled across this point.
#define MX_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

constexpr int P_EP_PITCH = 144;                              // output staging: 128 bytes of payload per row, padded
constexpr int P_EP_BYTES = 32 * P_EP_PITCH;                  // per wave

// Lane index within the wave, computed anew at each use (two VALU instructions): code that
// needs lane-derived values once per tile does not hold registers for them across the K loop.
__device__ __forceinline__ uint32_t fresh_lane_id()
{
    uint32_t l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}

// Accumulators of one wave (64 rows x 128 columns) -> global through a 32-row LDS strip
// holding 128 bytes per row: 64 bf16 or 32 fp32 columns at a time.  A store instruction
// of the wave covers 8 whole 128-byte row segments.
// 16-byte store.  A final output is written with the nontemporal hint: it is not read again
// here, and without the hint an output larger than the last-level cache slows the whole kernel
// down while it drains (split-K partials keep the default policy, the reduction reads them).
template <bool STREAM>
__device__ __forceinline__ void store16(void* dst, v4i v)
{
    if (STREAM) __builtin_nontemporal_store(v, reinterpret_cast<v4i*>(dst));
    else        *reinterpret_cast<v4i*>(dst) = v;
}

typedef __attribute__((address_space(3))) uint8_t lds_u8;
typedef int v2i __attribute__((ext_vector_type(2)));

// The same output stage for a wave tile that lies wholly inside the matrix and whose rows can be
// stored 16 bytes at a time (the common case; every tile of a ViT-B product): no bounds tests, no
// per-store address arithmetic (a store's address is a uniform tile pointer plus one per-lane
// offset that is computed once), and no waits between the LDS writes and reads of a chunk (the LDS
// executes a wave's instructions in order; the compiler waits where a register needs its data).
// BIAS: add the 128 FP32 bias values at LDS address `bias` (column nbase first).
template <bool STREAM, bool BIAS>
__device__ __forceinline__ void gemm_epilogue_interior(const GemmArgs& g, lds_u8* ep, v16f (&acc)[2][4],
                                                       uint32_t mrow0, uint32_t nbase, uint32_t zsplit, int64_t ldc,
                                                       const lds_u8* bias)
{
    typedef __attribute__((address_space(3))) v4i lds_v4i;
    typedef __attribute__((address_space(3))) v2i lds_v2i;
    typedef __attribute__((address_space(3))) v4f lds_v4f;
    const uint32_t lane = fresh_lane_id();
    const uint32_t lrow = lane & 31, lhalf = lane >> 5;
    const uint32_t rrow = lane >> 3, rchunk = lane & 7;
    const lds_u8* rd = ep + rrow * P_EP_PITCH + rchunk * 16;
    auto bias4 = [&](int jb, int q) -> v4f {
        return *reinterpret_cast<const lds_v4f*>(bias + (32 * jb + 8 * q + 4 * lhalf) * 4);
    };
    // Four (bf16) or eight (FP32) chunks of 32 rows x 128 bytes pass through the wave's LDS strip.  The
    // strip's accesses execute in program order, so the writes of chunk c+1 are issued right after the
    // reads of chunk c and before the global stores that wait for those reads: the LDS round trip of a
    // chunk is hidden behind the next chunk's conversion instead of being waited for 16 times.
    if (g.c_bf16 && g.split_k == 1) {
        lds_u8* wr = ep + lrow * P_EP_PITCH + lhalf * 8;
        uint8_t* tile = static_cast<uint8_t*>(g.c) + ((size_t)mrow0 * ldc + nbase) * 2;       // uniform
        const uint32_t voff = rrow * (uint32_t)ldc * 2u + rchunk * 16u;
        auto write_chunk = [&](int i, int jp) {
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const v16f& a = acc[i][2 * jp + jj];
                    v2i pk;
                    if (BIAS) {
                        const v4f bv = bias4(2 * jp + jj, q);
                        pk.x = (int)f32x2_to_bf16x2(a[4 * q] + bv.x, a[4 * q + 1] + bv.y);
                        pk.y = (int)f32x2_to_bf16x2(a[4 * q + 2] + bv.z, a[4 * q + 3] + bv.w);
                    } else {
                        pk.x = (int)f32x2_to_bf16x2(a[4 * q], a[4 * q + 1]);
                        pk.y = (int)f32x2_to_bf16x2(a[4 * q + 2], a[4 * q + 3]);
                    }
                    *reinterpret_cast<lds_v2i*>(wr + (32 * jj + 8 * q) * 2) = pk;
                }
        };
        v4i v[4];
        write_chunk(0, 0);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int i = c >> 1, jp = c & 1;
#pragma unroll
            for (int it = 0; it < 4; ++it) v[it] = *reinterpret_cast<const lds_v4i*>(rd + it * 8 * P_EP_PITCH);
            if (c + 1 < 4) write_chunk((c + 1) >> 1, (c + 1) & 1);
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                uint8_t* dst = tile + ((size_t)(i * 32 + it * 8) * ldc + jp * 64) * 2;            // uniform
                store16<STREAM>(dst + voff, v[it]);
            }
        }
    } else {
        lds_u8* wr = ep + lrow * P_EP_PITCH + lhalf * 16;
        float* base = static_cast<float*>(g.c);
        if (g.split_k > 1) base += (size_t)zsplit * g.m * g.n;
        uint8_t* tile = reinterpret_cast<uint8_t*>(base) + ((size_t)mrow0 * ldc + nbase) * 4;
        const uint32_t voff = rrow * (uint32_t)ldc * 4u + rchunk * 16u;
        auto write_chunk = [&](int i, int j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                v4f o = v4f{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                if (BIAS) o += bias4(j, q);
                *reinterpret_cast<lds_v4f*>(wr + 8 * q * 4) = o;
            }
        };
        v4i v[4];
        write_chunk(0, 0);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int i = c >> 2, j = c & 3;
#pragma unroll
            for (int it = 0; it < 4; ++it) v[it] = *reinterpret_cast<const lds_v4i*>(rd + it * 8 * P_EP_PITCH);
            if (c + 1 < 8) write_chunk((c + 1) >> 2, (c + 1) & 3);
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                uint8_t* dst = tile + ((size_t)(i * 32 + it * 8) * ldc + j * 32) * 4;             // uniform
                store16<STREAM>(dst + voff, v[it]);
            }
        }
    }
}

// GELU(x) = x * Phi(x) with Phi(x) = erfc(-x / sqrt(2)) / 2 (the exact form, not the tanh approximation),
// FP32, branch-free, about 30 instructions.  With z = |x| / sqrt(2):
//     erfc(z) = exp(-z^2) * G(z),   G(z) = t * P8(t - t0),   t = 1 / (1 + z / 2),
// where P8 is a degree-8 fit of the scaled complementary error function over z in [0, 12.1] (relative error
// 4.4e-8 in exact arithmetic; coefficients from fit_gelu_erfcx.py beside the package's Python files).
// erfc keeps its relative accuracy in the negative tail, where 1 + erf would cancel; to keep it through the
// exponential, z^2 = x^2 / 2 is carried as an FP32 product and its exact remainder, and the exponent of two as
// a rounded product and its remainder, both folded in as first-order corrections.  Against the FP64 value the
// result is within 5.5e-7 |GELU(x)| (2^-18 is 3.8e-6) for every x where |GELU(x)| >= 2^-100, and below
// 2^-120 in absolute terms beyond (checked on 6e6 points by the fitting script's FP32 emulation).  |x| is
// clamped at 17 before squaring: erfc has long underflowed there, and no infinity can arise.
__device__ __forceinline__ float gelu_f32(float x)
{
    constexpr float T0 = 0.5709219574928284f;
    constexpr float C0 = 0.562385082244873f, C1 = 0.768385112285614f, C2 = 0.584431529045105f,
                    C3 = 0.09252145141363144f, C4 = -0.20070798695087433f, C5 = -0.058531392365694046f,
                    C6 = 0.11107011884450912f, C7 = 0.014878340996801853f, C8 = -0.05936833471059799f;
    constexpr float HALF_LOG2E_HI = 0.72134751f;                    // log2(e) / 2 rounded to FP32 ...
    constexpr float HALF_LOG2E_LO = (float)(0.72134752044448170368 - (double)HALF_LOG2E_HI);   // ... and what it lost
    const float ax = __builtin_fminf(__builtin_fabsf(x), 17.0f);
    const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(ax, 0.35355339059327376f, 1.0f));     // 1 / (1 + z / 2)
    const float w = t - T0;
    float g = C8;
    g = __builtin_fmaf(g, w, C7); g = __builtin_fmaf(g, w, C6); g = __builtin_fmaf(g, w, C5);
    g = __builtin_fmaf(g, w, C4); g = __builtin_fmaf(g, w, C3); g = __builtin_fmaf(g, w, C2);
    g = __builtin_fmaf(g, w, C1); g = __builtin_fmaf(g, w, C0);
    g = __fmul_rn(g, t);
    const float s = __fmul_rn(ax, ax);
    const float r = __builtin_fmaf(ax, ax, -s);                     // x^2 = s + r exactly
    const float yh = __fmul_rn(s, HALF_LOG2E_HI);
    float yl = __builtin_fmaf(s, HALF_LOG2E_HI, -yh);               // z^2 log2(e) = yh + yl + r log2(e) / 2 (to first order)
    yl = __builtin_fmaf(s, HALF_LOG2E_LO, yl);
    const float e = __builtin_amdgcn_exp2f(-yh);
    float c = __builtin_fmaf(yl, -0.69314718f, 1.0f);               // 2^-yl
    c = __builtin_fmaf(r, -0.5f, c);                                // exp(-r / 2)
    const float half_erfc = __fmul_rn(__fmul_rn(__fmul_rn(g, e), c), 0.5f);
    const float phi = x < 0.0f ? half_erfc : 1.0f - half_erfc;
    return __fmul_rn(x, phi);
}

// Second output stage of the fused forward product of an MLP's first layer: the next layer's forward
// quantizer Q(1) (Eq. 3; 1x32 groups along the output columns, which are the next layer's contraction
// dimension, round_D) applied to GELU(product + bias), from the FP32 accumulators.  Runs after the stage
// that stores the pre-activation and reuses the wave's LDS strip.
// A lane holds, of each 32 x 32 MFMA tile (i, j), 16 of the 32 columns of one row: the four runs
// 8q + 4 * lhalf + (0..3); the other 16 are in the lane 32 away.  Group maximum: the lane's 16 values, then one
// exchange with that lane.  The 16 codes of a lane are four 2-byte pieces of the group's 16 bytes; they go to
// the strip ([64 rows][64 B] codes, then [64 rows][4] scale bytes) and leave as 16-byte pieces, 64 contiguous
// bytes per row.  Rows beyond m and column groups beyond n (n % 32 == 0) are not stored.
template <bool FLOOR>
__device__ __forceinline__ void gemm_epilogue_gelu_quant(const GemmArgs& g, lds_u8* ep, v16f (&acc)[2][4],
                                                         uint32_t mrow0, uint32_t nbase, const lds_u8* bias)
{
    typedef __attribute__((address_space(3))) v4f lds_v4f;
    typedef __attribute__((address_space(3))) v4i lds_v4i;
    typedef __attribute__((address_space(3))) uint16_t lds_u16;
    typedef __attribute__((address_space(3))) uint32_t lds_u32;
    const uint32_t lane = fresh_lane_id();
    const uint32_t lrow = lane & 31, lhalf = lane >> 5;
    lds_u8* scale_strip = ep + 4096;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float v[16];
            uint32_t m = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const v4f bv = *reinterpret_cast<const lds_v4f*>(bias + (32 * j + 8 * q + 4 * lhalf) * 4);
                v[4 * q] = gelu_f32(acc[i][j][4 * q] + bv.x);
                v[4 * q + 1] = gelu_f32(acc[i][j][4 * q + 1] + bv.y);
                v[4 * q + 2] = gelu_f32(acc[i][j][4 * q + 2] + bv.z);
                v[4 * q + 3] = gelu_f32(acc[i][j][4 * q + 3] + bv.w);
                m = mxd::absmax3_bits(v[4 * q], v[4 * q + 1], m);
                m = mxd::absmax3_bits(v[4 * q + 2], v[4 * q + 3], m);
            }
            const auto sw = __builtin_amdgcn_permlane32_swap(m, m, false, false);
            m = sw[0] > sw[1] ? sw[0] : sw[1];
            const uint32_t byte = mxd::scale_byte(m, FLOOR);
            const int e = mxd::grid_exponent(byte);
            mxd::f32_round_toward_minus_inf();              // round_D's mode for inexact subnormal scalings
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t pk = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r) pk |= mxd::rtn_code<FLOOR>(v[4 * q + r], e) << (4 * r);
                *reinterpret_cast<lds_u16*>(ep + (i * 32 + lrow) * 64 + 16 * j + 4 * q + 2 * lhalf) = (uint16_t)pk;
            }
            mxd::f32_round_to_nearest_even();
            if (lhalf == 0) scale_strip[(i * 32 + lrow) * 4 + j] = (uint8_t)byte;
        }
    asm volatile("" ::: "memory");          // the strip is read back below through other lanes' addresses
    // codes: 4 lanes per row (one column group each), 16 rows per instruction
    const uint32_t half_n = g.n >> 1, grp_n = g.n >> 5;
    const uint32_t piece = lane & 3, prow = lane >> 2;
    const bool group_ok = nbase + 32 * piece < g.n;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const uint32_t row = it * 16 + prow;
        const v4i c = *reinterpret_cast<const lds_v4i*>(ep + row * 64 + piece * 16);
        if (group_ok && mrow0 + row < g.m)
            *reinterpret_cast<v4i*>(g.q_codes + (size_t)(mrow0 + row) * half_n + (nbase >> 1) + piece * 16) = c;
    }
    // scale bytes: one row per lane
    {
        const uint32_t sc = *reinterpret_cast<const lds_u32*>(scale_strip + lane * 4);
        if (mrow0 + lane < g.m) {
            uint8_t* dst = g.q_scales + (size_t)(mrow0 + lane) * grp_n + (nbase >> 5);
            if (nbase + 128 <= g.n && (grp_n & 3u) == 0u && (reinterpret_cast<uintptr_t>(g.q_scales) & 3u) == 0u) {
                *reinterpret_cast<uint32_t*>(dst) = sc;
            } else {
                for (uint32_t b = 0; b < 4; ++b)
                    if (nbase + 32 * b < g.n) dst[b] = (uint8_t)(sc >> (8 * b));
            }
        }
    }
}

// bias: LDS address of the bias value of column nbase (FP32, 128 values), or null.
template <bool STREAM>
__device__ __forceinline__ void gemm_epilogue_chunked(const GemmArgs& g, uint8_t* ep, v16f (&acc)[2][4],
                                                      uint32_t mrow0, uint32_t nbase, int lane_in, uint32_t zsplit,
                                                      const __attribute__((address_space(3))) uint8_t* bias)
{
    // bias of the four columns a lane holds in accumulator registers 4q..4q+3 of column block jb
    auto bias4 = [&](int jb, int q, uint32_t lhalf) -> v4f {
        if (bias == nullptr) return v4f{0.f, 0.f, 0.f, 0.f};
        return *reinterpret_cast<const __attribute__((address_space(3))) v4f*>(bias + (32 * jb + 8 * q + 4 * lhalf) * 4);
    };
    // lane-derived indices are recomputed at every call instead of living across the K loop
    (void)lane_in;
    const uint32_t lane = fresh_lane_id();
    const uint32_t lrow = lane & 31, lhalf = lane >> 5;
    const uint32_t rrow = lane >> 3, rchunk = lane & 7;
    float* cf = static_cast<float*>(g.c);
    uint16_t* ch = static_cast<uint16_t*>(g.c);
    int64_t ldc = g.ldc;
    if (g.split_k > 1) {
        cf += (size_t)zsplit * g.m * g.n;
        ldc = g.n;
    }
    const bool as_bf16 = g.c_bf16 && g.split_k == 1;
    if (as_bf16) {
        const bool vec_ok = (ldc & 7) == 0 && (reinterpret_cast<uintptr_t>(ch) & 15) == 0;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) {
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const v16f& a = acc[i][2 * jp + jj];
                        const v4f bv = bias4(2 * jp + jj, q, lhalf);
                        uint2 pk;
                        pk.x = f32x2_to_bf16x2(a[4 * q] + bv.x, a[4 * q + 1] + bv.y);
                        pk.y = f32x2_to_bf16x2(a[4 * q + 2] + bv.z, a[4 * q + 3] + bv.w);
                        *reinterpret_cast<uint2*>(ep + lrow * P_EP_PITCH + (32 * jj + 8 * q + 4 * lhalf) * 2) = pk;
                    }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const uint32_t row = it * 8 + rrow;
                    const uint32_t mm = mrow0 + i * 32 + row, nn = nbase + jp * 64 + rchunk * 8;
                    uint4 v = *reinterpret_cast<const uint4*>(ep + row * P_EP_PITCH + rchunk * 16);
                    if (mm < g.m && nn < g.n) {
                        uint16_t* dst = ch + (size_t)mm * ldc + nn;
                        if (nn + 8 <= g.n && vec_ok) {
                            store16<STREAM>(dst, v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w});
                        } else {
                            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
                            for (int e = 0; e < 8; ++e)
                                if (nn + e < g.n) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                        }
                    }
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
    } else {
        const bool vec_ok = (ldc & 3) == 0 && (reinterpret_cast<uintptr_t>(cf) & 15) == 0;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const v4f bv = bias4(j, q, lhalf);
                    *reinterpret_cast<float4*>(ep + lrow * P_EP_PITCH + (8 * q + 4 * lhalf) * 4) =
                        make_float4(acc[i][j][4 * q] + bv.x, acc[i][j][4 * q + 1] + bv.y, acc[i][j][4 * q + 2] + bv.z,
                                    acc[i][j][4 * q + 3] + bv.w);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const uint32_t row = it * 8 + rrow;
                    const uint32_t mm = mrow0 + i * 32 + row, nn = nbase + j * 32 + rchunk * 4;
                    float4 v = *reinterpret_cast<const float4*>(ep + row * P_EP_PITCH + rchunk * 16);
                    if (mm < g.m && nn < g.n) {
                        float* dst = cf + (size_t)mm * ldc + nn;
                        if (nn + 4 <= g.n && vec_ok) {
                            store16<STREAM>(dst, v4i{__float_as_int(v.x), __float_as_int(v.y), __float_as_int(v.z), __float_as_int(v.w)});
                        } else {
                            const float w[4] = {v.x, v.y, v.z, v.w};
                            for (int e = 0; e < 4; ++e)
                                if (nn + e < g.n) dst[e] = w[e];
                        }
                    }
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
    }
}

// ---------------------------------------------------------------------------
// Ping-pong form of the main path: one workgroup of 8 waves per CU, tile 256 x 256.
// Waves 0-3 (group 0) and 4-7 (group 1) own the left and right 128 columns; wave w and
// wave w+4 sit on the same SIMD.  Time is cut into slots separated by workgroup barriers.
// In every slot one group issues its 16 MFMAs of a K step (M phase) while the other group
// reads the operands of its next K step from LDS and issues DMA loads (L phase); then they
// swap.  The matrix pipe of a SIMD always has exactly one wave feeding it, and no LDS or
// DMA latency sits between two MFMA bursts of the same wave.
//   Per 256 x 256 x 128 step the CU loads 32 KB through L2 -> LDS instead of the 2 x 24 KB of
//   two 256 x 128 workgroups.
//   LDS: 3 code stages x 32 KB | 3 scale slots x [512 rows][16 B] | output staging 8 x 4.5 KB |
//        2 x 1 KB of bias values (the tile being multiplied and the one being loaded).
// Two cursors run over the workgroup's tile list.  The read cursor names the K step whose
// operands the next L phase reads; the issue cursor runs two stages ahead of it (also across
// tile boundaries) and names the stage the same L phase loads.  Stage q of a tile lives in
// buffer (global stage count) % 3, scale block j in slot (global block count) % 3.
// Safety of the ring: the L phase of step s reads stage s and overwrites the buffer of stage
// s-1, whose last readers (the other group's L phase of step s-1, and this group's) finished
// before the previous barrier.  Each wave ends an L phase with a wait for all loads it issued
// in earlier phases, so stage s+1 is complete, and visible after the barrier, before its first
// reader.  Scale block j of a tile is issued with stage 4j-1 (block 0 with stage 0), at least
// two steps before its first reader and after the last reader of the slot's previous block.
// ---------------------------------------------------------------------------
constexpr int Q_BM = 256, Q_BN = 256, Q_NT = 512, Q_WAVES = 8, Q_STAGES = 3;
constexpr int Q_STAGE_BYTES = (Q_BM + Q_BN) * 64;                       // 32768
constexpr int Q_SCALE_OFF = Q_STAGES * Q_STAGE_BYTES;                   // 98304
constexpr int Q_SCALE_SLOT = (Q_BM + Q_BN) * 16;                        // 8192
constexpr int Q_EP_OFF = Q_SCALE_OFF + 3 * Q_SCALE_SLOT;                // 122880
constexpr int Q_BIAS_OFF = Q_EP_OFF + Q_WAVES * P_EP_BYTES;             // 159744: two slots of 256 bias values
constexpr int Q_LDS_BYTES = Q_BIAS_OFF + 2 * 1024;                      // 161792
static_assert(Q_LDS_BYTES <= 160 * 1024, "one workgroup per CU");
constexpr unsigned Q_SLOTS = 256;

__device__ __forceinline__ void barrier_after_mfma(v16f (&acc)[2][4])
{
    // the accumulators pass through the statement: the MFMAs before it stay before it
    asm volatile("s_barrier"
                 : "+v"(acc[0][0]), "+v"(acc[0][1]), "+v"(acc[0][2]), "+v"(acc[0][3]),
                   "+v"(acc[1][0]), "+v"(acc[1][1]), "+v"(acc[1][2]), "+v"(acc[1][3])
                 :
                 : "memory");
}

// DMA load, 16 bytes per lane: lane i's bytes [base + voff, +16) land at LDS byte address
// lds_addr + 16 * i.  Written as an assembly statement for two reasons.  The compiler then keeps no
// record of outstanding loads into LDS: with the builtin it waits for all of them (vmcnt(0)) before
// the first LDS write that might overlap, which here is the output staging that runs while the
// next tile's loads are in flight; this kernel places every such wait itself.  And the address
// takes the scalar-base form directly (uniform 64-bit base, 32-bit lane offset) instead of 64-bit
// per-lane addresses.  M0 (the LDS destination) is listed as clobbered.
__device__ __forceinline__ void dma_load16_at(uint32_t lds_addr, const uint8_t* base, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory", "m0");
}

// The whole tile walk of one wave; GRP (0: columns 0-127, M phase first; 1: columns 128-255, L phase
// first) is a template parameter so that each group's loop is straight-line code.  All cursor
// state is wave-uniform (scalar registers) and advanced with compares and adds only.
template <int GRP, bool BIAS, bool GELUQ>
__device__ __forceinline__ void pingpong_wave(const GemmArgs& g, lds_u8* lds, const int wave)
{
    const uint32_t tiles = g.tiles_m * g.tiles_n, total = tiles * (uint32_t)g.split_k;
    const uint32_t xcd = blockIdx.x % 8, per = total / 8, rem = total % 8;
    const uint32_t range_end = (xcd + 1) * per + min(xcd + 1, rem);
    const uint32_t stride = (gridDim.x - xcd + 7) / 8;          // workgroups on this XCD
    const uint32_t first = xcd * per + min(xcd, rem) + blockIdx.x / 8;
    if (first >= range_end) return;

    MX_PROBE_INIT
    const uint32_t kbytes = g.k >> 1, kgroups = g.k >> 5;
    const int lane = threadIdx.x & 63;
    const int wm = wave & 3;
    const uint32_t lrow = lane & 31, lhalf = lane >> 5;
    const uint32_t swz = (lrow >> 2) & 3;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;

    // K steps per tile: the same for every tile but those of the last K split
    const int nk_full = (int)(g.k_per_split >> 7);
    const int nk_tail = (int)((g.k - (uint32_t)(g.split_k - 1) * g.k_per_split) >> 7);
    const uint32_t tail_first = tiles * (uint32_t)(g.split_k - 1);
    auto tile_steps = [&](uint32_t t) -> int { return t >= tail_first ? nk_tail : nk_full; };

    // ---- issue cursor: next stage to load.  The common path of a phase is straight-line
    //      scalar code; everything rare (a scale block is due, the tile ends) sits behind one
    //      branch each.  When the tile list is exhausted the cursor keeps re-loading the last
    //      stage (i_step = 0) into buffers that no longer have readers. ----
    uint32_t a_off[2], b_off[2], s_off;
    const uint8_t *a_ptr, *b_ptr, *s_base;
    uint32_t i_tile = first;
    int i_nk = 0, i_q = 0;              // K steps of the issue tile, next stage of it to load
    int i_due = 0, i_j = 0;             // stage that scale block i_j travels with
    uint32_t i_step = 64;               // bytes the code pointers advance per stage
    uint32_t i_dst = lds0 + wave * 2048;                          // this wave's A piece of the stage buffer
    uint32_t i_sdst = lds0 + Q_SCALE_OFF + wave * 1024;           // this wave's piece of the scale slot
    int i_buf = 0, i_slot = 0;
    uint32_t i_bias = lds0 + Q_BIAS_OFF;                          // bias slot of the next tile to be issued
    auto set_issue_tile = [&](uint32_t t) {
        const uint32_t z = t / tiles, r = t - z * tiles, tm = r / g.tiles_n;
        const uint32_t m0 = tm * Q_BM, n0 = (r - tm * g.tiles_n) * Q_BN;
        const uint32_t kbeg = z * g.k_per_split;
        const uint32_t mlast = g.m - 1 - m0, nlast = g.n - 1 - n0;
        a_ptr = g.a_codes + (size_t)m0 * kbytes + (kbeg >> 1);
        b_ptr = g.b_codes + (size_t)n0 * kbytes + (kbeg >> 1);
        const uint32_t ln = fresh_lane_id();
        const uint32_t lr = ln >> 2, lc = ((ln & 3) ^ ((ln >> 4) & 3)) << 4;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            a_off[u] = min(lr + (2 * wave + u) * 16, mlast) * kbytes + lc;
            b_off[u] = min(lr + (2 * wave + u) * 16, nlast) * kbytes + lc;
        }
        // scale rows: waves 0-3 fetch the A rows [64w, 64w+64), waves 4-7 the B rows [64(w-4), +64)
        if (GRP == 0) {
            s_base = g.a_scales + (size_t)m0 * kgroups + (kbeg >> 5);
            s_off = min((uint32_t)(wm * 64) + ln, mlast) * kgroups;
        } else {
            s_base = g.b_scales + (size_t)n0 * kgroups + (kbeg >> 5);
            s_off = min((uint32_t)(wm * 64) + ln, nlast) * kgroups;
        }
        i_nk = tile_steps(t);
        i_q = 0;
        i_due = 0;
        i_j = 0;
        // The tile's 256 bias values go to the slot that the tile before the previous one used; that tile's
        // output stage ended, in every wave, before the barriers of the previous tile's K loop (>= 4 steps),
        // and this point lies inside that loop.  One wave loads; its later waits cover the load (loads
        // complete in order) and barriers follow before any wave reads the slot.
        if (BIAS && GRP == 0 && wave == 0) {
            dma_load16_at(i_bias, reinterpret_cast<const uint8_t*>(g.bias + n0), min(4u * ln, g.n - 4u - n0) * 4u);
            i_bias = i_bias == lds0 + Q_BIAS_OFF ? i_bias + 1024u : i_bias - 1024u;
        }
    };
    // Loads the next stage (and the scale block that travels with it) and waits for every load
    // issued in earlier phases.
    auto issue_and_wait = [&]() {
        if (i_q == i_due) {                                      // once per 4 K steps
            const int off = min(4 * i_j, i_nk - 4) * 4;
            dma_load16_at(i_sdst, s_base + off, s_off);
            i_sdst += Q_SCALE_SLOT;
            if (++i_slot == 3) { i_slot = 0; i_sdst -= 3 * Q_SCALE_SLOT; }
            ++i_j;
            i_due = 4 * i_j < i_nk ? 4 * i_j - 1 : 0x7FFFFFFF;
            dma_load16_at(i_dst, a_ptr, a_off[0]);
            dma_load16_at(i_dst + 1024, a_ptr, a_off[1]);
            dma_load16_at(i_dst + Q_BM * 64, b_ptr, b_off[0]);
            dma_load16_at(i_dst + Q_BM * 64 + 1024, b_ptr, b_off[1]);
            MX_PROBE(1);
            asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
        } else {
            dma_load16_at(i_dst, a_ptr, a_off[0]);
            dma_load16_at(i_dst + 1024, a_ptr, a_off[1]);
            dma_load16_at(i_dst + Q_BM * 64, b_ptr, b_off[0]);
            dma_load16_at(i_dst + Q_BM * 64 + 1024, b_ptr, b_off[1]);
            MX_PROBE(1);
            asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        }
        MX_PROBE(2);
        a_ptr += i_step;
        b_ptr += i_step;
        i_dst = i_buf == 2 ? i_dst - 2 * Q_STAGE_BYTES : i_dst + Q_STAGE_BYTES;
        i_buf = i_buf == 2 ? 0 : i_buf + 1;
        if (++i_q == i_nk) {                                     // once per tile
            i_tile += stride;
            if (i_tile < range_end) {
                set_issue_tile(i_tile);
            } else {                                             // nothing left: stay on the last stage
                a_ptr -= 64;
                b_ptr -= 64;
                i_step = 0;
                i_q = 0;
                i_nk = 0x7FFFFFFF;
                i_due = -1;
            }
        }
    };

    // ---- read cursor: K step whose operands the next L phase reads (past the end of the tile
    //      list it keeps reading the buffers; those operands are never used) ----
    uint32_t r_tile = first;
    int r_nk = tile_steps(first), r_s = 0;
    int r_buf = 0, r_slot = 0;
    uint32_t r_src = 0;                 // byte offset of the stage buffer
    uint32_t r_sc = Q_SCALE_OFF;        // byte offset of this step's scale dwords: slot + 4 * (step within block)

    // per-lane parts of the LDS read addresses
    const uint32_t a_rd = (wm * 64 + lrow) * 64, b_rd = Q_BM * 64 + (GRP * 128 + lrow) * 64;
    const uint32_t a_rd0 = a_rd + (((0 + lhalf) ^ swz) << 4), a_rd1 = a_rd + (((2 + lhalf) ^ swz) << 4);
    const uint32_t b_rd0 = b_rd + (((0 + lhalf) ^ swz) << 4), b_rd1 = b_rd + (((2 + lhalf) ^ swz) << 4);
    const uint32_t sa_rd = (wm * 64 + lane) * 16, sb_rd = (Q_BM + GRP * 128 + lane) * 16;    // lane, not lane % 32

    struct Frag { v4i a[2]; v4i b[4]; };
    Frag f[2];
    uint32_t sca[2], scb[4];
    v16f acc[2][4];

    auto load_phase = [&]() {
        uint32_t va, vb0, vb1;
        MX_PROBE(0);
        {
            // scale dwords of this K step: one read serves two 32-row blocks (lanes 0-31 the first,
            // lanes 32-63 the second; the 16-byte row pitch makes each read a 4-way bank conflict
            // whether or not the two half waves read the same rows), then the halves are exchanged
            const lds_u8* sp = lds + r_sc;
            va = *reinterpret_cast<const __attribute__((address_space(3))) uint32_t*>(sp + sa_rd);
            vb0 = *reinterpret_cast<const __attribute__((address_space(3))) uint32_t*>(sp + sb_rd);
            vb1 = *reinterpret_cast<const __attribute__((address_space(3))) uint32_t*>(sp + sb_rd + 1024);
            const lds_u8* base = lds + r_src;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                f[0].a[i] = *reinterpret_cast<const __attribute__((address_space(3))) v4i*>(base + a_rd0 + i * 2048);
                f[1].a[i] = *reinterpret_cast<const __attribute__((address_space(3))) v4i*>(base + a_rd1 + i * 2048);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f[0].b[j] = *reinterpret_cast<const __attribute__((address_space(3))) v4i*>(base + b_rd0 + j * 2048);
                f[1].b[j] = *reinterpret_cast<const __attribute__((address_space(3))) v4i*>(base + b_rd1 + j * 2048);
            }
            // advance to the next K step
            r_src = r_buf == 2 ? 0 : r_src + Q_STAGE_BYTES;
            r_buf = r_buf == 2 ? 0 : r_buf + 1;
            r_sc += 4;
            ++r_s;
            if (r_s == r_nk || (r_s & 3) == 0) {                 // it starts a scale block (once per <= 4 steps)
                if (r_s == r_nk) {                               // ... of the next tile
                    r_tile += stride;
                    r_s = 0;
                    r_nk = r_tile < range_end ? tile_steps(r_tile) : 0x7FFFFFFF;
                }
                r_slot = r_slot == 2 ? 0 : r_slot + 1;
                // the last block of a K range is shifted back to end where the range ends
                const int within = r_s + 4 > r_nk ? r_s - (r_nk - 4) : 0;
                r_sc = Q_SCALE_OFF + r_slot * Q_SCALE_SLOT + within * 4;
            }
        }
        issue_and_wait();
        // (the compiler waits for the LDS reads here)
        const auto pa = __builtin_amdgcn_permlane32_swap(va, va, false, false);
        const auto pb0 = __builtin_amdgcn_permlane32_swap(vb0, vb0, false, false);
        const auto pb1 = __builtin_amdgcn_permlane32_swap(vb1, vb1, false, false);
        sca[0] = pa[0] >> 8 * lhalf; sca[1] = pa[1] >> 8 * lhalf;
        scb[0] = pb0[0] >> 8 * lhalf; scb[1] = pb0[1] >> 8 * lhalf;
        scb[2] = pb1[0] >> 8 * lhalf; scb[3] = pb1[1] >> 8 * lhalf;
        MX_PROBE(3);
    };
    // FIRST: the first K step of a tile; its first 64-K slice starts the accumulators from zero (the
    // matrix instruction takes a constant 0 as its addend), so they are never cleared by separate moves.
    auto mma_phase = [&](auto first_c) {
        constexpr bool FIRST = decltype(first_c)::value;
        MX_PROBE(4);
        MX_SCHED_FENCE();
        const v16f zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                v8i xa = v8i{f[kk].a[i].x, f[kk].a[i].y, f[kk].a[i].z, f[kk].a[i].w, 0, 0, 0, 0};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    v8i xb = v8i{f[kk].b[j].x, f[kk].b[j].y, f[kk].b[j].z, f[kk].b[j].w, 0, 0, 0, 0};
                    if (kk == 0)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(xb, xa, FIRST ? zero : acc[i][j], 4, 4, 0, (int)scb[j], 0, (int)sca[i]);
                    else
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(xb, xa, acc[i][j], 4, 4, 2, (int)scb[j], 2, (int)sca[i]);
                }
            }
        MX_SCHED_FENCE();
        MX_PROBE(5);
    };
    // ---- prologue: stages 0 and 1 (scale block 0 travels with stage 0) ----
    set_issue_tile(first);
    issue_and_wait();
    issue_and_wait();                                                 // (ends with vmcnt(4): all but stage 1)
    asm volatile("s_barrier" ::: "memory");                           // stage 0 and scale block 0 are in
    if (GRP == 0) load_phase();                                       // operands of step 0

    // ---- per K step one barrier: group 0 runs  M(k) | barrier | L(k+1),  group 1 runs
    //      L(k) | barrier | M(k).  At the barrier every read of stage k has returned (group 0's were
    //      consumed by M(k), group 1 waits for its own), so the loads issued after it may overwrite
    //      that buffer; and every wave has waited for its part of stage k+1, which group 0 reads
    //      right after it.  Between barriers the two waves of a SIMD drift freely: one is in its
    //      MFMA burst while the other reads and loads. ----
    uint32_t c_bias = Q_BIAS_OFF;                                 // bias slot of the tile being multiplied
    for (uint32_t c_tile = first; c_tile < range_end; c_tile += stride) {
        const int nk = tile_steps(c_tile);
        // step 0 starts the accumulators, the others add to them (nk >= 4)
        if (GRP == 0) {
            mma_phase(std::true_type{});
            barrier_after_mfma(acc);
            load_phase();
        } else {
            load_phase();
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            mma_phase(std::true_type{});
        }
        for (int k = 1; k < nk; ++k) {
            if (GRP == 0) {
                mma_phase(std::false_type{});
                barrier_after_mfma(acc);
                load_phase();
            } else {
                load_phase();
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                mma_phase(std::false_type{});
            }
        }
        const uint32_t z = c_tile / tiles, r = c_tile - z * tiles, tm = r / g.tiles_n;
        const uint32_t m0 = tm * Q_BM + wm * 64, n0 = (r - tm * g.tiles_n) * Q_BN + GRP * 128;
        uint8_t* ep = (uint8_t*)(lds + Q_EP_OFF + wave * P_EP_BYTES);
        const lds_u8* bias = BIAS ? lds + c_bias + GRP * 512 : nullptr;
        const uint32_t c_bias_now = c_bias;
        if (BIAS) c_bias = c_bias == (uint32_t)Q_BIAS_OFF ? c_bias + 1024u : c_bias - 1024u;
        MX_PROBE(6);
        // wave tile wholly inside the matrix, rows storable 16 bytes at a time, lane offsets within 32 bits
        const bool final_out = g.split_k == 1;
        const int64_t ldc = final_out ? g.ldc : (int64_t)g.n;
        const uint32_t ebytes = (final_out && g.c_bf16) ? 2u : 4u;
        const bool interior = m0 + 64 <= g.m && n0 + 128 <= g.n && ldc < (1 << 27) &&
                              ((reinterpret_cast<uintptr_t>(g.c) | (uintptr_t)(ldc * ebytes)) & 15) == 0;
        if (interior) {
            if (final_out) gemm_epilogue_interior<true, BIAS>(g, lds + Q_EP_OFF + wave * P_EP_BYTES, acc, m0, n0, z, ldc, BIAS ? lds + c_bias_now + GRP * 512 : nullptr);
            else           gemm_epilogue_interior<false, false>(g, lds + Q_EP_OFF + wave * P_EP_BYTES, acc, m0, n0, z, ldc, nullptr);
        } else {
            if (final_out) gemm_epilogue_chunked<true>(g, ep, acc, m0, n0, lane, z, bias);
            else           gemm_epilogue_chunked<false>(g, ep, acc, m0, n0, lane, z, nullptr);
        }
        if (GELUQ) {
            // BIAS is set with GELUQ: the bias slot of this tile is still valid (it is reused two tiles later)
            if (g.q_floor) gemm_epilogue_gelu_quant<true>(g, lds + Q_EP_OFF + wave * P_EP_BYTES, acc, m0, n0, lds + c_bias_now + GRP * 512);
            else           gemm_epilogue_gelu_quant<false>(g, lds + Q_EP_OFF + wave * P_EP_BYTES, acc, m0, n0, lds + c_bias_now + GRP * 512);
        }
        MX_PROBE(7);
    }
    // the cursor's trailing loads target this workgroup's LDS: they must land before it is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// BIAS: a bias row is added in the output stage (a separate instance: the plain product's code is
// the same with and without this feature in the source).
// GELUQ (only with BIAS): a second output stage quantizes GELU(product + bias) for the next layer.
template <bool BIAS, bool GELUQ = false>
__global__ __launch_bounds__(Q_NT, 2) void mx_gemm_pingpong_kernel(GemmArgs g)
{
    __shared__ __attribute__((aligned(1024))) uint8_t lds[BIAS ? Q_LDS_BYTES : Q_BIAS_OFF];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Short-K tiles spend as long storing as multiplying.  Started together, all compute units store
    // at the same time, the burst (33 MB per round) takes longer to drain than the next K loop has
    // loads in flight for, and the loop stalls behind it; the stalled units then stay in step.  Half
    // of the workgroups start half a K loop later, so that one half stores while the other multiplies.
    if ((blockIdx.x >> 3) & 1)
        for (int i = 0; i < g.stagger; ++i) __builtin_amdgcn_s_sleep(32);
    if (wave < 4) pingpong_wave<0, BIAS, GELUQ>(g, (lds_u8*)lds, wave);
    else          pingpong_wave<1, BIAS, GELUQ>(g, (lds_u8*)lds, wave);
}

// ---------------------------------------------------------------------------
// Calibration: the products' MFMA in a register-resident loop.  8 waves per workgroup (two per
// SIMD, as in the main kernel), each with the main kernel's 8 independent accumulator tiles; every lane
// loads its 12 operand registers (two 64-K slices of 2 m-side and 4 n-side fragments) once from the
// caller's buffer and then issues 16 MFMAs per iteration with no memory or LDS access in between.
// What it measures is the rate the matrix pipe sustains for these operand bytes; that rate depends
// on the bytes (switching activity against the power limit), which is why the caller supplies them.
// ---------------------------------------------------------------------------
constexpr int CAL_WAVES = 8, CAL_FRAGS = 12;
constexpr size_t CAL_OPERAND_BYTES = (size_t)CAL_WAVES * CAL_FRAGS * 64 * 16;      // 98304

__global__ __launch_bounds__(CAL_WAVES * 64, 1) void calibration_mfma_kernel(const v4i* __restrict__ operands, int iterations,
                                                                            float* sink)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v4i f[CAL_FRAGS];
#pragma unroll
    for (int q = 0; q < CAL_FRAGS; ++q) f[q] = operands[(wave * CAL_FRAGS + q) * 64 + lane];
    v16f acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const v4i a = f[kk * 6 + i];
                const v8i xa = v8i{a.x, a.y, a.z, a.w, 0, 0, 0, 0};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const v4i b = f[kk * 6 + 2 + j];
                    const v8i xb = v8i{b.x, b.y, b.z, b.w, 0, 0, 0, 0};
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(xb, xa, acc[i][j], 4, 4, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
                }
            }
        MX_SCHED_FENCE();
    }
    // keep the accumulators alive; one value per lane leaves the kernel
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) t += acc[i][j][r];
    sink[(size_t)blockIdx.x * (CAL_WAVES * 64) + threadIdx.x] = t;
}

}  // namespace

namespace mxl {

size_t calibration_mfma_operand_bytes() { return CAL_OPERAND_BYTES; }

hipError_t launch_calibration_mfma(const uint8_t* operands, int workgroups, int iterations, float* sink, hipStream_t st)
{
    hipLaunchKernelGGL(calibration_mfma_kernel, dim3((unsigned)workgroups), dim3(CAL_WAVES * 64), 0, st,
                       reinterpret_cast<const v4i*>(operands), iterations, sink);
    return hipGetLastError();
}

int gemm_split_k(int64_t m, int64_t n, int64_t k)
{
    // Split K only when the output has too few tiles to fill the machine and K is long.  A split
    // product runs in the main kernel (at least 8 K steps per split): one 256 x 256 workgroup per
    // CU, 256 slots; the split is the largest that still fits in one round of slots, so that
    // every partial tile is written once and the second, emptier round does not exist.
    const bool fast = (k & 127) == 0;
    const int64_t bm = fast ? Q_BM : G_BM, bn = fast ? Q_BN : G_BN, slots = 256;
    int64_t tiles = ((m + bm - 1) / bm) * ((n + bn - 1) / bn);
    if (tiles * 2 > slots || k < 4096) return 1;
    int64_t s = slots / tiles;
    int64_t max_by_k = k / 1024;                 // keep at least 8 K steps per split
    if (s > max_by_k) s = max_by_k;
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    return (int)s;
}

bool gemm_takes_fused_quantizer(int64_t m, int64_t n, int64_t k)
{
    // the main kernel: K a multiple of 128 with at least four K steps, and no K split
    return (k & 127) == 0 && k >= 512 && (n & 31) == 0 && gemm_split_k(m, n, k) == 1;
}

hipError_t launch_gemm(const GemmParams& p, hipStream_t st)
{
    GemmArgs g{};
    g.a_codes = p.a_codes; g.a_scales = p.a_scales; g.b_codes = p.b_codes; g.b_scales = p.b_scales;
    g.m = (uint32_t)p.m; g.n = (uint32_t)p.n; g.k = (uint32_t)p.k;
    g.split_k = p.split_k;
    uint32_t ksteps = (uint32_t)((p.k + 127) / 128);
    uint32_t steps_per = (ksteps + p.split_k - 1) / p.split_k;
    g.k_per_split = steps_per * 128;
    g.split_k = (int)((ksteps + steps_per - 1) / steps_per);   // drop empty splits
    g.c = g.split_k > 1 ? p.workspace : p.c;
    g.ldc = p.ldc; g.c_bf16 = p.c_bf16;
    g.bias = g.split_k > 1 ? nullptr : p.bias;                  // partial sums get none: the reduction adds it
    if ((p.k & 127) == 0) {
        g.tiles_m = (uint32_t)((p.m + D_BM - 1) / D_BM);
        g.tiles_n = (uint32_t)((p.n + D_BN - 1) / D_BN);
        dim3 grid(g.tiles_m * g.tiles_n * g.split_k);
        const uint32_t last_steps = ksteps - (uint32_t)(g.split_k - 1) * steps_per;
        if (steps_per >= 4 && last_steps >= 4) {
            g.tiles_m = (uint32_t)((p.m + Q_BM - 1) / Q_BM);
            g.tiles_n = (uint32_t)((p.n + Q_BN - 1) / Q_BN);
            const unsigned nblk = g.tiles_m * g.tiles_n * g.split_k;
            // measured on the ViT-B products: 2.5 us (3 x 2048 clocks) gains 5-15 % at K = 768 and
            // 3-5 % at K = 2304, nothing at K = 3072; pointless below two rounds of tiles
            g.stagger = (g.split_k == 1 && nblk >= 2 * Q_SLOTS && p.k <= 2304) ? 3 : 0;
            const dim3 pgrid(nblk < Q_SLOTS ? nblk : Q_SLOTS);
            if (p.q_codes) {
                if (!g.bias || g.split_k != 1) return hipErrorInvalidValue;
                g.q_codes = p.q_codes; g.q_scales = p.q_scales; g.q_floor = p.q_floor ? 1 : 0;
                hipLaunchKernelGGL((mx_gemm_pingpong_kernel<true, true>), pgrid, dim3(Q_NT), 0, st, g);
            } else if (g.bias) {
                hipLaunchKernelGGL(mx_gemm_pingpong_kernel<true>, pgrid, dim3(Q_NT), 0, st, g);
            } else {
                hipLaunchKernelGGL(mx_gemm_pingpong_kernel<false>, pgrid, dim3(Q_NT), 0, st, g);
            }
        } else {
            if (p.q_codes) return hipErrorInvalidValue;          // the fused quantizer lives in the main kernel only
            hipLaunchKernelGGL(mx_gemm_dma_kernel, grid, dim3(D_NT), 0, st, g);
        }
    } else {
        if (p.q_codes) return hipErrorInvalidValue;
        g.tiles_m = (uint32_t)((p.m + G_BM - 1) / G_BM);
        g.tiles_n = (uint32_t)((p.n + G_BN - 1) / G_BN);
        dim3 grid(g.tiles_m * g.tiles_n, 1, g.split_k);
        dim3 block((G_BM / G_WM) * (G_BN / G_WN) * 64);
        hipLaunchKernelGGL((mx_gemm_kernel<G_BM, G_BN, G_WM, G_WN>), grid, block, 0, st, g);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (g.split_k > 1) {
        size_t total = (size_t)p.m * p.n;
        const size_t out_bytes = p.c_bf16 ? 2 : 4;
        const bool vec = (p.n & 3) == 0 && ((size_t)p.ldc * out_bytes & 15) == 0 &&
                         (reinterpret_cast<uintptr_t>(p.c) & 15) == 0 && (reinterpret_cast<uintptr_t>(p.workspace) & 15) == 0;
        if (vec) {
            dim3 rgrid((unsigned)((total / 4 + 255) / 256)), rblock(256);
            hipLaunchKernelGGL(splitk_reduce4_kernel, rgrid, rblock, 0, st,
                               static_cast<const float*>(p.workspace), g.split_k, g.m, g.n, p.c, p.ldc, (int)p.c_bf16, p.bias);
        } else {
            dim3 rgrid((unsigned)((total + 255) / 256)), rblock(256);
            hipLaunchKernelGGL(splitk_reduce_kernel, rgrid, rblock, 0, st,
                               static_cast<const float*>(p.workspace), g.split_k, g.m, g.n, p.c, p.ldc, (int)p.c_bf16, p.bias);
        }
        e = hipGetLastError();
    }
    return e;
}

}  // namespace mxl

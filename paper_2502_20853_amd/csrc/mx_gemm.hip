// C[m x n] = A[m x k] . B[n x k]^T on packed MXFP4 operands, FP32 accumulation
// on gfx950's block-scaled FP4 matrix cores (V_MFMA_SCALE_F32_16X16X128_F8F6F4).
// All three products of the layer (Eqs. 3-5, Sec. 3.3) have this form because
// every operand is stored along its own contraction dimension.
//
// Kernel structure
//   - workgroup tile BM x BN, K step 128 (= 64 bytes of codes and 4 scale bytes
//     per row), double-buffered in LDS;
//   - one 16x16x128 MFMA consumes, per lane, 32 consecutive K elements (16 bytes,
//     exactly one MX group) of row (lane % 16), K block (lane / 16), and that
//     group's E8M0 scale byte;
//   - code tiles sit in LDS row-major with the 16-byte chunk index XOR-swizzled
//     by (row >> 2) & 3 so that both the 16-byte stores (4 lanes per row) and
//     the MFMA operand reads (16 rows per K block) are bank-conflict free;
//   - scale tiles sit in LDS as [k block][row % 16][row-tile % 4] per group of
//     four 16-row tiles, so one 32-bit LDS read hands a lane the scale bytes of
//     four MFMAs, picked by the instruction's op_sel;
//   - the MFMA's first operand is the B (n) side, so that a lane ends up with
//     four consecutive n of one m and stores 8 or 16 contiguous bytes.
#include "mx_launch.hpp"

#include <type_traits>

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

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);   // NaN stays NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
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
            size_t off = (size_t)mm * ldc + nn;
            if (nn + 3 < g.n && vec_ok) {
                if (as_bf16) {
                    uint2 pk;
                    pk.x = (uint32_t)f32_to_bf16_rne(v.x) | ((uint32_t)f32_to_bf16_rne(v.y) << 16);
                    pk.y = (uint32_t)f32_to_bf16_rne(v.z) | ((uint32_t)f32_to_bf16_rne(v.w) << 16);
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
                                     void* c, int64_t ldc, int c_bf16)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)m * n;
    if (idx >= total) return;
    float s = 0.f;
    for (int z = 0; z < split; ++z) s += part[(size_t)z * total + idx];
    uint32_t r = (uint32_t)(idx / n), col = (uint32_t)(idx - (size_t)r * n);
    if (c_bf16) static_cast<uint16_t*>(c)[(size_t)r * ldc + col] = f32_to_bf16_rne(s);
    else        static_cast<float*>(c)[(size_t)r * ldc + col] = s;
}

constexpr int G_BM = 256, G_BN = 256, G_WM = 128, G_WN = 64;

}  // namespace

namespace mxl {

int gemm_split_k(int64_t m, int64_t n, int64_t k)
{
    // Split K only when the output has too few tiles to fill the 256 CUs and K is long.
    int64_t tiles = ((m + G_BM - 1) / G_BM) * ((n + G_BN - 1) / G_BN);
    if (tiles >= 128 || k < 4096) return 1;
    int64_t want = (256 + tiles - 1) / tiles;
    int64_t max_by_k = k / 1024;                 // keep at least 8 K steps per split
    int64_t s = want < max_by_k ? want : max_by_k;
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    return (int)s;
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
    g.tiles_m = (uint32_t)((p.m + G_BM - 1) / G_BM);
    g.tiles_n = (uint32_t)((p.n + G_BN - 1) / G_BN);
    dim3 grid(g.tiles_m * g.tiles_n, 1, g.split_k), block((G_BM / G_WM) * (G_BN / G_WN) * 64);
    hipLaunchKernelGGL((mx_gemm_kernel<G_BM, G_BN, G_WM, G_WN>), grid, block, 0, st, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (g.split_k > 1) {
        size_t total = (size_t)p.m * p.n;
        dim3 rgrid((unsigned)((total + 255) / 256)), rblock(256);
        hipLaunchKernelGGL(splitk_reduce_kernel, rgrid, rblock, 0, st,
                           static_cast<const float*>(p.workspace), g.split_k, g.m, g.n, p.c, p.ldc, (int)p.c_bf16);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace mxl

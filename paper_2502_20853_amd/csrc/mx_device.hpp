// Device-side building blocks of the MXFP4 quantizers (gfx950).
//
// Everything here works on FP32 bit patterns so that each decision (shared
// exponent, bracket, rounding direction) is an exact integer or exact FP32
// operation: the scaled value y = x * 2^-s and the position k of |y| inside its
// E2M1 binade are power-of-two multiples of the input and therefore exact.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mxd {

// ---- shared exponent (Sec. 3.2) -------------------------------------------
// amax_bits: FP32 bits of M = max |x| over the group (sign cleared).
// Returns the scale byte s + 127.
//   truncation-free: s = ceil(log2(M/6)).  With M = m * 2^e, 1 <= m < 2 and
//     6 = 1.5 * 2^2 this is e - 2 when m <= 1.5 and e - 1 otherwise.
//   Eq. 2:           s = floor(log2 M) - 2 = e - 2.
// The biased exponent field is e + 127, so byte = field - 2 (+1).  Clamping s
// to >= -127 is byte >= 0; subnormal M has field 0 and lands on that clamp.
// M = 0 uses epsilon = 1e-8, for which both rules give s = -29.
__device__ __forceinline__ uint32_t scale_byte(uint32_t amax_bits, bool floor_mode)
{
    uint32_t field = amax_bits >> 23;
    uint32_t inc = (!floor_mode && (amax_bits & 0x7FFFFFu) > 0x400000u) ? 1u : 0u;
    int b = (int)field - 2 + (int)inc;
    b = b < 0 ? 0 : b;
    return amax_bits == 0u ? 98u : (uint32_t)b;
}

// 2^-s as FP32 for scale byte b = s + 127 (s in [-127, 126]: always normal).
__device__ __forceinline__ float inv_scale(uint32_t byte)
{
    return __uint_as_float((254u - byte) << 23);
}

// 2^s as FP32 (s = -127 is the subnormal 2^-127).
__device__ __forceinline__ float fwd_scale(uint32_t byte)
{
    return __uint_as_float(byte ? (byte << 23) : 0x00400000u);
}

// ---- E2M1 rounding (Sec. 3.2) ----------------------------------------------
// y is the scaled value x / S.  Let a = |y| and E its binade, with everything
// below 1 treated as the binade of 1 (E2M1's subnormal step equals the step of
// [1,2)).  k = a / step(E) * ... lies in [0,4): floor(k) and floor(k)+1 are the
// two neighbouring codes relative to 2*(E-127), and frac(k) is
// p = (a - m1)/(m2 - m1).
struct Bracket {
    uint32_t base;   // code of the lower magnitude m1
    float frac;      // p in [0,1)
    uint32_t sign;   // 8 if the sign bit of y is set
};

__device__ __forceinline__ Bracket bracket(float y, bool floor_mode)
{
    uint32_t yb = __float_as_uint(y);
    uint32_t ab = yb & 0x7FFFFFFFu;
    if (floor_mode) ab = ab > 0x40C00000u ? 0x40C00000u : ab;   // Eq. 2 truncates to |y| <= 6
    uint32_t E = ab >> 23;
    E = E < 127u ? 127u : E;
    float k = __uint_as_float(ab) * __uint_as_float((255u - E) << 23);   // exact
    float fl = floorf(k);
    Bracket br;
    br.frac = k - fl;                                                    // exact
    br.base = 2u * (E - 127u) + (uint32_t)fl;
    br.sign = (yb >> 28) & 8u;
    return br;
}

// round_D: q1 iff strictly nearer, so a midpoint goes to q2, the larger signed
// value: up in magnitude for y > 0, down in magnitude for y < 0.
__device__ __forceinline__ uint32_t round_rtn(float y, bool floor_mode)
{
    Bracket br = bracket(y, floor_mode);
    bool up = br.sign ? (br.frac > 0.5f) : (br.frac >= 0.5f);
    return (br.base + (up ? 1u : 0u)) | br.sign;
}

// round_S with 16 random bits: larger magnitude iff r16 < 65536 * p.
__device__ __forceinline__ uint32_t round_sr(float y, uint32_t r16, bool floor_mode)
{
    Bracket br = bracket(y, floor_mode);
    bool up = (float)r16 < br.frac * 65536.0f;                           // both sides exact
    return (br.base + (up ? 1u : 0u)) | br.sign;
}

// Q-EMA (Algorithm 1): bracket from y = w/S, choice by z = w_ema/S.
__device__ __forceinline__ uint32_t round_ema(float y, float z, bool floor_mode)
{
    uint32_t yb = __float_as_uint(y);
    uint32_t ab = yb & 0x7FFFFFFFu;
    if (floor_mode) ab = ab > 0x40C00000u ? 0x40C00000u : ab;
    uint32_t E = ab >> 23;
    E = E < 127u ? 127u : E;
    float f = __uint_as_float((255u - E) << 23);
    float k = __uint_as_float(ab) * f;
    float fl = floorf(k);
    float fr = k - fl;
    uint32_t neg = yb >> 31;
    // z mirrored so that the bracket is [fl, fl+1] on a positive axis
    float zk = __uint_as_float(__float_as_uint(z) ^ (neg << 31)) * f;
    float mid = fl + 0.5f;
    bool up = neg ? (zk > mid) : (zk >= mid);   // |z-q1| < |z-q2| picks q1, else q2
    up = up && (fr != 0.0f);                    // w/S already an E2M1 value: keep it
    return (2u * (E - 127u) + (uint32_t)fl + (up ? 1u : 0u)) | ((yb >> 28) & 8u);
}

// value of an E2M1 code times 2^s, exact in FP32 (may be subnormal)
__device__ __forceinline__ float dequant(uint32_t code, float scale)
{
    uint32_t n = code & 7u;
    uint32_t bits = (((n >> 1) + 126u) << 23) | ((n & 1u) << 22);
    bits = n < 2u ? (n ? 0x3F000000u : 0u) : bits;
    return __uint_as_float(bits | ((code & 8u) << 28)) * scale;
}

// ---- Philox4x32-10 (Salmon et al., SC'11) ----------------------------------
struct U4 { uint32_t w[4]; };

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1)
{
    const uint32_t MUL_A = 0xD2511F53u, MUL_B = 0xCD9E8D57u;
    const uint32_t WEYL_A = 0x9E3779B9u, WEYL_B = 0xBB67AE85u;
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        uint64_t pa = (uint64_t)MUL_A * c0;
        uint64_t pb = (uint64_t)MUL_B * c2;
        uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)pb;
        c3 = (uint32_t)pa;
        c0 = n0;
        c2 = n2;
        k0 += WEYL_A;
        k1 += WEYL_B;
    }
    U4 r;
    r.w[0] = c0; r.w[1] = c1; r.w[2] = c2; r.w[3] = c3;
    return r;
}

// The eight 16-bit fields for the 8-element block `blk` (= element index >> 3).
__device__ __forceinline__ U4 sr_block(uint64_t blk, uint32_t tensor_id, uint32_t k0, uint32_t k1)
{
    return philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), tensor_id, 0u, k0, k1);
}

__device__ __forceinline__ uint32_t sr_field(const U4& r, int t)
{
    uint32_t w = r.w[t >> 1];
    return (t & 1) ? (w >> 16) : (w & 0xFFFFu);
}

// ---- cross-lane max over aligned groups of 4 lanes (one 32-element group) ---
__device__ __forceinline__ uint32_t quad_max(uint32_t v)
{
    uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);  // lane ^ 1
    v = v > o ? v : o;
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);           // lane ^ 2
    return v > o ? v : o;
}

// ---- source loads: 8 consecutive elements as FP32 --------------------------
struct F8 { float v[8]; };

__device__ __forceinline__ F8 load8(const float* p)
{
    const float4* q = reinterpret_cast<const float4*>(p);
    float4 a = q[0], b = q[1];
    F8 r;
    r.v[0] = a.x; r.v[1] = a.y; r.v[2] = a.z; r.v[3] = a.w;
    r.v[4] = b.x; r.v[5] = b.y; r.v[6] = b.z; r.v[7] = b.w;
    return r;
}

__device__ __forceinline__ F8 load8(const uint16_t* p)   // bf16 bit patterns
{
    uint4 a = *reinterpret_cast<const uint4*>(p);
    F8 r;
    r.v[0] = __uint_as_float(a.x << 16); r.v[1] = __uint_as_float(a.x & 0xFFFF0000u);
    r.v[2] = __uint_as_float(a.y << 16); r.v[3] = __uint_as_float(a.y & 0xFFFF0000u);
    r.v[4] = __uint_as_float(a.z << 16); r.v[5] = __uint_as_float(a.z & 0xFFFF0000u);
    r.v[6] = __uint_as_float(a.w << 16); r.v[7] = __uint_as_float(a.w & 0xFFFF0000u);
    return r;
}

__device__ __forceinline__ F8 zero8()
{
    F8 r;
#pragma unroll
    for (int t = 0; t < 8; ++t) r.v[t] = 0.0f;
    return r;
}

__device__ __forceinline__ uint32_t amax_bits8(const F8& x)
{
    uint32_t m = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        uint32_t b = __float_as_uint(x.v[t]) & 0x7FFFFFFFu;
        m = b > m ? b : m;
    }
    return m;
}

}  // namespace mxd

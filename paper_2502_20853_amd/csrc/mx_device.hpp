// Device-side building blocks of the MXFP4 quantizers (gfx950).
//
// Everything here works on FP32 bit patterns so that each decision (shared
// exponent, bracket, rounding direction) is an exact integer operation on a value
// that is a power-of-two multiple of the input.
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
    // adding 0x3FFFFF carries into the exponent field exactly when the mantissa exceeds 0x400000
    uint32_t field = (amax_bits + (floor_mode ? 0u : 0x3FFFFFu)) >> 23;
    uint32_t b;
    asm("v_sub_u32_e64 %0, %1, 2 clamp" : "=v"(b) : "v"(field));     // max(field - 2, 0) in one instruction
    return amax_bits == 0u ? 98u : b;
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
// The quantizers never form y = x / S itself.  They form v = x * 2^(-s-126) (one ldexp), which
// puts |y| in [0, 6] onto FP32 bit patterns whose layout IS the E2M1 grid: |y| < 1 lands
// in FP32's subnormal range (uniform spacing, like E2M1's subnormals 0 and 0.5), [1,2)
// in the first normal binade, and so on, so that
//     bits(v) >> 22           = code of the largest E2M1 magnitude m1 <= |y|,
//     bits(v) & 0x3FFFFF      = p * 2^22,   p = (|y| - m1) / (m2 - m1).
// Rounding is then one integer add that carries into bit 22.  The scaling is exact except
// when the result is subnormal and x has bits below 2^-149; the FP32 rounding mode is set
// so that the inexact case still decides correctly (v_ldexp_f32 rounds a subnormal result
// by the mode, like a multiplication does):
//   round_D, ties to the larger value: y > 0 goes up iff p >= 1/2, which floor(p * 2^22)
//     decides; y < 0 goes up in magnitude iff p > 1/2, which ceil(p * 2^22) decides.  Both
//     are what round-toward-minus-infinity does to the signed value.
//   round_S: up iff r16 < 65536 * p  <=>  p * 2^22 > 64 * r16, which ceil decides:
//     round-toward-plus-infinity on |x|.
__device__ __forceinline__ void f32_round_toward_plus_inf()  { __builtin_amdgcn_s_setreg(0x801, 1); }   // MODE[1:0]
__device__ __forceinline__ void f32_round_toward_minus_inf() { __builtin_amdgcn_s_setreg(0x801, 2); }
__device__ __forceinline__ void f32_round_to_nearest_even()  { __builtin_amdgcn_s_setreg(0x801, 0); }

constexpr uint32_t GRID_MAX_BITS = 0x01C00000u;      // 6 * 2^-126

// Exponent to hand to ldexp for scale byte b = s + 127:  -s - 126 = 1 - b.
__device__ __forceinline__ int grid_exponent(uint32_t byte) { return 1 - (int)byte; }

// round_D.  Call with the rounding mode set toward minus infinity.  e = grid_exponent(byte).
// FLOOR: Eq. 2's scale, which truncates to |y| <= 6.
template <bool FLOOR>
__device__ __forceinline__ uint32_t rtn_code(float x, int e)
{
    uint32_t vb = __float_as_uint(__builtin_ldexpf(x, e));
    uint32_t mag = vb & 0x7FFFFFFFu;
    if (FLOOR) mag = mag > GRID_MAX_BITS ? GRID_MAX_BITS : mag;
    // + 2^21, minus 1 for negative values: a negative midpoint stays at the smaller magnitude
    uint32_t t = mag + 0x200000u + (uint32_t)((int32_t)vb >> 31);
    return (t >> 22) | ((vb >> 28) & 8u);
}

// round_S.  Call with the rounding mode set toward plus infinity.
// rinv = ((65535 - r16) << 6) | 63: the add carries into bit 22 iff p * 2^22 > 64 * r16.
template <bool FLOOR>
__device__ __forceinline__ uint32_t sr_code(float x, int e, uint32_t rinv)
{
    uint32_t mag = __float_as_uint(__builtin_ldexpf(__builtin_fabsf(x), e));
    if (FLOOR) mag = mag > GRID_MAX_BITS ? GRID_MAX_BITS : mag;
    return ((mag + rinv) >> 22) | ((__float_as_uint(x) >> 28) & 8u);
}

// round_D that also hands back the rounded value on the grid's bit layout with its sign,
// i.e. sign | (code & 7) << 22 = +-m * 2^-126, for the double quantization that follows.
// The sum keeps the sign in bit 31 (the magnitude stays below 2^25, so nothing carries into it, and
// the -1 of a negative value only borrows from the low bits), which saves taking |v| apart first;
// bits 30..25 of the sum are zero, so sum >> 28 is the sign nibble as it stands.
template <bool FLOOR>
__device__ __forceinline__ uint32_t rtn_code_keep(float x, int e, uint32_t& grid_bits)
{
    uint32_t vb = __float_as_uint(__builtin_ldexpf(x, e));
    if (FLOOR) {
        uint32_t mag = vb & 0x7FFFFFFFu;
        mag = mag > GRID_MAX_BITS ? GRID_MAX_BITS : mag;
        vb = mag | (vb & 0x80000000u);
    }
    uint32_t t = vb + 0x200000u + (uint32_t)((int32_t)vb >> 31);
    grid_bits = t & 0xFFC00000u;
    return ((t >> 22) & 7u) | (t >> 28);
}

template <bool FLOOR>
__device__ __forceinline__ uint32_t sr_code_keep(float x, int e, uint32_t rinv, uint32_t& grid_bits)
{
    uint32_t mag = __float_as_uint(__builtin_ldexpf(__builtin_fabsf(x), e));
    if (FLOOR) mag = mag > GRID_MAX_BITS ? GRID_MAX_BITS : mag;
    uint32_t t = mag + rinv;
    grid_bits = t & 0xFFC00000u;
    return (t >> 22) | ((__float_as_uint(x) >> 28) & 8u);
}

// round_S of a non-negative value whose sign nibble (0 or 8) is supplied separately.
template <bool FLOOR>
__device__ __forceinline__ uint32_t sr_code_mag(float a, int e, uint32_t rinv, uint32_t sign8)
{
    uint32_t mag = __float_as_uint(__builtin_ldexpf(a, e));
    if (FLOOR) mag = mag > GRID_MAX_BITS ? GRID_MAX_BITS : mag;
    return ((mag + rinv) >> 22) | sign8;
}

// round_D of a non-negative value a with the sign supplied separately (sign8 = 0 or 8).
// Only for values whose scaled form is exact (E2M1 x 2^s or bf16 sources near a
// threshold are): the tie then goes up in magnitude for +, down for -.
template <bool FLOOR>
__device__ __forceinline__ uint32_t rtn_code_mag(float a, int e, uint32_t sign8)
{
    uint32_t mag = __float_as_uint(__builtin_ldexpf(a, e));
    if (FLOOR) mag = mag > GRID_MAX_BITS ? GRID_MAX_BITS : mag;
    return ((mag + 0x200000u - (sign8 >> 3)) >> 22) | sign8;
}

// |value| of an E2M1 code times 2^s, from the same bit layout: (code & 7) << 22 is
// m * 2^-126 as an FP32 pattern.  Exact in any rounding mode.
__device__ __forceinline__ float dequant_mag(uint32_t code, uint32_t byte)
{
    return __builtin_ldexpf(__uint_as_float((code & 7u) << 22), (int)byte - 1);
}

// Q-EMA (Algorithm 1): bracket from y = w/S, choice by z = w_ema/S.
// y_is_exact_zero: w itself is +-0 (then y = 0 is an E2M1 value and is kept); a nonzero w whose
// y underflowed to 0 in FP32 still has the bracket [0, 0.5].
__device__ __forceinline__ uint32_t round_ema(float y, float z, bool floor_mode, bool w_is_zero)
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
    up = up && (fr != 0.0f || (ab == 0u && !w_is_zero));   // w/S already an E2M1 value: keep it
    return (2u * (E - 127u) + (uint32_t)fl + (up ? 1u : 0u)) | ((yb >> 28) & 8u);
}

// signed value of an E2M1 code times 2^s (byte = s + 127), exact in FP32 (may be subnormal)
__device__ __forceinline__ float dequant(uint32_t code, uint32_t byte)
{
    return __uint_as_float(__float_as_uint(dequant_mag(code, byte)) | ((code & 8u) << 28));
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
        uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(pb >> 32), c1, k0, 0x96);   // three-way xor
        uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(pa >> 32), c3, k1, 0x96);
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

// The eight rounding addends ((65535 - r16) << 6) | 63 of an 8-element block, for sr_code().
struct U8 { uint32_t w[8]; };

// (16-bit field of w) * 64 + 63 in one instruction; HIGH selects the upper field.
template <bool HIGH>
__device__ __forceinline__ uint32_t field16_times64_plus63(uint32_t w)
{
    uint32_t r;
    if (HIGH) asm("v_mad_u32_u16 %0, %1, 64, 63 op_sel:[1,0,0,0]" : "=v"(r) : "v"(w));
    else      asm("v_mad_u32_u16 %0, %1, 64, 63" : "=v"(r) : "v"(w));
    return r;
}

__device__ __forceinline__ U8 sr_addends(uint64_t blk, uint32_t tensor_id, uint32_t k0, uint32_t k1)
{
    U4 r = sr_block(blk, tensor_id, k0, k1);
    U8 a;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t inv = ~r.w[i];                       // both 16-bit fields become 65535 - r16
        a.w[2 * i] = field16_times64_plus63<false>(inv);
        a.w[2 * i + 1] = field16_times64_plus63<true>(inv);
    }
    return a;
}

// ---- E3M0 elements (the other 4-bit format of the paper's format ablation, Table 7) -------------
// Code = sign << 3 | exponent field E (3 bits, no mantissa bit); magnitude 0 for E = 0 and 2^(E-3)
// otherwise: 0, 0.25, 0.5, 1, 2, 4, 8, 16 (bias 3, no Inf/NaN codes), Q_p = 16, E_max = 4.
// The same construction as for E2M1 works one bit higher: v = x * 2^(-s-124) puts |y| in [0, 16] onto
// FP32 patterns whose exponent field IS the code of the lower neighbour (|y| < 0.25 lands in the
// subnormals, the bracket [0, 0.25]) and whose 23 mantissa bits are p * 2^23.
//   truncation-free scale: s = ceil(log2(M / 16)) = e - 4 for M = 2^e exactly, e - 3 otherwise;
//   Eq. 2's scale:         s = floor(log2 M) - 4.
// epsilon = 1e-8 = 1.34 * 2^-27 for an all-zero group gives s = -30 resp. -31.
__device__ __forceinline__ uint32_t scale_byte_e3m0(uint32_t amax_bits, bool floor_mode)
{
    uint32_t field = (amax_bits + (floor_mode ? 0u : 0x7FFFFFu)) >> 23;   // carries iff the mantissa is not zero
    uint32_t b;
    asm("v_sub_u32_e64 %0, %1, 4 clamp" : "=v"(b) : "v"(field));
    return amax_bits == 0u ? (floor_mode ? 96u : 97u) : b;
}

constexpr uint32_t GRID_MAX_BITS_E3M0 = 7u << 23;     // 16 * 2^-124

__device__ __forceinline__ int grid_exponent_e3m0(uint32_t byte) { return 3 - (int)byte; }

// round_D; rounding mode toward minus infinity (see rtn_code).
template <bool FLOOR>
__device__ __forceinline__ uint32_t rtn_code_e3m0(float x, int e)
{
    uint32_t vb = __float_as_uint(__builtin_ldexpf(x, e));
    uint32_t mag = vb & 0x7FFFFFFFu;
    if (FLOOR) mag = mag > GRID_MAX_BITS_E3M0 ? GRID_MAX_BITS_E3M0 : mag;
    uint32_t t = mag + 0x400000u + (uint32_t)((int32_t)vb >> 31);
    return (t >> 23) | ((vb >> 28) & 8u);
}

// round_S; rounding mode toward plus infinity; rinv = ((65535 - r16) << 7) | 127.
template <bool FLOOR>
__device__ __forceinline__ uint32_t sr_code_e3m0(float x, int e, uint32_t rinv)
{
    uint32_t mag = __float_as_uint(__builtin_ldexpf(__builtin_fabsf(x), e));
    if (FLOOR) mag = mag > GRID_MAX_BITS_E3M0 ? GRID_MAX_BITS_E3M0 : mag;
    return ((mag + rinv) >> 23) | ((__float_as_uint(x) >> 28) & 8u);
}

__device__ __forceinline__ U8 sr_addends_e3m0(uint64_t blk, uint32_t tensor_id, uint32_t k0, uint32_t k1)
{
    U4 r = sr_block(blk, tensor_id, k0, k1);
    U8 a;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a.w[2 * i] = ((65535u - (r.w[i] & 0xFFFFu)) << 7) | 127u;
        a.w[2 * i + 1] = ((65535u - (r.w[i] >> 16)) << 7) | 127u;
    }
    return a;
}

// signed value of an E3M0 code times 2^s: (E << 23) is 2^(E-127) as an FP32 pattern (0 for E = 0)
__device__ __forceinline__ float dequant_e3m0(uint32_t code, uint32_t byte)
{
    float mag = __builtin_ldexpf(__uint_as_float((code & 7u) << 23), (int)byte - 3);
    return __uint_as_float(__float_as_uint(mag) | ((code & 8u) << 28));
}

// ---- cross-lane max over aligned groups of 4 lanes (one 32-element group) ---
__device__ __forceinline__ uint32_t quad_max(uint32_t v)
{
    uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);  // lane ^ 1
    v = v > o ? v : o;
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);           // lane ^ 2
    return v > o ? v : o;
}

// ---- source loads: 8 consecutive elements as FP32; a source is read once, so the loads
//      carry the nontemporal hint --------------------------
struct F8 { float v[8]; };

__device__ __forceinline__ F8 load8(const float* p)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4* q = reinterpret_cast<const f4*>(p);
    const f4 a = __builtin_nontemporal_load(q), b = __builtin_nontemporal_load(q + 1);
    F8 r;
    r.v[0] = a.x; r.v[1] = a.y; r.v[2] = a.z; r.v[3] = a.w;
    r.v[4] = b.x; r.v[5] = b.y; r.v[6] = b.z; r.v[7] = b.w;
    return r;
}

__device__ __forceinline__ F8 load8(const uint16_t* p)   // bf16 bit patterns
{
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    const u4 a = __builtin_nontemporal_load(reinterpret_cast<const u4*>(p));
    F8 r;
    r.v[0] = __uint_as_float(a.x << 16); r.v[1] = __uint_as_float(a.x & 0xFFFF0000u);
    r.v[2] = __uint_as_float(a.y << 16); r.v[3] = __uint_as_float(a.y & 0xFFFF0000u);
    r.v[4] = __uint_as_float(a.z << 16); r.v[5] = __uint_as_float(a.z & 0xFFFF0000u);
    r.v[6] = __uint_as_float(a.w << 16); r.v[7] = __uint_as_float(a.w & 0xFFFF0000u);
    return r;
}

// The same in two steps, for loads issued ahead of their use: 4 registers hold 8 bf16 values.
typedef uint32_t bf16x8_raw __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8_raw load8_raw(const uint16_t* p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const bf16x8_raw*>(p));
}
__device__ __forceinline__ F8 expand8(bf16x8_raw a)
{
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

// max(|a|, |b|, m) on FP32 bit patterns in one instruction: for finite values the order of the
// magnitudes is the order of their bit patterns, and the source modifiers take the absolute values
// (the separate AND and the two-operand maximum cost more issue cycles than this one instruction).
__device__ __forceinline__ uint32_t absmax3_bits(float a, float b, uint32_t m)
{
    float r;
    asm("v_max3_f32 %0, |%1|, |%2|, %3" : "=v"(r) : "v"(a), "v"(b), "v"(__uint_as_float(m)));
    return __float_as_uint(r);
}

__device__ __forceinline__ uint32_t amax_bits8(const F8& x)
{
    uint32_t m = 0;
#pragma unroll
    for (int t = 0; t < 8; t += 2) m = absmax3_bits(x.v[t], x.v[t + 1], m);
    return m;
}

}  // namespace mxd

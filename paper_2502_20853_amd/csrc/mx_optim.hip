// Q-Ramping's customised AdamW (Algorithm 2; Sec. 6.2) for gfx950: one streaming pass over the
// weights of the quantized layers, bound by memory.
//
// A weight element with amplification factor N_w has N_w times the global batch size -- its
// gradient is accumulated over N_w steps -- and N_w times the global learning rate.  Per element
// and step:
//     g_acc += grad;  acc_steps += 1;
//     if acc_steps >= N_w:
//         g = g_acc / acc_steps;  lr_w = N_w * lr;  u = ++updates;
//         w = w * (1 - lr_w * weight_decay)
//         m = beta1 * m + (1 - beta1) * g;   v = beta2 * v + (1 - beta2) * g * g
//         w = w - (lr_w / (1 - beta1^u)) * m / (sqrt(v) / sqrt(1 - beta2^u) + eps)
//         g_acc = 0;  acc_steps = 0
// An element with factor N thus follows AdamW at learning rate N * lr on the means of N consecutive
// gradients, with the bias correction counting its own updates.  FP32 arithmetic; 1 - beta and
// ln(beta) come from the host in double precision, and 1 - beta^u = -expm1(u * ln(beta)) keeps its
// relative accuracy when u is small.
//
// Work split: one lane owns 4 consecutive elements (16-byte accesses on every array).
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdint>
#include "mx_launch.hpp"

namespace {

constexpr int OPT_THREADS = 256;

typedef float v4f __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));

struct AdamArgs {
    float* w;
    const void* grad;
    float* m;
    float* v;
    float* g_acc;                 // null iff factor is null
    const int32_t* factor;        // null: 1 everywhere
    int32_t* acc_steps;           // null iff factor is null
    int32_t* updates;
    int64_t quads;                // count / 4
    float lr, beta1, beta2, eps, weight_decay;
    float one_minus_beta1, one_minus_beta2, ln_beta1, ln_beta2;
};

__device__ __forceinline__ float4 load_grad4(const float* g, int64_t q)
{
    const v4f r = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(g) + q);
    return make_float4(r.x, r.y, r.z, r.w);
}

__device__ __forceinline__ float4 load_grad4(const uint16_t* g, int64_t q)       // bf16 bit patterns
{
    const v2u r = __builtin_nontemporal_load(reinterpret_cast<const v2u*>(g) + q);
    return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u),
                       __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xFFFF0000u));
}

struct ElemState { float w, m, v, acc; int32_t steps, upd; };

__device__ __forceinline__ void adamw_element(const AdamArgs& a, ElemState& s, float g, int32_t n_w)
{
    s.acc = s.acc + g;
    s.steps += 1;
    if (s.steps < n_w) return;                          // this element's batch is not full yet
    const float gm = __fdiv_rn(s.acc, (float)s.steps);
    const float lr_w = (float)n_w * a.lr;
    s.upd += 1;
    const float u = (float)s.upd;
    s.w = s.w * (1.0f - lr_w * a.weight_decay);
    s.m = a.beta1 * s.m + a.one_minus_beta1 * gm;
    s.v = a.beta2 * s.v + a.one_minus_beta2 * gm * gm;
    const float bc1 = -expm1f(u * a.ln_beta1);
    const float bc2 = -expm1f(u * a.ln_beta2);
    const float denom = __fdiv_rn(__fsqrt_rn(s.v), __fsqrt_rn(bc2)) + a.eps;
    s.w = s.w - __fdiv_rn(__fdiv_rn(lr_w, bc1) * s.m, denom);
    s.acc = 0.0f;
    s.steps = 0;
}

template <typename GradT, bool RAMPING>
__global__ __launch_bounds__(OPT_THREADS) void ramping_adamw_kernel(AdamArgs a)
{
    const int64_t q = (int64_t)blockIdx.x * OPT_THREADS + threadIdx.x;
    if (q >= a.quads) return;
    // every array is touched once per step and the state of a model is far larger than the
    // last-level cache: all accesses are marked streaming
    const float4 g4 = load_grad4(static_cast<const GradT*>(a.grad), q);
    v4f* wp = reinterpret_cast<v4f*>(a.w) + q;
    v4f* mp = reinterpret_cast<v4f*>(a.m) + q;
    v4f* vp = reinterpret_cast<v4f*>(a.v) + q;
    v4i* up = reinterpret_cast<v4i*>(a.updates) + q;
    const v4f w4 = __builtin_nontemporal_load(wp), m4 = __builtin_nontemporal_load(mp),
              v4 = __builtin_nontemporal_load(vp);
    const v4i u4 = __builtin_nontemporal_load(up);
    v4f acc4 = {0.f, 0.f, 0.f, 0.f};
    v4i n4 = {1, 1, 1, 1}, c4 = {0, 0, 0, 0};
    if (RAMPING) {
        acc4 = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(a.g_acc) + q);
        n4 = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.factor) + q);
        c4 = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(a.acc_steps) + q);
    }
    ElemState e[4] = {{w4.x, m4.x, v4.x, acc4.x, c4.x, u4.x}, {w4.y, m4.y, v4.y, acc4.y, c4.y, u4.y},
                      {w4.z, m4.z, v4.z, acc4.z, c4.z, u4.z}, {w4.w, m4.w, v4.w, acc4.w, c4.w, u4.w}};
    const float g[4] = {g4.x, g4.y, g4.z, g4.w};
    const int32_t n[4] = {n4.x, n4.y, n4.z, n4.w};
#pragma unroll
    for (int t = 0; t < 4; ++t) adamw_element(a, e[t], g[t], n[t]);
    const v4f wo = {e[0].w, e[1].w, e[2].w, e[3].w}, mo = {e[0].m, e[1].m, e[2].m, e[3].m},
              vo = {e[0].v, e[1].v, e[2].v, e[3].v};
    const v4i uo = {e[0].upd, e[1].upd, e[2].upd, e[3].upd};
    __builtin_nontemporal_store(wo, wp);
    __builtin_nontemporal_store(mo, mp);
    __builtin_nontemporal_store(vo, vp);
    __builtin_nontemporal_store(uo, up);
    if (RAMPING) {
        const v4f ao = {e[0].acc, e[1].acc, e[2].acc, e[3].acc};
        const v4i co = {e[0].steps, e[1].steps, e[2].steps, e[3].steps};
        __builtin_nontemporal_store(ao, reinterpret_cast<v4f*>(a.g_acc) + q);
        __builtin_nontemporal_store(co, reinterpret_cast<v4i*>(a.acc_steps) + q);
    }
}

}  // namespace

namespace mxl {

hipError_t launch_ramping_adamw(const RampingAdamwParams& p, hipStream_t st)
{
    AdamArgs a{};
    a.w = p.w; a.grad = p.grad; a.m = p.m; a.v = p.v; a.g_acc = p.g_acc; a.factor = p.factor;
    a.acc_steps = p.acc_steps; a.updates = p.updates; a.quads = p.count / 4;
    a.lr = p.lr; a.beta1 = p.beta1; a.beta2 = p.beta2; a.eps = p.eps; a.weight_decay = p.weight_decay;
    a.one_minus_beta1 = (float)(1.0 - (double)p.beta1);
    a.one_minus_beta2 = (float)(1.0 - (double)p.beta2);
    a.ln_beta1 = (float)std::log((double)p.beta1);
    a.ln_beta2 = (float)std::log((double)p.beta2);
    dim3 grid((unsigned)((a.quads + OPT_THREADS - 1) / OPT_THREADS)), block(OPT_THREADS);
    const bool ramping = p.factor != nullptr;
    if (p.grad_bf16) {
        if (ramping) hipLaunchKernelGGL((ramping_adamw_kernel<uint16_t, true>), grid, block, 0, st, a);
        else         hipLaunchKernelGGL((ramping_adamw_kernel<uint16_t, false>), grid, block, 0, st, a);
    } else {
        if (ramping) hipLaunchKernelGGL((ramping_adamw_kernel<float, true>), grid, block, 0, st, a);
        else         hipLaunchKernelGGL((ramping_adamw_kernel<float, false>), grid, block, 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace mxl

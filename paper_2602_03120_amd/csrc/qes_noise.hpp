// Device-side noise generator of the QES hot path for gfx950.
//
// Implements docs/NOISE_SPEC.md (paper §3.2 Eq. 3; App. A.1 for the 4-bit container):
// Philox4x32-10 -> exactly specified Box-Muller -> stochastic rounding. Every floating-point
// operation that can reach an integer is written out (explicit fma, no contraction: this file is
// compiled with -ffp-contract=off), so the integers match the CPU oracle bit for bit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qes {

constexpr uint32_t kPhiloxM0 = 0xD2511F53u;
constexpr uint32_t kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u;
constexpr uint32_t kPhiloxW1 = 0xBB67AE85u;

struct Words {
    uint32_t w0, w1, w2, w3;
};

// N1. Ten rounds on counter (c0,c1,c2,c3) with key (k0,k1). Arguments that are wave-uniform
// (key, tensor id, high counter words) stay in scalar registers; the first rounds then cost less.
__device__ __forceinline__ Words philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    return Words{c0, c1, c2, c3};
}

// Three-input xor in one instruction (gfx950 v_bitop3_b32, truth table 0x96).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// N1 + N2 for the tensor kernels: counter (pair, 0, tensor_id, 0) with a wave-uniform key and
// tensor id. Same function as philox4x32_10(pair, 0, tensor_id, 0, k0, k1); written round by round
// so that everything that does not depend on the lane is computed on the scalar unit (the second
// product of the first Philox round, the first product of the second, the pre-xored round keys) and every
// three-input xor of lane data is a single instruction.
__device__ __forceinline__ Words philox_tensor(uint32_t pair, uint32_t tensor_id, uint32_t k0, uint32_t k1)
{
    // first Philox round
    uint64_t p0 = (uint64_t)kPhiloxM0 * (uint64_t)pair;
    const uint64_t u1 = (uint64_t)kPhiloxM1 * (uint64_t)tensor_id;           // uniform
    const uint32_t c0_1 = (uint32_t)(u1 >> 32) ^ k0;                          // uniform
    const uint32_t c1_1 = (uint32_t)u1;                                       // uniform
    uint32_t c2 = (uint32_t)(p0 >> 32) ^ k1;
    uint32_t c3 = (uint32_t)p0;
    k0 += kPhiloxW0;
    k1 += kPhiloxW1;
    // second Philox round
    const uint64_t u0 = (uint64_t)kPhiloxM0 * (uint64_t)c0_1;                 // uniform
    uint64_t p1 = (uint64_t)kPhiloxM1 * (uint64_t)c2;
    uint32_t c0 = (uint32_t)(p1 >> 32) ^ (c1_1 ^ k0);
    uint32_t c1 = (uint32_t)p1;
    c2 = c3 ^ ((uint32_t)(u0 >> 32) ^ k1);
    const uint32_t c3_2 = (uint32_t)u0;                                       // uniform
    k0 += kPhiloxW0;
    k1 += kPhiloxW1;
    // third Philox round
    p0 = (uint64_t)kPhiloxM0 * (uint64_t)c0;
    p1 = (uint64_t)kPhiloxM1 * (uint64_t)c2;
    c0 = xor3((uint32_t)(p1 >> 32), c1, k0);
    c2 = (uint32_t)(p0 >> 32) ^ (c3_2 ^ k1);
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    // Philox rounds four to ten
#pragma unroll
    for (int r = 3; r < 10; ++r) {
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
        p0 = (uint64_t)kPhiloxM0 * (uint64_t)c0;
        p1 = (uint64_t)kPhiloxM1 * (uint64_t)c2;
        c0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        c2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
    }
    return Words{c0, c1, c2, c3};
}

// Correctly rounded sqrt for x in {-0} U [2^-24, 64): the hardware approximation (within one
// ulp) followed by the usual one-ulp correction against the exact residual. No range scaling is
// needed because x = -2 ln(u1) is never subnormal.
__device__ __forceinline__ float sqrt_rn_bounded(float x)
{
    const float s = __builtin_amdgcn_sqrtf(x);
    const float s_dn = __uint_as_float(__float_as_uint(s) - 1u);
    const float s_up = __uint_as_float(__float_as_uint(s) + 1u);
    const float r_dn = __builtin_fmaf(-s_dn, s, x);
    const float r_up = __builtin_fmaf(-s_up, s, x);
    float r = (r_dn <= 0.0f) ? s_dn : s;
    r = (r_up > 0.0f) ? s_up : r;
    return r;
}

// N4. ln(m * 2^-24) for integer m in [1, 2^24]; result <= 0.
__device__ __forceinline__ float ln_u1(uint32_t m)
{
    const float xf = (float)m;
    const uint32_t ix = __float_as_uint(xf) - 0x3F3504F3u;
    // float(e - 24) for e = ix >> 23 in [0,24]: 2^23 + e is exact, so is the subtraction
    const float ef = __uint_as_float((ix >> 23) | 0x4B000000u) - 8388632.0f;
    const float t = __uint_as_float((ix & 0x007FFFFFu) + 0x3F3504F3u) - 1.0f;
    float p = -0x1.a7d988p-4f;
    p = __builtin_fmaf(p, t, 0x1.4d64acp-3f);
    p = __builtin_fmaf(p, t, -0x1.6049d0p-3f);
    p = __builtin_fmaf(p, t, 0x1.976dd8p-3f);
    p = __builtin_fmaf(p, t, -0x1.ff7476p-3f);
    p = __builtin_fmaf(p, t, 0x1.5559f0p-2f);
    p = __builtin_fmaf(p, t, -0x1.000060p-1f);
    const float l1 = __builtin_fmaf(t * t, p, t);
    return __builtin_fmaf(ef, 0x1.62e430p-1f, l1);
}

// N3 + N4. The two standard Gaussians of one Philox call (lane 0: even element, lane 1: odd).
__device__ __forceinline__ void gauss_pair(uint32_t w0, uint32_t w1, float &eps0, float &eps1)
{
    const float L = ln_u1((w0 >> 8) + 1u);
    const float r = sqrt_rn_bounded(-2.0f * L);
    const float f = (float)(w1 & 0x3FFFFFC0u) * 0x1p-30f;   // = ((w1 >> 6) & 0xFFFFFF) * 2^-24, exact
    const float z = f * f;
    float sp = 0x1.3e17cap-13f;
    sp = __builtin_fmaf(sp, z, -0x1.32535ap-8f);
    sp = __builtin_fmaf(sp, z, 0x1.4668f2p-4f);
    sp = __builtin_fmaf(sp, z, -0x1.4abbc4p-1f);
    sp = __builtin_fmaf(sp, z, 0x1.921fb6p+0f);
    float c = 0x1.c1f064p-11f;
    c = __builtin_fmaf(c, z, -0x1.54f61ap-6f);
    c = __builtin_fmaf(c, z, 0x1.03bd06p-2f);
    c = __builtin_fmaf(c, z, -0x1.3bd3a6p+0f);
    c = __builtin_fmaf(c, z, 0x1.fffffep-1f);
    const float s = f * sp;
    // quadrant q = w1 >> 30: (c,s), (-s,c), (-c,-s), (s,-c)
    const bool swap = (w1 & 0x40000000u) != 0u;
    const float a = swap ? s : c;
    const float b = swap ? c : s;
    const uint32_t sign_a = (w1 ^ (w1 << 1)) & 0x80000000u;   // q = 1 or 2
    const uint32_t sign_b = w1 & 0x80000000u;                 // q = 2 or 3
    const float ca = __uint_as_float(__float_as_uint(a) ^ sign_a);
    const float sb = __uint_as_float(__float_as_uint(b) ^ sign_b);
    eps0 = r * ca;
    eps1 = r * sb;
}

// N5 + N6. One lane's integer perturbation from its Gaussian and its rounding word.
__device__ __forceinline__ int32_t delta_of(float eps, uint32_t wround, float sigma)
{
    const float ub = (float)(wround >> 8) * 0x1p-24f;
    const float t = sigma * eps;
    const float fl = __builtin_floorf(t);
    const float fr = t - fl;
    int32_t d = (int32_t)fl + ((ub < fr) ? 1 : 0);
    d = d < -8 ? -8 : d;
    d = d > 7 ? 7 : d;
    return d;
}

// N5 + N6 with the result kept in fp32 (every value is a small integer, so this is the same number):
// saves the two int<->float conversions when the consumer is the fp32 sum of Eq. 5. CLAMP = false
// is valid when sigma <= 1.2: |sigma*eps| < 7, so the container clamp cannot fire.
template <bool CLAMP>
__device__ __forceinline__ float delta_f32(float eps, uint32_t wround, float sigma)
{
    const float ub = (float)(wround >> 8) * 0x1p-24f;
    const float t = sigma * eps;
    const float fl = __builtin_floorf(t);
    const float fr = t - fl;
    float d = fl + ((ub < fr) ? 1.0f : 0.0f);
    if (CLAMP) d = __builtin_amdgcn_fmed3f(d, -8.0f, 7.0f);
    return d;
}

template <bool CLAMP>
__device__ __forceinline__ void delta_pair_f32(uint32_t k0, uint32_t k1, uint32_t tensor_id, uint32_t pair,
                                               float sigma, float &d0, float &d1)
{
    const Words w = philox_tensor(pair, tensor_id, k0, k1);
    float e0, e1;
    gauss_pair(w.w0, w.w1, e0, e1);
    d0 = delta_f32<CLAMP>(e0, w.w2, sigma);
    d1 = delta_f32<CLAMP>(e1, w.w3, sigma);
}

// The two perturbations of pair `pair` (32-bit pair index, high counter word 0) of a tensor.
__device__ __forceinline__ void delta_pair(uint32_t k0, uint32_t k1, uint32_t tensor_id,
                                           uint32_t pair, float sigma, int32_t &d0, int32_t &d1)
{
    const Words w = philox_tensor(pair, tensor_id, k0, k1);
    float e0, e1;
    gauss_pair(w.w0, w.w1, e0, e1);
    d0 = delta_of(e0, w.w2, sigma);
    d1 = delta_of(e1, w.w3, sigma);
}

// N7 with the operands held in fp32: base and delta are small integers, so base + delta is exact
// and the range test is a median. Returns base + delta if qmin <= base + delta <= qmax, else base.
__device__ __forceinline__ float gate_f32(float base, float delta, float qmin, float qmax)
{
    const float v = base + delta;
    return (__builtin_amdgcn_fmed3f(v, qmin, qmax) == v) ? v : base;
}

// N7 / Alg. 2 gate: v if qmin <= v <= qmax else keep.
__device__ __forceinline__ int32_t gate(int32_t base, int32_t delta, int32_t qmin, uint32_t qspan)
{
    const uint32_t v = (uint32_t)base + (uint32_t)delta;   // wraps instead of overflowing
    return (v - (uint32_t)qmin <= qspan) ? (int32_t)v : base;
}

}  // namespace qes

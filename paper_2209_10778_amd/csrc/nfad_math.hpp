// nfad_math.hpp -- fp32 device arithmetic for the four activations and their derivatives.
//
// Every activation here has the shape f(x) = x * s(x) with s a smooth step from 0 to 1
// (Table I of the paper; GELU-erf is the textbook x*Phi(x)).  Pushing the dual number
// (x, 1) through it (Sec. II-C eq. 3) gives
//     y = x * s(x),      dydx = s(x) + x * s'(x).
// The pair is evaluated from ONE hardware exponential (v_exp_f32, base 2) and one hardware
// reciprocal (v_rcp_f32); all arithmetic is fp32 whatever the storage type.
//
// Two tiers, chosen by the storage type the result is rounded to (kWide = fp32 storage):
//
//  * wide   -- results must be good to a few fp32 ulps everywhere.  The code works with the
//    small "complement" p of the step on each side of zero instead of with s itself:
//        for the three odd-symmetric steps (s(x) + s(-x) = 1):   p = s(-|x|)  in [0, 1/2]
//        y    = max(x, 0) - |x| * p            (x - x p for x > 0,  x p for x < 0)
//        s(x) = x > 0 ? 1 - p : p
//    so nothing of the form 1 + tanh, 1 + erf or 1 - sigmoid is formed where it cancels and
//    only non-positive arguments are exponentiated.
//
//  * narrow -- results are rounded to fp16/bf16 (>= 2^-12 relative), so an fp32 ulp of
//    absolute error in a quantity near 1 is invisible and a few instructions are dropped:
//    s is formed directly, 1 - s by subtraction, y = x * s.  Small results (x << 0) stay
//    relatively accurate because s itself is still computed without cancellation there.
//    With twice the elements per byte, this is the tier where VALU cycles show next to HBM.
//
// Both tiers return finite results for every finite x (y -> x, dydx -> 1 as x -> +inf;
// y -> -0, dydx -> 0 as x -> -inf): an exponential that overflows to +inf only ever
// reaches a reciprocal (1/inf = 0), never a product with zero.
#pragma once
#ifndef __HIPCC_RTC__
#include <hip/hip_runtime.h>
#endif

namespace nfad {

__device__ __forceinline__ float ex2(float v) { return __builtin_amdgcn_exp2f(v); }  // 2^v
__device__ __forceinline__ float rcp(float v) { return __builtin_amdgcn_rcpf(v); }   // 1/v
__device__ __forceinline__ float fma_(float a, float b, float c) { return __builtin_fmaf(a, b, c); }

static constexpr float kLog2e = 1.44269504088896340736f;

enum Kind : int { kGeluTanh = 0, kGeluErf = 1, kSwish = 2, kMish = 3 };

// 0.5 erfcx(a / sqrt 2) ~= t P(t), t = 1/(1 + Q a): struct ErfcxWide (degree 8), ErfcxNarrow (degree 6);
// logit(Phi(a)) / a as a polynomial in a: struct PhiLogitNarrow
#include "nfad_erfcx_coeffs.inc"

// Phi(-a) / exp(-a^2/2) for a >= 0, i.e. the scaled complementary error function.
template <class Fit>
__device__ __forceinline__ float half_erfcx(float a) {
  const float t = rcp(fma_(Fit::kQ, a, 1.0f));
  float P = Fit::kC[Fit::kDeg];
#pragma unroll
  for (int i = Fit::kDeg - 1; i >= 0; --i) P = fma_(P, t, Fit::kC[i]);
  return P * t;
}

template <int KIND>
struct Act;

// ---------------------------------------------------------------- Swish (Table I, Table II)
// s = sigmoid, s' = sigmoid(x) sigmoid(-x).
template <>
struct Act<kSwish> {
  template <bool kWide>
  __device__ __forceinline__ static void eval(float x, float& y, float& d) {
    if constexpr (kWide) {
      // e = exp(-|x|): sigmoid(|x|) = 1/(1+e) =: r, sigmoid(-|x|) = e r =: p, s' = r p.
      const float a = __builtin_fabsf(x);
      const float e = ex2(-kLog2e * a);
      const float r = rcp(1.0f + e);
      const float p = e * r;
      y = fma_(-a, p, __builtin_fmaxf(x, 0.0f));
      const float s = x > 0.0f ? r : p;
      d = fma_(x, r * p, s);
    } else {
      const float s = rcp(1.0f + ex2(-kLog2e * x));
      y = x * s;
      d = fma_(y, 1.0f - s, s);  // s + x s (1 - s): Table II as printed
    }
  }
};

// ---------------------------------------------------------------- GELU, tanh form (Table I)
// 0.5 (1 + tanh u) = sigmoid(2u), u = c (x + k x^3) odd in x, so the Swish scheme applies
// with exponent 2u and  s' = sigmoid(2u) sigmoid(-2u) * 2u',  2u' = 2c (1 + 3 k x^2).
// x^2 is capped so that a huge finite |x| cannot produce inf * 0 in the derivative; the cap
// is far beyond the point (|x| ~ 6) where exp(-2|u|) has underflowed to zero.
template <>
struct Act<kGeluTanh> {
  static constexpr float kC = 0.79788456080286535588f;  // sqrt(2/pi)
  static constexpr float kK = 0.044715f;
  template <bool kWide>
  __device__ __forceinline__ static void eval(float x, float& y, float& d) {
    const float x2 = __builtin_fminf(x * x, 1.0e30f);
    const float du2 = fma_(6.0f * kC * kK, x2, 2.0f * kC);  // 2u'
    if constexpr (kWide) {
      const float a = __builtin_fabsf(x);
      const float v = a * fma_(2.0f * kC * kK * kLog2e, x2, 2.0f * kC * kLog2e);  // 2|u| log2 e
      const float e = ex2(-v);
      const float r = rcp(1.0f + e);
      const float p = e * r;
      y = fma_(-a, p, __builtin_fmaxf(x, 0.0f));
      const float s = x > 0.0f ? r : p;
      d = fma_(x, (r * p) * du2, s);
    } else {
      const float w = x * fma_(-2.0f * kC * kK * kLog2e, x2, -2.0f * kC * kLog2e);  // -2u log2 e
      const float s = rcp(1.0f + ex2(w));
      y = x * s;
      d = fma_(y * (1.0f - s), du2, s);
    }
  }
};

// ---------------------------------------------------------------- GELU, erf form
// s = Phi, s' = phi.  Phi(-a) = exp(-a^2/2) * half_erfcx(a); the same exponential gives the
// density phi = exp(-a^2/2)/sqrt(2 pi).
template <>
struct Act<kGeluErf> {
  static constexpr float kInvSqrt2Pi = 0.39894228040143267794f;
  template <bool kWide>
  __device__ __forceinline__ static void eval(float x, float& y, float& d) {
    const float a = __builtin_fabsf(x);
    const float E = ex2((-0.5f * kLog2e) * (x * x));
    if constexpr (kWide) {
      const float p = half_erfcx<ErfcxWide>(a) * E;  // Phi(-|x|)
      y = fma_(-a, p, __builtin_fmaxf(x, 0.0f));
      const float s = x > 0.0f ? 1.0f - p : p;
      d = fma_(x, E * kInvSqrt2Pi, s);
    } else {
      const float p = half_erfcx<ErfcxNarrow>(a) * E;
      const float s = x > 0.0f ? 1.0f - p : p;
      y = x * s;
      d = fma_(x, E * kInvSqrt2Pi, s);
    }
  }
};

// ---------------------------------------------------------------- Mish (Table I)
// With e = exp(x) and n = e (e + 2):  tanh(ln(1 + e)) = n / (n + 2) =: t  (no log, no tanh),
// 1 - t^2 = 4 (e + 1)^2 / (n + 2)^2, softplus' = e / (e + 1), hence
//     dydx = t + x * 4 e (e + 1) / (n + 2)^2.
// x is capped at 41.5 (< 60 ln 2) inside the exponential (t and dydx are already 1 to fp32
// precision far below that) so that n cannot overflow; the cap is a compare-and-select, not
// a min, so that a NaN input stays NaN in both results.  Wide tier: for x > 0,
// y = x - 2x/(n+2) keeps the last bits that x * t would lose.
__device__ __forceinline__ float mish_cap(float x) { return x > 41.5f ? 41.5f : x; }
template <>
struct Act<kMish> {
  template <bool kWide>
  __device__ __forceinline__ static void eval(float x, float& y, float& d) {
    const float xc = mish_cap(x);
    const float e = ex2(kLog2e * xc);
    const float n = fma_(e, e, e + e);
    const float R = rcp(n + 2.0f);
    const float t = n * R;
    if constexpr (kWide) y = x > 0.0f ? fma_(x, -2.0f * R, x) : x * t;
    else y = x * t;
    const float g = fma_(4.0f, e, 4.0f) * e;  // 4 e (e + 1)
    d = fma_(g * R, xc * R, t);
  }
};

// Value only / derivative only: the unused half of eval() is dead code the compiler drops.
template <int KIND, bool kWide>
__device__ __forceinline__ float act_value(float x) {
  float y, d;
  Act<KIND>::template eval<kWide>(x, y, d);
  return y;
}
// GELU-erf, value only, for 16-bit storage: x Phi(x) with Phi(x) = sigmoid(x L(|x|)), L a degree-6
// polynomial (logit(Phi(a)) / a on [0, 6.5]; the argument is clamped beyond, where Phi(-a) < 1e-10).
// One exponential, one reciprocal, no select: at 4 bytes per element (one 16-bit read, one
// 16-bit write) the erfcx form above is bound by the vector ALU, this one is not.  The polynomial's
// error stays below a fifth of an fp16 ulp wherever the result is above the absolute floor.
template <>
__device__ __forceinline__ float act_value<kGeluErf, false>(float x) {
  const float a = __builtin_fminf(__builtin_fabsf(x), PhiLogitNarrow::kMaxA);
  float M = PhiLogitNarrow::kC[PhiLogitNarrow::kDeg];
#pragma unroll
  for (int i = PhiLogitNarrow::kDeg - 1; i >= 0; --i) M = fma_(M, a, PhiLogitNarrow::kC[i]);
  return x * rcp(1.0f + ex2(x * M));
}
template <int KIND, bool kWide>
__device__ __forceinline__ float act_deriv(float x) {
  float y, d;
  Act<KIND>::template eval<kWide>(x, y, d);
  return d;
}

// ---------------------------------------------------------------- primitives of the save-all baseline
// The stand-alone primitive operators of ordinary back-propagation (sigmoid, tanh, erf):
// each result is rounded to storage and re-read in backward.
__device__ __forceinline__ float sigmoid_f(float x) {
  const float a = __builtin_fabsf(x);
  const float e = ex2(-kLog2e * a);
  const float r = rcp(1.0f + e);
  return x > 0.0f ? r : e * r;
}
// tanh(u) = sign(u) (1 - e)/(1 + e), e = exp(-2|u|); for tiny |u| the quotient form loses
// relative accuracy, which is harmless here (absolute error stays at the fp32 ulp of 1).
__device__ __forceinline__ float tanh_f(float u) {
  const float a = __builtin_fabsf(u);
  const float e = ex2((-2.0f * kLog2e) * a);
  const float t = (1.0f - e) * rcp(1.0f + e);
  return __builtin_copysignf(t, u);
}
// erf(z) = sign(z) (1 - erfc|z|), erfc|z| = 2 Phi(-sqrt2 |z|).
__device__ __forceinline__ float erf_f(float z) {
  const float a = 1.41421356237309504880f * __builtin_fabsf(z);
  const float E = ex2((-0.5f * kLog2e) * (a * a));
  const float erfc_a = 2.0f * half_erfcx<ErfcxWide>(a) * E;
  return __builtin_copysignf(1.0f - erfc_a, z);
}

}  // namespace nfad

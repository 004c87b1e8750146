// nfad_ops.hpp -- the per-element operations of the method and its two baselines, as plug-ins
// of the streaming skeleton (nfad_stream_device.hpp).  The arithmetic of the activations is
// in nfad_math.hpp.  The dual-number tangent (seed 1, Sec. II-C eq. 3) never touches memory.
#pragma once
#include "nfad_math.hpp"

namespace nfad {

// ------------------------------------------------------------------ per-element operations
// An Op maps kIn input elements to kOut output elements, all fp32 in registers.  kWide says
// whether the results will be stored as fp32 (true) or rounded to fp16/bf16 (false); the
// activations use it to pick their arithmetic tier, the other operations ignore it.

// Forward pass of the method: (x) -> (y, dydx).                       Sec. II-C eq. 3
template <int KIND>
struct FwdOp {
  static constexpr int kIn = 1, kOut = 2;
  // Swish and GELU-tanh: one exponential, one reciprocal and a handful of multiply-adds per element
  static constexpr bool kLight = KIND == kSwish || KIND == kGeluTanh;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    Act<KIND>::template eval<kWide>(in[0], out[0], out[1]);
  }
};
// Backward pass of the method: (gy, dydx) -> gx = gy * dydx.          Sec. II-C eq. 4
struct BwdOp {
  static constexpr int kIn = 2, kOut = 1;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    out[0] = in[0] * in[1];
  }
};
// Backward pass of a chain with M outputs: the tangents of all consumers merge at the source,
// gx = sum_m gy_m * dydx_m.  Inputs in the order gy0, dydx0, gy1, dydx1, ...        Sec. II-E, IV-B
template <int M>
struct BwdMultiOp {
  static constexpr int kIn = 2 * M, kOut = 1;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    float acc = in[0] * in[1];
#pragma unroll
    for (int m = 1; m < M; ++m) acc = fma_(in[2 * m], in[2 * m + 1], acc);
    out[0] = acc;
  }
};
// Recomputation baseline: forward keeps nothing but x.               Sec. II-C "Recomputation"
template <int KIND>
struct RecomputeFwdOp {
  static constexpr int kIn = 1, kOut = 1;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    out[0] = act_value<KIND, kWide>(in[0]);
  }
};
template <int KIND>
struct RecomputeBwdOp {  // (gy, x) -> gy * f'(x)
  static constexpr int kIn = 2, kOut = 1;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    out[0] = in[0] * act_deriv<KIND, kWide>(in[1]);
  }
};

// Save-all baseline: ordinary back-propagation through the primitive operations, keeping
// what each primitive's backward needs (Sec. II-C eqs. 1-2 for Swish; same recipe for the
// others).  Forward: (x) -> (y, new saved tensors).  Backward: (gy, x, saved...) -> gx.
template <int KIND>
struct SaveAllFwdOp;
template <int KIND>
struct SaveAllBwdOp;

template <>
struct SaveAllFwdOp<kSwish> {  // v1 = sigmoid(x), v2 = x, v3 = v1 v2; saves v1
  static constexpr int kIn = 1, kOut = 2;
  static constexpr bool kLight = true;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    const float v1 = sigmoid_f(in[0]);
    out[0] = v1 * in[0];
    out[1] = v1;
  }
};
template <>
struct SaveAllBwdOp<kSwish> {  // (g, x, v1):  x' = g v2 [v1 (1 - v1)] + g v1      eqs. 1-2
  static constexpr int kIn = 3, kOut = 1;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    const float g = in[0], v2 = in[1], v1 = in[2];
    out[0] = fma_(g * v2, v1 * (1.0f - v1), g * v1);
  }
};

template <>
struct SaveAllFwdOp<kMish> {  // t = tanh(softplus x), y = x t; saves t
  static constexpr int kIn = 1, kOut = 2;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    const float x = in[0];
    const float e = ex2(kLog2e * mish_cap(x));
    const float n = fma_(e, e, e + e);
    const float t = n * rcp(n + 2.0f);
    out[0] = x * t;
    out[1] = t;
  }
};
template <>
struct SaveAllBwdOp<kMish> {  // (g, x, t)
  static constexpr int kIn = 3, kOut = 1;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    const float g = in[0], x = in[1], t = in[2];
    const float g_t = g * x;                       // product node, towards tanh
    const float g_sp = g_t * fma_(-t, t, 1.0f);    // tanh keeps its output
    const float g_x1 = g_sp * sigmoid_f(x);        // softplus keeps its input
    out[0] = fma_(g, t, g_x1);                     // + product node, towards x
  }
};

template <>
struct SaveAllFwdOp<kGeluErf> {  // h = 0.5 x, s = 1 + erf(x/sqrt 2), y = h s; saves h, s
  static constexpr int kIn = 1, kOut = 3;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    const float x = in[0];
    const float h = 0.5f * x;
    const float s = 1.0f + erf_f(0.70710678118654752440f * x);
    out[0] = h * s;
    out[1] = h;
    out[2] = s;
  }
};
template <>
struct SaveAllBwdOp<kGeluErf> {  // (g, x, h, s)
  static constexpr int kIn = 4, kOut = 1;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    const float g = in[0], x = in[1], h = in[2], s = in[3];
    const float g_h = g * s, g_s = g * h;          // product node
    // erf keeps its input z = x/sqrt 2: erf'(z) = 2/sqrt(pi) exp(-z^2); chain 1/sqrt 2
    const float dz = 0.79788456080286535588f * ex2((-0.5f * kLog2e) * (x * x));
    out[0] = fma_(g_s, dz, 0.5f * g_h);
  }
};

template <>
struct SaveAllFwdOp<kGeluTanh> {  // t = tanh u, h = 0.5 x, s = 1 + t, y = h s; saves t, h, s
  static constexpr int kIn = 1, kOut = 4;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    const float x = in[0];
    const float x2 = __builtin_fminf(x * x, 1.0e30f);
    const float u = x * fma_(Act<kGeluTanh>::kC * Act<kGeluTanh>::kK, x2, Act<kGeluTanh>::kC);
    const float t = tanh_f(u);
    const float h = 0.5f * x;
    const float s = 1.0f + t;
    out[0] = h * s;
    out[1] = t;
    out[2] = h;
    out[3] = s;
  }
};
template <>
struct SaveAllBwdOp<kGeluTanh> {  // (g, x, t, h, s)
  static constexpr int kIn = 5, kOut = 1;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    const float g = in[0], x = in[1], t = in[2], h = in[3], s = in[4];
    const float g_h = g * s, g_s = g * h;          // product node
    const float g_u = g_s * fma_(-t, t, 1.0f);     // tanh keeps its output
    const float x2 = __builtin_fminf(x * x, 1.0e30f);
    const float du = fma_(3.0f * Act<kGeluTanh>::kC * Act<kGeluTanh>::kK, x2, Act<kGeluTanh>::kC);
    out[0] = fma_(g_u, du, 0.5f * g_h);            // the cubic keeps x
  }
};

}  // namespace nfad

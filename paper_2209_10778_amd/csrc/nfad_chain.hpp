// nfad_chain.hpp -- compile-time composer for forward-AD chains of element-wise primitives.
//
// The paper's method applies to any composition of "fad" primitive operations that maps one
// source element to one result (Sec. III-A: unary operations, binary operations with a
// constant, binary operations whose two inputs come from the same source; the symbolic
// primitives tanh, sigmoid, softplus; Sec. V-A lists add, mul, exp, tanh, softplus, sigmoid
// "etc."; the piecewise primitives relu, abs, min, max and sqrt are added here so that ELU,
// hard-swish, softsign and the like are chains too).
// Here such a chain is a TYPE built from the templates below; evaluating it pushes the dual
// number (x, 1) through the primitives (Sec. II-C eq. 3, Sec. II-D: v' = sum dv/du * u'), all
// in registers, and the result (value, tangent) is (y, dydx) of the fused forward kernel.
// The seed tangent is the literal 1, so the multiply-by-one of a single-operation chain is
// folded away by the compiler (the paper's NY->YN shortcut, Sec. IV-B "Efficiency").
//
//   using Mish = Mul<X, Tanh<Softplus<X>>>;          // x * tanh(softplus(x))
//   Dual r = Mish::eval(seed(x));                    // r.v = y, r.d = dy/dx
//
// Shared sub-expressions are written twice in the type but evaluated once: everything is
// inlined and pure, so the compiler merges them.
//
// All arithmetic is fp32 with the hardware exp2/log2/rcp; each primitive is written so that
// its value AND its tangent stay accurate where the textbook formula cancels (1 - tanh^2,
// s (1 - s), log(1 + e)).
#pragma once
#include "nfad_math.hpp"

namespace nfad {
namespace chain {

struct Dual {
  float v;  // value
  float d;  // tangent d v / d x
};

__device__ __forceinline__ Dual seed(float x) { return Dual{x, 1.0f}; }

__device__ __forceinline__ float lg2(float v) { return __builtin_amdgcn_logf(v); }  // log2 v
static constexpr float kLn2 = 0.69314718055994530942f;

// ---------------------------------------------------------------- leaves
struct X {  // the source element, tangent 1
  __device__ __forceinline__ static Dual eval(Dual x) { return x; }
};
// A constant: C is any type with `static constexpr float value`.
template <class C>
struct Const {
  __device__ __forceinline__ static Dual eval(Dual) { return Dual{C::value, 0.0f}; }
};
#define NFAD_CHAIN_CONSTANT(Name, Value) \
  struct Name {                          \
    static constexpr float value = (Value); \
  }

// ---------------------------------------------------------------- binary, same source
template <class A, class B>
struct Add {
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x), b = B::eval(x);
    return Dual{a.v + b.v, a.d + b.d};
  }
};
template <class A, class B>
struct Sub {
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x), b = B::eval(x);
    return Dual{a.v - b.v, a.d - b.d};
  }
};
template <class A, class B>
struct Mul {  // product rule: v3' = v1 v2' + v1' v2  (Sec. II-C eq. 3)
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x), b = B::eval(x);
    return Dual{a.v * b.v, fma_(a.v, b.d, a.d * b.v)};
  }
};
template <class A, class B>
struct Div {  // (a/b)' = (a' - (a/b) b') / b
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x), b = B::eval(x);
    const float r = rcp(b.v);
    const float q = a.v * r;
    return Dual{q, fma_(-q, b.d, a.d) * r};
  }
};

template <class A, class B>
struct Min {  // the tangent follows the selected operand (the first on a tie)
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x), b = B::eval(x);
    return a.v <= b.v ? a : (b.v < a.v ? b : Dual{a.v + b.v, a.d + b.d});  // last arm: a NaN stays NaN
  }
};
template <class A, class B>
struct Max {
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x), b = B::eval(x);
    return a.v >= b.v ? a : (b.v > a.v ? b : Dual{a.v + b.v, a.d + b.d});
  }
};

// ---------------------------------------------------------------- unary
template <class A>
struct Relu {  // max(v, 0); tangent 0 at and below the kink
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x);
    return a.v > 0.0f ? a : Dual{a.v * 0.0f, a.d * 0.0f};  // v * 0 keeps NaN, gives -0 for v < 0
  }
};
template <class A>
struct Abs {  // tangent sign(v) v', 0 at the kink
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x);
    const float sgn = a.v > 0.0f ? 1.0f : (a.v < 0.0f ? -1.0f : a.v * 0.0f);
    return Dual{__builtin_fabsf(a.v), sgn * a.d};
  }
};
template <class A>
struct Sqrt {  // (sqrt v)' = v' / (2 sqrt v)
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x);
    const float r = __builtin_amdgcn_sqrtf(a.v);
    return Dual{r, (0.5f * a.d) * rcp(r)};
  }
};
template <class A>
struct Neg {
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x);
    return Dual{-a.v, -a.d};
  }
};
template <class A>
struct Exp {
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x);
    const float e = ex2(kLog2e * a.v);
    return Dual{e, e * a.d};
  }
};
template <class A>
struct Log {
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x);
    return Dual{kLn2 * lg2(a.v), a.d * rcp(a.v)};
  }
};
template <class A>
struct Sigmoid {  // s' = s (1 - s) = sigmoid(v) sigmoid(-v), both from e = exp(-|v|)
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x);
    const float e = ex2(-kLog2e * __builtin_fabsf(a.v));
    const float r = rcp(1.0f + e);
    const float p = e * r;
    return Dual{a.v > 0.0f ? r : p, (r * p) * a.d};
  }
};
template <class A>
struct Tanh {  // tanh v = sign(v) (1 - e)/(1 + e), 1 - tanh^2 = 4 e/(1 + e)^2, e = exp(-2|v|)
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x);
    const float av = __builtin_fabsf(a.v);
    const float e = ex2((-2.0f * kLog2e) * av);
    const float r = rcp(1.0f + e);
    // for tiny |v| the quotient (1-e)/(1+e) would lose relative accuracy: tanh v = v - v^3/3 there
    const float small = a.v * fma_(a.v * a.v, -0.33333333f, 1.0f);
    const float big = __builtin_copysignf((1.0f - e) * r, a.v);
    return Dual{av < 0.03125f ? small : big, (4.0f * e) * (r * r) * a.d};
  }
};
template <class A>
struct Softplus {  // ln(1 + e^v) = max(v, 0) + log1p(exp(-|v|)),  softplus' = sigmoid
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x);
    const float e = ex2(-kLog2e * __builtin_fabsf(a.v));
    // log1p(e): e - e^2/2 while 1 + e would round e away, log2(1 + e) ln 2 otherwise
    const float l1p = e < 0.0009765625f ? e * fma_(-0.5f, e, 1.0f) : kLn2 * lg2(1.0f + e);
    const float r = rcp(1.0f + e);
    return Dual{__builtin_fmaxf(a.v, 0.0f) + l1p, (a.v > 0.0f ? r : e * r) * a.d};
  }
};
template <class A>
struct Erf {  // erf' = 2/sqrt(pi) exp(-v^2)
  __device__ __forceinline__ static Dual eval(Dual x) {
    const Dual a = A::eval(x);
    const float s = 1.41421356237309504880f * __builtin_fabsf(a.v);
    const float E = ex2((-0.5f * kLog2e) * (s * s));  // exp(-v^2)
    const float erfc_a = 2.0f * half_erfcx<ErfcxWide>(s) * E;
    // small |v|: 1 - erfc cancels; use the series 2/sqrt(pi) (v - v^3/3 + v^5/10)
    const float v2 = a.v * a.v;
    const float series = 1.12837916709551257390f * a.v * fma_(v2, fma_(v2, 0.1f, -0.33333333f), 1.0f);
    const float big = __builtin_copysignf(1.0f - erfc_a, a.v);
    return Dual{__builtin_fabsf(a.v) < 0.125f ? series : big, (1.12837916709551257390f * E) * a.d};
  }
};

}  // namespace chain

// Forward pass of a composed chain as a per-element operation of the streaming skeleton:
// (x) -> (value, tangent) of Chain at the dual number (x, 1).              Sec. II-C eq. 3
template <class Chain>
struct ChainFwdOp {
  static constexpr int kIn = 1, kOut = 2;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    const chain::Dual r = Chain::eval(chain::seed(in[0]));
    out[0] = r.v;
    out[1] = r.d;
  }
};

// One source element, M chains, 2M results: R^1 -> R^M with one saved tangent per output
// (Sec. II-D "f: R^1 -> R^M", Sec. IV-A).  Output order: y0, dydx0, y1, dydx1, ...
template <class... Chains>
struct ChainFwdMultiOp {
  static constexpr int kIn = 1, kOut = 2 * (int)sizeof...(Chains);
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut]) {
    const chain::Dual r[] = {Chains::eval(chain::seed(in[0]))...};
#pragma unroll
    for (int m = 0; m < (int)sizeof...(Chains); ++m) {
      out[2 * m] = r[m].v;
      out[2 * m + 1] = r[m].d;
    }
  }
};

}  // namespace nfad

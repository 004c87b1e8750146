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
//   Dual r = to_dual(Mish::eval<true>(seed(x), args));   // r.v = y, r.d = dy/dx
//
// Shared sub-expressions are written twice in the type but evaluated once: everything is
// inlined and pure, so the compiler merges them.
//
// All arithmetic is fp32 with the hardware exp2/log2/rcp; each primitive is written so that
// its value AND its tangent stay accurate where the textbook formula cancels (1 - tanh^2,
// s (1 - s), log(1 + e)).
//
// Three things keep a composed chain close to a hand-minimised kernel: constants are a type
// of their own (Konst), so a binary operation with a constant costs one instruction and not
// a product rule against a zero tangent; every node is evaluated for a storage tier (kWide,
// as in nfad_math.hpp) and drops refinements that 16-bit storage cannot show; and two pairs
// of primitives are recognised and evaluated in one step: tanh(softplus(.)), the core of
// Mish, and 1 + erf(.), the core of GELU.
#pragma once
#include "nfad_math.hpp"

namespace nfad {
namespace chain {

struct Dual {
  float v;  // value
  float d;  // tangent d v / d x
};
// Run-time constants of a chain: passed to the kernel by value, so chains that differ only in
// these numbers are the same kernel.  Read by the leaf Arg<I>; the leaf Const<C> is a constant
// fixed at compile time instead (the built-in chains, and the few values -- 0, +-1, +-2, +-0.5 --
// whose presence changes what the composer can simplify).
static constexpr int kMaxArgs = 24;
struct Args {
  float c[kMaxArgs];
};
// A value that does not depend on x.  Its tangent is identically zero, and carrying that in
// the TYPE lets the binary operations with a constant operand (Sec. III-A) drop the dead
// half of the sum/product/quotient rule: with a run-time 0.0f the compiler may not (0 * inf).
struct Konst {
  float v;
};

__device__ __forceinline__ Dual seed(float x) { return Dual{x, 1.0f}; }
__device__ __forceinline__ Dual to_dual(Dual a) { return a; }
__device__ __forceinline__ Dual to_dual(Konst a) { return Dual{a.v, 0.0f}; }

__device__ __forceinline__ float lg2(float v) { return __builtin_amdgcn_logf(v); }  // log2 v
static constexpr float kLn2 = 0.69314718055994530942f;

// ---------------------------------------------------------------- rules of the binary operations
__device__ __forceinline__ Dual add_(Dual a, Dual b) { return Dual{a.v + b.v, a.d + b.d}; }
__device__ __forceinline__ Dual add_(Konst a, Dual b) { return Dual{a.v + b.v, b.d}; }
__device__ __forceinline__ Dual add_(Dual a, Konst b) { return Dual{a.v + b.v, a.d}; }
__device__ __forceinline__ Konst add_(Konst a, Konst b) { return Konst{a.v + b.v}; }

__device__ __forceinline__ Dual sub_(Dual a, Dual b) { return Dual{a.v - b.v, a.d - b.d}; }
__device__ __forceinline__ Dual sub_(Konst a, Dual b) { return Dual{a.v - b.v, -b.d}; }
__device__ __forceinline__ Dual sub_(Dual a, Konst b) { return Dual{a.v - b.v, a.d}; }
__device__ __forceinline__ Konst sub_(Konst a, Konst b) { return Konst{a.v - b.v}; }

// product rule: v3' = v1 v2' + v1' v2  (Sec. II-C eq. 3)
__device__ __forceinline__ Dual mul_(Dual a, Dual b) { return Dual{a.v * b.v, fma_(a.v, b.d, a.d * b.v)}; }
__device__ __forceinline__ Dual mul_(Konst a, Dual b) { return Dual{a.v * b.v, a.v * b.d}; }
__device__ __forceinline__ Dual mul_(Dual a, Konst b) { return Dual{a.v * b.v, a.d * b.v}; }
__device__ __forceinline__ Konst mul_(Konst a, Konst b) { return Konst{a.v * b.v}; }

// quotient rule: (a/b)' = (a' - (a/b) b') / b.  A denominator that has overflowed (an exponential
// of a large argument: 1/b = 0) drags its tangent to infinity with it, and 0 * inf is NaN where
// the true derivative tends to 0; the tangent is therefore 0 whenever 1/b is.  (A NaN
// denominator still gives NaN: NaN == 0 is false.)
__device__ __forceinline__ Dual div_(Dual a, Dual b) {
  const float r = rcp(b.v);
  const float q = a.v * r;
  const float t = fma_(-q, b.d, a.d) * r;
  return Dual{q, r == 0.0f ? q * 0.0f : t};   // q * 0 keeps a NaN numerator NaN
}
__device__ __forceinline__ Dual div_(Konst a, Dual b) {
  const float r = rcp(b.v);
  const float q = a.v * r;
  const float t = (-q * b.d) * r;
  return Dual{q, r == 0.0f ? 0.0f : t};
}
__device__ __forceinline__ Dual div_(Dual a, Konst b) {
  const float r = rcp(b.v);  // folded at compile time for a literal constant
  return Dual{a.v * r, a.d * r};
}
__device__ __forceinline__ Konst div_(Konst a, Konst b) { return Konst{a.v * rcp(b.v)}; }

// ---------------------------------------------------------------- leaves
// Every node has   template <bool kWide> static eval(Dual x, const Args& g)   returning Dual or Konst; kWide
// says that the result will be stored as fp32 (see the tiers in nfad_math.hpp): a few
// primitives drop a refinement that only shows at fp32 resolution when it is false.
struct X {  // the source element, tangent 1
  template <bool kWide>
  __device__ __forceinline__ static Dual eval(Dual x, const Args&) {
    return x;
  }
};
// A constant: C is any type with `static constexpr float value`.
template <class C>
struct Const {
  template <bool kWide>
  __device__ __forceinline__ static Konst eval(Dual, const Args&) {
    return Konst{C::value};
  }
};
// The I-th run-time constant.
template <int I>
struct Arg {
  template <bool kWide>
  __device__ __forceinline__ static Konst eval(Dual, const Args& g) {
    return Konst{g.c[I]};
  }
};
#define NFAD_CHAIN_CONSTANT(Name, Value) \
  struct Name {                          \
    static constexpr float value = (Value); \
  }
// The constants that stay compile-time in run-time compiled chains too.
NFAD_CHAIN_CONSTANT(KZero, 0.0f);
NFAD_CHAIN_CONSTANT(KOne, 1.0f);
NFAD_CHAIN_CONSTANT(KMinusOne, -1.0f);
NFAD_CHAIN_CONSTANT(KTwo, 2.0f);
NFAD_CHAIN_CONSTANT(KMinusTwo, -2.0f);
NFAD_CHAIN_CONSTANT(KHalf, 0.5f);
NFAD_CHAIN_CONSTANT(KMinusHalf, -0.5f);

// ---------------------------------------------------------------- binary, same source
#define NFAD_CHAIN_BINARY(Name, rule)                                  \
  template <class A, class B>                                          \
  struct Name {                                                        \
    template <bool kWide>                                              \
    __device__ __forceinline__ static auto eval(Dual x, const Args& g) {              \
      return rule(A::template eval<kWide>(x, g), B::template eval<kWide>(x, g)); \
    }                                                                  \
  }
NFAD_CHAIN_BINARY(Add, add_);
NFAD_CHAIN_BINARY(Sub, sub_);
NFAD_CHAIN_BINARY(Mul, mul_);
NFAD_CHAIN_BINARY(Div, div_);
#undef NFAD_CHAIN_BINARY

template <class A, class B>
struct Min {  // the tangent follows the selected operand (the first on a tie)
  template <bool kWide>
  __device__ __forceinline__ static Dual eval(Dual x, const Args& g) {
    const Dual a = to_dual(A::template eval<kWide>(x, g)), b = to_dual(B::template eval<kWide>(x, g));
    return a.v <= b.v ? a : (b.v < a.v ? b : Dual{a.v + b.v, a.d + b.d});  // last arm: a NaN stays NaN
  }
};
template <class A, class B>
struct Max {
  template <bool kWide>
  __device__ __forceinline__ static Dual eval(Dual x, const Args& g) {
    const Dual a = to_dual(A::template eval<kWide>(x, g)), b = to_dual(B::template eval<kWide>(x, g));
    return a.v >= b.v ? a : (b.v > a.v ? b : Dual{a.v + b.v, a.d + b.d});
  }
};

// ---------------------------------------------------------------- unary
// Each rule maps the operand's (value, tangent) to the result's; NFAD_CHAIN_UNARY wraps it
// into a node.
__device__ __forceinline__ Dual relu_(Dual a) {  // max(v, 0); tangent 0 at and below the kink
  return a.v > 0.0f ? a : Dual{a.v * 0.0f, a.d * 0.0f};  // v * 0 keeps NaN, gives -0 for v < 0
}
__device__ __forceinline__ Dual abs_(Dual a) {  // tangent sign(v) v', 0 at the kink
  const float sgn = a.v > 0.0f ? 1.0f : (a.v < 0.0f ? -1.0f : a.v * 0.0f);
  return Dual{__builtin_fabsf(a.v), sgn * a.d};
}
__device__ __forceinline__ Dual sqrt_(Dual a) {  // (sqrt v)' = v' / (2 sqrt v)
  const float r = __builtin_amdgcn_sqrtf(a.v);
  return Dual{r, (0.5f * a.d) * rcp(r)};
}
__device__ __forceinline__ Dual neg_(Dual a) { return Dual{-a.v, -a.d}; }
__device__ __forceinline__ Dual exp_(Dual a) {
  const float e = ex2(kLog2e * a.v);
  return Dual{e, e * a.d};
}
__device__ __forceinline__ Dual log_(Dual a) { return Dual{kLn2 * lg2(a.v), a.d * rcp(a.v)}; }
__device__ __forceinline__ Dual sigmoid_(Dual a) {  // s' = s (1 - s) = sigmoid(v) sigmoid(-v), both from e = exp(-|v|)
  const float e = ex2(-kLog2e * __builtin_fabsf(a.v));
  const float r = rcp(1.0f + e);
  const float p = e * r;
  return Dual{a.v > 0.0f ? r : p, (r * p) * a.d};
}
template <bool kWide>
__device__ __forceinline__ Dual tanh_(Dual a) {  // tanh v = sign(v) (1 - e)/(1 + e), 1 - tanh^2 = 4 e/(1 + e)^2, e = exp(-2|v|)
  const float av = __builtin_fabsf(a.v);
  const float e = ex2((-2.0f * kLog2e) * av);
  const float r = rcp(1.0f + e);
  const float big = __builtin_copysignf((1.0f - e) * r, a.v);
  const float dt = (4.0f * e) * (r * r) * a.d;
  if constexpr (kWide) {
    // for tiny |v| the quotient (1-e)/(1+e) loses relative accuracy (its absolute error stays
    // at the fp32 ulp of 1, which 16-bit storage cannot see): tanh v = v - v^3/3 there
    const float small = a.v * fma_(a.v * a.v, -0.33333333f, 1.0f);
    return Dual{av < 0.03125f ? small : big, dt};
  } else {
    return Dual{big, dt};
  }
}
template <bool kWide>
__device__ __forceinline__ Dual softplus_(Dual a) {  // ln(1 + e^v) = max(v, 0) + log1p(exp(-|v|)),  softplus' = sigmoid
  const float e = ex2(-kLog2e * __builtin_fabsf(a.v));
  float l1p = kLn2 * lg2(1.0f + e);
  // log1p(e) = e - e^2/2 where 1 + e would round e away (an absolute error of at most 2^-24, again
  // invisible after rounding to 16 bits next to max(v, 0) or below the smallest fp16 normal)
  if constexpr (kWide) l1p = e < 0.0009765625f ? e * fma_(-0.5f, e, 1.0f) : l1p;
  const float r = rcp(1.0f + e);
  return Dual{__builtin_fmaxf(a.v, 0.0f) + l1p, (a.v > 0.0f ? r : e * r) * a.d};
}
template <bool kWide>
__device__ __forceinline__ float erfc_abs_(float v, float& E) {  // erfc(|v|), and E = exp(-v^2)
  const float s = 1.41421356237309504880f * __builtin_fabsf(v);
  E = ex2((-0.5f * kLog2e) * (s * s));
  if constexpr (kWide) return 2.0f * half_erfcx<ErfcxWide>(s) * E;
  else return 2.0f * half_erfcx<ErfcxNarrow>(s) * E;
}
template <bool kWide>
__device__ __forceinline__ Dual erf_(Dual a) {  // erf' = 2/sqrt(pi) exp(-v^2)
  float E;
  const float erfc_a = erfc_abs_<kWide>(a.v, E);
  // small |v|: 1 - erfc cancels; use the series 2/sqrt(pi) (v - v^3/3 + v^5/10)
  const float v2 = a.v * a.v;
  const float series = 1.12837916709551257390f * a.v * fma_(v2, fma_(v2, 0.1f, -0.33333333f), 1.0f);
  const float big = __builtin_copysignf(1.0f - erfc_a, a.v);
  return Dual{__builtin_fabsf(a.v) < 0.125f ? series : big, (1.12837916709551257390f * E) * a.d};
}
// 1 + erf(v) = erfc(-v) in one step: erfc(|v|) on the negative side, 2 - erfc(|v|) on the positive
// one.  No cancellation anywhere (1 + erf(v) computed literally loses everything below v ~ -4),
// so neither the small-argument series of erf nor its select is needed.
template <bool kWide>
__device__ __forceinline__ Dual one_plus_erf_(Dual a) {
  float E;
  const float erfc_a = erfc_abs_<kWide>(a.v, E);
  return Dual{a.v < 0.0f ? erfc_a : 2.0f - erfc_a, (1.12837916709551257390f * E) * a.d};
}
// tanh(softplus(v)) in one step: with e = exp(v) and n = e (e + 2) it is n / (n + 2), and its
// derivative is 4 e (e + 1) / (n + 2)^2: one exponential and one reciprocal instead of two
// exponentials, a logarithm and two reciprocals.  v is capped at 41.5 inside the exponential
// (the result is 1 and its derivative 0 to fp32 precision far below that) so that n stays
// finite; the cap is a compare-and-select so that NaN stays NaN.
__device__ __forceinline__ Dual tanh_softplus_(Dual a) {
  const float vc = mish_cap(a.v);
  const float e = ex2(kLog2e * vc);
  const float n = fma_(e, e, e + e);
  const float R = rcp(n + 2.0f);
  const float g = fma_(4.0f, e, 4.0f) * e;
  return Dual{n * R, (g * R) * R * a.d};
}

#define NFAD_CHAIN_UNARY(Name, rule)                                \
  template <class A>                                                \
  struct Name {                                                     \
    template <bool kWide>                                           \
    __device__ __forceinline__ static Dual eval(Dual x, const Args& g) {           \
      return rule(to_dual(A::template eval<kWide>(x, g)));             \
    }                                                               \
  }
NFAD_CHAIN_UNARY(Relu, relu_);
NFAD_CHAIN_UNARY(Abs, abs_);
NFAD_CHAIN_UNARY(Sqrt, sqrt_);
NFAD_CHAIN_UNARY(Neg, neg_);
NFAD_CHAIN_UNARY(Exp, exp_);
NFAD_CHAIN_UNARY(Log, log_);
NFAD_CHAIN_UNARY(Sigmoid, sigmoid_);
NFAD_CHAIN_UNARY(Tanh, tanh_<kWide>);
NFAD_CHAIN_UNARY(Softplus, softplus_<kWide>);
NFAD_CHAIN_UNARY(Erf, erf_<kWide>);
#undef NFAD_CHAIN_UNARY

// Fused pairs (the composer's two peepholes): 1 + erf, the core of GELU as usually written ...
template <class C, class A>
struct Add<Const<C>, Erf<A>> {
  template <bool kWide>
  __device__ __forceinline__ static Dual eval(Dual x, const Args& g) {
    const Dual a = to_dual(A::template eval<kWide>(x, g));
    if constexpr (C::value == 1.0f) return one_plus_erf_<kWide>(a);
    else return add_(Konst{C::value}, erf_<kWide>(a));
  }
};
template <class A, class C>
struct Add<Erf<A>, Const<C>> : Add<Const<C>, Erf<A>> {};
// ... and tanh directly on a softplus, the core of Mish.
template <class A>
struct Tanh<Softplus<A>> {
  template <bool kWide>
  __device__ __forceinline__ static Dual eval(Dual x, const Args& g) {
    return tanh_softplus_(to_dual(A::template eval<kWide>(x, g)));
  }
};

}  // namespace chain

// Forward pass of a composed chain as a per-element operation of the streaming skeleton:
// (x) -> (value, tangent) of Chain at the dual number (x, 1).              Sec. II-C eq. 3
template <class Chain>
struct ChainFwdOp {
  static constexpr int kIn = 1, kOut = 2;
  using Params = chain::Args;   // run-time constants, a by-value kernel argument
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut], const Params& g) {
    const chain::Dual r = chain::to_dual(Chain::template eval<kWide>(chain::seed(in[0]), g));
    out[0] = r.v;
    out[1] = r.d;
  }
};

// One source element, M chains, 2M results: R^1 -> R^M with one saved tangent per output
// (Sec. II-D "f: R^1 -> R^M", Sec. IV-A).  Output order: y0, dydx0, y1, dydx1, ...
template <class... Chains>
struct ChainFwdMultiOp {
  static constexpr int kIn = 1, kOut = 2 * (int)sizeof...(Chains);
  using Params = chain::Args;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[kIn], float (&out)[kOut], const Params& g) {
    const chain::Dual r[] = {chain::to_dual(Chains::template eval<kWide>(chain::seed(in[0]), g))...};
#pragma unroll
    for (int m = 0; m < (int)sizeof...(Chains); ++m) {
      out[2 * m] = r[m].v;
      out[2 * m + 1] = r[m].d;
    }
  }
};

}  // namespace nfad

// nfad_chain.hip -- fused forward-AD kernels for chains composed from primitive operations
// (nfad_chain.hpp), and their C ABI.  A chain is fused into ONE kernel on the same streaming
// skeleton as the hand-tuned activations: read x, write y and dydx; backward is nfad_bwd.
#include "nfad_stream.hpp"
#include "nfad_chain.hpp"

namespace nfad {

// Forward pass of a composed chain: (x) -> (value, tangent) of Chain at (x, 1).   Sec. II-C eq. 3
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

namespace chain {
NFAD_CHAIN_CONSTANT(kOne, 1.0f);
NFAD_CHAIN_CONSTANT(kHalf, 0.5f);
NFAD_CHAIN_CONSTANT(kSqrt2OverPi, 0.79788456080286535588f);
NFAD_CHAIN_CONSTANT(kGeluCubic, 0.044715f);
NFAD_CHAIN_CONSTANT(kInvSqrt2, 0.70710678118654752440f);

// The built-in chains.  Each is spelled as the paper's Table I spells the activation (or as the
// plain primitive), NOT as the hand-minimised forms of nfad_math.hpp: they demonstrate that any
// composition of the primitives fuses into one forward kernel.  `program` is the same chain
// in postfix notation over the primitive names, for callers (and tests) to inspect.
using SigmoidC = Sigmoid<X>;
using TanhC = Tanh<X>;
using SoftplusC = Softplus<X>;
using ExpC = Exp<X>;
using SwishC = Div<X, Add<Const<kOne>, Exp<Neg<X>>>>;                       // x / (1 + e^-x)
using MishC = Mul<X, Tanh<Softplus<X>>>;                                    // x tanh(softplus x)
using GeluTanhC = Mul<Mul<Const<kHalf>, X>,                                  // 0.5 x (1 + tanh(c (x + k x^3)))
                      Add<Const<kOne>, Tanh<Mul<Const<kSqrt2OverPi>,
                                                Add<X, Mul<Const<kGeluCubic>, Mul<Mul<X, X>, X>>>>>>>;
using GeluErfC = Mul<Mul<Const<kHalf>, X>, Add<Const<kOne>, Erf<Mul<Const<kInvSqrt2>, X>>>>;
using TanhShrinkC = Sub<X, Tanh<X>>;                                         // x - tanh x
using LogSigmoidC = Neg<Softplus<Neg<X>>>;                                   // -softplus(-x)
using SwishSigmoidC = Mul<Sigmoid<X>, X>;                                    // v1 = sigmoid(x), v2 = x, v3 = v1 v2
}  // namespace chain

struct ChainEntry {
  const char* name;
  const char* program;
};
static const ChainEntry kChains[] = {
    {"sigmoid", "x sigmoid"},
    {"tanh", "x tanh"},
    {"softplus", "x softplus"},
    {"exp", "x exp"},
    {"swish_table1", "x 1 x neg exp + /"},
    {"mish_table1", "x x softplus tanh *"},
    {"gelu_tanh_table1", "0.5 x * 1 0.79788456080286535588 x 0.044715 x x * x * * + * tanh + *"},
    {"gelu_erf", "0.5 x * 1 0.70710678118654752440 x * erf + *"},
    {"tanhshrink", "x x tanh -"},
    {"logsigmoid", "x neg softplus neg"},
    {"swish_sigmoid", "x sigmoid x *"},
};
static constexpr int kNumChains = (int)(sizeof(kChains) / sizeof(kChains[0]));

}  // namespace nfad

using namespace nfad;

extern "C" {

int nfad_chain_count(void) { return kNumChains; }

const char* nfad_chain_name(int chain_id) {
  return (chain_id >= 0 && chain_id < kNumChains) ? kChains[chain_id].name : nullptr;
}

const char* nfad_chain_program(int chain_id) {
  return (chain_id >= 0 && chain_id < kNumChains) ? kChains[chain_id].program : nullptr;
}

int nfad_chain_fwd(int chain_id, const void* x, void* y, void* dydx, size_t n, int dtype, void* stream) {
  if (chain_id < 0 || chain_id >= kNumChains) return NFAD_EINVAL_KIND;
  const void* const in[1] = {x};
  void* const out[2] = {y, dydx};
  switch (chain_id) {
    case 0: return run<ChainFwdOp<chain::SigmoidC>>(dtype, in, out, n, stream);
    case 1: return run<ChainFwdOp<chain::TanhC>>(dtype, in, out, n, stream);
    case 2: return run<ChainFwdOp<chain::SoftplusC>>(dtype, in, out, n, stream);
    case 3: return run<ChainFwdOp<chain::ExpC>>(dtype, in, out, n, stream);
    case 4: return run<ChainFwdOp<chain::SwishC>>(dtype, in, out, n, stream);
    case 5: return run<ChainFwdOp<chain::MishC>>(dtype, in, out, n, stream);
    case 6: return run<ChainFwdOp<chain::GeluTanhC>>(dtype, in, out, n, stream);
    case 7: return run<ChainFwdOp<chain::GeluErfC>>(dtype, in, out, n, stream);
    case 8: return run<ChainFwdOp<chain::TanhShrinkC>>(dtype, in, out, n, stream);
    case 9: return run<ChainFwdOp<chain::LogSigmoidC>>(dtype, in, out, n, stream);
    case 10: return run<ChainFwdOp<chain::SwishSigmoidC>>(dtype, in, out, n, stream);
  }
  return NFAD_EINVAL_KIND;
}

}  // extern "C"

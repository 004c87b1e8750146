// nfad_chain.hip -- fused forward-AD kernels for chains composed from primitive operations
// (nfad_chain.hpp), and their C ABI.  A chain is fused into ONE kernel on the same streaming
// skeleton as the hand-tuned activations: read x, write y and dydx; backward is nfad_bwd.
#include "nfad_stream.hpp"
#include "nfad_chain.hpp"

namespace nfad {

namespace chain {
using kOne = KOne;
using kHalf = KHalf;
using kZero = KZero;
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
NFAD_CHAIN_CONSTANT(kThree, 3.0f);
NFAD_CHAIN_CONSTANT(kSix, 6.0f);
using EluC = Add<Relu<X>, Sub<Exp<Min<X, Const<kZero>>>, Const<kOne>>>;      // relu(x) + exp(min(x,0)) - 1
using HardSwishC = Div<Mul<X, Min<Max<Add<X, Const<kThree>>, Const<kZero>>, Const<kSix>>>, Const<kSix>>;
using SoftsignC = Div<X, Add<Const<kOne>, Abs<X>>>;                          // x / (1 + |x|)
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
    {"elu", "x relu x 0 min exp 1 - +"},
    {"hardswish", "x x 3 + 0 max 6 min * 6 /"},
    {"softsign", "x 1 x abs + /"},
};
static constexpr int kNumChains = (int)(sizeof(kChains) / sizeof(kChains[0]));

}  // namespace nfad

namespace nfad {
namespace jit {
static const char* name_of(int chain_id);
static const char* program_of(int chain_id);
static int outputs_of(int chain_id);
static int forward(int chain_id, int want_m, const void* x, void* const* y, void* const* dydx, size_t n, int dtype,
                   void* stream);
}  // namespace jit
}  // namespace nfad

using namespace nfad;

extern "C" {

int nfad_chain_count(void) { return kNumChains; }

const char* nfad_chain_name(int chain_id) {
  if (chain_id >= NFAD_CHAIN_JIT_BASE) return jit::name_of(chain_id);
  return (chain_id >= 0 && chain_id < kNumChains) ? kChains[chain_id].name : nullptr;
}

const char* nfad_chain_program(int chain_id) {
  if (chain_id >= NFAD_CHAIN_JIT_BASE) return jit::program_of(chain_id);
  return (chain_id >= 0 && chain_id < kNumChains) ? kChains[chain_id].program : nullptr;
}

int nfad_chain_fwd(int chain_id, const void* x, void* y, void* dydx, size_t n, int dtype, void* stream) {
  if (chain_id >= NFAD_CHAIN_JIT_BASE) {
    void* const ys[1] = {y};
    void* const ds[1] = {dydx};
    return jit::forward(chain_id, 1, x, ys, ds, n, dtype, stream);
  }
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
    case 11: return run<ChainFwdOp<chain::EluC>>(dtype, in, out, n, stream);
    case 12: return run<ChainFwdOp<chain::HardSwishC>>(dtype, in, out, n, stream);
    case 13: return run<ChainFwdOp<chain::SoftsignC>>(dtype, in, out, n, stream);
  }
  return NFAD_EINVAL_KIND;
}

}  // extern "C"

// ==================================================================== run-time composed chains
// A caller can hand the library ANY chain over the primitives, as a postfix program; the
// library translates it into the same expression-template type the built-in chains use,
// compiles that one instantiation of the streaming kernel with the run-time compiler
// (hiprtc, for the architecture of the current device) and keeps the loaded kernel.  The
// program text is parsed against a closed grammar (the primitive names, `x`, decimal
// constants): nothing from the caller's string reaches the compiler verbatim.
//
// Constants do not reach the compiler at all: sub-expressions without x are folded on the
// host, and every remaining constant becomes a run-time argument of the kernel (Arg<i>, passed
// by value with each launch), so programs that differ only in their numbers -- x * 0.1 and
// x * 0.2 -- are ONE kernel, compiled once.  Only the values 0, +-1, +-2 and +-0.5 stay
// compile-time constants, because their presence changes what the composer can simplify
// (1 + erf, multiplication by 1, ...).  Division by a constant is multiplication by its
// reciprocal, taken on the host.
#include <hip/hiprtc.h>

#include <math.h>
#include <stdio.h>
#include <string.h>

#include <memory>
#include <string>
#include <vector>

#include "nfad_chain_table.hpp"
#include "nfad_embedded.inc"

namespace nfad {
namespace jit {

static constexpr int kMaxTokens = 256;
static constexpr int kDefaultMaxChains = 4096;

// One compiled forward kernel (all storage types, both launch shapes, the element-at-a-time form).
struct Kernel {
  int uid = -1;
  int m = 1;                                              // number of outputs (chains over the same x)
  hipModule_t module = nullptr;
  hipFunction_t vec[3] = {nullptr, nullptr, nullptr};     // indexed by nfad_dtype_t: the shape for large launches,
  hipFunction_t vec_small[3] = {nullptr, nullptr, nullptr};   // ... the one for small launches,
  hipFunction_t scalar[3] = {nullptr, nullptr, nullptr};  // ... and the element-at-a-time kernel
  ~Kernel() {
    if (module) (void)hipModuleUnload(module);
  }
};
using Table = ChainTable<Kernel, chain::Args>;

// NFAD_MAX_CHAINS (environment, read once) lowers the capacity: the hook the slot-reuse tests use.
static Table& table() {
  static Table* t = [] {
    int cap = kDefaultMaxChains;
    if (const char* s = getenv("NFAD_MAX_CHAINS")) {
      const long v = atol(s);
      if (v >= 1 && v < cap) cap = (int)v;
    }
    return new Table(cap);   // never destroyed: kernels must not be unloaded during process teardown
  }();
  return *t;
}
static int g_next_uid = 0;   // under g_uid_mu
static std::mutex g_uid_mu;
static thread_local std::string g_log;

// ---- postfix program -> expression-template type with the constants taken out
struct Item {
  std::string type;    // type expression over nfad::chain templates (empty while the item is a pure constant)
  bool is_const;
  double value;
};
struct Translation {
  std::string types[NFAD_MAX_OUTPUTS];   // one per program
  chain::Args args;                      // values of Arg<0> .. Arg<nargs - 1>
  int nargs = 0;
};

static bool emit_constant(double v, Translation& tr, std::string& type, std::string& err) {
  const float f = (float)v;
  if (!isfinite(f)) { err = "a constant sub-expression is not finite"; return false; }
  static const struct { float v; const char* name; } kStructural[] = {
      {0.0f, "KZero"}, {1.0f, "KOne"}, {-1.0f, "KMinusOne"}, {2.0f, "KTwo"}, {-2.0f, "KMinusTwo"},
      {0.5f, "KHalf"}, {-0.5f, "KMinusHalf"}};
  for (const auto& k : kStructural)
    if (f == k.v) { type = std::string("nfc::Const<nfc::") + k.name + ">"; return true; }
  if (tr.nargs >= chain::kMaxArgs) { err = "more than " + std::to_string(chain::kMaxArgs) + " constants"; return false; }
  tr.args.c[tr.nargs] = f;
  type = "nfc::Arg<" + std::to_string(tr.nargs++) + ">";
  return true;
}
static bool materialise(Item& it, Translation& tr, std::string& err) {   // a constant item becomes a leaf
  if (!it.is_const) return true;
  if (!emit_constant(it.value, tr, it.type, err)) return false;
  it.is_const = false;
  return true;
}
static double fold_unary(const std::string& op, double v) {
  if (op == "neg") return -v;
  if (op == "relu") return v > 0 ? v : 0.0;
  if (op == "abs") return fabs(v);
  if (op == "sqrt") return sqrt(v);
  if (op == "exp") return exp(v);
  if (op == "log") return log(v);
  if (op == "tanh") return tanh(v);
  if (op == "sigmoid") return 1.0 / (1.0 + exp(-v));
  if (op == "softplus") return v > 0 ? v + log1p(exp(-v)) : log1p(exp(v));
  return erf(v);   // "erf"
}
static double fold_binary(const std::string& op, double a, double b) {
  if (op == "+") return a + b;
  if (op == "-") return a - b;
  if (op == "*") return a * b;
  if (op == "/") return a / b;
  if (op == "min") return a <= b ? a : b;
  return a >= b ? a : b;   // "max"
}

static bool translate(const char* program, int index, Translation& tr, std::string& err) {
  static const struct { const char* tok; const char* tmpl; int arity; } kOps[] = {
      {"+", "Add", 2}, {"-", "Sub", 2}, {"*", "Mul", 2}, {"/", "Div", 2}, {"min", "Min", 2}, {"max", "Max", 2},
      {"neg", "Neg", 1}, {"relu", "Relu", 1}, {"abs", "Abs", 1}, {"sqrt", "Sqrt", 1},
      {"exp", "Exp", 1}, {"log", "Log", 1}, {"tanh", "Tanh", 1}, {"sigmoid", "Sigmoid", 1},
      {"softplus", "Softplus", 1}, {"erf", "Erf", 1}};
  std::vector<Item> stack;
  int ntok = 0;
  bool uses_x = false;
  const char* p = program;
  while (*p) {
    while (*p == ' ' || *p == '\t' || *p == '\n') ++p;
    if (!*p) break;
    const char* q = p;
    while (*q && *q != ' ' && *q != '\t' && *q != '\n') ++q;
    const std::string tok(p, q);
    p = q;
    if (++ntok > kMaxTokens) { err = "program too long"; return false; }
    if (tok == "x") { stack.push_back({"nfc::X", false, 0.0}); uses_x = true; continue; }
    bool matched = false;
    for (const auto& op : kOps) {
      if (tok != op.tok) continue;
      if ((int)stack.size() < op.arity) { err = "operator '" + tok + "' lacks operands"; return false; }
      if (op.arity == 1) {
        Item& a = stack.back();
        if (a.is_const) a.value = fold_unary(tok, a.value);
        else a.type = std::string("nfc::") + op.tmpl + "<" + a.type + ">";
      } else {
        Item b = stack.back();
        stack.pop_back();
        Item& a = stack.back();
        if (a.is_const && b.is_const) {
          a.value = fold_binary(tok, a.value, b.value);
        } else if (tok == "/" && b.is_const) {   // division by a constant: multiply by its reciprocal
          Item r = {"", true, 1.0 / b.value};
          if (!materialise(r, tr, err)) { if (b.value == 0.0) err = "division by the constant 0"; return false; }
          a.type = "nfc::Mul<" + a.type + ", " + r.type + ">";
        } else {
          // the left operand's constants are numbered before the right operand's
          if (!materialise(a, tr, err) || !materialise(b, tr, err)) return false;
          a.type = std::string("nfc::") + op.tmpl + "<" + a.type + ", " + b.type + ">";
        }
      }
      matched = true;
      break;
    }
    if (matched) continue;
    char* end = nullptr;
    const double c = strtod(tok.c_str(), &end);
    if (end == tok.c_str() || *end != '\0' || !isfinite(c) || !isfinite((float)c)) { err = "unknown token '" + tok + "'"; return false; }
    stack.push_back({"", true, c});
  }
  if (stack.size() != 1) { err = "program leaves " + std::to_string(stack.size()) + " values"; return false; }
  if (!uses_x) { err = "program does not use x"; return false; }
  tr.types[index] = stack[0].type;
  return true;
}

static const char* kTypeNames[3] = {"float", "_Float16", "__bf16"};   // indexed by nfad_dtype_t

// Compiles and loads the kernel of `op` (a ChainFwdOp / ChainFwdMultiOp type expression with m outputs).
static int build_kernel(const std::string& op, int m, std::shared_ptr<Kernel>& out) {
  const std::string src = "#include \"nfad_stream_device.hpp\"\n#include \"nfad_chain.hpp\"\n"
                          "namespace nfc = nfad::chain;\n";
  hiprtcProgram prog = nullptr;
  if (hiprtcCreateProgram(&prog, src.c_str(), "nfad_user_chain.hip", kNumEmbedded, const_cast<const char**>(kEmbeddedSources),
                          const_cast<const char**>(kEmbeddedNames)) != HIPRTC_SUCCESS) {
    g_log = "hiprtcCreateProgram failed";
    return NFAD_ECOMPILE;
  }
  std::string names[9];
  for (int t = 0; t < 3; ++t) {
    const std::string rule = "nfad::ShapeRule<1, " + std::to_string(2 * m) + ", " + kTypeNames[t] + ">";
    names[t] = "nfad::ew_vec_kernel<" + op + ", " + kTypeNames[t] + ", " + rule + "::Large>";
    names[3 + t] = "nfad::ew_scalar_kernel<" + op + ", " + kTypeNames[t] + ">";
    names[6 + t] = "nfad::ew_vec_kernel<" + op + ", " + kTypeNames[t] + ", " + rule + "::Small>";
  }
  for (auto& nm : names) hiprtcAddNameExpression(prog, nm.c_str());

  int dev = 0;
  hipDeviceProp_t prop;
  std::string arch = "gfx950";
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.gcnArchName[0])
    arch = prop.gcnArchName;
  const std::string arch_opt = "--offload-arch=" + arch;
  const char* opts[] = {arch_opt.c_str(), "-O3", "-std=c++17",
                        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
  const hiprtcResult rc = hiprtcCompileProgram(prog, (int)(sizeof(opts) / sizeof(opts[0])), opts);
  size_t log_size = 0;
  if (hiprtcGetProgramLogSize(prog, &log_size) == HIPRTC_SUCCESS && log_size > 1) {
    g_log.resize(log_size);
    hiprtcGetProgramLog(prog, &g_log[0]);
  }
  if (rc != HIPRTC_SUCCESS) { hiprtcDestroyProgram(&prog); return NFAD_ECOMPILE; }

  size_t code_size = 0;
  std::vector<char> code;
  if (hiprtcGetCodeSize(prog, &code_size) != HIPRTC_SUCCESS) { hiprtcDestroyProgram(&prog); return NFAD_ECOMPILE; }
  code.resize(code_size);
  hiprtcGetCode(prog, code.data());

  std::shared_ptr<Kernel> k(new Kernel);
  k->m = m;
  bool ok = hipModuleLoadData(&k->module, code.data()) == hipSuccess;
  for (int t = 0; ok && t < 9; ++t) {
    const char* lowered = nullptr;
    hipFunction_t* slot = t < 3 ? &k->vec[t] : (t < 6 ? &k->scalar[t - 3] : &k->vec_small[t - 6]);
    ok = hiprtcGetLoweredName(prog, names[t].c_str(), &lowered) == HIPRTC_SUCCESS && lowered &&
         hipModuleGetFunction(slot, k->module, lowered) == hipSuccess;
  }
  hiprtcDestroyProgram(&prog);
  if (!ok) {
    if (g_log.empty()) g_log = "loading the compiled chain failed";
    return NFAD_ECOMPILE;   // k's destructor unloads what was loaded
  }
  {
    std::lock_guard<std::mutex> lock(g_uid_mu);
    k->uid = g_next_uid++;
  }
  out = std::move(k);
  return NFAD_OK;
}

static int compile(const char* const* programs, int m, int* chain_id) {
  std::string list, joined, err;
  Translation tr;
  memset(&tr.args, 0, sizeof tr.args);
  g_log.clear();
  for (int j = 0; j < m; ++j) {
    if (!programs[j]) { g_log = "null program"; return NFAD_ENULL; }
    if (!translate(programs[j], j, tr, err)) {
      g_log = (m > 1 ? "program " + std::to_string(j) + ": " : std::string()) + err;
      return NFAD_EPROGRAM;
    }
    list += (j ? ", " : "") + tr.types[j];
    joined += (j ? " ; " : "") + std::string(programs[j]);
  }
  // the structure of the chain(s) with the constants left open: the identity of the kernel
  const std::string op = m == 1 ? "nfad::ChainFwdOp<" + list + ">" : "nfad::ChainFwdMultiOp<" + list + ">";
  Table& t = table();
  if (!t.has_room()) {   // before any compiler work
    g_log = "too many live chains (" + std::to_string(t.capacity()) + "): release some first";
    return NFAD_ECOMPILE;
  }
  std::shared_ptr<Kernel> kernel = t.find_kernel(op);
  if (!kernel) {
    std::shared_ptr<Kernel> fresh;
    const int rc = build_kernel(op, m, fresh);
    if (rc != NFAD_OK) return rc;
    kernel = t.adopt(op, fresh);   // another thread may have compiled the same structure meanwhile
  }
  const int slot = t.insert(joined, op, kernel, tr.args);
  if (slot < 0) {
    g_log = "too many live chains (" + std::to_string(t.capacity()) + "): release some first";
    return NFAD_ECOMPILE;
  }
  *chain_id = NFAD_CHAIN_JIT_BASE + slot;
  return NFAD_OK;
}

static const char* name_of(int chain_id) {
  const Table::Chain* c = table().peek(chain_id - NFAD_CHAIN_JIT_BASE);
  return c ? c->name.c_str() : nullptr;
}
static const char* program_of(int chain_id) {
  const Table::Chain* c = table().peek(chain_id - NFAD_CHAIN_JIT_BASE);
  return c ? c->program.c_str() : nullptr;
}
static int outputs_of(int chain_id) {
  Table::Chain c;
  return table().get(chain_id - NFAD_CHAIN_JIT_BASE, c) ? c.kernel->m : -1;
}
static int kernel_of(int chain_id) {
  Table::Chain c;
  return table().get(chain_id - NFAD_CHAIN_JIT_BASE, c) ? c.kernel->uid : -1;
}

template <int M>
static int forward_m(const Table::Chain& c, const void* x, void* const* y, void* const* dydx, size_t n, int dtype,
                     void* stream) {
  const void* const in[1] = {x};
  void* out[2 * M];
  for (int j = 0; j < M; ++j) { out[2 * j] = y[j]; out[2 * j + 1] = dydx[j]; }
  const int rc = validate<1, 2 * M>(in, out, n, dtype);
  if (rc != NFAD_OK || n == 0) return rc;
  using P = Ptrs<1, 2 * M>;
  P p;
  p.in[0] = x;
  for (int o = 0; o < 2 * M; ++o) p.out[o] = out[o];
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const Kernel& k = *c.kernel;
  chain::Args consts = c.args;
  auto enqueue = [s, &consts](hipFunction_t f, const P& q, size_t m, Geometry g) {
    P ptrs = q;
    void* params[3] = {&ptrs, &m, &consts};
    return hipModuleLaunchKernel(f, g.grid, 1, 1, g.threads, 1, 1, g.lds, s, params, nullptr);
  };
  return launch_planned(
      p, n, dtype,
      [&](const P& q, size_t m, Geometry g) { return enqueue(g.small ? k.vec_small[dtype] : k.vec[dtype], q, m, g); },
      [&](const P& q, size_t m, Geometry g) { return enqueue(k.scalar[dtype], q, m, g); });
}

// want_m: the number of outputs the entry point serves (1 for nfad_chain_fwd), 0 = any.
static int forward(int chain_id, int want_m, const void* x, void* const* y, void* const* dydx, size_t n, int dtype,
                   void* stream) {
  Table::Chain c;   // a copy: its kernel reference keeps the module loaded until this call returns
  if (!table().get(chain_id - NFAD_CHAIN_JIT_BASE, c)) return NFAD_EINVAL_KIND;
  if (want_m && c.kernel->m != want_m) return NFAD_EINVAL_KIND;
  if (!dtype_ok(dtype)) return NFAD_EINVAL_DTYPE;
  if (n == 0) return NFAD_OK;
  if (!y || !dydx) return NFAD_ENULL;
  switch (c.kernel->m) {
    case 1: return forward_m<1>(c, x, y, dydx, n, dtype, stream);
    case 2: return forward_m<2>(c, x, y, dydx, n, dtype, stream);
    case 3: return forward_m<3>(c, x, y, dydx, n, dtype, stream);
    case 4: return forward_m<4>(c, x, y, dydx, n, dtype, stream);
  }
  return NFAD_EINVAL_KIND;
}

}  // namespace jit
}  // namespace nfad

extern "C" {

int nfad_chain_compile(const char* program, int* chain_id) {
  if (!program || !chain_id) return NFAD_ENULL;
  const char* const programs[1] = {program};
  return jit::compile(programs, 1, chain_id);
}

int nfad_chain_compile_multi(const char* const* programs, int m, int* chain_id) {
  if (!programs || !chain_id) return NFAD_ENULL;
  if (m < 1 || m > NFAD_MAX_OUTPUTS) return NFAD_EINVAL_KIND;
  return jit::compile(programs, m, chain_id);
}

int nfad_chain_num_outputs(int chain_id) {
  if (chain_id >= NFAD_CHAIN_JIT_BASE) return jit::outputs_of(chain_id);
  return (chain_id >= 0 && chain_id < kNumChains) ? 1 : -1;
}

int nfad_chain_kernel(int chain_id) {
  return chain_id >= NFAD_CHAIN_JIT_BASE ? jit::kernel_of(chain_id) : -1;
}

int nfad_chain_fwd_multi(int chain_id, const void* x, void* const* y, void* const* dydx, size_t n, int dtype,
                         void* stream) {
  if (chain_id < NFAD_CHAIN_JIT_BASE) return NFAD_EINVAL_KIND;
  return jit::forward(chain_id, 0, x, y, dydx, n, dtype, stream);
}

int nfad_chain_release(int chain_id) {
  if (chain_id < NFAD_CHAIN_JIT_BASE) return NFAD_EINVAL_KIND;
  return jit::table().release(chain_id - NFAD_CHAIN_JIT_BASE) ? NFAD_OK : NFAD_EINVAL_KIND;
}

const char* nfad_chain_log(void) { return jit::g_log.c_str(); }

}  // extern "C"

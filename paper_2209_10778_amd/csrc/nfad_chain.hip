// nfad_chain.hip -- fused forward-AD kernels for chains composed from primitive operations
// (nfad_chain.hpp), and their C ABI.  A chain is fused into ONE kernel on the same streaming
// skeleton as the hand-tuned activations: read x, write y and dydx; backward is nfad_bwd.
#include "nfad_stream.hpp"
#include "nfad_chain.hpp"

namespace nfad {

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
NFAD_CHAIN_CONSTANT(kZero, 0.0f);
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
struct Compiled;
static const Compiled* find(int chain_id);
static int forward(const Compiled* c, const void* x, void* const* y, void* const* dydx, size_t n, int dtype,
                   void* stream);
static int outputs_of(const Compiled* c);
static const char* name_of(const Compiled* c);
static const char* program_of(const Compiled* c);
}  // namespace jit
}  // namespace nfad

using namespace nfad;

extern "C" {

int nfad_chain_count(void) { return kNumChains; }

const char* nfad_chain_name(int chain_id) {
  if (chain_id >= NFAD_CHAIN_JIT_BASE) {
    const jit::Compiled* c = jit::find(chain_id);
    return c ? jit::name_of(c) : nullptr;
  }
  return (chain_id >= 0 && chain_id < kNumChains) ? kChains[chain_id].name : nullptr;
}

const char* nfad_chain_program(int chain_id) {
  if (chain_id >= NFAD_CHAIN_JIT_BASE) {
    const jit::Compiled* c = jit::find(chain_id);
    return c ? jit::program_of(c) : nullptr;
  }
  return (chain_id >= 0 && chain_id < kNumChains) ? kChains[chain_id].program : nullptr;
}

int nfad_chain_fwd(int chain_id, const void* x, void* y, void* dydx, size_t n, int dtype, void* stream) {
  if (chain_id >= NFAD_CHAIN_JIT_BASE) {
    const jit::Compiled* c = jit::find(chain_id);
    if (!c || jit::outputs_of(c) != 1) return NFAD_EINVAL_KIND;
    void* const ys[1] = {y};
    void* const ds[1] = {dydx};
    return jit::forward(c, x, ys, ds, n, dtype, stream);
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
// (hiprtc, for the architecture of the current device) and keeps the loaded kernel under a
// new chain id.  The program text is parsed against a closed grammar (the primitive names,
// `x`, decimal constants): nothing from the caller's string reaches the compiler verbatim.
#include <hip/hiprtc.h>

#include <math.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <string>
#include <vector>

#include "nfad_embedded.inc"

namespace nfad {
namespace jit {

static constexpr int kMaxTokens = 256;
static constexpr int kMaxChains = 4096;

struct Compiled {
  std::string program, name;
  int m = 1;                                              // number of outputs (chains over the same x)
  hipModule_t module = nullptr;
  hipFunction_t vec[3] = {nullptr, nullptr, nullptr};     // indexed by nfad_dtype_t: the shape for large launches,
  hipFunction_t vec_small[3] = {nullptr, nullptr, nullptr};   // ... the one for small launches,
  hipFunction_t scalar[3] = {nullptr, nullptr, nullptr};  // ... and the element-at-a-time kernel
  bool live = false;
};
static std::mutex g_mu;
static std::vector<Compiled*> g_chains;          // index = id - NFAD_CHAIN_JIT_BASE; never shrinks
static thread_local std::string g_log;

// postfix program -> C++ type expression over nfad::chain templates (+ constant definitions)
static bool translate(const char* program, int index, std::string& consts, std::string& type, std::string& err) {
  static const struct { const char* tok; const char* tmpl; int arity; } kOps[] = {
      {"+", "Add", 2}, {"-", "Sub", 2}, {"*", "Mul", 2}, {"/", "Div", 2}, {"min", "Min", 2}, {"max", "Max", 2},
      {"neg", "Neg", 1}, {"relu", "Relu", 1}, {"abs", "Abs", 1}, {"sqrt", "Sqrt", 1},
      {"exp", "Exp", 1}, {"log", "Log", 1}, {"tanh", "Tanh", 1}, {"sigmoid", "Sigmoid", 1},
      {"softplus", "Softplus", 1}, {"erf", "Erf", 1}};
  std::vector<std::string> stack;
  int ntok = 0, nconst = 0;
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
    if (tok == "x") { stack.push_back("X"); uses_x = true; continue; }
    bool matched = false;
    for (const auto& op : kOps) {
      if (tok != op.tok) continue;
      if ((int)stack.size() < op.arity) { err = "operator '" + tok + "' lacks operands"; return false; }
      if (op.arity == 1) {
        stack.back() = std::string(op.tmpl) + "<" + stack.back() + ">";
      } else {
        const std::string b = stack.back(); stack.pop_back();
        stack.back() = std::string(op.tmpl) + "<" + stack.back() + ", " + b + ">";
      }
      matched = true;
      break;
    }
    if (matched) continue;
    char* end = nullptr;
    const float c = strtof(tok.c_str(), &end);
    if (end == tok.c_str() || *end != '\0' || !isfinite(c)) { err = "unknown token '" + tok + "'"; return false; }
    char buf[96];
    snprintf(buf, sizeof buf, "NFAD_CHAIN_CONSTANT(K%d_%d, %af);\n", index, nconst, (double)c);  // exact hex-float literal
    consts += buf;
    stack.push_back("Const<K" + std::to_string(index) + "_" + std::to_string(nconst) + ">");
    ++nconst;
  }
  if (stack.size() != 1) { err = "program leaves " + std::to_string(stack.size()) + " values"; return false; }
  if (!uses_x) { err = "program does not use x"; return false; }
  type = stack[0];
  return true;
}

static const char* kTypeNames[3] = {"float", "_Float16", "__bf16"};   // indexed by nfad_dtype_t

static int compile(const char* const* programs, int m, int* chain_id) {
  std::string consts, aliases, list, joined, err;
  g_log.clear();
  for (int j = 0; j < m; ++j) {
    std::string type;
    if (!programs[j]) { g_log = "null program"; return NFAD_ENULL; }
    if (!translate(programs[j], j, consts, type, err)) {
      g_log = (m > 1 ? "program " + std::to_string(j) + ": " : std::string()) + err;
      return NFAD_EPROGRAM;
    }
    aliases += "using UserChain" + std::to_string(j) + " = " + type + ";\n";
    list += (j ? ", nfad::chain::UserChain" : "nfad::chain::UserChain") + std::to_string(j);
    joined += (j ? " ; " : "") + std::string(programs[j]);
  }
  // m == 1 uses the same operation type as the built-in chains
  const std::string op = m == 1 ? "nfad::ChainFwdOp<" + list + ">" : "nfad::ChainFwdMultiOp<" + list + ">";

  const std::string src = "#include \"nfad_stream_device.hpp\"\n#include \"nfad_chain.hpp\"\n"
                          "namespace nfad { namespace chain {\n" + consts + aliases + "} }\n";
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

  Compiled* c = new Compiled;
  c->program = joined;
  c->m = m;
  bool ok = hipModuleLoadData(&c->module, code.data()) == hipSuccess;
  for (int t = 0; ok && t < 9; ++t) {
    const char* lowered = nullptr;
    hipFunction_t* slot = t < 3 ? &c->vec[t] : (t < 6 ? &c->scalar[t - 3] : &c->vec_small[t - 6]);
    ok = hiprtcGetLoweredName(prog, names[t].c_str(), &lowered) == HIPRTC_SUCCESS && lowered &&
         hipModuleGetFunction(slot, c->module, lowered) == hipSuccess;
  }
  hiprtcDestroyProgram(&prog);
  if (!ok) {
    if (c->module) (void)hipModuleUnload(c->module);
    delete c;
    if (g_log.empty()) g_log = "loading the compiled chain failed";
    return NFAD_ECOMPILE;
  }
  c->live = true;
  std::lock_guard<std::mutex> lock(g_mu);
  if ((int)g_chains.size() >= kMaxChains) {
    (void)hipModuleUnload(c->module);
    delete c;
    g_log = "too many compiled chains";
    return NFAD_ECOMPILE;
  }
  c->name = "jit:" + std::to_string(g_chains.size());
  g_chains.push_back(c);
  *chain_id = NFAD_CHAIN_JIT_BASE + (int)g_chains.size() - 1;
  return NFAD_OK;
}

// Copies the launch handles of a live chain out under the lock; nullptr if the id is dead.
static const Compiled* find(int chain_id) {
  std::lock_guard<std::mutex> lock(g_mu);
  const int i = chain_id - NFAD_CHAIN_JIT_BASE;
  if (i < 0 || i >= (int)g_chains.size() || !g_chains[i]->live) return nullptr;
  return g_chains[i];
}

template <int M>
static int forward_m(const Compiled* c, const void* x, void* const* y, void* const* dydx, size_t n, int dtype,
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
  auto enqueue = [s](hipFunction_t f, const P& q, size_t m, Geometry g) {
    P args = q;
    void* params[2] = {&args, &m};
    return hipModuleLaunchKernel(f, g.grid, 1, 1, g.threads, 1, 1, g.lds, s, params, nullptr);
  };
  return launch_planned(
      p, n, dtype,
      [&](const P& q, size_t m, Geometry g) { return enqueue(g.small ? c->vec_small[dtype] : c->vec[dtype], q, m, g); },
      [&](const P& q, size_t m, Geometry g) { return enqueue(c->scalar[dtype], q, m, g); });
}

static int forward(const Compiled* c, const void* x, void* const* y, void* const* dydx, size_t n, int dtype,
                   void* stream) {
  if (!dtype_ok(dtype)) return NFAD_EINVAL_DTYPE;
  if (n == 0) return NFAD_OK;
  if (!y || !dydx) return NFAD_ENULL;
  switch (c->m) {
    case 1: return forward_m<1>(c, x, y, dydx, n, dtype, stream);
    case 2: return forward_m<2>(c, x, y, dydx, n, dtype, stream);
    case 3: return forward_m<3>(c, x, y, dydx, n, dtype, stream);
    case 4: return forward_m<4>(c, x, y, dydx, n, dtype, stream);
  }
  return NFAD_EINVAL_KIND;
}

static int outputs_of(const Compiled* c) { return c->m; }
static const char* name_of(const Compiled* c) { return c->name.c_str(); }
static const char* program_of(const Compiled* c) { return c->program.c_str(); }

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
  if (chain_id >= NFAD_CHAIN_JIT_BASE) {
    const jit::Compiled* c = jit::find(chain_id);
    return c ? jit::outputs_of(c) : -1;
  }
  return (chain_id >= 0 && chain_id < kNumChains) ? 1 : -1;
}

int nfad_chain_fwd_multi(int chain_id, const void* x, void* const* y, void* const* dydx, size_t n, int dtype,
                         void* stream) {
  if (chain_id < NFAD_CHAIN_JIT_BASE) return NFAD_EINVAL_KIND;
  const jit::Compiled* c = jit::find(chain_id);
  return c ? jit::forward(c, x, y, dydx, n, dtype, stream) : NFAD_EINVAL_KIND;
}

int nfad_chain_release(int chain_id) {
  std::lock_guard<std::mutex> lock(jit::g_mu);
  const int i = chain_id - NFAD_CHAIN_JIT_BASE;
  if (i < 0 || i >= (int)jit::g_chains.size() || !jit::g_chains[i]->live) return NFAD_EINVAL_KIND;
  jit::g_chains[i]->live = false;
  (void)hipModuleUnload(jit::g_chains[i]->module);
  jit::g_chains[i]->module = nullptr;
  return NFAD_OK;
}

const char* nfad_chain_log(void) { return jit::g_log.c_str(); }

}  // extern "C"

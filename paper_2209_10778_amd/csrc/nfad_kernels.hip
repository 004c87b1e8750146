// nfad_kernels.hip -- the per-element operations of the method and its two baselines, and
// the C ABI of libnfad (include/nfad.h).  The streaming kernel skeleton and the launch code
// are in nfad_stream.hpp; the arithmetic of the activations is in nfad_math.hpp.  The
// dual-number tangent (seed 1, Sec. II-C eq. 3) never touches memory.
#include "nfad_stream.hpp"
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

// ------------------------------------------------------------------ streaming probes
// The launch shape of the kernels above with the arithmetic taken out: N_IN tensors read,
// N_OUT written, one block per tile, the same block sizes, unroll, cache hints and cap on
// resident waves.  They measure what the memory system gives a traffic pattern on the part
// at hand, so that a kernel's throughput can be read against its own pattern's ceiling.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

template <int N_IN, int N_OUT>
struct ProbeShape {
  static constexpr int kThreads = N_IN <= 1 ? NFAD_THREADS_1IN : NFAD_THREADS_NIN;
  static constexpr int kUnroll = NFAD_UNROLL;
  static constexpr bool kNtLoad = N_IN == 1 ? (NFAD_NT_LOAD_1IN != 0) : (NFAD_NT_LOAD_NIN != 0);
  static constexpr int kWavesRaw = NFAD_INFLIGHT_KIB / (kUnroll * (N_IN + N_OUT));
  static constexpr int kWavesPerCu = kWavesRaw < 8 ? 8 : (kWavesRaw > 32 ? 32 : kWavesRaw);
};
struct ProbePtrs {
  const u32x4* in[2];
  u32x4* out[2];
};

template <int N_IN, int N_OUT>
__global__ __launch_bounds__((ProbeShape<N_IN, N_OUT>::kThreads)) void probe_kernel(ProbePtrs p, size_t nvec) {
  using Shape = ProbeShape<N_IN, N_OUT>;
  constexpr int kThreads = Shape::kThreads, kUnroll = Shape::kUnroll;
  const size_t base = (size_t)blockIdx.x * kThreads * kUnroll + threadIdx.x;
  u32x4 v[kUnroll];
#pragma unroll
  for (int j = 0; j < kUnroll; ++j) {
    const size_t idx = base + (size_t)j * kThreads;
    // with nothing to read, write a pattern with busy bits (not a constant)
    const unsigned h = (unsigned)idx * 2654435761u;
    v[j] = u32x4{h, h ^ 0x9e3779b9u, h * 31u, ~h};
    if (N_IN > 0 && idx < nvec) {
      v[j] = stream_load<Shape::kNtLoad>(p.in[0] + idx);
      if (N_IN > 1) v[j] ^= stream_load<Shape::kNtLoad>(p.in[1] + idx);
    }
  }
  if constexpr (N_OUT > 0) {
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      const size_t idx = base + (size_t)j * kThreads;
      if (idx < nvec) {
        stream_store(p.out[0] + idx, v[j]);
        if (N_OUT > 1) stream_store(p.out[1] + idx, ~v[j]);
      }
    }
  } else {
    // keep the loads alive: one 16-byte write that practically never happens
    u32x4 acc = v[0];
#pragma unroll
    for (int j = 1; j < kUnroll; ++j) acc ^= v[j];
    if (acc.x == 0x7fc12345u && acc.y == 0x7fc54321u && acc.z == 0x12345678u && acc.w == 0x87654321u) p.out[0][0] = acc;
  }
}

template <int N_IN, int N_OUT>
static int launch_probe(const ProbePtrs& p, size_t nvec, hipStream_t stream) {
  using Shape = ProbeShape<N_IN, N_OUT>;
  const size_t tile = (size_t)Shape::kThreads * Shape::kUnroll;
  const size_t grid = (nvec + tile - 1) / tile;
  if (grid == 0) return NFAD_OK;
  if (grid > max_grid()) return NFAD_ELAUNCH;   // probes do not stride: 2^24 tiles is 64 GiB per tensor
  const unsigned lds = lds_reservation(Shape::kWavesPerCu, Shape::kThreads, device_info().lds_per_cu);
  hipLaunchKernelGGL((probe_kernel<N_IN, N_OUT>), dim3((unsigned)grid), dim3(Shape::kThreads), lds, stream, p, nvec);
  return hipGetLastError() == hipSuccess ? NFAD_OK : NFAD_ELAUNCH;
}

}  // namespace nfad

using namespace nfad;

#define NFAD_DISPATCH_KIND(kind, OPT, ...)                         \
  switch (kind) {                                                  \
    case NFAD_GELU_TANH: return run<OPT<kGeluTanh>>(__VA_ARGS__);  \
    case NFAD_GELU_ERF: return run<OPT<kGeluErf>>(__VA_ARGS__);    \
    case NFAD_SWISH: return run<OPT<kSwish>>(__VA_ARGS__);         \
    case NFAD_MISH: return run<OPT<kMish>>(__VA_ARGS__);           \
  }                                                                \
  return NFAD_EINVAL_KIND

extern "C" {

int nfad_fwd(int kind, const void* x, void* y, void* dydx, size_t n, int dtype, void* stream) {
  if (!kind_ok(kind)) return NFAD_EINVAL_KIND;
  const void* const in[1] = {x};
  void* const out[2] = {y, dydx};
  NFAD_DISPATCH_KIND(kind, FwdOp, dtype, in, out, n, stream);
}

int nfad_bwd(const void* gy, const void* dydx, void* gx, size_t n, int dtype, void* stream) {
  const void* const in[2] = {gy, dydx};
  void* const out[1] = {gx};
  return run<BwdOp>(dtype, in, out, n, stream);
}

int nfad_bwd_multi(const void* const* gy, const void* const* dydx, int m, void* gx, size_t n, int dtype,
                   void* stream) {
  if (m < 1 || m > NFAD_MAX_OUTPUTS) return NFAD_EINVAL_KIND;
  if (!dtype_ok(dtype)) return NFAD_EINVAL_DTYPE;
  if (n == 0) return NFAD_OK;
  if (!gy || !dydx) return NFAD_ENULL;
  void* const out[1] = {gx};
  switch (m) {
    case 1: {
      const void* const in[2] = {gy[0], dydx[0]};
      return run<BwdMultiOp<1>>(dtype, in, out, n, stream);
    }
    case 2: {
      const void* const in[4] = {gy[0], dydx[0], gy[1], dydx[1]};
      return run<BwdMultiOp<2>>(dtype, in, out, n, stream);
    }
    case 3: {
      const void* const in[6] = {gy[0], dydx[0], gy[1], dydx[1], gy[2], dydx[2]};
      return run<BwdMultiOp<3>>(dtype, in, out, n, stream);
    }
    case 4: {
      const void* const in[8] = {gy[0], dydx[0], gy[1], dydx[1], gy[2], dydx[2], gy[3], dydx[3]};
      return run<BwdMultiOp<4>>(dtype, in, out, n, stream);
    }
  }
  return NFAD_EINVAL_KIND;
}

int nfad_recompute_fwd(int kind, const void* x, void* y, size_t n, int dtype, void* stream) {
  if (!kind_ok(kind)) return NFAD_EINVAL_KIND;
  const void* const in[1] = {x};
  void* const out[1] = {y};
  NFAD_DISPATCH_KIND(kind, RecomputeFwdOp, dtype, in, out, n, stream);
}

int nfad_recompute_bwd(int kind, const void* gy, const void* x, void* gx, size_t n, int dtype,
                       void* stream) {
  if (!kind_ok(kind)) return NFAD_EINVAL_KIND;
  const void* const in[2] = {gy, x};
  void* const out[1] = {gx};
  NFAD_DISPATCH_KIND(kind, RecomputeBwdOp, dtype, in, out, n, stream);
}

int nfad_saveall_num_saved(int kind) {
  switch (kind) {
    case NFAD_GELU_TANH: return 4;
    case NFAD_GELU_ERF: return 3;
    case NFAD_SWISH: return 2;
    case NFAD_MISH: return 2;
  }
  return -1;
}

int nfad_saveall_fwd(int kind, const void* x, void* y, void* const* saved, size_t n, int dtype,
                     void* stream) {
  if (!kind_ok(kind)) return NFAD_EINVAL_KIND;
  if (!dtype_ok(dtype)) return NFAD_EINVAL_DTYPE;
  if (n == 0) return NFAD_OK;
  if (!saved) return NFAD_ENULL;
  const void* const in[1] = {x};
  switch (kind) {
    case NFAD_SWISH: {
      void* const out[2] = {y, saved[1]};
      return run<SaveAllFwdOp<kSwish>>(dtype, in, out, n, stream);
    }
    case NFAD_MISH: {
      void* const out[2] = {y, saved[1]};
      return run<SaveAllFwdOp<kMish>>(dtype, in, out, n, stream);
    }
    case NFAD_GELU_ERF: {
      void* const out[3] = {y, saved[1], saved[2]};
      return run<SaveAllFwdOp<kGeluErf>>(dtype, in, out, n, stream);
    }
    case NFAD_GELU_TANH: {
      void* const out[4] = {y, saved[1], saved[2], saved[3]};
      return run<SaveAllFwdOp<kGeluTanh>>(dtype, in, out, n, stream);
    }
  }
  return NFAD_EINVAL_KIND;
}

int nfad_saveall_bwd(int kind, const void* gy, const void* const* saved, void* gx, size_t n,
                     int dtype, void* stream) {
  if (!kind_ok(kind)) return NFAD_EINVAL_KIND;
  if (!dtype_ok(dtype)) return NFAD_EINVAL_DTYPE;
  if (n == 0) return NFAD_OK;
  if (!saved) return NFAD_ENULL;
  void* const out[1] = {gx};
  switch (kind) {
    case NFAD_SWISH: {
      const void* const in[3] = {gy, saved[0], saved[1]};
      return run<SaveAllBwdOp<kSwish>>(dtype, in, out, n, stream);
    }
    case NFAD_MISH: {
      const void* const in[3] = {gy, saved[0], saved[1]};
      return run<SaveAllBwdOp<kMish>>(dtype, in, out, n, stream);
    }
    case NFAD_GELU_ERF: {
      const void* const in[4] = {gy, saved[0], saved[1], saved[2]};
      return run<SaveAllBwdOp<kGeluErf>>(dtype, in, out, n, stream);
    }
    case NFAD_GELU_TANH: {
      const void* const in[5] = {gy, saved[0], saved[1], saved[2], saved[3]};
      return run<SaveAllBwdOp<kGeluTanh>>(dtype, in, out, n, stream);
    }
  }
  return NFAD_EINVAL_KIND;
}

const char* nfad_status_string(int status) {
  switch (status) {
    case NFAD_OK: return "ok";
    case NFAD_EINVAL_KIND: return "invalid activation kind";
    case NFAD_EINVAL_DTYPE: return "invalid dtype";
    case NFAD_ENULL: return "null pointer with n > 0";
    case NFAD_EALIGN: return "pointer not aligned to the element size";
    case NFAD_EALIAS: return "two outputs of one call coincide";
    case NFAD_ELAUNCH: return "HIP kernel launch failed";
    case NFAD_EPROGRAM: return "malformed chain program";
    case NFAD_ECOMPILE: return "run-time compilation of a chain failed";
  }
  return "unknown status";
}

int nfad_version(void) { return 100; }

#ifdef NFAD_EXPERIMENT
void nfad_experiment_set_waves(int waves) { nfad::g_waves_experiment = waves; }
#endif

int nfad_probe_stream(int n_in, int n_out, const void* const* in, void* const* out, size_t bytes, void* stream) {
  using namespace nfad;
  if (n_in < 0 || n_in > 2 || n_out < 0 || n_out > 2 || n_in + n_out == 0) return NFAD_EINVAL_KIND;
  if ((n_in > 0 && !in) || !out) return NFAD_ENULL;
  ProbePtrs p = {{nullptr, nullptr}, {nullptr, nullptr}};
  for (int i = 0; i < n_in; ++i) {
    if (!in[i]) return NFAD_ENULL;
    if ((uintptr_t)in[i] & 15u) return NFAD_EALIGN;
    p.in[i] = static_cast<const u32x4*>(in[i]);
  }
  for (int o = 0; o < (n_out > 0 ? n_out : 1); ++o) {   // with n_out == 0, out[0] is the 16-byte sink
    if (!out[o]) return NFAD_ENULL;
    if ((uintptr_t)out[o] & 15u) return NFAD_EALIGN;
    p.out[o] = static_cast<u32x4*>(out[o]);
  }
  if (bytes & 15u) return NFAD_EALIGN;
  const size_t nvec = bytes / 16;
  hipStream_t st = static_cast<hipStream_t>(stream);
  switch (n_in * 3 + n_out) {
    case 0 * 3 + 1: return launch_probe<0, 1>(p, nvec, st);
    case 0 * 3 + 2: return launch_probe<0, 2>(p, nvec, st);
    case 1 * 3 + 0: return launch_probe<1, 0>(p, nvec, st);
    case 1 * 3 + 1: return launch_probe<1, 1>(p, nvec, st);
    case 1 * 3 + 2: return launch_probe<1, 2>(p, nvec, st);
    case 2 * 3 + 0: return launch_probe<2, 0>(p, nvec, st);
    case 2 * 3 + 1: return launch_probe<2, 1>(p, nvec, st);
    case 2 * 3 + 2: return launch_probe<2, 2>(p, nvec, st);
  }
  return NFAD_EINVAL_KIND;
}

}  // extern "C"

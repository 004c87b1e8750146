// nfad_kernels.hip -- gfx950 element-wise kernels and the C ABI of libnfad (include/nfad.h).
//
// One streaming skeleton serves every pass: each lane moves 16 bytes per access (4 fp32 or
// 8 fp16/bf16 elements), consecutive lanes touch consecutive 16-byte words (1 KiB per
// wave64 access), kUnroll independent accesses per tensor are in flight per lane, and
// blocks take the tensor tile by tile in address order.  All arithmetic is fp32 in
// registers; the dual-number tangent (seed 1, Sec. II-C eq. 3) never touches memory.
// There is no LDS, no atomics and no scratch memory: the path is a pure HBM stream.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/nfad.h"
#include "nfad_math.hpp"

// Launch-shape overrides for experiments (the defaults below are the measured choices).
#ifndef NFAD_THREADS_1IN   /* block size of kernels that read one tensor  */
#define NFAD_THREADS_1IN 128
#endif
#ifndef NFAD_THREADS_NIN   /* block size of kernels that read several     */
#define NFAD_THREADS_NIN 64
#endif
#ifndef NFAD_UNROLL        /* 16-byte accesses in flight per lane and tensor */
#define NFAD_UNROLL 2
#endif
#ifndef NFAD_NT_LOAD_1IN   /* nontemporal loads, one-input kernels        */
#define NFAD_NT_LOAD_1IN 0
#endif
#ifndef NFAD_NT_LOAD_NIN   /* nontemporal loads, several-input kernels    */
#define NFAD_NT_LOAD_NIN 1
#endif
#ifndef NFAD_INFLIGHT_KIB  /* target KiB of 16-byte accesses in flight per compute unit */
#define NFAD_INFLIGHT_KIB 96
#endif

namespace nfad {

// Launch shape of a streaming kernel with NIN input and NOUT output tensors.
//
// The path is bound by HBM, and HBM runs best when just enough requests are in flight to
// cover its latency (bandwidth x latency ~ 16 MB over the chip, ~64 KiB per compute unit):
// more than that only lengthens the queues in front of the DRAM banks and costs row hits
// and read/write turnarounds.  So every kernel uses small blocks, kUnroll independent
// 16-byte accesses per lane and tensor, and a cap on resident waves per compute unit of
//     kInflightKiB / (kUnroll * (NIN + NOUT))        (one wave64 access = 1 KiB),
// enforced by reserving an idle slice of the 160 KiB LDS per block at launch.
template <int NIN, int NOUT>
struct LaunchShape {
  static constexpr int kThreads = NIN == 1 ? NFAD_THREADS_1IN : NFAD_THREADS_NIN;
  static constexpr int kUnroll = NFAD_UNROLL;
  static constexpr bool kNtLoad = NIN == 1 ? (NFAD_NT_LOAD_1IN != 0) : (NFAD_NT_LOAD_NIN != 0);
  static constexpr int kWavesRaw = NFAD_INFLIGHT_KIB / (kUnroll * (NIN + NOUT));
  static constexpr int kWavesPerCu = kWavesRaw < 8 ? 8 : (kWavesRaw > 32 ? 32 : kWavesRaw);
};

// ------------------------------------------------------------------ storage formats
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Loads: the nontemporal hint pays when several input streams compete; a single input
// stream does better without it.  Stores are always nontemporal (written once, never re-read).
template <bool NT, typename V>
__device__ __forceinline__ V stream_load(const V* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <typename V>
__device__ __forceinline__ void stream_store(V* p, V v) {
  __builtin_nontemporal_store(v, p);
}

// Storage<T>: T is the element type in memory; kVec elements make one 16-byte word.
// Conversions to storage round to nearest even (the hardware default mode).
template <typename T>
struct Storage;

template <>
struct Storage<float> {
  using Elem = float;
  using Vec = f32x4;
  static constexpr int kVec = 4;
  __device__ __forceinline__ static float up(float v) { return v; }
  __device__ __forceinline__ static float down(float v) { return v; }
};
template <>
struct Storage<_Float16> {
  using Elem = _Float16;
  using Vec = f16x8;
  static constexpr int kVec = 8;
  __device__ __forceinline__ static float up(_Float16 v) { return (float)v; }
  __device__ __forceinline__ static _Float16 down(float v) { return (_Float16)v; }
};
template <>
struct Storage<__bf16> {
  using Elem = __bf16;
  using Vec = bf16x8;
  static constexpr int kVec = 8;
  __device__ __forceinline__ static float up(__bf16 v) { return (float)v; }
  __device__ __forceinline__ static __bf16 down(float v) { return (__bf16)v; }
};

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

// ------------------------------------------------------------------ kernels
template <int NIN, int NOUT>
struct Ptrs {
  const void* in[NIN];
  void* out[NOUT];
};

static constexpr int kScalarThreads = 256;

// 16-byte vector body.  Requires every pointer 16-byte aligned.  Tile = kThreads * kUnroll
// vectors; block b takes tiles b, b + gridDim.x, ... (the host launches one block per full
// tile, so the hardware dispatcher hands tiles out in address order).  Full tiles run
// unguarded; the one partial tile and the < kVec scalar tail elements are taken by a single
// block.  The kernel uses no LDS: the dynamic LDS size of the launch only limits how many
// blocks fit on a compute unit.
template <class Op, typename T>
__global__ __launch_bounds__((LaunchShape<Op::kIn, Op::kOut>::kThreads)) void ew_vec_kernel(
    Ptrs<Op::kIn, Op::kOut> p, size_t n) {
  using S = Storage<T>;
  using Vec = typename S::Vec;
  using Shape = LaunchShape<Op::kIn, Op::kOut>;
  constexpr int kVec = S::kVec;
  constexpr bool kWide = sizeof(T) == 4;
  constexpr int kThreads = Shape::kThreads;
  constexpr int kUnroll = Shape::kUnroll;
  constexpr bool kNt = Shape::kNtLoad;
  constexpr size_t kTile = (size_t)kThreads * kUnroll;
  const size_t nvec = n / kVec;
  const size_t full_tiles = nvec / kTile;

  for (size_t tile = blockIdx.x; tile < full_tiles; tile += gridDim.x) {
    const size_t base = tile * kTile + threadIdx.x;
    Vec vin[kUnroll][Op::kIn];
#pragma unroll
    for (int j = 0; j < kUnroll; ++j)
#pragma unroll
      for (int i = 0; i < Op::kIn; ++i)
        vin[j][i] = stream_load<kNt>(reinterpret_cast<const Vec*>(p.in[i]) + (base + (size_t)j * kThreads));
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      Vec vout[Op::kOut];
#pragma unroll
      for (int e = 0; e < kVec; ++e) {
        float fin[Op::kIn], fout[Op::kOut];
#pragma unroll
        for (int i = 0; i < Op::kIn; ++i) fin[i] = S::up(vin[j][i][e]);
        Op::template apply<kWide>(fin, fout);
#pragma unroll
        for (int o = 0; o < Op::kOut; ++o) vout[o][e] = S::down(fout[o]);
      }
#pragma unroll
      for (int o = 0; o < Op::kOut; ++o)
        stream_store(reinterpret_cast<Vec*>(p.out[o]) + (base + (size_t)j * kThreads), vout[o]);
    }
  }

  // Ragged end: vectors [full_tiles*kTile, nvec) and elements [nvec*kVec, n).
  if (blockIdx.x == full_tiles % gridDim.x) {
    for (size_t v = full_tiles * kTile + threadIdx.x; v < nvec; v += kThreads) {
      Vec vin[Op::kIn], vout[Op::kOut];
#pragma unroll
      for (int i = 0; i < Op::kIn; ++i) vin[i] = stream_load<kNt>(reinterpret_cast<const Vec*>(p.in[i]) + v);
#pragma unroll
      for (int e = 0; e < kVec; ++e) {
        float fin[Op::kIn], fout[Op::kOut];
#pragma unroll
        for (int i = 0; i < Op::kIn; ++i) fin[i] = S::up(vin[i][e]);
        Op::template apply<kWide>(fin, fout);
#pragma unroll
        for (int o = 0; o < Op::kOut; ++o) vout[o][e] = S::down(fout[o]);
      }
#pragma unroll
      for (int o = 0; o < Op::kOut; ++o) stream_store(reinterpret_cast<Vec*>(p.out[o]) + v, vout[o]);
    }
    const size_t k = nvec * kVec + threadIdx.x;
    if (threadIdx.x < kVec && k < n) {
      float fin[Op::kIn], fout[Op::kOut];
#pragma unroll
      for (int i = 0; i < Op::kIn; ++i) fin[i] = S::up(reinterpret_cast<const T*>(p.in[i])[k]);
      Op::template apply<kWide>(fin, fout);
#pragma unroll
      for (int o = 0; o < Op::kOut; ++o) reinterpret_cast<T*>(p.out[o])[k] = S::down(fout[o]);
    }
  }
}

// Element-at-a-time kernel for pointers that are not all 16-byte aligned: same values,
// lower bandwidth.
template <class Op, typename T>
__global__ __launch_bounds__(kScalarThreads) void ew_scalar_kernel(Ptrs<Op::kIn, Op::kOut> p, size_t n) {
  using S = Storage<T>;
  constexpr bool kWide = sizeof(T) == 4;
  const size_t stride = (size_t)gridDim.x * kScalarThreads;
  for (size_t k = (size_t)blockIdx.x * kScalarThreads + threadIdx.x; k < n; k += stride) {
    float fin[Op::kIn], fout[Op::kOut];
#pragma unroll
    for (int i = 0; i < Op::kIn; ++i) fin[i] = S::up(reinterpret_cast<const T*>(p.in[i])[k]);
    Op::template apply<kWide>(fin, fout);
#pragma unroll
    for (int o = 0; o < Op::kOut; ++o) reinterpret_cast<T*>(p.out[o])[k] = S::down(fout[o]);
  }
}

// ------------------------------------------------------------------ host side
// Compute units and LDS bytes per compute unit of the current device (256 and 160 KiB on
// MI355X), queried once per device.
struct DeviceInfo {
  int cus;
  int lds_per_cu;
};
static DeviceInfo device_info() {
  static DeviceInfo cached[64];
  static int ready[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return {256, 160 * 1024};
  if (!__atomic_load_n(&ready[dev], __ATOMIC_ACQUIRE)) {
    int cus = 0, lds = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess ||
        lds < 64 * 1024)
      lds = 64 * 1024;
    cached[dev] = {cus, lds};   // every thread that races here writes the same values
    __atomic_store_n(&ready[dev], 1, __ATOMIC_RELEASE);
  }
  return cached[dev];
}

// NFAD_WAVES_PER_CU (environment, read once): tuning aid that replaces the built-in cap on
// resident waves per compute unit; 0 disables the cap.
static int waves_per_cu_override() {
  static int cached = -2;
  int v = __atomic_load_n(&cached, __ATOMIC_RELAXED);
  if (v == -2) {
    const char* s = getenv("NFAD_WAVES_PER_CU");
    v = s ? atoi(s) : -1;
    if (v < -1 || v > 64) v = -1;
    __atomic_store_n(&cached, v, __ATOMIC_RELAXED);
  }
  return v;
}

// Dynamic-LDS bytes per block so that at most waves_per_cu waves are resident per CU.
static unsigned lds_reservation(int waves_per_cu, int threads, int lds_per_cu) {
  const int waves_per_block = threads / 64;
  const int blocks = waves_per_cu / waves_per_block;
  if (waves_per_cu <= 0 || blocks * waves_per_block >= 32) return 0;  // 32 waves/CU is the hardware limit
  if (blocks < 3) return 64 * 1024;                                   // 64 KiB is the per-block maximum
  return (unsigned)((lds_per_cu / blocks) & ~1023);
}

template <class Op, typename T>
static int launch(const void* const (&in)[Op::kIn], void* const (&out)[Op::kOut], size_t n,
                  hipStream_t stream) {
  using S = Storage<T>;
  using Shape = LaunchShape<Op::kIn, Op::kOut>;
  Ptrs<Op::kIn, Op::kOut> p;
  uintptr_t bits = 0;
  for (int i = 0; i < Op::kIn; ++i) { p.in[i] = in[i]; bits |= (uintptr_t)in[i]; }
  for (int o = 0; o < Op::kOut; ++o) { p.out[o] = out[o]; bits |= (uintptr_t)out[o]; }
  const size_t max_grid = 1u << 30;
  const DeviceInfo di = device_info();
  if ((bits & 15u) == 0) {
    const size_t nvec = n / S::kVec;
    size_t grid = nvec / ((size_t)Shape::kThreads * Shape::kUnroll);   // one block per full tile
    if (grid == 0) grid = 1;
    if (grid > max_grid) grid = max_grid;
    int waves = waves_per_cu_override();
    if (waves < 0) waves = Shape::kWavesPerCu;
    const unsigned lds = lds_reservation(waves, Shape::kThreads, di.lds_per_cu);
    hipLaunchKernelGGL((ew_vec_kernel<Op, T>), dim3((unsigned)grid), dim3(Shape::kThreads), lds, stream, p, n);
  } else {
    size_t grid = (n + kScalarThreads - 1) / kScalarThreads;
    const size_t cap = (size_t)di.cus * 32;
    if (grid > cap) grid = cap;
    hipLaunchKernelGGL((ew_scalar_kernel<Op, T>), dim3((unsigned)grid), dim3(kScalarThreads), 0, stream, p, n);
  }
  return hipGetLastError() == hipSuccess ? NFAD_OK : NFAD_ELAUNCH;
}

template <class Op>
static int launch_dtype(int dtype, const void* const (&in)[Op::kIn], void* const (&out)[Op::kOut],
                        size_t n, void* stream) {
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  switch (dtype) {
    case NFAD_F32: return launch<Op, float>(in, out, n, s);
    case NFAD_F16: return launch<Op, _Float16>(in, out, n, s);
    case NFAD_BF16: return launch<Op, __bf16>(in, out, n, s);
  }
  return NFAD_EINVAL_DTYPE;
}

static size_t elem_size(int dtype) { return dtype == NFAD_F32 ? 4 : 2; }
static bool kind_ok(int kind) { return kind >= 0 && kind <= 3; }
static bool dtype_ok(int dtype) { return dtype >= 0 && dtype <= 2; }

// Host-only argument checks shared by every entry point; no HIP call is made here.
template <int NIN, int NOUT>
static int validate(const void* const (&in)[NIN], void* const (&out)[NOUT], size_t n, int dtype) {
  if (!dtype_ok(dtype)) return NFAD_EINVAL_DTYPE;
  if (n == 0) return NFAD_OK;
  const uintptr_t mask = elem_size(dtype) - 1;
  for (int i = 0; i < NIN; ++i) {
    if (!in[i]) return NFAD_ENULL;
    if ((uintptr_t)in[i] & mask) return NFAD_EALIGN;
  }
  for (int o = 0; o < NOUT; ++o) {
    if (!out[o]) return NFAD_ENULL;
    if ((uintptr_t)out[o] & mask) return NFAD_EALIGN;
    for (int q = 0; q < o; ++q)
      if (out[q] == out[o]) return NFAD_EALIAS;
  }
  return NFAD_OK;
}

template <class Op>
static int run(int dtype, const void* const (&in)[Op::kIn], void* const (&out)[Op::kOut], size_t n,
               void* stream) {
  const int rc = validate<Op::kIn, Op::kOut>(in, out, n, dtype);
  if (rc != NFAD_OK || n == 0) return rc;
  return launch_dtype<Op>(dtype, in, out, n, stream);
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
  }
  return "unknown status";
}

int nfad_version(void) { return 100; }

}  // extern "C"

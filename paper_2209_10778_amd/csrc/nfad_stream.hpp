// nfad_stream.hpp -- host half of the streaming skeleton: argument validation, launch-shape
// arithmetic and the launch itself.  The kernels are in nfad_stream_device.hpp.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/nfad.h"
#include "nfad_stream_device.hpp"

namespace nfad {

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
#ifdef NFAD_EXPERIMENT   /* experiment builds only: the override can be changed between launches */
static int g_waves_experiment = -1;
static int waves_per_cu_override() { return g_waves_experiment; }
#else
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
#endif

// Dynamic-LDS bytes per block so that at most waves_per_cu waves are resident per CU.
static unsigned lds_reservation(int waves_per_cu, int threads, int lds_per_cu) {
  const int waves_per_block = threads / 64;
  const int blocks = waves_per_cu / waves_per_block;
  if (waves_per_cu <= 0 || blocks * waves_per_block >= 32) return 0;  // 32 waves/CU is the hardware limit
  if (blocks < 3) return 64 * 1024;                                   // 64 KiB is the per-block maximum
  return (unsigned)((lds_per_cu / blocks) & ~1023);
}

// Grid, block and idle-LDS reservation of a launch.
struct Geometry {
  unsigned grid, threads, lds;
};
template <int NIN, int NOUT>
static Geometry vec_geometry(size_t n, int elems_per_vec) {
  using Shape = LaunchShape<NIN, NOUT>;
  const size_t nvec = n / (size_t)elems_per_vec;
  size_t grid = nvec / ((size_t)Shape::kThreads * Shape::kUnroll);   // one block per full tile
  if (grid == 0) grid = 1;
  if (grid > (1u << 30)) grid = 1u << 30;
  int waves = waves_per_cu_override();
  if (waves < 0) waves = Shape::kWavesPerCu;
  return {(unsigned)grid, (unsigned)Shape::kThreads,
          lds_reservation(waves, Shape::kThreads, device_info().lds_per_cu)};
}
static Geometry scalar_geometry(size_t n) {
  size_t grid = (n + kScalarThreads - 1) / kScalarThreads;
  const size_t cap = (size_t)device_info().cus * 32;
  if (grid > cap) grid = cap;
  return {(unsigned)grid, (unsigned)kScalarThreads, 0u};
}
// The 16-byte vector body needs every pointer of the call 16-byte aligned.
template <int NIN, int NOUT>
static bool all_aligned16(const Ptrs<NIN, NOUT>& p) {
  uintptr_t bits = 0;
  for (int i = 0; i < NIN; ++i) bits |= (uintptr_t)p.in[i];
  for (int o = 0; o < NOUT; ++o) bits |= (uintptr_t)p.out[o];
  return (bits & 15u) == 0;
}

template <class Op, typename T>
static int launch(const void* const (&in)[Op::kIn], void* const (&out)[Op::kOut], size_t n,
                  hipStream_t stream) {
  Ptrs<Op::kIn, Op::kOut> p;
  for (int i = 0; i < Op::kIn; ++i) p.in[i] = in[i];
  for (int o = 0; o < Op::kOut; ++o) p.out[o] = out[o];
  if (all_aligned16(p)) {
    const Geometry g = vec_geometry<Op::kIn, Op::kOut>(n, Storage<T>::kVec);
    hipLaunchKernelGGL((ew_vec_kernel<Op, T>), dim3(g.grid), dim3(g.threads), g.lds, stream, p, n);
  } else {
    const Geometry g = scalar_geometry(n);
    hipLaunchKernelGGL((ew_scalar_kernel<Op, T>), dim3(g.grid), dim3(g.threads), 0, stream, p, n);
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

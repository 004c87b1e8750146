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

// Largest grid of the vector kernel.  One block per tile up to this many blocks; beyond it the
// kernel's grid stride takes over.  2^24 blocks keeps grid x block below 2^32 threads.
// NFAD_MAX_GRID (environment, read once) lowers it, which is how the striding path is tested.
static size_t max_grid() {
  static size_t cached = 0;
  size_t v = __atomic_load_n(&cached, __ATOMIC_RELAXED);
  if (v == 0) {
    v = (size_t)1 << 24;
    const char* s = getenv("NFAD_MAX_GRID");
    if (s) {
      const long long w = atoll(s);
      if (w >= 1 && w < (long long)v) v = (size_t)w;
    }
    __atomic_store_n(&cached, v, __ATOMIC_RELAXED);
  }
  return v;
}

// Dynamic-LDS bytes per block so that at most waves_per_cu waves are resident per CU.  The
// hardware hands out LDS in granules of 1/128 of a compute unit's LDS (1280 bytes of 160 KiB;
// measured with blocks that only wait) and keeps floor(128 / granules per block) blocks resident,
// so the caps that exist for one-wave blocks are 32, 25, 21, 18, 16, 14, 12, 11, ...: the
// reservation is the smallest number of granules that admits no more than the blocks asked for.
static unsigned lds_reservation(int waves_per_cu, int threads, int lds_per_cu) {
  const int waves_per_block = threads / 64;
  const int blocks = waves_per_cu / waves_per_block;
  if (waves_per_cu <= 0 || blocks * waves_per_block >= 32) return 0;  // 32 waves/CU is the hardware limit
  if (blocks < 3) return 64 * 1024;                                   // the per-block maximum: two blocks stay resident
  const int granules = 128 / (blocks + 1) + 1;                        // smallest g with floor(128 / g) <= blocks
  return (unsigned)(granules * (lds_per_cu / 128));
}

// Grid, block and idle-LDS reservation of a launch, and which of the operation's two shapes it uses.
struct Geometry {
  unsigned grid, threads, lds;
  bool small;
};
template <class Sh>
static Geometry shape_geometry(size_t n, int elems_per_vec, int waves_per_cu, bool small) {
  const size_t nvec = n / (size_t)elems_per_vec;
  size_t grid = nvec / ((size_t)Sh::kThreads * Sh::kUnroll);   // one block per full tile
  if (grid == 0) grid = 1;
  if (grid > max_grid()) grid = max_grid();
  return {(unsigned)grid, (unsigned)Sh::kThreads, lds_reservation(waves_per_cu, Sh::kThreads, device_info().lds_per_cu),
          small};
}
template <int NIN, int NOUT, typename T, bool LIGHT>
static Geometry rule_geometry(size_t n) {
  using R = ShapeRule<NIN, NOUT, T, LIGHT>;
  constexpr int kVec = 16 / (int)sizeof(T);
  const unsigned long long moved = (unsigned long long)n * sizeof(T) * (NIN + NOUT);
  if (R::kTwoShapes && moved >= R::kSmallFromBytes && moved < R::kSmallBytes)
    return shape_geometry<typename R::Small>(n, kVec, R::kSmallWavesPerCu, true);
  return shape_geometry<typename R::Large>(n, kVec, R::kLargeWavesPerCu, false);
}
// Geometry of the vector kernel of an operation with NIN inputs and NOUT outputs on `dtype` storage.
template <int NIN, int NOUT, bool LIGHT>
static Geometry default_geometry(int dtype, size_t n) {
  switch (dtype) {
    case NFAD_F32: return rule_geometry<NIN, NOUT, float, LIGHT>(n);
    case NFAD_F16: return rule_geometry<NIN, NOUT, _Float16, LIGHT>(n);
    default: return rule_geometry<NIN, NOUT, __bf16, LIGHT>(n);
  }
}
static Geometry scalar_geometry(size_t n) {
  size_t grid = (n + kScalarThreads - 1) / kScalarThreads;
  const size_t cap = (size_t)device_info().cus * 32;
  if (grid > cap) grid = cap;
  return {(unsigned)grid, (unsigned)kScalarThreads, 0u, false};
}
// How a call is carried out.  The 16-byte vector kernel needs every pointer 16-byte aligned.
// If all pointers are misaligned by the SAME amount (a view such as t[1:] of aligned tensors),
// `head` leading elements go through the scalar kernel and the rest, now aligned, through the
// vector kernel; pointers with different misalignments take the scalar kernel throughout.
struct Plan {
  bool vec;
  size_t head;
};
template <int NIN, int NOUT>
static Plan make_plan(const Ptrs<NIN, NOUT>& p, size_t n, size_t elem_bytes) {
  const uintptr_t mis = (uintptr_t)p.out[0] & 15u;
  for (int i = 0; i < NIN; ++i)
    if (((uintptr_t)p.in[i] & 15u) != mis) return {false, 0};
  for (int o = 0; o < NOUT; ++o)
    if (((uintptr_t)p.out[o] & 15u) != mis) return {false, 0};
  if (mis == 0) return {true, 0};
  const size_t head = (16 - mis) / elem_bytes;   // pointers are element-aligned, so this is exact
  if (n <= head) return {false, 0};
  return {true, head};
}
template <int NIN, int NOUT>
static Ptrs<NIN, NOUT> advanced(const Ptrs<NIN, NOUT>& p, size_t bytes) {
  Ptrs<NIN, NOUT> q;
  for (int i = 0; i < NIN; ++i) q.in[i] = static_cast<const char*>(p.in[i]) + bytes;
  for (int o = 0; o < NOUT; ++o) q.out[o] = static_cast<char*>(p.out[o]) + bytes;
  return q;
}
// Runs a call according to its plan.  launch_vec(ptrs, n, geometry) and launch_scalar(ptrs, n,
// geometry) enqueue the two kernels and return a hipError_t.
template <int NIN, int NOUT, bool LIGHT = false, class LaunchVec, class LaunchScalar>
static int launch_planned(const Ptrs<NIN, NOUT>& p, size_t n, int dtype, LaunchVec launch_vec,
                          LaunchScalar launch_scalar) {
  const size_t elem_bytes = dtype == NFAD_F32 ? 4 : 2;
  const Plan plan = make_plan(p, n, elem_bytes);
  hipError_t e = hipSuccess;
  if (!plan.vec) {
    e = launch_scalar(p, n, scalar_geometry(n));
  } else {
    if (plan.head) e = launch_scalar(p, plan.head, scalar_geometry(plan.head));
    if (e == hipSuccess) {
      const size_t rest = n - plan.head;
      e = launch_vec(advanced(p, plan.head * elem_bytes), rest, default_geometry<NIN, NOUT, LIGHT>(dtype, rest));
    }
  }
  return e == hipSuccess ? NFAD_OK : NFAD_ELAUNCH;
}

template <class Op, typename T, int DTYPE>
static int launch(const void* const (&in)[Op::kIn], void* const (&out)[Op::kOut], size_t n,
                  hipStream_t stream, const typename OpParams<Op>::type& prm) {
  using P = Ptrs<Op::kIn, Op::kOut>;
  using R = ShapeRule<Op::kIn, Op::kOut, T, OpLight<Op>::value>;
  P p;
  for (int i = 0; i < Op::kIn; ++i) p.in[i] = in[i];
  for (int o = 0; o < Op::kOut; ++o) p.out[o] = out[o];
  return launch_planned<Op::kIn, Op::kOut, OpLight<Op>::value>(
      p, n, DTYPE,
      [stream, &prm](const P& q, size_t m, Geometry g) {
        if (R::kTwoShapes && g.small)
          hipLaunchKernelGGL((ew_vec_kernel<Op, T, typename R::Small>), dim3(g.grid), dim3(g.threads), g.lds, stream, q, m, prm);
        else
          hipLaunchKernelGGL((ew_vec_kernel<Op, T, typename R::Large>), dim3(g.grid), dim3(g.threads), g.lds, stream, q, m, prm);
        return hipGetLastError();
      },
      [stream, &prm](const P& q, size_t m, Geometry g) {
        hipLaunchKernelGGL((ew_scalar_kernel<Op, T>), dim3(g.grid), dim3(g.threads), 0, stream, q, m, prm);
        return hipGetLastError();
      });
}

template <class Op>
static int launch_dtype(int dtype, const void* const (&in)[Op::kIn], void* const (&out)[Op::kOut],
                        size_t n, void* stream, const typename OpParams<Op>::type& prm) {
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  switch (dtype) {
    case NFAD_F32: return launch<Op, float, NFAD_F32>(in, out, n, s, prm);
    case NFAD_F16: return launch<Op, _Float16, NFAD_F16>(in, out, n, s, prm);
    case NFAD_BF16: return launch<Op, __bf16, NFAD_BF16>(in, out, n, s, prm);
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
               void* stream, const typename OpParams<Op>::type& prm = typename OpParams<Op>::type{}) {
  const int rc = validate<Op::kIn, Op::kOut>(in, out, n, dtype);
  if (rc != NFAD_OK || n == 0) return rc;
  return launch_dtype<Op>(dtype, in, out, n, stream, prm);
}

}  // namespace nfad

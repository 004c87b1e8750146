// nfad_stream_device.hpp -- device half of the streaming skeleton every libnfad kernel is an
// instance of (the host half, which validates and launches, is nfad_stream.hpp).  This file
// compiles both with hipcc and with the runtime compiler, so it includes nothing but the
// HIP runtime header.
//
// Each lane moves 16 bytes per access (4 fp32 or 8 fp16/bf16 elements), consecutive lanes
// touch consecutive 16-byte words (1 KiB per wave64 access), kUnroll independent accesses per
// tensor are in flight per lane (each stored as soon as it is computed), and blocks take the
// tensor tile by tile in address order.
// All arithmetic is fp32 in registers.  There is no LDS use, no atomics and no scratch
// memory: every pass is a pure HBM stream.
#pragma once
#ifndef __HIPCC_RTC__
#include <hip/hip_runtime.h>
#endif

namespace nfad {

// ------------------------------------------------------------------ launch shape
// The compile-time half of a launch shape: block size, independent 16-byte accesses in flight
// per lane and tensor, and whether loads carry the nontemporal hint.  (The run-time half, the
// cap on resident waves per compute unit, is applied by the host through an idle LDS
// reservation.)
template <int THREADS, int UNROLL, bool NT_LOAD>
struct Shape {
  static constexpr int kThreads = THREADS;
  static constexpr int kUnroll = UNROLL;
  static constexpr bool kNtLoad = NT_LOAD;
};

// The shapes the library's kernels run in, chosen from interleaved in-process sweeps over block
// size x unroll x load hint x cap on resident waves, with the arithmetic in place, on tensors
// from 12 MB to 805 MB per launch.  The path is bound by HBM, and HBM runs best when just
// enough requests are in flight to cover its latency: more only lengthens the queues in front
// of the DRAM banks.  The simplest stream wins almost everywhere: one-wave blocks, ONE 16-byte
// access per lane and tensor, nontemporal loads.
//  * Kernels that read several tensors (backward passes) and one-read/one-write kernels run it
//    with no cap on resident waves: best or within 1-2 % of best at every size.
//  * Kernels that read one tensor and write several (the forward pass of the method) run it
//    capped at 21 waves per compute unit for fp32 storage and 25 for 16-bit storage (twice the
//    arithmetic per byte keeps a wave alive longer; an operation that declares kLight, the
//    cheaper arithmetic, keeps 21 for 16-bit storage too; 21 and 25 are two of the caps the LDS
//    granule can express, see lds_reservation).  A launch that moves 9 to 48 MiB is over
//    before a steady state forms, and then what counts is how fast the grid is handed out:
//    four times fewer, fatter blocks (two waves, two accesses per lane) and no cap.  Below
//    9 MiB there are too few tiles for that (the fatter blocks would leave compute units
//    idle), and one-wave blocks win again.
template <bool C, class A, class B>
struct SelectType {
  using type = A;
};
template <class A, class B>
struct SelectType<false, A, B> {
  using type = B;
};
template <int NIN, int NOUT, typename T, bool LIGHT = false>
struct ShapeRule {
  static constexpr bool kFanOut = NIN == 1 && NOUT >= 2;
  using Large = Shape<64, 1, true>;
  using Small = typename SelectType<kFanOut, Shape<128, 2, true>, Large>::type;
  static constexpr int kLargeWavesPerCu = kFanOut ? ((sizeof(T) == 4 || LIGHT) ? 21 : 25) : 0;   // 0 = no cap
  static constexpr int kSmallWavesPerCu = 0;
  static constexpr bool kTwoShapes = kFanOut;
  static constexpr unsigned long long kSmallFromBytes = 9ull << 20;   // Small shape for launches that move
  static constexpr unsigned long long kSmallBytes = 48ull << 20;      // [kSmallFromBytes, kSmallBytes) bytes
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

// ------------------------------------------------------------------ kernels
template <int NIN, int NOUT>
struct Ptrs {
  const void* in[NIN];
  void* out[NOUT];
};

// An operation may take a block of run-time parameters (a by-value kernel argument): it then
// declares `using Params = ...` and its apply() takes the block as a third argument.  The others
// get an empty block.
struct NoParams {};
template <class...>
struct VoidType {
  using type = void;
};
// An operation whose arithmetic is so light that its waves live hardly longer than their memory
// accesses declares `static constexpr bool kLight = true` (see ShapeRule).
template <class Op, class = void>
struct OpLight {
  static constexpr bool value = false;
};
template <class Op>
struct OpLight<Op, typename VoidType<decltype(Op::kLight)>::type> {
  static constexpr bool value = Op::kLight;
};
template <class Op, class = void>
struct OpParams {
  using type = NoParams;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[Op::kIn], float (&out)[Op::kOut], const type&) {
    Op::template apply<kWide>(in, out);
  }
};
template <class Op>
struct OpParams<Op, typename VoidType<typename Op::Params>::type> {
  using type = typename Op::Params;
  template <bool kWide>
  __device__ __forceinline__ static void apply(const float (&in)[Op::kIn], float (&out)[Op::kOut], const type& prm) {
    Op::template apply<kWide>(in, out, prm);
  }
};

static constexpr int kScalarThreads = 256;

// 16-byte vector body.  Requires every pointer 16-byte aligned.  Tile = kThreads * kUnroll
// vectors; block b takes tiles b, b + gridDim.x, ... (the host launches one block per full
// tile, so the hardware dispatcher hands tiles out in address order).  Full tiles run
// unguarded; the one partial tile and the < kVec scalar tail elements are taken by a single
// block.  The kernel uses no LDS: the dynamic LDS size of the launch only limits how many
// blocks fit on a compute unit.
template <class Op, typename T, class Sh>
__global__ __launch_bounds__((Sh::kThreads)) void ew_vec_kernel(Ptrs<Op::kIn, Op::kOut> p, size_t n,
                                                                typename OpParams<Op>::type prm) {
  using S = Storage<T>;
  using Vec = typename S::Vec;
  constexpr int kVec = S::kVec;
  constexpr bool kWide = sizeof(T) == 4;
  constexpr int kThreads = Sh::kThreads;
  constexpr int kUnroll = Sh::kUnroll;
  constexpr bool kNt = Sh::kNtLoad;
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
        OpParams<Op>::template apply<kWide>(fin, fout, prm);
#pragma unroll
        for (int o = 0; o < Op::kOut; ++o) vout[o][e] = S::down(fout[o]);
      }
#pragma unroll
      for (int o = 0; o < Op::kOut; ++o)
        stream_store(reinterpret_cast<Vec*>(p.out[o]) + (base + (size_t)j * kThreads), vout[o]);
      // Keep the vectors apart in the instruction stream: vector j is stored before vector
      // j + 1 is waited for and computed, so stores leave the wave in pairs spread over its
      // compute phase instead of in one burst at the end (measured: forward kernels 1-3 %
      // faster, the others unchanged).
      __builtin_amdgcn_sched_barrier(0);
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
        OpParams<Op>::template apply<kWide>(fin, fout, prm);
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
      OpParams<Op>::template apply<kWide>(fin, fout, prm);
#pragma unroll
      for (int o = 0; o < Op::kOut; ++o) reinterpret_cast<T*>(p.out[o])[k] = S::down(fout[o]);
    }
  }
}

// Element-at-a-time kernel for pointers that are not all 16-byte aligned: same values,
// lower bandwidth.
template <class Op, typename T>
__global__ __launch_bounds__(kScalarThreads) void ew_scalar_kernel(Ptrs<Op::kIn, Op::kOut> p, size_t n,
                                                                   typename OpParams<Op>::type prm) {
  using S = Storage<T>;
  constexpr bool kWide = sizeof(T) == 4;
  const size_t stride = (size_t)gridDim.x * kScalarThreads;
  for (size_t k = (size_t)blockIdx.x * kScalarThreads + threadIdx.x; k < n; k += stride) {
    float fin[Op::kIn], fout[Op::kOut];
#pragma unroll
    for (int i = 0; i < Op::kIn; ++i) fin[i] = S::up(reinterpret_cast<const T*>(p.in[i])[k]);
    OpParams<Op>::template apply<kWide>(fin, fout, prm);
#pragma unroll
    for (int o = 0; o < Op::kOut; ++o) reinterpret_cast<T*>(p.out[o])[k] = S::down(fout[o]);
  }
}

}  // namespace nfad

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

}  // namespace nfad

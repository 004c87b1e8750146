// nfad_sweep.hip -- libnfad_sweep.so, a MEASUREMENT library that is not part of libnfad.
//
// It launches the traffic patterns of the libnfad kernels -- with their real arithmetic or
// with none -- in ANY launch shape: block size, 16-byte accesses in flight per lane, the
// order of a lane's accesses, cache hints, cap on resident waves per compute unit, one
// block per tile or a persistent grid, and the tile -> compute-die mapping are arguments of
// one call.  paper_2209_10778_amd/sweep.py times these launches next to libnfad's own to
// find, per traffic pattern and size, the best shape the part offers (the ceiling a kernel
// is read against) and to record what each design choice of the library is worth.
//
// Patterns with arithmetic are libnfad's own kernel template and operations (nfad_stream_device.hpp,
// nfad_ops.hpp), instantiated for a grid of shapes; patterns without arithmetic use a kernel of
// their own with the whole shape as run-time arguments.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nfad_stream.hpp"
#include "nfad_ops.hpp"

namespace nfad {
namespace sweep {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

template <bool NT, typename V>
__device__ __forceinline__ void store_as(V* p, V v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// Workgroups are dealt round-robin to the 8 compute dies (XCDs), each with its own L2.  With
// chunk = c > 0 die k takes runs of c consecutive tiles (tiles [g*8c + k*c, g*8c + (k+1)*c) of
// every group g of 8c tiles) instead of every eighth tile; tiles beyond the last whole group
// keep the identity mapping.  A bijection on [0, tiles).
__device__ __forceinline__ size_t die_remap(size_t b, size_t tiles, unsigned chunk) {
  if (chunk == 0) return b;
  const size_t group = (size_t)8 * chunk;
  if (b >= (tiles / group) * group) return b;
  const size_t g = b / group, r = b % group;
  return g * group + (r % 8) * chunk + r / 8;
}

struct Geometry {
  size_t nvec;        // 16-byte vectors per tensor
  unsigned adjacent;  // 0: a lane's j-th access is blockDim.x vectors after its (j-1)-th; 1: the next vector
  unsigned chunk;     // die_remap chunk; applied only when the grid has one block per tile
};

// No arithmetic: N_IN tensors read, N_OUT written (XOR of the inputs, complement in out[1];
// an index pattern when nothing is read; a practically-never store when nothing is written).
template <int N_IN, int N_OUT, int U, bool NTL, bool NTS>
__global__ __launch_bounds__(1024) void stream_kernel(const u32x4* in0, const u32x4* in1, u32x4* out0, u32x4* out1,
                                                      Geometry g) {
  const unsigned T = blockDim.x;
  const size_t tile = (size_t)T * U;
  const size_t full = g.nvec / tile;
  const bool remap = g.chunk != 0 && gridDim.x == full;
  u32x4 sink = u32x4{0u, 0u, 0u, 0u};
  for (size_t b = blockIdx.x; b < full; b += gridDim.x) {
    const size_t t = remap ? die_remap(b, full, g.chunk) : b;
    const size_t first = t * tile + (g.adjacent ? (size_t)threadIdx.x * U : (size_t)threadIdx.x);
    const size_t step = g.adjacent ? 1 : T;
    u32x4 v[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const size_t idx = first + (size_t)j * step;
      if constexpr (N_IN == 0) {
        const unsigned h = (unsigned)idx * 2654435761u;
        v[j] = u32x4{h, h ^ 0x9e3779b9u, h * 31u, ~h};
      } else {
        v[j] = stream_load<NTL>(in0 + idx);
        if constexpr (N_IN > 1) v[j] ^= stream_load<NTL>(in1 + idx);
      }
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const size_t idx = first + (size_t)j * step;
      if constexpr (N_OUT > 0) store_as<NTS>(out0 + idx, v[j]);
      if constexpr (N_OUT > 1) store_as<NTS>(out1 + idx, ~v[j]);
      if constexpr (N_OUT == 0) sink ^= v[j];
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  if (blockIdx.x == full % gridDim.x) {   // ragged end, one block
    for (size_t idx = full * tile + threadIdx.x; idx < g.nvec; idx += T) {
      u32x4 w;
      if constexpr (N_IN == 0) {
        const unsigned h = (unsigned)idx * 2654435761u;
        w = u32x4{h, h ^ 0x9e3779b9u, h * 31u, ~h};
      } else {
        w = in0[idx];
        if constexpr (N_IN > 1) w ^= in1[idx];
      }
      if constexpr (N_OUT > 0) out0[idx] = w;
      if constexpr (N_OUT > 1) out1[idx] = ~w;
      if constexpr (N_OUT == 0) sink ^= w;
    }
  }
  if constexpr (N_OUT == 0) {   // keep the loads alive: a 16-byte write that practically never happens
    if (sink.x == 0x7fc12345u && sink.y == 0x7fc54321u && sink.z == 0x12345678u && sink.w == 0x87654321u)
      out0[0] = sink;
  }
}

struct Launch {
  unsigned grid, threads, lds;
  hipStream_t stream;
};

// ------------------------------------------------------------------ phased traffic (experiment)
// Pure read streams and pure write streams both run faster on this part than any mix of the
// two (the DRAM bus pays for every change of direction).  The kernels below separate reads
// from writes IN TIME across the whole chip without any communication: every wave reads the
// chip-wide constant-rate clock and issues loads only while (clock mod period) < read_ticks
// and stores only during the rest of the period.  One wave64 per block, a persistent grid;
// per period each wave loads one chunk of U 16-byte vectors per lane and tensor, holds it in
// registers, and stores the results in the write phase.  period == 0 switches the waiting off
// (a plain persistent big-chunk kernel).  Every wait is bounded: after kMaxSpins polls a wave
// proceeds regardless, so the grid always drains.
struct Phase {
  unsigned period;      // clock ticks (10 ns each); 0 = no phasing
  unsigned read_ticks;  // loads are issued while (clock % period) < read_ticks, stores otherwise
};
static constexpr int kMaxSpins = 4096;
__device__ __forceinline__ void wait_for(bool want_read, Phase ph) {
  if (ph.period == 0) return;
  for (int spin = 0; spin < kMaxSpins; ++spin) {
    const unsigned t = (unsigned)__builtin_amdgcn_s_memrealtime() % ph.period;
    if ((t < ph.read_ticks) == want_read) return;
    __builtin_amdgcn_s_sleep(2);
  }
}

template <class Op, typename T, int U, bool NTL>
__global__ __launch_bounds__(64) void phased_op_kernel(Ptrs<Op::kIn, Op::kOut> p, size_t nvec, Phase ph) {
  using S = Storage<T>;
  using Vec = typename S::Vec;
  constexpr int kVec = S::kVec;
  constexpr bool kWide = sizeof(T) == 4;
  constexpr size_t kTile = (size_t)64 * U;
  const size_t full = nvec / kTile;
  for (size_t t = blockIdx.x; t < full; t += gridDim.x) {
    const size_t first = t * kTile + threadIdx.x;
    Vec vin[U][Op::kIn];
    wait_for(true, ph);
#pragma unroll
    for (int j = 0; j < U; ++j)
#pragma unroll
      for (int i = 0; i < Op::kIn; ++i)
        vin[j][i] = stream_load<NTL>(reinterpret_cast<const Vec*>(p.in[i]) + (first + (size_t)j * 64));
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    wait_for(false, ph);
#pragma unroll
    for (int j = 0; j < U; ++j) {
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
        stream_store(reinterpret_cast<Vec*>(p.out[o]) + (first + (size_t)j * 64), vout[o]);
    }
  }
  if (blockIdx.x == full % gridDim.x) {   // ragged end, one wave, unphased
    for (size_t idx = full * kTile + threadIdx.x; idx < nvec; idx += 64) {
      Vec vout[Op::kOut];
#pragma unroll
      for (int e = 0; e < kVec; ++e) {
        float fin[Op::kIn], fout[Op::kOut];
#pragma unroll
        for (int i = 0; i < Op::kIn; ++i) fin[i] = S::up(reinterpret_cast<const Vec*>(p.in[i])[idx][e]);
        Op::template apply<kWide>(fin, fout);
#pragma unroll
        for (int o = 0; o < Op::kOut; ++o) vout[o][e] = S::down(fout[o]);
      }
#pragma unroll
      for (int o = 0; o < Op::kOut; ++o) reinterpret_cast<Vec*>(p.out[o])[idx] = vout[o];
    }
  }
}

template <class Op, typename T>
static hipError_t launch_phased_t(int unroll, bool ntl, const void* const* in, void* const* out, size_t nvec,
                                  Phase ph, unsigned grid, unsigned lds, hipStream_t stream) {
  Ptrs<Op::kIn, Op::kOut> p;
  for (int i = 0; i < Op::kIn; ++i) p.in[i] = in[i];
  for (int o = 0; o < Op::kOut; ++o) p.out[o] = out[o];
#define NFAD_SWEEP_GO(U)                                                                                             \
  do {                                                                                                               \
    if (ntl) hipLaunchKernelGGL((phased_op_kernel<Op, T, U, true>), dim3(grid), dim3(64), lds, stream, p, nvec, ph);  \
    else hipLaunchKernelGGL((phased_op_kernel<Op, T, U, false>), dim3(grid), dim3(64), lds, stream, p, nvec, ph);     \
  } while (0)
  switch (unroll) {
    case 2: NFAD_SWEEP_GO(2); break;
    case 4: NFAD_SWEEP_GO(4); break;
    case 8: NFAD_SWEEP_GO(8); break;
    case 16: NFAD_SWEEP_GO(16); break;
    default: return hipErrorInvalidValue;
  }
#undef NFAD_SWEEP_GO
  return hipGetLastError();
}
template <class Op>
static hipError_t launch_phased(int dtype, int unroll, bool ntl, const void* const* in, void* const* out, size_t nvec,
                                Phase ph, unsigned grid, unsigned lds, hipStream_t stream) {
  switch (dtype) {
    case NFAD_F32: return launch_phased_t<Op, float>(unroll, ntl, in, out, nvec, ph, grid, lds, stream);
    case NFAD_BF16: return launch_phased_t<Op, __bf16>(unroll, ntl, in, out, nvec, ph, grid, lds, stream);
  }
  return hipErrorInvalidValue;
}

template <int N_IN, int N_OUT, int U>
static hipError_t launch_stream_u(bool ntl, bool nts, const void* const* in, void* const* out, Geometry g, Launch l) {
  const u32x4* i0 = N_IN > 0 ? static_cast<const u32x4*>(in[0]) : nullptr;
  const u32x4* i1 = N_IN > 1 ? static_cast<const u32x4*>(in[1]) : nullptr;
  u32x4* o0 = static_cast<u32x4*>(out[0]);
  u32x4* o1 = N_OUT > 1 ? static_cast<u32x4*>(out[1]) : nullptr;
#define NFAD_SWEEP_GO(L, S) \
  hipLaunchKernelGGL((stream_kernel<N_IN, N_OUT, U, L, S>), dim3(l.grid), dim3(l.threads), l.lds, l.stream, i0, i1, o0, o1, g)
  if (ntl && nts) NFAD_SWEEP_GO(true, true);
  else if (ntl) NFAD_SWEEP_GO(true, false);
  else if (nts) NFAD_SWEEP_GO(false, true);
  else NFAD_SWEEP_GO(false, false);
#undef NFAD_SWEEP_GO
  return hipGetLastError();
}
template <int N_IN, int N_OUT>
static hipError_t launch_stream(int unroll, bool ntl, bool nts, const void* const* in, void* const* out, Geometry g,
                                Launch l) {
  switch (unroll) {
    case 1: return launch_stream_u<N_IN, N_OUT, 1>(ntl, nts, in, out, g, l);
    case 2: return launch_stream_u<N_IN, N_OUT, 2>(ntl, nts, in, out, g, l);
    case 4: return launch_stream_u<N_IN, N_OUT, 4>(ntl, nts, in, out, g, l);
    case 8: return launch_stream_u<N_IN, N_OUT, 8>(ntl, nts, in, out, g, l);
  }
  return hipErrorInvalidValue;
}

// libnfad's own kernel template (nfad_stream_device.hpp) with libnfad's arithmetic, instantiated
// for a grid of compile-time shapes: block size x unroll x load hint.  The cap on resident waves
// and the grid (one block per tile, or fewer blocks striding) stay run-time arguments.
template <class Op, typename T, int THREADS, int UNROLL>
static hipError_t launch_op_tu(bool ntl, const Ptrs<Op::kIn, Op::kOut>& p, size_t n, Launch l) {
  if (ntl)
    hipLaunchKernelGGL((ew_vec_kernel<Op, T, Shape<THREADS, UNROLL, true>>), dim3(l.grid), dim3(THREADS), l.lds,
                       l.stream, p, n, NoParams{});
  else
    hipLaunchKernelGGL((ew_vec_kernel<Op, T, Shape<THREADS, UNROLL, false>>), dim3(l.grid), dim3(THREADS), l.lds,
                       l.stream, p, n, NoParams{});
  return hipGetLastError();
}
template <class Op, typename T>
static hipError_t launch_op_t(int unroll, bool ntl, const void* const* in, void* const* out, size_t n, Launch l) {
  Ptrs<Op::kIn, Op::kOut> p;
  for (int i = 0; i < Op::kIn; ++i) p.in[i] = in[i];
  for (int o = 0; o < Op::kOut; ++o) p.out[o] = out[o];
  switch (l.threads * 16 + unroll) {
#define NFAD_SWEEP_CASE(TH, U) case TH * 16 + U: return launch_op_tu<Op, T, TH, U>(ntl, p, n, l)
    NFAD_SWEEP_CASE(64, 1); NFAD_SWEEP_CASE(64, 2); NFAD_SWEEP_CASE(64, 4);
    NFAD_SWEEP_CASE(128, 1); NFAD_SWEEP_CASE(128, 2); NFAD_SWEEP_CASE(128, 4);
    NFAD_SWEEP_CASE(256, 1); NFAD_SWEEP_CASE(256, 2); NFAD_SWEEP_CASE(256, 4);
    NFAD_SWEEP_CASE(512, 1); NFAD_SWEEP_CASE(512, 2); NFAD_SWEEP_CASE(512, 4);
#undef NFAD_SWEEP_CASE
  }
  return hipErrorInvalidValue;
}
template <class Op>
static hipError_t launch_op(int dtype, int unroll, bool ntl, const void* const* in, void* const* out, size_t n,
                            Launch l) {
  switch (dtype) {
    case NFAD_F32: return launch_op_t<Op, float>(unroll, ntl, in, out, n, l);
    case NFAD_BF16: return launch_op_t<Op, __bf16>(unroll, ntl, in, out, n, l);
  }
  return hipErrorInvalidValue;   // fp16 storage behaves as bf16 does and is not instantiated here
}

}  // namespace sweep
}  // namespace nfad

// ------------------------------------------------------------------ residency probe
// How many blocks with a given idle LDS reservation the hardware keeps resident per compute unit:
// every block waits `ticks` ticks of the constant 100 MHz clock (bounded: at most kProbeSpins
// polls, so the grid always drains) and then writes its index.  With R blocks resident per
// compute unit a grid of G blocks takes ceil(G / (CUs * R)) * ticks.
namespace nfad {
namespace sweep {
static constexpr int kProbeSpins = 1 << 16;
__global__ __launch_bounds__(1024) void residency_probe_kernel(unsigned ticks, unsigned* out) {
  const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
  for (int spin = 0; spin < kProbeSpins; ++spin) {
    if (__builtin_amdgcn_s_memrealtime() - t0 >= ticks) break;
    __builtin_amdgcn_s_sleep(8);
  }
  if (threadIdx.x == 0) out[blockIdx.x] = blockIdx.x;
}
}  // namespace sweep
}  // namespace nfad

using namespace nfad;

extern "C" {

// Patterns.  0..6: no arithmetic, (reads, writes) = (1,2) (2,1) (1,1) (1,0) (0,1) (0,2) (2,0).
// 10..13: nfad_fwd's arithmetic for kind 0..3 (in: x; out: y, dydx).  20: nfad_bwd's (in: gy, dydx; out: gx).
// 30..33: nfad_recompute_fwd's for kind 0..3 (in: x; out: y).
enum {
  NFAD_SWEEP_R1W2 = 0, NFAD_SWEEP_R2W1 = 1, NFAD_SWEEP_R1W1 = 2, NFAD_SWEEP_R1W0 = 3, NFAD_SWEEP_R0W1 = 4,
  NFAD_SWEEP_R0W2 = 5, NFAD_SWEEP_R2W0 = 6, NFAD_SWEEP_FWD = 10, NFAD_SWEEP_BWD = 20, NFAD_SWEEP_RECOMPUTE_FWD = 30
};

// One launch of `pattern` over n elements of `dtype` per tensor (n a multiple of 16 / element size;
// every pointer 16-byte aligned; device pointers in the host arrays `in` and `out`; a pattern
// without output still needs out[0] -> 16 writable bytes).  Shape arguments:
//   threads       block size, a multiple of 64 up to 1024 (arithmetic patterns: 64, 128, 256 or 512)
//   unroll        1, 2, 4 or 8 16-byte accesses in flight per lane and tensor (arithmetic: 1, 2 or 4)
//   adjacent      (patterns without arithmetic only) 0: a lane's accesses are `threads` vectors apart (each wave instruction covers 1 KiB
//                 contiguous); 1: they are consecutive (each lane owns unroll*16 contiguous bytes)
//   nt_load/store nontemporal hint on loads / stores (the arithmetic patterns always store nontemporal)
//   waves_per_cu  cap on resident waves per compute unit through an idle LDS reservation; <= 0: none
//   max_grid      0: one block per tile; > 0: at most that many blocks, each striding over the tiles
//   die_chunk     (patterns without arithmetic only) 0: identity tile order; c > 0: each compute die takes runs of c consecutive tiles
// Returns an nfad_status_t.  Asynchronous on `stream`, capturable.
int nfad_sweep_launch(int pattern, int dtype, int threads, int unroll, int adjacent, int nt_load, int nt_store,
                      int waves_per_cu, long long max_grid, int die_chunk, const void* const* in, void* const* out,
                      size_t n, void* stream) {
  if (!dtype_ok(dtype)) return NFAD_EINVAL_DTYPE;
  if (threads < 64 || threads > 1024 || threads % 64) return NFAD_EINVAL_KIND;
  if (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8) return NFAD_EINVAL_KIND;
  if (max_grid < 0 || die_chunk < 0 || !out) return NFAD_EINVAL_KIND;
  int n_in = 0, n_out = 0;
  switch (pattern) {
    case NFAD_SWEEP_R1W2: n_in = 1; n_out = 2; break;
    case NFAD_SWEEP_R2W1: n_in = 2; n_out = 1; break;
    case NFAD_SWEEP_R1W1: n_in = 1; n_out = 1; break;
    case NFAD_SWEEP_R1W0: n_in = 1; n_out = 0; break;
    case NFAD_SWEEP_R0W1: n_in = 0; n_out = 1; break;
    case NFAD_SWEEP_R0W2: n_in = 0; n_out = 2; break;
    case NFAD_SWEEP_R2W0: n_in = 2; n_out = 0; break;
    case NFAD_SWEEP_FWD: case NFAD_SWEEP_FWD + 1: case NFAD_SWEEP_FWD + 2: case NFAD_SWEEP_FWD + 3:
      n_in = 1; n_out = 2; break;
    case NFAD_SWEEP_BWD: n_in = 2; n_out = 1; break;
    case NFAD_SWEEP_RECOMPUTE_FWD: case NFAD_SWEEP_RECOMPUTE_FWD + 1: case NFAD_SWEEP_RECOMPUTE_FWD + 2:
    case NFAD_SWEEP_RECOMPUTE_FWD + 3:
      n_in = 1; n_out = 1; break;
    default: return NFAD_EINVAL_KIND;
  }
  if (n_in > 0 && !in) return NFAD_ENULL;
  for (int i = 0; i < n_in; ++i) {
    if (!in[i]) return NFAD_ENULL;
    if ((uintptr_t)in[i] & 15u) return NFAD_EALIGN;
  }
  for (int o = 0; o < (n_out > 0 ? n_out : 1); ++o) {
    if (!out[o]) return NFAD_ENULL;
    if ((uintptr_t)out[o] & 15u) return NFAD_EALIGN;
  }
  const size_t per_vec = 16 / elem_size(dtype);
  if (n % per_vec) return NFAD_EALIGN;
  if (n == 0) return NFAD_OK;
  sweep::Geometry g = {n / per_vec, adjacent ? 1u : 0u, (unsigned)die_chunk};
  const size_t tile = (size_t)threads * unroll;
  size_t grid = g.nvec / tile;
  if (grid == 0) grid = 1;
  if (max_grid > 0 && grid > (size_t)max_grid) grid = (size_t)max_grid;
  if (grid > ((size_t)1 << 24)) return NFAD_ELAUNCH;
  const sweep::Launch l = {(unsigned)grid, (unsigned)threads,
                           waves_per_cu > 0 ? lds_reservation(waves_per_cu, threads, device_info().lds_per_cu) : 0u,
                           static_cast<hipStream_t>(stream)};
  const bool ntl = nt_load != 0, nts = nt_store != 0;
  if (pattern >= NFAD_SWEEP_FWD && (adjacent || die_chunk)) return NFAD_EINVAL_KIND;   // stream patterns only
  hipError_t e = hipErrorInvalidValue;
  switch (pattern) {
    case NFAD_SWEEP_R1W2: e = sweep::launch_stream<1, 2>(unroll, ntl, nts, in, out, g, l); break;
    case NFAD_SWEEP_R2W1: e = sweep::launch_stream<2, 1>(unroll, ntl, nts, in, out, g, l); break;
    case NFAD_SWEEP_R1W1: e = sweep::launch_stream<1, 1>(unroll, ntl, nts, in, out, g, l); break;
    case NFAD_SWEEP_R1W0: e = sweep::launch_stream<1, 0>(unroll, ntl, nts, in, out, g, l); break;
    case NFAD_SWEEP_R0W1: e = sweep::launch_stream<0, 1>(unroll, ntl, nts, in, out, g, l); break;
    case NFAD_SWEEP_R0W2: e = sweep::launch_stream<0, 2>(unroll, ntl, nts, in, out, g, l); break;
    case NFAD_SWEEP_R2W0: e = sweep::launch_stream<2, 0>(unroll, ntl, nts, in, out, g, l); break;
    case NFAD_SWEEP_FWD + 0: e = sweep::launch_op<FwdOp<kGeluTanh>>(dtype, unroll, ntl, in, out, n, l); break;
    case NFAD_SWEEP_FWD + 1: e = sweep::launch_op<FwdOp<kGeluErf>>(dtype, unroll, ntl, in, out, n, l); break;
    case NFAD_SWEEP_FWD + 2: e = sweep::launch_op<FwdOp<kSwish>>(dtype, unroll, ntl, in, out, n, l); break;
    case NFAD_SWEEP_FWD + 3: e = sweep::launch_op<FwdOp<kMish>>(dtype, unroll, ntl, in, out, n, l); break;
    case NFAD_SWEEP_BWD: e = sweep::launch_op<BwdOp>(dtype, unroll, ntl, in, out, n, l); break;
    case NFAD_SWEEP_RECOMPUTE_FWD + 0: e = sweep::launch_op<RecomputeFwdOp<kGeluTanh>>(dtype, unroll, ntl, in, out, n, l); break;
    case NFAD_SWEEP_RECOMPUTE_FWD + 1: e = sweep::launch_op<RecomputeFwdOp<kGeluErf>>(dtype, unroll, ntl, in, out, n, l); break;
    case NFAD_SWEEP_RECOMPUTE_FWD + 2: e = sweep::launch_op<RecomputeFwdOp<kSwish>>(dtype, unroll, ntl, in, out, n, l); break;
    case NFAD_SWEEP_RECOMPUTE_FWD + 3: e = sweep::launch_op<RecomputeFwdOp<kMish>>(dtype, unroll, ntl, in, out, n, l); break;
  }
  return e == hipSuccess ? NFAD_OK : NFAD_ELAUNCH;
}

// Phased variant (see "phased traffic" above) of the arithmetic patterns NFAD_SWEEP_FWD + kind and
// NFAD_SWEEP_BWD, fp32 or bf16 storage: a persistent grid of waves_per_cu one-wave blocks per
// compute unit (persistent != 0), or one one-wave block per tile with at most waves_per_cu of them
// resident per compute unit (persistent == 0); unroll (2, 4, 8 or 16) 16-byte vectors per lane and tensor per period; loads are
// issued in the first read_ticks of every period of `period_ticks` 10 ns clock ticks, stores in
// the rest; period_ticks == 0 disables the waiting.  Other arguments as nfad_sweep_launch.
int nfad_sweep_launch_phased(int pattern, int dtype, int unroll, int nt_load, int waves_per_cu, int persistent,
                             int period_ticks, int read_ticks, const void* const* in, void* const* out, size_t n,
                             void* stream) {
  if (dtype != NFAD_F32 && dtype != NFAD_BF16) return NFAD_EINVAL_DTYPE;
  if (waves_per_cu < 1 || waves_per_cu > 32 || period_ticks < 0 || read_ticks < 0 || read_ticks > period_ticks)
    return NFAD_EINVAL_KIND;
  int n_in = 0, n_out = 0;
  if (pattern >= NFAD_SWEEP_FWD && pattern < NFAD_SWEEP_FWD + 4) { n_in = 1; n_out = 2; }
  else if (pattern == NFAD_SWEEP_BWD) { n_in = 2; n_out = 1; }
  else return NFAD_EINVAL_KIND;
  if (!in || !out) return NFAD_ENULL;
  for (int i = 0; i < n_in; ++i) {
    if (!in[i]) return NFAD_ENULL;
    if ((uintptr_t)in[i] & 15u) return NFAD_EALIGN;
  }
  for (int o = 0; o < n_out; ++o) {
    if (!out[o]) return NFAD_ENULL;
    if ((uintptr_t)out[o] & 15u) return NFAD_EALIGN;
  }
  const size_t per_vec = 16 / elem_size(dtype);
  if (n % per_vec) return NFAD_EALIGN;
  if (n == 0) return NFAD_OK;
  const size_t nvec = n / per_vec;
  const DeviceInfo di = device_info();
  const size_t tiles = nvec / ((size_t)64 * unroll);
  size_t grid = persistent ? (size_t)di.cus * waves_per_cu : tiles;   // else one block per tile, each waiting for its phases
  if (grid > tiles) grid = tiles;
  if (grid == 0) grid = 1;
  if (grid > ((size_t)1 << 24)) return NFAD_ELAUNCH;
  const unsigned lds = lds_reservation(waves_per_cu, 64, di.lds_per_cu);
  const sweep::Phase ph = {(unsigned)period_ticks, (unsigned)read_ticks};
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool ntl = nt_load != 0;
  hipError_t e = hipErrorInvalidValue;
  switch (pattern) {
    case NFAD_SWEEP_FWD + 0: e = sweep::launch_phased<FwdOp<kGeluTanh>>(dtype, unroll, ntl, in, out, nvec, ph, (unsigned)grid, lds, st); break;
    case NFAD_SWEEP_FWD + 1: e = sweep::launch_phased<FwdOp<kGeluErf>>(dtype, unroll, ntl, in, out, nvec, ph, (unsigned)grid, lds, st); break;
    case NFAD_SWEEP_FWD + 2: e = sweep::launch_phased<FwdOp<kSwish>>(dtype, unroll, ntl, in, out, nvec, ph, (unsigned)grid, lds, st); break;
    case NFAD_SWEEP_FWD + 3: e = sweep::launch_phased<FwdOp<kMish>>(dtype, unroll, ntl, in, out, nvec, ph, (unsigned)grid, lds, st); break;
    case NFAD_SWEEP_BWD: e = sweep::launch_phased<BwdOp>(dtype, unroll, ntl, in, out, nvec, ph, (unsigned)grid, lds, st); break;
  }
  return e == hipSuccess ? NFAD_OK : NFAD_ELAUNCH;
}

// Residency probe: `grid` blocks of `threads` threads (a multiple of 64, at most 1024), each with
// `lds_bytes` of dynamic LDS (at most 64 KiB) it never touches, each waiting `ticks` (at most
// 100000 = 1 ms) ticks of the 100 MHz clock before it writes its index to out[block] (device
// memory, grid * 4 bytes).  The launch's duration tells how many blocks were resident at a time.
int nfad_sweep_residency(int threads, unsigned lds_bytes, unsigned grid, unsigned ticks, void* out, void* stream) {
  if (threads < 64 || threads > 1024 || threads % 64 || lds_bytes > 64u * 1024u || grid == 0 || grid > (1u << 24) ||
      ticks > 100000u)
    return NFAD_EINVAL_KIND;
  if (!out) return NFAD_ENULL;
  if ((uintptr_t)out & 3u) return NFAD_EALIGN;
  hipLaunchKernelGGL(sweep::residency_probe_kernel, dim3(grid), dim3((unsigned)threads), lds_bytes,
                     static_cast<hipStream_t>(stream), ticks, static_cast<unsigned*>(out));
  return hipGetLastError() == hipSuccess ? NFAD_OK : NFAD_ELAUNCH;
}

// The idle LDS reservation libnfad's launcher makes for a cap of waves_per_cu resident waves with
// blocks of `threads` threads on the current device (0 = no reservation).
unsigned nfad_sweep_lds_for_cap(int waves_per_cu, int threads) {
  if (threads < 64 || threads > 1024 || threads % 64) return 0;
  return lds_reservation(waves_per_cu, threads, device_info().lds_per_cu);
}

}  // extern "C"

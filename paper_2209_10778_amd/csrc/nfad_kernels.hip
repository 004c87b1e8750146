// nfad_kernels.hip -- the C ABI of libnfad (include/nfad.h) for the method and its two
// baselines.  The per-element operations are in nfad_ops.hpp, the streaming kernel skeleton
// and the launch code in nfad_stream.hpp, the arithmetic of the activations in nfad_math.hpp.
#include "nfad_stream.hpp"
#include "nfad_ops.hpp"

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

int nfad_version(void) { return 200; }

}  // extern "C"

/* nfad_c_check.c -- the C ABI of libnfad exercised from a plain C99 program: no Python, no
 * PyTorch.  Device memory comes from the HIP runtime's C API; expected values come from the
 * fp64 CPU oracle (linked as a library; this program is test infrastructure).
 *
 * For each activation (Table I of the paper + the erf form of GELU) and each storage type
 * that C can hold natively (fp32), on n seeded pseudo-random inputs with a ragged n:
 *   fused forward   y = f(x), dydx = f'(x)           (Sec. II-C eq. 3)
 *   backward        gx = gy * dydx                    (Sec. II-C eq. 4)
 *   recomputation and save-all baselines
 * every result against max(2e-6, one fp32 ulp of the reference) -- with |x| <= 6 that is the flat
 * 2e-6 wherever the reference is below 16 -- plus the error paths that need no launch.
 * Backward passes consume the ORACLE's forward results rounded to fp32 (uploaded from the host),
 * on the GPU and in the oracle alike: no oracle input comes from the GPU.
 * Exit status 0 = all checks passed. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "nfad.h"

/* the oracle's C entry points (oracle/nfad_oracle.c) */
int nfad_oracle_fwd(int kind, const double* x, double* y, double* dydx, size_t n, int threads);
int nfad_oracle_bwd(const double* gy, const double* dydx, double* gx, size_t n, int threads);
int nfad_oracle_recompute_fwd(int kind, const double* x, double* y, size_t n, int threads);
int nfad_oracle_recompute_bwd(int kind, const double* gy, const double* x, double* gx, size_t n, int threads);
int nfad_oracle_num_saved(int kind);
int nfad_oracle_saveall_fwd(int kind, const double* x, double* y, double* const* saved, size_t n, int threads);
int nfad_oracle_saveall_bwd(int kind, const double* gy, const double* const* saved, double* gx, size_t n, int threads);

#define HIP_OK(call)                                                              \
  do {                                                                            \
    hipError_t e_ = (call);                                                       \
    if (e_ != hipSuccess) {                                                       \
      fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_)); \
      exit(2);                                                                    \
    }                                                                             \
  } while (0)
#define NFAD_OK_(call)                                                                      \
  do {                                                                                      \
    int s_ = (call);                                                                        \
    if (s_ != NFAD_OK) {                                                                    \
      fprintf(stderr, "%s:%d: status %d (%s)\n", __FILE__, __LINE__, s_, nfad_status_string(s_)); \
      exit(2);                                                                              \
    }                                                                                       \
  } while (0)

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static double uniform01(void) { /* splitmix64 */
  uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  return (double)(z >> 11) / 9007199254740992.0;
}

static int g_failures = 0;
/* |got - ref| <= max(2e-6, ulp_f32(ref)) + allowance[i] (allowance may be NULL) */
static void check(const char* what, int kind, const float* got, const double* ref, size_t n, const double* allowance) {
  double worst = 0.0, worst_over_bar = 0.0;
  size_t at = 0, bad = 0;
  for (size_t i = 0; i < n; ++i) {
    const double err = fabs((double)got[i] - ref[i]);
    int e;
    frexp(ref[i], &e);
    const double ulp = ldexp(1.0, (e - 1 < -126 ? -126 : e - 1) - 23);
    const double bar = ulp > 2e-6 ? ulp : 2e-6;
    if (!(err <= bar + (allowance ? allowance[i] : 0.0))) ++bad;
    if (err > worst || err != err) { worst = err; at = i; }
    if (err / bar > worst_over_bar) worst_over_bar = err / bar;
  }
  printf("  %-22s kind %d  max |err| %.3e at %zu (%.3f of the bar)  %s\n", what, kind, worst, at, worst_over_bar,
         bad ? "FAIL" : "ok");
  if (bad) ++g_failures;
}

int main(void) {
  const size_t n = 3 * 8192 + 5 * 256 + 77 + 3; /* several tiles, a partial tile, a scalar tail */
  const size_t bytes = n * sizeof(float);
  int ndev = 0;
  HIP_OK(hipGetDeviceCount(&ndev));
  if (ndev < 1) { fprintf(stderr, "no GPU\n"); return 2; }
  HIP_OK(hipSetDevice(0));
  printf("libnfad version %d, %d device(s)\n", nfad_version(), ndev);

  float* hx = malloc(bytes); float* hgy = malloc(bytes); float* hout = malloc(bytes); float* hout2 = malloc(bytes);
  double* x64 = malloc(n * 8); double* gy64 = malloc(n * 8); double* y64 = malloc(n * 8);
  double* d64 = malloc(n * 8); double* gx64 = malloc(n * 8); double* dst64 = malloc(n * 8);
  double* sv64[NFAD_MAX_SAVED];
  for (int j = 0; j < NFAD_MAX_SAVED; ++j) sv64[j] = malloc(n * 8);
  for (size_t i = 0; i < n; ++i) {
    hx[i] = (float)(12.0 * uniform01() - 6.0);
    hgy[i] = (float)(2.0 * uniform01() - 1.0);
    x64[i] = hx[i];
    gy64[i] = hgy[i];
  }
  void *dx, *dgy, *dy, *dd, *dgx, *dsv[NFAD_MAX_SAVED];
  HIP_OK(hipMalloc(&dx, bytes)); HIP_OK(hipMalloc(&dgy, bytes)); HIP_OK(hipMalloc(&dy, bytes));
  HIP_OK(hipMalloc(&dd, bytes)); HIP_OK(hipMalloc(&dgx, bytes));
  for (int j = 0; j < NFAD_MAX_SAVED; ++j) HIP_OK(hipMalloc(&dsv[j], bytes));
  HIP_OK(hipMemcpy(dx, hx, bytes, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dgy, hgy, bytes, hipMemcpyHostToDevice));
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));

  for (int kind = 0; kind < 4; ++kind) {
    /* the method: fused forward; then backward on the ORACLE's tangent rounded to fp32 */
    NFAD_OK_(nfad_fwd(kind, dx, dy, dd, n, NFAD_F32, stream));
    HIP_OK(hipStreamSynchronize(stream));
    nfad_oracle_fwd(kind, x64, y64, d64, n, 1);
    HIP_OK(hipMemcpy(hout, dy, bytes, hipMemcpyDeviceToHost));
    check("nfad_fwd y", kind, hout, y64, n, NULL);
    HIP_OK(hipMemcpy(hout, dd, bytes, hipMemcpyDeviceToHost));
    check("nfad_fwd dydx", kind, hout, d64, n, NULL);
    for (size_t i = 0; i < n; ++i) { hout2[i] = (float)d64[i]; dst64[i] = hout2[i]; } /* stored tangent of record */
    HIP_OK(hipMemcpy(dd, hout2, bytes, hipMemcpyHostToDevice));
    NFAD_OK_(nfad_bwd(dgy, dd, dgx, n, NFAD_F32, stream));
    HIP_OK(hipStreamSynchronize(stream));
    nfad_oracle_bwd(gy64, dst64, gx64, n, 1);
    HIP_OK(hipMemcpy(hout2, dgx, bytes, hipMemcpyDeviceToHost));
    check("nfad_bwd gx", kind, hout2, gx64, n, NULL);

    /* recomputation baseline */
    NFAD_OK_(nfad_recompute_fwd(kind, dx, dy, n, NFAD_F32, stream));
    NFAD_OK_(nfad_recompute_bwd(kind, dgy, dx, dgx, n, NFAD_F32, stream));
    HIP_OK(hipStreamSynchronize(stream));
    nfad_oracle_recompute_fwd(kind, x64, y64, n, 1);
    nfad_oracle_recompute_bwd(kind, gy64, x64, gx64, n, 1);
    HIP_OK(hipMemcpy(hout, dy, bytes, hipMemcpyDeviceToHost));
    check("recompute_fwd y", kind, hout, y64, n, NULL);
    HIP_OK(hipMemcpy(hout, dgx, bytes, hipMemcpyDeviceToHost));
    check("recompute_bwd gx", kind, hout, gx64, n, NULL);

    /* save-all baseline: the library and the oracle must agree on the number of saved tensors */
    const int k = nfad_saveall_num_saved(kind);
    if (k != nfad_oracle_num_saved(kind) || k < 1 || k > NFAD_MAX_SAVED) {
      printf("  saved-tensor count mismatch for kind %d: %d\n", kind, k);
      ++g_failures;
      continue;
    }
    void* saved[NFAD_MAX_SAVED];
    saved[0] = dx; /* stands for x, not written */
    for (int j = 1; j < k; ++j) saved[j] = dsv[j];
    NFAD_OK_(nfad_saveall_fwd(kind, dx, dy, saved, n, NFAD_F32, stream));
    HIP_OK(hipStreamSynchronize(stream));
    nfad_oracle_saveall_fwd(kind, x64, y64, sv64, n, 1);
    HIP_OK(hipMemcpy(hout, dy, bytes, hipMemcpyDeviceToHost));
    check("saveall_fwd y", kind, hout, y64, n, NULL);
    for (int j = 1; j < k; ++j) {
      char what[32];
      snprintf(what, sizeof what, "saveall_fwd saved[%d]", j);
      HIP_OK(hipMemcpy(hout, dsv[j], bytes, hipMemcpyDeviceToHost));
      check(what, kind, hout, sv64[j], n, NULL);
      /* backward reads the ORACLE's intermediates rounded to fp32, on both sides */
      for (size_t i = 0; i < n; ++i) { hout[i] = (float)sv64[j][i]; sv64[j][i] = hout[i]; }
      HIP_OK(hipMemcpy(dsv[j], hout, bytes, hipMemcpyHostToDevice));
    }
    memcpy(sv64[0], x64, n * 8);
    NFAD_OK_(nfad_saveall_bwd(kind, dgy, (const void* const*)saved, dgx, n, NFAD_F32, stream));
    HIP_OK(hipStreamSynchronize(stream));
    nfad_oracle_saveall_bwd(kind, gy64, (const double* const*)sv64, gx64, n, 1);
    HIP_OK(hipMemcpy(hout, dgx, bytes, hipMemcpyDeviceToHost));
    check("saveall_bwd gx", kind, hout, gx64, n, NULL);
  }

  /* error paths: validation happens before any launch */
  if (nfad_fwd(7, dx, dy, dd, n, NFAD_F32, stream) != NFAD_EINVAL_KIND) { puts("  bad kind accepted"); ++g_failures; }
  if (nfad_fwd(0, dx, dy, dd, n, 9, stream) != NFAD_EINVAL_DTYPE) { puts("  bad dtype accepted"); ++g_failures; }
  if (nfad_fwd(0, NULL, dy, dd, n, NFAD_F32, stream) != NFAD_ENULL) { puts("  null x accepted"); ++g_failures; }
  if (nfad_fwd(0, dx, dy, dy, n, NFAD_F32, stream) != NFAD_EALIAS) { puts("  dydx == y accepted"); ++g_failures; }
  if (nfad_fwd(0, NULL, NULL, NULL, 0, NFAD_F32, stream) != NFAD_OK) { puts("  n == 0 rejected"); ++g_failures; }

  /* a chain compiled at run time, from C */
  int id = -1;
  NFAD_OK_(nfad_chain_compile("x x softplus tanh *", &id));
  NFAD_OK_(nfad_chain_fwd(id, dx, dy, dd, n, NFAD_F32, stream));
  HIP_OK(hipStreamSynchronize(stream));
  nfad_oracle_fwd(NFAD_MISH, x64, y64, d64, n, 1);
  /* a composed chain: the bar plus 5e-7 * max(1,|x|) * max(1,|ref|) (a dozen fp32 primitives) */
  double* allow = malloc(n * 8);
  for (size_t i = 0; i < n; ++i) allow[i] = 5e-7 * fmax(1.0, fabs(x64[i])) * fmax(1.0, fabs(y64[i]));
  HIP_OK(hipMemcpy(hout, dy, bytes, hipMemcpyDeviceToHost));
  check("chain(mish) y", NFAD_MISH, hout, y64, n, allow);
  for (size_t i = 0; i < n; ++i) allow[i] = 5e-7 * fmax(1.0, fabs(x64[i])) * fmax(1.0, fabs(d64[i]));
  HIP_OK(hipMemcpy(hout, dd, bytes, hipMemcpyDeviceToHost));
  check("chain(mish) dydx", NFAD_MISH, hout, d64, n, allow);
  free(allow);
  NFAD_OK_(nfad_chain_release(id));

  HIP_OK(hipStreamDestroy(stream));
  printf(g_failures ? "FAILED: %d check(s)\n" : "all checks passed\n", g_failures);
  return g_failures ? 1 : 0;
}

/*
 * nfad_oracle.c -- slow, plain, fp64 CPU oracle for nested forward-mode AD of
 * element-wise activations.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the yardstick the GPU library is
 * checked against and the CPU baseline the benchmark times beside it.  It is
 * never part of the product path, it shares no code, header, table or
 * constant generator with the GPU kernels, and nothing in it is tuned.
 *
 * What it computes (all in IEEE double, libm only, one element at a time):
 *
 *   fwd      : y = f(x) and dydx = f'(x)          (method: Sec. II-C eq. 3,
 *              the dual number (x, 1) pushed through the activation; the
 *              result is exactly the textbook value and derivative, so the
 *              oracle is the definition written out)
 *   fwd_dual : the same pair, but obtained by literally propagating
 *              (value, tangent) pairs through the primitive operations in
 *              the order of Sec. II-C eq. 3 / Sec. II-D (seed tangent 1).
 *              Kept separate so that the two derivations can be compared.
 *   bwd      : gx = gy * dydx                      (Sec. II-C eq. 4, Sec. II-E)
 *   saveall  : ordinary back-propagation that keeps every intermediate its
 *              primitives need (Sec. II-C eqs. 1-2 for Swish; the same
 *              recipe applied to the other activations)
 *   recompute: keep only x, rebuild the derivative in backward (Sec. II-C,
 *              "Recomputation")
 *
 * Activation definitions: Table I (GELU tanh form, Mish, Swish); the Swish
 * derivative is Table II.  The erf form of GELU, x*Phi(x), is the textbook
 * one (it is not printed in the paper).
 *
 * Stable evaluation, and why each rewriting is the same function:
 *   sigmoid(v)            evaluated with a non-positive exponent on each side
 *   0.5*(1+tanh u)        = sigmoid(2u)            (identity; avoids 1+(-1))
 *   0.5*(1-tanh^2 u)      = 2*sigmoid(2u)*sigmoid(-2u)
 *   Phi(x)                = 0.5*erfc(-x/sqrt 2)    (no 1+erf cancellation)
 *   softplus(x)           = log1p(exp(x)) for x<=0, x+log1p(exp(-x)) else
 * These identities are themselves pinned by the CPU tests against 50-digit
 * evaluation of the unrewritten definitions.
 *
 * Kinds: 0 GELU-tanh, 1 GELU-erf, 2 Swish (beta = 1), 3 Mish.
 * `threads` <= 0 means "all cores OpenMP reports"; 1 means serial.
 * Every function returns 0 on success, 1 on a bad kind or null pointer.
 */
#include <math.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define KIND_GELU_TANH 0
#define KIND_GELU_ERF 1
#define KIND_SWISH 2
#define KIND_MISH 3

/* sqrt(2/pi), 1/sqrt(2*pi), 1/sqrt(2): computed, not typed in. */
static double c_sqrt_2_over_pi(void) { return sqrt(2.0 / acos(-1.0)); }
static double c_inv_sqrt_2pi(void) { return 1.0 / sqrt(2.0 * acos(-1.0)); }
static double c_inv_sqrt_2(void) { return 1.0 / sqrt(2.0); }
static const double GELU_CUBIC = 0.044715; /* Table I */

static double sigmoid(double v) {
  if (v >= 0.0) return 1.0 / (1.0 + exp(-v));
  double e = exp(v);
  return e / (1.0 + e);
}

static double softplus(double v) {
  if (v <= 0.0) return log1p(exp(v));
  return v + log1p(exp(-v));
}

/* ---------------------------------------------------------------- */
/* Closed form: value and derivative of each activation.            */
/* ---------------------------------------------------------------- */

/* Swish: Table I, derivative Table II: s + x*s*(1-s), with 1-s = sigmoid(-x). */
static void swish_vd(double x, double *y, double *d) {
  double s = sigmoid(x), sc = sigmoid(-x);
  *y = x * s;
  *d = s + x * s * sc;
}

/* GELU, tanh form: Table I.  u = sqrt(2/pi)*(x + 0.044715 x^3). */
static void gelu_tanh_vd(double x, double *y, double *d) {
  double c = c_sqrt_2_over_pi();
  double u = c * (x + GELU_CUBIC * x * x * x);
  double du = c * (1.0 + 3.0 * GELU_CUBIC * x * x);
  double s = sigmoid(2.0 * u);   /* 0.5*(1+tanh u)   */
  double sc = sigmoid(-2.0 * u); /* 0.5*(1-tanh u)   */
  *y = x * s;
  /* d/dx [x * 0.5(1+tanh u)] = 0.5(1+tanh u) + x * 0.5(1-tanh^2 u) * u' */
  *d = s + x * (2.0 * s * sc) * du;
}

/* GELU, erf form: x*Phi(x); derivative Phi(x) + x*phi(x). */
static void gelu_erf_vd(double x, double *y, double *d) {
  double Phi = 0.5 * erfc(-x * c_inv_sqrt_2());
  double phi = exp(-0.5 * x * x) * c_inv_sqrt_2pi();
  *y = x * Phi;
  *d = Phi + x * phi;
}

/* Mish: Table I.  softplus' = sigmoid, tanh' = 1 - tanh^2. */
static void mish_vd(double x, double *y, double *d) {
  double sp = softplus(x);
  double t = tanh(sp);
  *y = x * t;
  *d = t + x * (1.0 - t * t) * sigmoid(x);
}

static int closed_form(int kind, double x, double *y, double *d) {
  switch (kind) {
    case KIND_GELU_TANH: gelu_tanh_vd(x, y, d); return 0;
    case KIND_GELU_ERF: gelu_erf_vd(x, y, d); return 0;
    case KIND_SWISH: swish_vd(x, y, d); return 0;
    case KIND_MISH: mish_vd(x, y, d); return 0;
  }
  return 1;
}

/* ---------------------------------------------------------------- */
/* Dual-number propagation (Sec. II-C eq. 3, Sec. II-D).            */
/* A node carries (v, dv) with dv = d v / d x; the head is (x, 1).  */
/* ---------------------------------------------------------------- */
typedef struct { double v, dv; } dual;

static dual d_seed(double x) { dual r = {x, 1.0}; return r; }
static dual d_const(double c) { dual r = {c, 0.0}; return r; }
static dual d_add(dual a, dual b) { dual r = {a.v + b.v, a.dv + b.dv}; return r; }
static dual d_mul(dual a, dual b) { dual r = {a.v * b.v, a.v * b.dv + a.dv * b.v}; return r; }
static dual d_sigmoid(dual a) { double s = sigmoid(a.v); dual r = {s, s * sigmoid(-a.v) * a.dv}; return r; }
static dual d_tanh(dual a) {
  double t = tanh(a.v);
  /* 1 - tanh^2 = 4 sigmoid(2v) sigmoid(-2v): the same number without cancellation */
  dual r = {t, 4.0 * sigmoid(2.0 * a.v) * sigmoid(-2.0 * a.v) * a.dv};
  return r;
}
static dual d_softplus(dual a) { dual r = {softplus(a.v), sigmoid(a.v) * a.dv}; return r; }
static dual d_erf(dual a) {
  dual r = {erf(a.v), 2.0 / sqrt(acos(-1.0)) * exp(-a.v * a.v) * a.dv};
  return r;
}

static int dual_form(int kind, double x, double *y, double *d) {
  dual X = d_seed(x), out;
  switch (kind) {
    case KIND_SWISH: { /* v1 = sigmoid(x), v2 = x, v3 = v1*v2 */
      dual v1 = d_sigmoid(X), v2 = X;
      out = d_mul(v1, v2);
      break;
    }
    case KIND_GELU_TANH: { /* 0.5*x*(1 + tanh(c*(x + k*x^3))) */
      dual x3 = d_mul(d_mul(X, X), X);
      dual u = d_mul(d_const(c_sqrt_2_over_pi()), d_add(X, d_mul(d_const(GELU_CUBIC), x3)));
      dual s = d_add(d_const(1.0), d_tanh(u));
      out = d_mul(d_mul(d_const(0.5), X), s);
      break;
    }
    case KIND_GELU_ERF: { /* 0.5*x*(1 + erf(x/sqrt 2)) */
      dual z = d_mul(d_const(c_inv_sqrt_2()), X);
      dual s = d_add(d_const(1.0), d_erf(z));
      out = d_mul(d_mul(d_const(0.5), X), s);
      break;
    }
    case KIND_MISH: { /* x * tanh(softplus(x)) */
      out = d_mul(X, d_tanh(d_softplus(X)));
      break;
    }
    default: return 1;
  }
  *y = out.v;
  *d = out.dv;
  return 0;
}

/* ---------------------------------------------------------------- */
/* Ordinary back-propagation with saved intermediates.              */
/*                                                                  */
/* Saved set = what each primitive's backward needs (a product      */
/* keeps both operands, tanh and sigmoid keep their output,         */
/* softplus, erf and the cubic keep their input, sums and constant  */
/* scalings keep nothing), duplicates removed; slot 0 is always x:  */
/*   Swish     {x, s=sigmoid(x)}                   (eqs. 1-2)       */
/*   Mish      {x, t=tanh(softplus x)}                              */
/*   GELU-erf  {x, h=0.5x, s=1+erf(x/sqrt 2)}                       */
/*   GELU-tanh {x, t=tanh u, h=0.5x, s=1+t}                         */
/* ---------------------------------------------------------------- */
static int num_saved(int kind) {
  switch (kind) {
    case KIND_SWISH: return 2;
    case KIND_MISH: return 2;
    case KIND_GELU_ERF: return 3;
    case KIND_GELU_TANH: return 4;
  }
  return -1;
}

static void saveall_fwd_one(int kind, double x, double *y, double *sv) {
  sv[0] = x;
  switch (kind) {
    case KIND_SWISH: { /* v1 = sigmoid(x), v2 = x, v3 = v1*v2 */
      double v1 = sigmoid(x);
      sv[1] = v1;
      *y = v1 * x;
      break;
    }
    case KIND_MISH: {
      double t = tanh(softplus(x));
      sv[1] = t;
      *y = x * t;
      break;
    }
    case KIND_GELU_ERF: {
      double h = 0.5 * x;
      double s = 1.0 + erf(x * c_inv_sqrt_2());
      sv[1] = h;
      sv[2] = s;
      *y = h * s;
      break;
    }
    case KIND_GELU_TANH: {
      double u = c_sqrt_2_over_pi() * (x + GELU_CUBIC * x * x * x);
      double t = tanh(u);
      double h = 0.5 * x;
      double s = 1.0 + t;
      sv[1] = t;
      sv[2] = h;
      sv[3] = s;
      *y = h * s;
      break;
    }
  }
}

static double saveall_bwd_one(int kind, double g, const double *sv) {
  double x = sv[0];
  switch (kind) {
    case KIND_SWISH: { /* eq. 1 and eq. 2: x' = g*v2*[v1(1-v1)] + g*v1 */
      double v1 = sv[1], v2 = x;
      return g * v2 * (v1 * (1.0 - v1)) + g * v1;
    }
    case KIND_MISH: {
      double t = sv[1];
      double g_t = g * x;                 /* product node, towards tanh   */
      double g_sp = g_t * (1.0 - t * t);  /* tanh keeps its output        */
      double g_x1 = g_sp * sigmoid(x);    /* softplus keeps its input     */
      double g_x2 = g * t;                /* product node, towards x      */
      return g_x1 + g_x2;
    }
    case KIND_GELU_ERF: {
      double h = sv[1], s = sv[2];
      double g_h = g * s, g_s = g * h;    /* product node                 */
      double z = x * c_inv_sqrt_2();      /* erf keeps its input          */
      double g_z = g_s * 2.0 / sqrt(acos(-1.0)) * exp(-z * z);
      return 0.5 * g_h + c_inv_sqrt_2() * g_z;
    }
    case KIND_GELU_TANH: {
      double t = sv[1], h = sv[2], s = sv[3];
      double g_h = g * s, g_s = g * h;    /* product node                 */
      double g_u = g_s * (1.0 - t * t);   /* tanh keeps its output        */
      double du = c_sqrt_2_over_pi() * (1.0 + 3.0 * GELU_CUBIC * x * x); /* cubic keeps x */
      return 0.5 * g_h + g_u * du;
    }
  }
  return 0.0;
}

/* ---------------------------------------------------------------- */
/* Exported array entry points.                                     */
/* ---------------------------------------------------------------- */
static int resolve_threads(int threads) {
#ifdef _OPENMP
  if (threads <= 0) return omp_get_max_threads();
  return threads;
#else
  (void)threads;
  return 1;
#endif
}

int nfad_oracle_max_threads(void) { return resolve_threads(0); }

int nfad_oracle_num_saved(int kind) { return num_saved(kind); }

int nfad_oracle_fwd(int kind, const double *x, double *y, double *dydx, size_t n, int threads) {
  if (kind < 0 || kind > 3) return 1;
  if (n && (!x || !y || !dydx)) return 1;
  int nt = resolve_threads(threads);
  (void)nt;
#pragma omp parallel for schedule(static) num_threads(nt)
  for (long long i = 0; i < (long long)n; ++i) closed_form(kind, x[i], &y[i], &dydx[i]);
  return 0;
}

int nfad_oracle_fwd_dual(int kind, const double *x, double *y, double *dydx, size_t n) {
  if (kind < 0 || kind > 3) return 1;
  if (n && (!x || !y || !dydx)) return 1;
  for (size_t i = 0; i < n; ++i) dual_form(kind, x[i], &y[i], &dydx[i]);
  return 0;
}

int nfad_oracle_bwd(const double *gy, const double *dydx, double *gx, size_t n, int threads) {
  if (n && (!gy || !dydx || !gx)) return 1;
  int nt = resolve_threads(threads);
  (void)nt;
#pragma omp parallel for schedule(static) num_threads(nt)
  for (long long i = 0; i < (long long)n; ++i) gx[i] = gy[i] * dydx[i];
  return 0;
}

int nfad_oracle_recompute_fwd(int kind, const double *x, double *y, size_t n, int threads) {
  if (kind < 0 || kind > 3) return 1;
  if (n && (!x || !y)) return 1;
  int nt = resolve_threads(threads);
  (void)nt;
#pragma omp parallel for schedule(static) num_threads(nt)
  for (long long i = 0; i < (long long)n; ++i) {
    double d;
    closed_form(kind, x[i], &y[i], &d);
  }
  return 0;
}

int nfad_oracle_recompute_bwd(int kind, const double *gy, const double *x, double *gx, size_t n,
                              int threads) {
  if (kind < 0 || kind > 3) return 1;
  if (n && (!gy || !x || !gx)) return 1;
  int nt = resolve_threads(threads);
  (void)nt;
#pragma omp parallel for schedule(static) num_threads(nt)
  for (long long i = 0; i < (long long)n; ++i) {
    double y, d;
    closed_form(kind, x[i], &y, &d);
    gx[i] = gy[i] * d;
  }
  return 0;
}

/* saved[j] (j = 0 .. num_saved-1) are n-element arrays; slot 0 receives a copy of x. */
int nfad_oracle_saveall_fwd(int kind, const double *x, double *y, double *const *saved, size_t n,
                            int threads) {
  int k = num_saved(kind);
  if (k < 0) return 1;
  if (n && (!x || !y || !saved)) return 1;
  for (int j = 0; j < k; ++j)
    if (n && !saved[j]) return 1;
  int nt = resolve_threads(threads);
  (void)nt;
#pragma omp parallel for schedule(static) num_threads(nt)
  for (long long i = 0; i < (long long)n; ++i) {
    double sv[4];
    saveall_fwd_one(kind, x[i], &y[i], sv);
    for (int j = 0; j < k; ++j) saved[j][i] = sv[j];
  }
  return 0;
}

int nfad_oracle_saveall_bwd(int kind, const double *gy, const double *const *saved, double *gx,
                            size_t n, int threads) {
  int k = num_saved(kind);
  if (k < 0) return 1;
  if (n && (!gy || !gx || !saved)) return 1;
  for (int j = 0; j < k; ++j)
    if (n && !saved[j]) return 1;
  int nt = resolve_threads(threads);
  (void)nt;
#pragma omp parallel for schedule(static) num_threads(nt)
  for (long long i = 0; i < (long long)n; ++i) {
    double sv[4];
    for (int j = 0; j < k; ++j) sv[j] = saved[j][i];
    gx[i] = saveall_bwd_one(kind, gy[i], sv);
  }
  return 0;
}

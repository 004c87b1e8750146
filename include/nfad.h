/*
 * nfad.h -- C ABI of libnfad: nested forward-mode automatic differentiation for
 * element-wise activation functions on AMD MI355X (gfx950).
 *
 * The method (Sec. II-C eq. 3-4, Sec. II-E of "Nesting Forward Automatic
 * Differentiation for Memory-Efficient Deep Neural Network Training"): during the
 * forward pass each element carries the dual number (x, 1) through the activation,
 * which yields y = f(x) and the local derivative dydx = f'(x) together.  Only dydx
 * is kept for the backward pass, which is then one multiply, gx = gy * dydx.
 * The two alternatives the paper compares against are exported beside it:
 * ordinary back-propagation that saves every intermediate (Sec. II-C eqs. 1-2) and
 * recomputation from x in the backward pass (Sec. II-C, "Recomputation").
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * Pointers  : DEVICE pointers (HIP global memory) to flat, contiguous arrays of `n`
 *             elements of `dtype`.  All tensors of one call share `dtype`.  Tensor
 *             shape (NCHW, row-major, ...) is irrelevant: the operation is
 *             element-wise.  `saved` is a HOST array of device pointers.
 * Ownership : the caller owns every buffer.  The library never allocates, frees or
 *             keeps a pointer, and has no state apart from the table of run-time compiled
 *             chains (thread-safe, re-entrant).
 * Stream    : `stream` is a hipStream_t passed as void*; NULL is the default stream.
 *             Calls enqueue work and return; they never synchronise, allocate or copy,
 *             so they may be captured into a HIP graph.
 * Math      : fp32 internally for all dtypes; fp16/bf16 results are rounded once,
 *             to nearest even, on store.  Swish uses beta = 1 (Table I).
 * Alignment : pointers must be aligned to the element size (else NFAD_EALIGN).
 *             If every pointer of a call is 16-byte aligned the 128-bit vector body
 *             runs.  If all are misaligned by the same amount (equal views of aligned
 *             tensors) a few leading elements take a scalar kernel and the rest the
 *             vector body; otherwise a scalar kernel produces the same values, slower.
 * Aliasing  : an output may coincide EXACTLY with an input of the same call
 *             (y == x, gx == gy, gx == dydx, gx == saved[j]); two outputs must not
 *             coincide (NFAD_EALIAS).  Partial overlap is undefined.
 * Errors    : every call returns an nfad_status_t as int.  Arguments are validated
 *             on the host before any HIP call; n == 0 returns NFAD_OK without a
 *             launch (pointers may then be NULL).  A failed launch gives NFAD_ELAUNCH.
 *             Nothing throws or aborts across this boundary.
 * Finite x  : for every finite input the results are finite: y -> x, dydx -> 1 as
 *             x -> +inf and y -> -0, dydx -> -0 as x -> -inf.  A NaN input gives NaN in
 *             every output of that element; +-inf inputs give unspecified values.
 */
#ifndef NFAD_H_
#define NFAD_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Activations: Table I (GELU tanh form, Swish, Mish); the erf form of GELU is the
 * textbook x*Phi(x). */
typedef enum {
  NFAD_GELU_TANH = 0, /* 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))) */
  NFAD_GELU_ERF = 1,  /* 0.5 x (1 + erf(x / sqrt 2))                      */
  NFAD_SWISH = 2,     /* x * sigmoid(x)                                   */
  NFAD_MISH = 3       /* x * tanh(ln(1 + e^x))                            */
} nfad_kind_t;

typedef enum { NFAD_F32 = 0, NFAD_F16 = 1, NFAD_BF16 = 2 } nfad_dtype_t;

typedef enum {
  NFAD_OK = 0,
  NFAD_EINVAL_KIND = 1,
  NFAD_EINVAL_DTYPE = 2,
  NFAD_ENULL = 3,   /* a required pointer is NULL while n > 0            */
  NFAD_EALIGN = 4,  /* a pointer is not aligned to the element size      */
  NFAD_EALIAS = 5,  /* two outputs of one call coincide                  */
  NFAD_ELAUNCH = 6, /* the HIP runtime refused the launch                */
  NFAD_EPROGRAM = 7, /* a chain program is malformed                      */
  NFAD_ECOMPILE = 8  /* run-time compilation or loading of a chain failed */
} nfad_status_t;

#define NFAD_MAX_SAVED 4
#define NFAD_MAX_OUTPUTS 4

/* Forward pass of the method (Sec. II-C eq. 3): y[i] = f(x[i]), dydx[i] = f'(x[i]).
 * x: in, n elements.  y, dydx: out, n elements each.  dydx is the only tensor the
 * caller needs to keep for nfad_bwd; x may be released afterwards. */
int nfad_fwd(int kind, const void* x, void* y, void* dydx, size_t n, int dtype, void* stream);

/* Backward pass of the method (Sec. II-C eq. 4, Sec. II-E): gx[i] = gy[i] * dydx[i].
 * gy: upstream gradient, in.  dydx: as written by nfad_fwd, in.  gx: out. */
int nfad_bwd(const void* gy, const void* dydx, void* gx, size_t n, int dtype, void* stream);

/* Recomputation baseline (Sec. II-C, "Recomputation"): forward writes y only and the
 * caller keeps x; backward re-derives f'(x) and writes gx[i] = gy[i] * f'(x[i]). */
int nfad_recompute_fwd(int kind, const void* x, void* y, size_t n, int dtype, void* stream);
int nfad_recompute_bwd(int kind, const void* gy, const void* x, void* gx, size_t n, int dtype,
                       void* stream);

/* Save-all baseline (Sec. II-C eqs. 1-2): ordinary back-propagation through the
 * activation's primitive operations, keeping what each primitive's backward needs:
 *   Swish     k = 2: saved = { x, s = sigmoid(x) }
 *   Mish      k = 2: saved = { x, t = tanh(softplus(x)) }
 *   GELU-erf  k = 3: saved = { x, h = 0.5 x, s = 1 + erf(x / sqrt 2) }
 *   GELU-tanh k = 4: saved = { x, t = tanh(u), h = 0.5 x, s = 1 + t }
 * nfad_saveall_num_saved returns k (or -1 for a bad kind).
 * `saved` is a host array of k device pointers.  saved[0] stands for x, which already
 * exists: the forward pass never writes it (it may be NULL there) and writes
 * saved[1..k-1]; the backward pass reads gy and all k tensors (saved[0] = x). */
int nfad_saveall_num_saved(int kind);
int nfad_saveall_fwd(int kind, const void* x, void* y, void* const* saved, size_t n, int dtype,
                     void* stream);
int nfad_saveall_bwd(int kind, const void* gy, const void* const* saved, void* gx, size_t n,
                     int dtype, void* stream);

/* Composed chains (Sec. III-A: any composition of "fad" primitive operations that maps one
 * source element to one result; primitives: + - * / min max neg exp log tanh sigmoid
 * softplus erf relu abs sqrt, constants, and the source x; at a kink the tangent of relu and
 * abs is 0 and min/max follow their first operand).  The library carries a table of chains built from those
 * primitives with a compile-time dual-number composer; each is fused into ONE forward
 * kernel with the contract of nfad_fwd: y[i] = f(x[i]), dydx[i] = f'(x[i]), f' obtained by
 * pushing the dual number (x, 1) through the primitives (Sec. II-C eq. 3, Sec. II-D).
 * The backward pass of a chain is nfad_bwd.
 *   nfad_chain_count    number of chains in the table (ids are 0 .. count-1)
 *   nfad_chain_name     short name, or NULL for a bad id
 *   nfad_chain_program  the chain in postfix notation over the primitive names, e.g.
 *                       "x x softplus tanh *" for x*tanh(softplus(x)); NULL for a bad id
 *   nfad_chain_fwd      as nfad_fwd; a bad id gives NFAD_EINVAL_KIND */
int nfad_chain_count(void);
const char* nfad_chain_name(int chain_id);
const char* nfad_chain_program(int chain_id);
int nfad_chain_fwd(int chain_id, const void* x, void* y, void* dydx, size_t n, int dtype,
                   void* stream);

/* Run-time composed chains: the counterpart of the paper's automatic graph rewrite
 * (Sec. III-B, Sec. IV), which finds a chain of fad operations and replaces its forward and
 * backward passes.  `program` is ANY chain in the postfix notation above (tokens separated
 * by blanks: x, decimal constants and the primitive names listed above; at most
 * 256 tokens and 24 constants; must use x and leave exactly one value).  The library compiles
 * one fused forward kernel for it on the current device (hiprtc; a fraction of a second) and
 * returns a chain id >= NFAD_CHAIN_JIT_BASE in *chain_id, valid for nfad_chain_fwd / _name /
 * _program on that device until released.
 * Constants are arguments of the kernel, not part of it (Sec. III-A "binary operation with a
 * constant"): programs that differ only in their numbers share ONE compiled kernel, so
 * compiling `x 0.1 *` after `x 0.2 *` costs no compiler run.  (Sub-expressions without x are
 * folded on the host; only 0, +-1, +-2 and +-0.5 are compiled in.)
 * This is the one stateful part of the library: a process-wide table of at most 4096 LIVE
 * chains, protected by a mutex; a released chain's id is handed out again, and a kernel is
 * unloaded with the last chain that uses it.
 *   nfad_chain_compile  NFAD_EPROGRAM for a malformed program (checked on the host before
 *                       any compiler or HIP call), NFAD_ECOMPILE if compiling or loading fails
 *                       or if the table is full (checked before compiling)
 *   nfad_chain_release  frees the id; the caller must first wait for launches of that
 *                       chain to finish.  NFAD_EINVAL_KIND for an id that is not live
 *   nfad_chain_kernel   identifier (>= 0) of the compiled kernel behind a run-time chain: equal
 *                       for chains that share a kernel; -1 for a built-in or dead id
 *   nfad_chain_log      the calling thread's message from its last nfad_chain_compile
 *                       (parse error or compiler log; empty string if none)
 * Results are finite wherever the true value is representable and every intermediate
 * exponential stays finite or overflows only into a denominator (then the limit is returned). */
#define NFAD_CHAIN_JIT_BASE 1000
int nfad_chain_compile(const char* program, int* chain_id);
int nfad_chain_release(int chain_id);
int nfad_chain_kernel(int chain_id);
const char* nfad_chain_log(void);

/* One source, several outputs (Sec. II-D "R^1 -> R^M", Sec. IV-A): m chains over the same x,
 * 1 <= m <= NFAD_MAX_OUTPUTS, fused into ONE forward kernel that reads x once and writes
 * y[j] and dydx[j] for j < m (one saved tangent per output); the backward pass merges the
 * m upstream gradients at the source, gx[i] = sum_j gy[j][i] * dydx[j][i].
 *   nfad_chain_compile_multi  `programs` = host array of m postfix programs; errors as
 *                             nfad_chain_compile, NFAD_EINVAL_KIND for a bad m.  The id
 *                             works with nfad_chain_fwd_multi / _release / _name;
 *                             nfad_chain_program returns the programs joined by " ; "
 *   nfad_chain_num_outputs    m of a run-time compiled chain, 1 for a built-in chain, -1 for
 *                             a bad id
 *   nfad_chain_fwd_multi      y, dydx: host arrays of m device pointers (all 2m outputs
 *                             distinct).  nfad_chain_fwd on an id with m > 1, or this call
 *                             on a built-in id, gives NFAD_EINVAL_KIND
 *   nfad_bwd_multi            gy, dydx: host arrays of m device pointers; gx may coincide
 *                             with any input */
int nfad_chain_compile_multi(const char* const* programs, int m, int* chain_id);
int nfad_chain_num_outputs(int chain_id);
int nfad_chain_fwd_multi(int chain_id, const void* x, void* const* y, void* const* dydx, size_t n,
                         int dtype, void* stream);
int nfad_bwd_multi(const void* const* gy, const void* const* dydx, int m, void* gx, size_t n,
                   int dtype, void* stream);

/* Static, NUL-terminated description of a status code (never NULL). */
const char* nfad_status_string(int status);

/* major * 10000 + minor * 100 + patch */
int nfad_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NFAD_H_ */

"""GPU parity of the composed chains: every chain the library carries, through the C ABI,
against the fp64 postfix dual-number interpreter on the same seeded storage-rounded inputs."""
import numpy as np
import pytest
import torch

from oracle import chain
import oracle
import paper_2209_10778_amd as nfad
from paper_2209_10778_amd import inputs
from chain_programs import random_programs
from parity import chain_allowance, compare, two_stage_budget

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
N = 3 * 8192 + 5 * 256 + 77 + 5


def chains():
    return [(i, nfad.nfad_chain_name(i)) for i in range(nfad.nfad_chain_count())]


def chain_inputs(name, dtype, seed):
    """N(0, 2.5) clipped to the range where the chain's VALUE is representable in the storage
    type (exp(x) leaves fp16 above 11)."""
    a = inputs.gaussian(N, 2.5, seed)
    lim = {"exp": 10.0}.get(name, 100.0)
    special = np.array([0.0, -0.0, 1e-4, -1e-4, 0.02, -0.02, 0.1, -0.1, 1.0, -1.0, 5.0, -5.0, 9.0, -9.0,
                        20.0, -20.0, 50.0, -50.0, 80.0, -80.0], np.float32)
    a[:special.size] = special
    return inputs.to_storage(np.clip(a, -lim, lim), dtype)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("cid,name", chains())
def test_chain_fwd_matches_interpreter(cid, name, dtype):
    td = DTYPES[dtype]
    x = chain_inputs(name, dtype, 7000 + cid)
    x64 = inputs.storage_to_f64(x)
    y_ref, d_ref = chain.eval_chain(nfad.nfad_chain_program(cid), x64)
    xd = x.to(DEV)
    y = torch.full_like(xd, float("nan"))
    d = torch.full_like(xd, float("nan"))
    nfad.nfad_chain_fwd(cid, xd, y, d)
    # a composition of fp32 primitives: the bar plus the chain allowance (parity.py)
    sy = compare(y, y_ref, td, f"chain {name} y {dtype}", extra_tol=chain_allowance(x64, y_ref))
    sd = compare(d, d_ref, td, f"chain {name} dydx {dtype}", extra_tol=chain_allowance(x64, d_ref))
    print(f"\n[chain {name} {dtype}] y err/bar {sy['max_over_bar']:.2f} max_abs {sy['max_abs']:.3e} max_ulp {sy['max_ulp']:.2f}; "
          f"dydx err/bar {sd['max_over_bar']:.2f} max_abs {sd['max_abs']:.3e} max_ulp {sd['max_ulp']:.2f}")


def test_chain_then_bwd_gives_the_chain_gradient():
    """Sec. II-E: dL/dx = (d chain/dx) * g, with the stored tangent of the fused forward."""
    td, dtype = torch.float32, "f32"
    cid = [i for i, n in chains() if n == "tanhshrink"][0]
    x = chain_inputs("tanhshrink", dtype, 7100)
    gy = inputs.to_storage(inputs.gaussian(N, 1.0, 7101), dtype)
    x64, gy64 = inputs.storage_to_f64(x), inputs.storage_to_f64(gy)
    _, d_ref = chain.eval_chain(nfad.nfad_chain_program(cid), x64)
    xd, gyd = x.to(DEV), gy.to(DEV)
    y, d, gx = torch.empty_like(xd), torch.empty_like(xd), torch.empty_like(xd)
    nfad.nfad_chain_fwd(cid, xd, y, d)
    nfad.nfad_bwd(gyd, d, gx)
    gx_ref = oracle.bwd(gy64, d_ref)
    compare(gx, gx_ref, td, "chain gradient",
            extra_tol=two_stage_budget(gy64, d_ref, gx_ref, td, d_allowance=chain_allowance(x64, d_ref)))


def test_chain_errors_and_edges():
    L = nfad.lib()
    A = 1 << 20
    assert L.nfad_chain_fwd(-1, A, A + 64, A + 128, 4, 0, None) == 1
    assert L.nfad_chain_fwd(nfad.nfad_chain_count(), A, A + 64, A + 128, 4, 0, None) == 1
    assert L.nfad_chain_fwd(0, None, None, None, 0, 0, None) == 0
    assert L.nfad_chain_fwd(0, None, A, A + 64, 4, 0, None) == 3
    for n in (1, 3, 7, 8, 9, 255, 257):
        x = chain_inputs("sigmoid", "bf16", 7200 + n)[:n].contiguous()
        y_ref, d_ref = chain.eval_chain("x sigmoid", inputs.storage_to_f64(x))
        xd = x.to(DEV)
        y, d = torch.empty_like(xd), torch.empty_like(xd)
        nfad.nfad_chain_fwd(0, xd, y, d)
        compare(y, y_ref, torch.bfloat16, f"n={n}")
        compare(d, d_ref, torch.bfloat16, f"n={n}")


# ------------------------------------------------------------------ run-time composed chains
JIT_PROGRAMS = [
    "x x * tanh",                               # tanh(x^2)
    "x sigmoid x tanh *",                       # sigmoid(x) tanh(x)
    "x 0.5 * exp 1 + log",                      # ln(1 + e^{x/2})
    "x x softplus tanh *",                      # Mish again, compiled at run time
    "x 1.702 x * sigmoid *",                    # the sigmoid approximation of GELU
    "x erf x * 0.25 x * -",                     # x erf(x) - x/4
    "1 x x * 1 + /",                            # 1/(1+x^2)
    "x relu 1.5 x 0 min exp 1 - * +",           # ELU with alpha = 1.5
    "x abs 1 + sqrt x *",                       # x sqrt(1 + |x|)
    "x -1 max 2.5 min x *",                     # x clamp(x, -1, 2.5)
    "x 0.75 * softplus tanh 2 *",               # the fused tanh-of-softplus pair on a scaled operand
    "2 x exp 1 + /",                            # constant / chain
    "x 3 / x -",                                # chain / constant
    "3 x - tanh",                               # constant - chain
    "x 1 2 + 4 * 8 / 0.5 - *",                  # a constant sub-expression: x * ((1 + 2) * 4 / 8 - 0.5)
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_runtime_compiled_chains_match_interpreter(dtype):
    td = DTYPES[dtype]
    ids = []
    for k, prog in enumerate(JIT_PROGRAMS):
        cid = nfad.nfad_chain_compile(prog)
        assert cid >= 1000 and nfad.nfad_chain_program(cid) == prog and nfad.nfad_chain_name(cid).startswith("jit:")
        ids.append(cid)
        a = inputs.gaussian(N, 2.0, 7300 + k)
        x = inputs.to_storage(np.clip(a, -9.0, 9.0), dtype)
        x64 = inputs.storage_to_f64(x)
        y_ref, d_ref = chain.eval_chain(prog, x64)
        xd = x.to(DEV)
        y = torch.full_like(xd, float("nan"))
        d = torch.full_like(xd, float("nan"))
        nfad.nfad_chain_fwd(cid, xd, y, d)
        compare(y, y_ref, td, f"jit {prog!r} y {dtype}", extra_tol=chain_allowance(x64, y_ref))
        compare(d, d_ref, td, f"jit {prog!r} dydx {dtype}", extra_tol=chain_allowance(x64, d_ref))
        # the scalar (misaligned) kernel of the same chain
        buf = torch.zeros(N + 8, dtype=td, device=DEV)
        buf[1:N + 1] = xd
        y2, d2 = torch.empty_like(xd), torch.empty_like(xd)
        nfad.nfad_chain_fwd(cid, buf[1:N + 1], y2, d2)
        assert torch.equal(y2, y) and torch.equal(d2, d)
    torch.cuda.synchronize()
    for cid in ids:
        nfad.nfad_chain_release(cid)
        assert nfad.nfad_chain_name(cid) is None
        with pytest.raises(nfad.NfadError):
            nfad.nfad_chain_fwd(cid, xd, y, d)
    with pytest.raises(nfad.NfadError):
        nfad.nfad_chain_release(ids[0])


# ------------------------------------------------------------------ one source, several outputs
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("m", [2, 3, 4])
def test_multi_output_chain_and_merged_backward(m, dtype):
    td = DTYPES[dtype]
    programs = ["x tanh x *", "x tanh sigmoid", "x x * neg exp", "x 0.5 * softplus"][:m]
    cid = nfad.nfad_chain_compile_multi(programs)
    assert nfad.nfad_chain_num_outputs(cid) == m and nfad.nfad_chain_program(cid) == " ; ".join(programs)
    a = inputs.gaussian(N, 2.0, 7400 + m)
    x = inputs.to_storage(np.clip(a, -9.0, 9.0), dtype)
    x64 = inputs.storage_to_f64(x)
    xd = x.to(DEV)
    ys = [torch.full_like(xd, float("nan")) for _ in range(m)]
    ds = [torch.full_like(xd, float("nan")) for _ in range(m)]
    nfad.nfad_chain_fwd_multi(cid, xd, ys, ds)
    refs = [chain.eval_chain(p, x64) for p in programs]
    for j in range(m):
        compare(ys[j], refs[j][0], td, f"multi y{j} {dtype}", extra_tol=chain_allowance(x64, refs[j][0]))
        compare(ds[j], refs[j][1], td, f"multi d{j} {dtype}", extra_tol=chain_allowance(x64, refs[j][1]))
    with pytest.raises(nfad.NfadError):
        nfad.nfad_chain_fwd(cid, xd, ys[0], ds[0])             # a multi-output id needs the multi call
    with pytest.raises(nfad.NfadError):
        nfad.nfad_chain_fwd_multi(cid, xd, ys, [ds[0]] * m)    # coinciding outputs

    # backward: tangents of all consumers merge at the source; inputs are the ORACLE's tangents, stored
    gys = [inputs.to_storage(inputs.gaussian(N, 1.0, 7500 + 10 * m + j), dtype) for j in range(m)]
    dst = [inputs.to_storage(refs[j][1].astype(np.float32), dtype) for j in range(m)]
    gx_ref = sum(inputs.storage_to_f64(gys[j]) * inputs.storage_to_f64(dst[j]) for j in range(m))
    gx = torch.full_like(xd, float("nan"))
    nfad.nfad_bwd_multi([g.to(DEV) for g in gys], [d.to(DEV) for d in dst], gx)
    # a sum of m exact products accumulated in fp32: each of the m - 1 additions rounds once (2^-24
    # relative) at a magnitude of at most sum_j |gy_j dydx_j|; then the one rounding to storage (the bar)
    mag = sum(np.abs(inputs.storage_to_f64(gys[j]) * inputs.storage_to_f64(dst[j])) for j in range(m))
    sm = compare(gx, gx_ref, td, f"bwd_multi m={m} {dtype}", extra_tol=(m - 1) * 2.0 ** -24 * mag)
    print(f"\n[bwd_multi m={m} {dtype}] err/bar {sm['max_over_bar']:.3f}")
    nfad.nfad_chain_release(cid)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chain_kernels_in_their_second_block_shape(dtype):
    """Launches that move 9 to 48 MiB take 128-thread blocks of two accesses per lane: a built-in
    chain, a run-time compiled chain and a two-output chain at a ragged size inside that window."""
    td = DTYPES[dtype]
    es = 4 if dtype == "f32" else 2
    n = (1_300_000 if dtype == "f32" else 2_600_000) + 3 * 256 * 8 + 777 + 3
    assert 9 * 2 ** 20 <= 3 * n * es and 5 * n * es < 48 * 2 ** 20
    x = inputs.to_storage(np.clip(inputs.gaussian(n, 2.0, 7700), -9.0, 9.0), dtype)
    x64 = inputs.storage_to_f64(x)
    xd = x.to(DEV)
    builtin = [i for i, name in chains() if name == "tanhshrink"][0]
    jit = nfad.nfad_chain_compile("x 0.25 * x tanh +")
    for cid in (builtin, jit):
        y, d = torch.full_like(xd, float("nan")), torch.full_like(xd, float("nan"))
        nfad.nfad_chain_fwd(cid, xd, y, d)
        y_ref, d_ref = chain.eval_chain(nfad.nfad_chain_program(cid), x64)
        compare(y, y_ref, td, f"second shape chain {cid} y {dtype}", extra_tol=chain_allowance(x64, y_ref))
        compare(d, d_ref, td, f"second shape chain {cid} dydx {dtype}", extra_tol=chain_allowance(x64, d_ref))
    nfad.nfad_chain_release(jit)
    programs = ["x tanh x *", "x 0.5 * softplus"]
    cid = nfad.nfad_chain_compile_multi(programs)
    ys = [torch.full_like(xd, float("nan")) for _ in programs]
    ds = [torch.full_like(xd, float("nan")) for _ in programs]
    nfad.nfad_chain_fwd_multi(cid, xd, ys, ds)
    for j, p in enumerate(programs):
        y_ref, d_ref = chain.eval_chain(p, x64)
        compare(ys[j], y_ref, td, f"second shape multi y{j} {dtype}", extra_tol=chain_allowance(x64, y_ref))
        compare(ds[j], d_ref, td, f"second shape multi d{j} {dtype}", extra_tol=chain_allowance(x64, d_ref))
    nfad.nfad_chain_release(cid)


def test_multi_output_autograd_front_end():
    from paper_2209_10778_amd import autograd as A
    programs = ["x tanh x *", "x tanh sigmoid"]
    x = inputs.to_storage(np.clip(inputs.gaussian(30_000, 2.0, 7600), -9, 9), "f32")
    x64 = inputs.storage_to_f64(x)
    xd = x.to(DEV).requires_grad_(True)
    a, b = A.chain_multi(xd, programs)
    assert len(a.grad_fn.saved_tensors) == 2
    (a.sum() + 2.0 * b.sum()).backward()
    d1 = chain.eval_chain(programs[0], x64)[1]
    d2 = chain.eval_chain(programs[1], x64)[1]
    g_ref = d1 + 2.0 * d2          # upstream gradients 1 and 2 on the GPU's own stored tangents
    compare(xd.grad, g_ref, torch.float32, "multi autograd",
            extra_tol=two_stage_budget(np.ones_like(x64), d1, g_ref, torch.float32, chain_allowance(x64, d1))
            + two_stage_budget(2.0 * np.ones_like(x64), d2, g_ref, torch.float32, chain_allowance(x64, d2)))


# ------------------------------------------------------------------ random programs
def test_random_programs_match_interpreter():
    """Thirty seeded random chains, compiled at run time, against the interpreter (fp32 and fp16)."""
    programs = random_programs(30)
    a = np.clip(inputs.gaussian(N, 2.0, 7600), -6.0, 6.0)
    for prog in programs:
        cid = nfad.nfad_chain_compile(prog)
        for dtype in ("f32", "f16"):
            td = DTYPES[dtype]
            x = inputs.to_storage(a, dtype)
            x64 = inputs.storage_to_f64(x)
            y_ref, d_ref = chain.eval_chain(prog, x64)
            assert np.isfinite(y_ref).all() and np.isfinite(d_ref).all(), prog
            xd = x.to(DEV)
            y = torch.full_like(xd, float("nan"))
            d = torch.full_like(xd, float("nan"))
            nfad.nfad_chain_fwd(cid, xd, y, d)
            compare(y, y_ref, td, f"random {prog!r} y {dtype}", extra_tol=chain_allowance(x64, y_ref))
            compare(d, d_ref, td, f"random {prog!r} dydx {dtype}", extra_tol=chain_allowance(x64, d_ref))
        nfad.nfad_chain_release(cid)


# ------------------------------------------------------------------ exhaustive 16-bit inputs
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_every_16bit_pattern_through_every_builtin_chain(dtype):
    """All finite fp16 / bf16 bit patterns within the range where the chain as spelled is finite
    (the same limits as the random-input test), through every built-in chain."""
    td = DTYPES[dtype]
    bits = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    x_all = bits.view(td)
    xf = x_all.to(torch.float64)
    report = {}
    for cid, name in chains():
        lim = {"exp": 10.0}.get(name, 100.0)
        x = x_all[torch.isfinite(xf) & (xf.abs() <= lim)].contiguous()
        x64 = inputs.storage_to_f64(x)
        y_ref, d_ref = chain.eval_chain(nfad.nfad_chain_program(cid), x64)
        xd = x.to(DEV)
        y = torch.full_like(xd, float("nan"))
        d = torch.full_like(xd, float("nan"))
        nfad.nfad_chain_fwd(cid, xd, y, d)
        sy = compare(y, y_ref, td, f"exhaustive chain {name} y {dtype}", extra_tol=chain_allowance(x64, y_ref))
        sd = compare(d, d_ref, td, f"exhaustive chain {name} dydx {dtype}", extra_tol=chain_allowance(x64, d_ref))
        report[name] = (round(sy["max_ulp"], 2), round(sd["max_ulp"], 2))
    print(f"\n[exhaustive chains {dtype}] max ulp (y, dydx): {report}")


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_quotient_with_an_overflowed_denominator_returns_the_limit(dtype):
    """x / (1 + e^-x) as Table I spells Swish: for x below -88.7 the exponential overflows in fp32 and
    the quotient rule meets 0 * inf.  Every finite input of the storage type must give the limits
    (y -> -0, dydx -> 0), not NaN; inside the fp64 interpreter's own range (|x| <= 700) the
    interpreter is the reference."""
    td = DTYPES[dtype]
    cid = [i for i, n in chains() if n == "swish_table1"][0]
    if dtype == "f32":
        x = torch.tensor([-3.0e38, -1e30, -1e10, -1e4, -700.0, -100.0, -89.0, -88.0, -60.0, 60.0, 88.0, 89.0, 700.0,
                          1e4, 1e10, 3.0e38], dtype=torch.float32)
    else:
        bits = torch.arange(65536, dtype=torch.int32).to(torch.int16)
        x = bits.view(td)
        x = x[torch.isfinite(x.to(torch.float64))].contiguous()
    x64 = inputs.storage_to_f64(x)
    xd = x.to(DEV)
    y = torch.full_like(xd, float("nan"))
    d = torch.full_like(xd, float("nan"))
    nfad.nfad_chain_fwd(cid, xd, y, d)
    assert bool(torch.isfinite(y.float()).all()) and bool(torch.isfinite(d.float()).all())
    inside = np.abs(x64) <= 700.0
    y_ref, d_ref = chain.eval_chain(nfad.nfad_chain_program(cid), x64[inside])
    keep = torch.from_numpy(inside).to(DEV)
    compare(y[keep], y_ref, td, f"swish_table1 y {dtype}", extra_tol=chain_allowance(x64[inside], y_ref))
    compare(d[keep], d_ref, td, f"swish_table1 dydx {dtype}", extra_tol=chain_allowance(x64[inside], d_ref))
    far = torch.from_numpy(~inside).to(DEV)
    neg = far & (xd < 0)
    pos = far & (xd > 0)
    assert bool((y[neg] == 0).all()) and bool((d[neg] == 0).all())
    assert bool((y[pos] == xd[pos]).all()) and bool((d[pos] == 1).all())


def test_programs_that_differ_only_in_constants_share_one_kernel():
    """Sec. III-A "binary operation with a constant": the constant is an argument of the kernel."""
    import time
    progs = ["x 0.1 * tanh x 1.25 + *", "x 0.2 * tanh x -3.5 + *", "x 7.0 * tanh x 0.001 + *"]
    t0 = time.perf_counter()
    ids = [nfad.nfad_chain_compile(progs[0])]
    t_first = time.perf_counter() - t0
    t0 = time.perf_counter()
    ids += [nfad.nfad_chain_compile(p) for p in progs[1:]]
    t_rest = (time.perf_counter() - t0) / 2
    kernels = [nfad.nfad_chain_kernel(i) for i in ids]
    assert kernels[0] >= 0 and kernels == [kernels[0]] * 3 and len(set(ids)) == 3
    other = nfad.nfad_chain_compile("x 0.1 * tanh x 1.25 - *")          # another structure: another kernel
    assert nfad.nfad_chain_kernel(other) not in (-1, kernels[0])
    print(f"\n[shared kernel] first compile {t_first * 1e3:.0f} ms, same structure again {t_rest * 1e3:.2f} ms")
    assert t_rest < 0.05                                                 # no compiler run
    a = np.clip(inputs.gaussian(N, 2.0, 7700), -9.0, 9.0)
    for dtype in ("f32", "bf16"):
        td = DTYPES[dtype]
        x = inputs.to_storage(a, dtype)
        x64 = inputs.storage_to_f64(x)
        xd = x.to(DEV)
        for cid, prog in zip(ids, progs):
            y_ref, d_ref = chain.eval_chain(prog, x64)
            y, d = torch.full_like(xd, float("nan")), torch.full_like(xd, float("nan"))
            nfad.nfad_chain_fwd(cid, xd, y, d)
            compare(y, y_ref, td, f"shared {prog!r} y {dtype}", extra_tol=chain_allowance(x64, y_ref))
            compare(d, d_ref, td, f"shared {prog!r} dydx {dtype}", extra_tol=chain_allowance(x64, d_ref))
    torch.cuda.synchronize()
    nfad.nfad_chain_release(ids[0])                                      # the kernel outlives its first chain
    y, d = torch.empty_like(xd), torch.empty_like(xd)
    nfad.nfad_chain_fwd(ids[1], xd, y, d)
    y_ref, d_ref = chain.eval_chain(progs[1], x64)
    compare(y, y_ref, td, "after release y", extra_tol=chain_allowance(x64, y_ref))
    torch.cuda.synchronize()
    for cid in ids[1:] + [other]:
        nfad.nfad_chain_release(cid)


def test_table_holds_live_chains_only_in_a_subprocess():
    """A process that compiles and releases chains for ever (a training loop with a step-dependent
    number in a traced expression) must never fill the table: with the capacity lowered to 4 through
    the NFAD_MAX_CHAINS hook, 40 compile / run / release rounds succeed, a fifth LIVE chain is
    refused before any compiler work, and releasing one makes room again.  (Child process: the hook
    is read once.)"""
    import os
    import subprocess
    import sys
    code = r"""
import sys, os, time
sys.path.insert(0, os.getcwd()); sys.path.insert(0, os.path.join(os.getcwd(), "tests"))
import numpy as np, torch
import paper_2209_10778_amd as nfad
from oracle import chain
from parity import chain_allowance, compare
x = torch.linspace(-4, 4, 4099, device="cuda:0")
x64 = x.double().cpu().numpy()
y, d = torch.empty_like(x), torch.empty_like(x)
for step in range(40):
    prog = f"x {0.5 + 0.01 * step} * tanh x *" if step % 2 else f"x {1 + step} + sigmoid"
    cid = nfad.nfad_chain_compile(prog)
    assert cid in (1000, 1001), cid
    nfad.nfad_chain_fwd(cid, x, y, d)
    torch.cuda.synchronize()
    y_ref, d_ref = chain.eval_chain(prog, x64)
    compare(y, y_ref, torch.float32, prog, extra_tol=chain_allowance(x64, y_ref))
    compare(d, d_ref, torch.float32, prog, extra_tol=chain_allowance(x64, d_ref))
    if step % 2:
        nfad.nfad_chain_release(cid)
    elif step:
        nfad.nfad_chain_release(cid)
# slot 1000 still holds step 0's chain
ids = [nfad.nfad_chain_compile(f"x {k} *  x exp +") for k in (3, 4, 5)]
assert sorted(ids) == [1001, 1002, 1003]
t0 = time.perf_counter()
try:
    nfad.nfad_chain_compile("x x * x * 7 +")
    raise SystemExit("a fifth live chain was accepted")
except nfad.NfadError as e:
    assert e.status == 8 and "too many live chains" in str(e), str(e)
assert time.perf_counter() - t0 < 0.05          # refused before compiling
nfad.nfad_chain_release(1002)
assert nfad.nfad_chain_compile("x x * x * 7 +") == 1002
print("table ok")
"""
    env = dict(os.environ, NFAD_MAX_CHAINS="4")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True, timeout=170)
    assert r.returncode == 0 and "table ok" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]

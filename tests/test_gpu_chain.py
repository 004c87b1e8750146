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
from parity import compare

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
N = 3 * 8192 + 5 * 256 + 77 + 5


def chains():
    return [(i, nfad.nfad_chain_name(i)) for i in range(nfad.nfad_chain_count())]


def chain_inputs(name, dtype, seed):
    """N(0, 2.5) clipped to the range where the chain as spelled is finite in fp32 and in the
    storage type (exp(x) leaves fp16 above 11; the quotient form of Swish needs e^-x finite)."""
    a = inputs.gaussian(N, 2.5, seed)
    lim = {"exp": 10.0, "swish_table1": 60.0}.get(name, 100.0)
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
    # fp32 arithmetic through a composition: a few fp32 ulps per primitive, and the exponent
    # argument's rounding scales with |x|; allow 2e-6 * max(1,|x|) relative on top of the usual bar
    rel = 2e-6 * np.maximum(1.0, np.abs(x64))
    sy = compare(y, y_ref, td, f"chain {name} y {dtype}", extra_tol=rel * np.maximum(1.0, np.abs(y_ref)))
    sd = compare(d, d_ref, td, f"chain {name} dydx {dtype}", extra_tol=rel * np.maximum(1.0, np.abs(d_ref)))
    print(f"\n[chain {name} {dtype}] y max_abs {sy['max_abs']:.3e} max_ulp {sy['max_ulp']:.2f}; "
          f"dydx max_abs {sd['max_abs']:.3e} max_ulp {sd['max_ulp']:.2f}")


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
    compare(gx, oracle.bwd(gy64, d_ref), td, "chain gradient", extra_tol=4e-6 * np.abs(gy64) * np.maximum(1.0, np.abs(x64)))


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
        rel = 2e-6 * np.maximum(1.0, np.abs(x64)) ** 2
        compare(y, y_ref, td, f"jit {prog!r} y {dtype}", extra_tol=rel * np.maximum(1.0, np.abs(y_ref)))
        compare(d, d_ref, td, f"jit {prog!r} dydx {dtype}", extra_tol=rel * np.maximum(1.0, np.abs(d_ref)))
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
    rel = 2e-6 * np.maximum(1.0, np.abs(x64)) ** 2
    refs = [chain.eval_chain(p, x64) for p in programs]
    for j in range(m):
        compare(ys[j], refs[j][0], td, f"multi y{j} {dtype}", extra_tol=rel * np.maximum(1.0, np.abs(refs[j][0])))
        compare(ds[j], refs[j][1], td, f"multi d{j} {dtype}", extra_tol=rel * np.maximum(1.0, np.abs(refs[j][1])))
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
    mag = sum(np.abs(inputs.storage_to_f64(gys[j]) * inputs.storage_to_f64(dst[j])) for j in range(m))
    compare(gx, gx_ref, td, f"bwd_multi m={m} {dtype}", extra_tol=4e-7 * mag)
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
    compare(xd.grad, d1 + 2.0 * d2, torch.float32, "multi autograd", extra_tol=1e-5 * np.maximum(1, np.abs(x64)))


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
            rel = 2e-6 * np.maximum(1.0, np.abs(x64)) ** 2
            compare(y, y_ref, td, f"random {prog!r} y {dtype}", extra_tol=rel * np.maximum(1.0, np.abs(y_ref)))
            compare(d, d_ref, td, f"random {prog!r} dydx {dtype}", extra_tol=rel * np.maximum(1.0, np.abs(d_ref)))
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
        lim = {"exp": 10.0, "swish_table1": 60.0}.get(name, 100.0)
        x = x_all[torch.isfinite(xf) & (xf.abs() <= lim)].contiguous()
        x64 = inputs.storage_to_f64(x)
        y_ref, d_ref = chain.eval_chain(nfad.nfad_chain_program(cid), x64)
        xd = x.to(DEV)
        y = torch.full_like(xd, float("nan"))
        d = torch.full_like(xd, float("nan"))
        nfad.nfad_chain_fwd(cid, xd, y, d)
        rel = 2e-6 * np.maximum(1.0, np.abs(x64))
        sy = compare(y, y_ref, td, f"exhaustive chain {name} y {dtype}", extra_tol=rel * np.maximum(1.0, np.abs(y_ref)))
        sd = compare(d, d_ref, td, f"exhaustive chain {name} dydx {dtype}", extra_tol=rel * np.maximum(1.0, np.abs(d_ref)))
        report[name] = (round(sy["max_ulp"], 2), round(sd["max_ulp"], 2))
    print(f"\n[exhaustive chains {dtype}] max ulp (y, dydx): {report}")

"""The chain detector's state machine and program builder, on host tensors (recording only:
nothing is executed, and materialising a chain on the host must fail loudly)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import chain as ochain
from paper_2209_10778_amd import trace


def test_classify_is_the_papers_four_states():
    assert [trace.classify(a, b) for a in (False, True) for b in (False, True)] == ["NN", "NY", "YN", "YY"]


def active(states):
    return [s for s in states if s != "NN"]


def test_user_written_mish_is_one_chain():
    x = torch.randn(5, 7)
    with trace.fuse(require_cuda=False) as t:
        y = x * torch.tanh(F.softplus(x))
    assert isinstance(y, trace.Lazy) and y.shape == x.shape and y.dtype == x.dtype
    assert " ".join(y._program) == "x x softplus tanh *"
    assert active(t.states) == ["NY", "YY", "YY"]          # softplus begins, tanh and mul continue
    assert t.kernels == []                                  # nothing has run


def test_user_written_gelu_tanh_program_evaluates_to_gelu():
    import numpy as np
    import oracle
    x = torch.randn(64)
    with trace.fuse(require_cuda=False):
        y = 0.5 * x * (1.0 + torch.tanh(0.7978845608028654 * (x + 0.044715 * x ** 3)))
    prog = " ".join(y._program)
    xs = np.linspace(-6, 6, 241)
    v, d = ochain.eval_chain(prog, xs)
    vr, dr = oracle.fwd(oracle.GELU_TANH, xs)
    assert np.max(np.abs(v - vr)) < 1e-13 and np.max(np.abs(d - dr)) < 1e-13


def test_builtin_functionals_expand_to_primitives():
    x = torch.randn(8)
    with trace.fuse(require_cuda=False):
        progs = {
            "silu": " ".join(F.silu(x)._program),
            "mish": " ".join(F.mish(x)._program),
            "square": " ".join(torch.square(x)._program),
            "rsub": " ".join((1 - x)._program),
            "rdiv": " ".join((2 / x)._program),
            "neg": " ".join((-x)._program),
            "sigmoid_method": " ".join(x.sigmoid()._program),
        }
    assert progs == {"silu": "x x sigmoid *", "mish": "x x softplus tanh *", "square": "x x *",
                     "rsub": "1.0 x -", "rdiv": "2.0 x /", "neg": "x neg", "sigmoid_method": "x sigmoid"}


def test_piecewise_functionals_expand_to_primitives():
    x = torch.randn(8)
    with trace.fuse(require_cuda=False):
        progs = {
            "relu": " ".join(F.relu(x)._program),
            "abs": " ".join(x.abs()._program),
            "elu": " ".join(F.elu(x, alpha=0.5)._program),
            "hardswish": " ".join(F.hardswish(x)._program),
            "softsign": " ".join(F.softsign(x)._program),
            "clamp": " ".join(torch.clamp(x, -1, 2.5)._program),
            "clamp_kw": " ".join(x.clamp(min=0.0)._program),
            "relu6": " ".join(F.relu6(x)._program),
        }
    assert progs == {"relu": "x relu", "abs": "x abs", "elu": "x relu 0.5 x 0 min exp 1 - * +",
                     "hardswish": "x x 3 + 0 max 6 min * 6 /", "softsign": "x 1 x abs + /",
                     "clamp": "x -1.0 max 2.5 min", "clamp_kw": "x 0.0 max", "relu6": "x 0 max 6 min"}


def test_binary_operator_needs_the_same_source():
    x, w = torch.randn(4, 4), torch.randn(4, 4)
    with trace.fuse(require_cuda=False) as t:
        a = torch.tanh(x)                 # NY
        b = torch.sigmoid(w)              # NY (another chain, another source)
        assert isinstance(a, trace.Lazy) and isinstance(b, trace.Lazy) and a._source is x and b._source is w
        c = a * b                         # different sources: nfad operator, YN for both chains
    assert active(t.states)[:3] == ["NY", "NY", "YN"]
    # each chain is ONE plain primitive: run natively, nothing fused (Sec. IV-B "Efficiency")
    assert t.kernels == [] and t.native_singles == 2 and not isinstance(c, trace.Lazy)
    assert torch.equal(c, torch.tanh(x) * torch.sigmoid(w))


def test_a_longer_chain_on_the_host_has_no_fallback():
    x = torch.randn(4, 4)
    with trace.fuse(require_cuda=False):
        a = torch.tanh(x) * x             # two operators: a real chain
        with pytest.raises((ValueError, RuntimeError, ImportError)):
            a.sum()                       # materialising needs the GPU library: no CPU fallback


def test_single_operator_rule():
    x = torch.randn(16)
    with trace.fuse(require_cuda=False) as t:
        assert torch.equal((x * 0.125).sum(), (x * 0.125).sum())          # lone x * c: native
        assert t.native_singles == 2 and t.kernels == []
        lone = F.silu(x)                                                  # a fused functional: replaced
        assert isinstance(lone, trace.Lazy) and lone._nops == 1 and lone._native is None
        two = torch.exp(-x)
        assert two._nops == 2 and two._native is None


def test_non_fad_operator_is_passed_through_untouched():
    x = torch.randn(3, 3)
    with trace.fuse(require_cuda=False) as t:
        y = torch.cumsum(x, 0) @ x        # neither is a fad primitive
    assert not isinstance(y, trace.Lazy) and active(t.states) == []
    assert torch.equal(y, torch.cumsum(x, 0) @ x)


def test_unsupported_variants_do_not_start_a_chain():
    x = torch.randn(6)
    xi = torch.arange(6)
    with trace.fuse(require_cuda=False):
        assert not isinstance(F.softplus(x, threshold=5.0), trace.Lazy)  # the linear branch would be visible
        assert not isinstance(F.leaky_relu(x, inplace=True), trace.Lazy)
        assert not isinstance(torch.tanh(xi.double()), trace.Lazy)      # float64 is not a storage type here
        assert not isinstance(x ** 2.5, trace.Lazy)
        assert not isinstance(x + torch.randn(1), trace.Lazy)           # broadcasting a different tensor
        assert not isinstance(x ** 9, trace.Lazy) and not isinstance(x ** True, trace.Lazy)
        assert isinstance(x ** 2, trace.Lazy) and isinstance(torch.pow(x, 3.0), trace.Lazy)


FUNCTIONALS = {
    "softplus_beta": (lambda t: F.softplus(t, beta=2.5), False),
    "leaky_relu": (lambda t: F.leaky_relu(t, 0.2), False),
    "leaky_relu_default": (lambda t: F.leaky_relu(t), False),
    "selu": (F.selu, False),
    "celu": (lambda t: F.celu(t, alpha=0.7), False),
    "hardtanh": (lambda t: F.hardtanh(t, -0.5, 1.5), False),
    "hardsigmoid": (F.hardsigmoid, False),
    "logsigmoid": (F.logsigmoid, False),
    "tanhshrink": (F.tanhshrink, False),
    "clamp_min": (lambda t: torch.clamp_min(t, -0.25), False),
    "clamp_max": (lambda t: t.clamp_max(0.75), False),
    "expm1": (torch.expm1, False),
    "erfc": (torch.erfc, False),
    "reciprocal": (torch.reciprocal, True),
    "rsqrt": (torch.rsqrt, True),
    "log1p": (torch.log1p, True),
    "gelu_tanh": (lambda t: F.gelu(t, approximate="tanh"), False),
    "elu": (lambda t: F.elu(t, alpha=1.3), False),
    "hardswish": (F.hardswish, False),
    "relu6": (F.relu6, False),
    "pow_float_3": (lambda t: torch.pow(t, 3.0), False),
    "pow_int_4": (lambda t: t ** 4, False),
    "pow_half": (lambda t: t ** 0.5, True),
    "pow_minus_one": (lambda t: torch.pow(t, -1), True),
    "pow_minus_half": (lambda t: t.pow(-0.5), True),
    "pow_of_a_chain": (lambda t: torch.pow(torch.tanh(t), 2.0), False),
}


@pytest.mark.parametrize("name", sorted(FUNCTIONALS))
def test_recorded_program_of_a_functional_means_what_the_framework_computes(name):
    """The detector's expansion of each functional into primitives, evaluated by the fp64 chain
    interpreter, against the framework's own fp64 value and autograd gradient."""
    from oracle import chain
    fn, positive = FUNCTIONALS[name]
    g = torch.Generator().manual_seed(11)
    x32 = torch.randn(4001, generator=g) * 2.5
    if positive:
        x32 = x32.abs() + 0.25
    with trace.fuse(require_cuda=False):
        lazy = fn(x32)
        assert isinstance(lazy, trace.Lazy), name
        program = " ".join(lazy._program)
    x64 = x32.double().requires_grad_(True)
    y64 = fn(x64)
    (d64,) = torch.autograd.grad(y64.sum(), x64)
    y, d = chain.eval_chain(program, x32.double().numpy())
    # 1e-7: the framework's own fp64 kernels carry a few fp32 constants (1/6, the softplus threshold)
    assert np.allclose(y, y64.detach().numpy(), rtol=1e-7, atol=1e-7), (name, program)
    assert np.allclose(d, d64.numpy(), rtol=1e-7, atol=1e-7), (name, program)


# ------------------------------------------------------------------ eager semantics under mutation
@pytest.fixture
def interpreted_chains(monkeypatch):
    """Chains resolve through the fp64 interpreter instead of the GPU library (host tests of the
    detector's bookkeeping only: which program runs on which values)."""
    from paper_2209_10778_amd import autograd as A

    def one(x, prog):
        v, _ = ochain.eval_chain(prog, x.detach().double().numpy())
        return torch.from_numpy(v).to(x.dtype).view(x.shape)

    monkeypatch.setattr(A, "chain", one)
    monkeypatch.setattr(A, "chain_multi", lambda x, progs: tuple(one(x, p) for p in progs))


def test_in_place_operator_on_a_resolved_chain_leaves_no_stale_program(interpreted_chains):
    x = torch.tensor([0.5, -0.7, 2.0, -3.0])
    with trace.fuse(require_cuda=False) as t:
        y = F.silu(x)
        y.mul_(2)                         # resolves y (YN) and writes the value in place
        z = torch.tanh(y)                 # must see 2 * silu(x): y is an ordinary tensor now
        out = z + torch.zeros(4)          # a non-fad use
    assert t.kernels == ["x x sigmoid *"]
    assert torch.allclose(out, torch.tanh(2 * F.silu(x)), atol=1e-6)


def test_in_place_operator_on_a_source_resolves_the_chains_recorded_over_it(interpreted_chains):
    x = torch.tensor([0.5, -0.7, 2.0, -3.0])
    x0 = x.clone()
    with trace.fuse(require_cuda=False) as t:
        y = torch.tanh(x) * x
        assert isinstance(y, trace.Lazy) and t.kernels == []
        x.add_(1)                         # the chain takes its value BEFORE the write
        assert t.kernels == ["x tanh x *"]
        out = y + torch.zeros(4)
    assert torch.allclose(out, torch.tanh(x0) * x0, atol=1e-6) and torch.equal(x, x0 + 1)
    # also through an augmented assignment and an out= argument
    for write in (lambda v: v.__iadd__(1.0), lambda v: torch.add(v, 1.0, out=v), lambda v: v.copy_(torch.ones(4))):
        x = x0.clone()
        with trace.fuse(require_cuda=False) as t:
            y = torch.exp(-x) * x
            write(x)
            out = y + torch.zeros(4)
        assert torch.allclose(out, torch.exp(-x0) * x0, atol=1e-6)


def test_source_modified_behind_the_detectors_back_is_an_error(interpreted_chains):
    x = torch.tensor([0.5, -0.7, 2.0])
    with trace.fuse(require_cuda=False):
        y = torch.tanh(x) * x
    x.add_(1)                             # outside the context: nothing can intercept this
    with pytest.raises(RuntimeError, match="modified in place"):
        y.sum()
    base = torch.tensor([0.5, -0.7, 2.0])
    with trace.fuse(require_cuda=False):
        y = torch.tanh(base) * base
        base.view(-1)[0:1].zero_()        # through a view: caught by the version counter
        with pytest.raises(RuntimeError, match="modified in place"):
            y.sum()


def test_chains_over_one_source_waiting_to_be_consumed_are_resolved_together(interpreted_chains):
    """R^1 -> R^M: two outputs recorded before the first non-fad use form ONE group; the shared
    prefix h is not an output; a chain recorded after the group was resolved gets its own kernel."""
    x = torch.tensor([0.5, -0.7, 2.0, -3.0])
    with trace.fuse(require_cuda=False) as t:
        h = torch.tanh(x)                 # continued by both chains below: a prefix, not an output
        a = h * x
        b = torch.sigmoid(h)
        sa = a.sum()                      # first non-fad use: a and b are resolved by one kernel
        assert t.kernels == ["x tanh x * ; x tanh sigmoid"] and b._value is not None and h._value is None
        sb = b.sum()                      # already resolved: no further kernel
        c = torch.exp(-x) * x
        sc = c.sum()
    assert t.kernels == ["x tanh x * ; x tanh sigmoid", "x neg exp x *"]
    assert torch.allclose(sa, (torch.tanh(x) * x).sum()) and torch.allclose(sb, torch.sigmoid(torch.tanh(x)).sum())
    assert torch.allclose(sc, (torch.exp(-x) * x).sum())


def test_numbers_fp32_cannot_hold_do_not_enter_a_chain():
    x = torch.randn(6)
    with trace.fuse(require_cuda=False):
        for c in (float("nan"), float("inf"), 1e39, -1e39):
            assert not isinstance(x * c, trace.Lazy)
        assert not isinstance(torch.clamp(x, max=float("inf")), trace.Lazy)
        with pytest.raises(OverflowError):
            x * 10 ** 400                     # what the framework itself does with such a number
        ok = x * 3.0e38
        assert isinstance(ok, trace.Lazy)
        ok._value = x                         # nothing to resolve on leaving the context

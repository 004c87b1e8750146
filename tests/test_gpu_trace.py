"""The chain detector end to end on the GPU: user-written PyTorch activations are fused into one
forward kernel each, values and gradients match the oracle, and one tensor is saved."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import chain as ochain
from paper_2209_10778_amd import inputs, trace
from parity import chain_allowance, compare, two_stage_budget

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def active(states):
    return [s for s in states if s != "NN"]


def _x(n, seed, dtype="f32"):
    return inputs.to_storage(np.clip(inputs.gaussian(n, 2.0, seed), -9, 9), dtype)


USER_CODE = {
    "mish": (lambda x: x * torch.tanh(F.softplus(x)), oracle.MISH, "x x softplus tanh *"),
    "swish": (lambda x: x * torch.sigmoid(x), oracle.SWISH, "x x sigmoid *"),
    "gelu_tanh": (lambda x: 0.5 * x * (1.0 + torch.tanh(0.7978845608028654 * (x + 0.044715 * x ** 3))),
                  oracle.GELU_TANH, None),
    "gelu_erf": (lambda x: x * 0.5 * (1.0 + torch.erf(x / 1.4142135623730951)), oracle.GELU_ERF, None),
}


@pytest.mark.parametrize("name", sorted(USER_CODE))
def test_user_written_activation_is_fused_and_correct(name):
    fn, kind, program = USER_CODE[name]
    n = 70_001
    x = _x(n, 9000 + kind)
    gy = inputs.to_storage(inputs.gaussian(n, 1.0, 9100 + kind), "f32")
    x64, gy64 = inputs.storage_to_f64(x), inputs.storage_to_f64(gy)
    xd = x.to(DEV).requires_grad_(True)
    with trace.fuse() as t:
        y = fn(xd)
        assert isinstance(y, trace.Lazy) and t.kernels == []       # nothing executed yet
        z = y.reshape(-1)                                          # non-fad use: the chain ends (YN)
    assert len(t.kernels) == 1 and (program is None or t.kernels[0] == program)
    # one or more branches begin at the source (NY), continue and merge (YY), and the chain ends once (YN)
    st = active(t.states)
    assert st[0] == "NY" and st[-1] == "YN" and set(st[1:-1]) <= {"NY", "YY"} and st.count("YN") == 1
    saved = z.grad_fn.next_functions[0][0].saved_tensors if z.grad_fn.name() != "_FadChainBackward" else z.grad_fn.saved_tensors
    assert len(saved) == 1                                          # dydx only
    z.backward(gy.to(DEV))
    y_ref, d_ref = oracle.fwd(kind, x64)
    compare(z.detach(), y_ref, torch.float32, f"traced {name} y", extra_tol=chain_allowance(x64, y_ref))
    compare(xd.grad, gy64 * d_ref, torch.float32, f"traced {name} grad",
            extra_tol=two_stage_budget(gy64, d_ref, gy64 * d_ref, torch.float32, chain_allowance(x64, d_ref)))


def test_chain_resolves_after_the_context_has_closed():
    x = _x(10_000, 9200).to(DEV).requires_grad_(True)
    with trace.fuse() as t:
        y = F.silu(x)
    assert isinstance(y, trace.Lazy) and t.kernels == []
    loss = y.sum()                    # outside the context: still resolves through the recorded chain
    loss.backward()
    assert t.kernels == ["x x sigmoid *"]
    x64 = inputs.storage_to_f64(x.detach().cpu())
    _, d_ref = oracle.fwd(oracle.SWISH, x64)
    compare(x.grad, d_ref, torch.float32, "late resolve grad", extra_tol=chain_allowance(x64, d_ref))


def test_two_consumers_of_one_source_give_two_outputs():
    """R^1 -> R^M: one source, two chains ending in different non-fad operators."""
    x = _x(20_000, 9300).to(DEV).requires_grad_(True)
    x64 = inputs.storage_to_f64(x.detach().cpu())
    with trace.fuse() as t:
        h = torch.tanh(x)             # shared prefix
        a = (h * x).sum()             # chain 1: x tanh x *
        b = torch.sigmoid(h).sum()    # chain 2: x tanh sigmoid
    (a + b).backward()
    assert sorted(t.kernels) == sorted(["x tanh x *", "x tanh sigmoid"])
    _, d1 = ochain.eval_chain("x tanh x *", x64)
    _, d2 = ochain.eval_chain("x tanh sigmoid", x64)
    compare(x.grad, d1 + d2, torch.float32, "merged tangents",
            extra_tol=chain_allowance(x64, d1) + chain_allowance(x64, d2))


def test_two_outputs_recorded_before_the_first_use_are_one_kernel_with_two_saved_tangents():
    """R^1 -> R^M inside the detector (Sec. IV-A, IV-B): both chains are recorded before anything
    consumes them, so ONE forward kernel reads x once and writes both values and both tangents,
    and ONE backward kernel merges the two upstream gradients at the source."""
    n = 20_000
    x = _x(n, 9350).to(DEV).requires_grad_(True)
    x64 = inputs.storage_to_f64(x.detach().cpu())
    w1 = inputs.to_storage(inputs.gaussian(n, 1.0, 9351), "f32")
    w2 = inputs.to_storage(inputs.gaussian(n, 1.0, 9352), "f32")
    with trace.fuse() as t:
        h = torch.tanh(x)             # shared prefix: continued twice, never an output itself
        a = h * x                     # output 1: x tanh x *
        b = torch.sigmoid(h)          # output 2: x tanh sigmoid
        assert t.kernels == []
        la = (a * w1.to(DEV)).sum()   # first non-fad use (a different source): both chains resolve here
        assert t.kernels == ["x tanh x * ; x tanh sigmoid"]
        lb = (b * w2.to(DEV)).sum()
        assert len(t.kernels) == 1
    node = a.materialize().grad_fn
    assert node is b.materialize().grad_fn and len(node.saved_tensors) == 2       # one node, M = 2 tangents
    (la + lb).backward()
    (y1, d1), (y2, d2) = ochain.eval_chain("x tanh x *", x64), ochain.eval_chain("x tanh sigmoid", x64)
    compare(a.materialize().detach(), y1, torch.float32, "fused output 1", extra_tol=chain_allowance(x64, y1))
    compare(b.materialize().detach(), y2, torch.float32, "fused output 2", extra_tol=chain_allowance(x64, y2))
    g1, g2 = inputs.storage_to_f64(w1), inputs.storage_to_f64(w2)
    g_ref = g1 * d1 + g2 * d2
    compare(x.grad, g_ref, torch.float32, "merged gradient",
            extra_tol=two_stage_budget(g1, d1, g_ref, torch.float32, chain_allowance(x64, d1))
            + two_stage_budget(g2, d2, g_ref, torch.float32, chain_allowance(x64, d2)))


def test_in_place_writes_keep_eager_semantics_on_the_gpu():
    """The two ways an in-place operator could meet a deferred chain (see the host tests), end to end."""
    x = _x(10_000, 9360).to(DEV)
    x0 = x.clone()
    x64 = inputs.storage_to_f64(x0.cpu())
    with trace.fuse() as t:
        y = F.silu(x)
        y.mul_(2)                                  # y resolves, then is written in place
        z = torch.tanh(y) * y                      # a new chain over the written tensor
        u = torch.tanh(x) * x                      # a chain over x ...
        x.add_(1)                                  # ... takes its value before x changes
        out_z, out_u = z + 0 * x0, u + 0 * x0
    s_ref = ochain.eval_chain("x x sigmoid *", x64)[0]
    y_ref = 2 * s_ref
    z_ref, dz_dy = ochain.eval_chain("x tanh x *", y_ref)
    u_ref = ochain.eval_chain("x tanh x *", x64)[0]
    # two stages: y carries its own bar and allowance (doubled by the in-place scaling), which the
    # second chain's derivative scales; then the second chain's own allowance
    from parity import tolerance
    tol_y = 2 * (tolerance(torch.from_numpy(s_ref), torch.float32).numpy() + chain_allowance(x64, s_ref))
    compare(out_z, z_ref, torch.float32, "chain over a written tensor",
            extra_tol=np.abs(dz_dy) * tol_y + chain_allowance(y_ref, z_ref))
    compare(out_u, u_ref, torch.float32, "chain resolved before its source was written",
            extra_tol=chain_allowance(x64, u_ref))
    assert torch.equal(x, x0 + 1)


def test_mixing_sources_ends_both_chains():
    x = _x(5_000, 9400).to(DEV)
    w = _x(5_000, 9401).to(DEV)
    with trace.fuse() as t:
        y = torch.tanh(x * 0.5) * torch.sigmoid(-w)     # operands from different sources: nfad operator
    assert not isinstance(y, trace.Lazy)
    assert sorted(t.kernels) == ["x 0.5 * tanh", "x neg sigmoid"]
    ref = np.tanh(0.5 * inputs.storage_to_f64(x.cpu())) * (1 / (1 + np.exp(inputs.storage_to_f64(w.cpu()))))
    xw = np.maximum(np.abs(inputs.storage_to_f64(x.cpu())), np.abs(inputs.storage_to_f64(w.cpu())))
    compare(y, ref, torch.float32, "mixed sources", extra_tol=chain_allowance(xw, ref))   # two chains and a product
    with trace.fuse() as t:                             # each side a lone primitive: both run natively
        y = torch.tanh(x) * torch.sigmoid(w)
    assert t.kernels == [] and t.native_singles == 2
    assert torch.equal(y, torch.tanh(x) * torch.sigmoid(w))


def test_a_small_network_with_user_written_mish_trains_a_step():
    torch.manual_seed(0)
    lin1, lin2 = torch.nn.Linear(64, 256).to(DEV), torch.nn.Linear(256, 8).to(DEV)
    x = torch.randn(32, 64, device=DEV)

    def net(v):
        h = lin1(v)
        return lin2(h * torch.tanh(F.softplus(h)))

    with trace.fuse() as t:
        net(x).square().mean().backward()
    assert t.kernels == ["x x softplus tanh *"]     # the activation; the loss's lone square runs natively
    assert t.native_singles == 1
    g1 = [p.grad.clone() for p in list(lin1.parameters()) + list(lin2.parameters())]
    for p in list(lin1.parameters()) + list(lin2.parameters()):
        p.grad = None
    net(x).square().mean().backward()              # plain PyTorch, no fusion
    g2 = [p.grad for p in list(lin1.parameters()) + list(lin2.parameters())]
    for a, b in zip(g1, g2):
        assert torch.allclose(a, b, rtol=2e-4, atol=2e-6)


FRAMEWORK_CODE = {
    "selu_gate": lambda x: F.selu(x) * torch.sigmoid(1.702 * x),
    "leaky_logsigmoid": lambda x: F.leaky_relu(x, 0.1) + F.logsigmoid(x),
    "celu_hardtanh": lambda x: F.celu(x, alpha=0.5) - F.hardtanh(x, -2.0, 2.0) * 0.25,
    "softplus_beta": lambda x: F.softplus(x, beta=3.0) * torch.tanh(x),
    "hardsigmoid_swish": lambda x: x * F.hardsigmoid(x) + torch.expm1(-x.abs()),
    "tanhshrink_erfc": lambda x: F.tanhshrink(x) * torch.erfc(0.5 * x).clamp_max(1.5),
}


@pytest.mark.parametrize("name", sorted(FRAMEWORK_CODE))
def test_framework_functionals_fuse_into_one_kernel_and_match_the_interpreter(name):
    """Compositions of the framework's own functionals: one fused kernel, value and gradient
    against the fp64 interpreter run on the program the detector recorded (the programs'
    meaning is pinned against the framework's fp64 results on the host)."""
    fn = FRAMEWORK_CODE[name]
    n = 50_003
    x = _x(n, 9300 + len(name))
    gy = inputs.to_storage(inputs.gaussian(n, 1.0, 9400 + len(name)), "f32")
    x64, gy64 = inputs.storage_to_f64(x), inputs.storage_to_f64(gy)
    xd = x.to(DEV).requires_grad_(True)
    with trace.fuse() as t:
        y = fn(xd)
        assert isinstance(y, trace.Lazy) and t.kernels == []
        z = y.reshape(-1)
    assert len(t.kernels) == 1
    z.backward(gy.to(DEV))
    y_ref, d_ref = ochain.eval_chain(t.kernels[0], x64)
    compare(z.detach(), y_ref, torch.float32, f"traced {name} y", extra_tol=chain_allowance(x64, y_ref))
    compare(xd.grad, gy64 * d_ref, torch.float32, f"traced {name} grad",
            extra_tol=two_stage_budget(gy64, d_ref, gy64 * d_ref, torch.float32, chain_allowance(x64, d_ref)))
    # and against the framework's own eager result in fp32 (loose: the framework's fp32 error is its own)
    x_e = x.to(DEV).requires_grad_(True)
    y_e = fn(x_e)
    y_e.backward(gy.to(DEV))
    assert torch.allclose(z.detach(), y_e.detach(), rtol=2e-5, atol=2e-5)
    assert torch.allclose(xd.grad, x_e.grad, rtol=2e-4, atol=2e-5)


def test_whole_layers_under_the_detector_match_eager_and_fuse_only_the_activations():
    """A transformer encoder layer and a ResNet bottleneck written with composite activations,
    run unchanged under the detector: same result and gradients as eager execution, one fused
    kernel per activation call, lone primitives elsewhere in the layer (q * scale, ...) left native."""
    from paper_2209_10778_amd import footprint as fp
    torch.manual_seed(3)
    enc = torch.nn.TransformerEncoderLayer(64, 4, 128, dropout=0.0, activation=fp.Act("gelu_tanh", "composite"),
                                           batch_first=True).to(DEV)
    res = fp.resnet_bottleneck(16, 8, "mish", "composite").to(DEV)
    for model, x, n_act in ((enc, torch.randn(5, 12, 64, device=DEV), 1), (res, torch.randn(3, 16, 10, 10, device=DEV), 3)):
        xe = x.clone().requires_grad_(True)
        ye = model(xe)
        ye.square().mean().backward()
        ge = [p.grad.clone() for p in model.parameters()]
        model.zero_grad(set_to_none=True)
        xt = x.clone().requires_grad_(True)
        with trace.fuse() as t:
            yt = model(xt)
        if isinstance(yt, trace.Lazy):
            yt = yt.materialize()
        yt.square().mean().backward()
        assert len(t.kernels) == n_act, t.kernels
        assert torch.allclose(yt, ye, rtol=1e-4, atol=1e-5)
        assert torch.allclose(xt.grad, xe.grad, rtol=1e-3, atol=1e-6)
        for p, g in zip(model.parameters(), ge):
            assert torch.allclose(p.grad, g, rtol=1e-3, atol=1e-5)
        model.zero_grad(set_to_none=True)

"""The autograd front end: values and input gradients against the oracle, and what it saves."""
import numpy as np
import pytest
import torch

import oracle
from oracle import chain as ochain
import paper_2209_10778_amd as nfad
from paper_2209_10778_amd import autograd as A
from paper_2209_10778_amd import inputs
from parity import chain_allowance, compare, saveall_two_stage_budget, two_stage_budget

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
KIND = {"gelu_tanh": 0, "gelu_erf": 1, "swish": 2, "mish": 3}


@pytest.mark.parametrize("mode", ["fad", "recompute", "saveall"])
@pytest.mark.parametrize("name", sorted(KIND))
def test_value_and_gradient(name, mode):
    shape = (7, 33, 129)
    n = int(np.prod(shape))
    x = inputs.to_storage(inputs.gaussian(n, 1.5, 8100 + KIND[name]), "f32")
    gy = inputs.to_storage(inputs.gaussian(n, 1.0, 8200 + KIND[name]), "f32")
    x64, gy64 = inputs.storage_to_f64(x), inputs.storage_to_f64(gy)
    y_ref, d_ref = oracle.fwd(KIND[name], x64)
    xd = x.to(DEV).view(shape).requires_grad_(True)
    y = A.activation(xd, name, mode=mode)
    assert y.shape == xd.shape
    y.backward(gy.to(DEV).view(shape))
    compare(y.detach(), y_ref, torch.float32, f"{name} {mode} y")
    g_ref = gy64 * d_ref
    # fad and save-all: the backward pass consumes what the GPU forward pass stored (two-stage
    # budgets); recomputation derives gy * f'(x) in one kernel (the stated bar, no allowance)
    extra = {"fad": lambda: two_stage_budget(gy64, d_ref, g_ref, torch.float32),
             "saveall": lambda: saveall_two_stage_budget(KIND[name], gy64, x64, torch.float32),
             "recompute": lambda: None}[mode]()
    st = compare(xd.grad, g_ref, torch.float32, f"{name} {mode} grad", extra_tol=extra)
    print(f"\n[autograd {name} {mode}] grad err / stated bar {st['max_over_bar']:.3f}")


def test_only_one_tensor_is_saved_by_fad():
    x = torch.randn(1 << 16, device=DEV, requires_grad=True)
    for name in KIND:
        y = A.activation(x, name)
        saved = y.grad_fn.saved_tensors
        assert len(saved) == 1 and saved[0].data_ptr() != x.data_ptr()      # dydx, not x
        k = nfad.nfad_saveall_num_saved(KIND[name])
        ys = A.activation(x, name, mode="saveall")
        assert len(ys.grad_fn.saved_tensors) == k
        yr = A.activation(x, name, mode="recompute")
        rec = yr.grad_fn.saved_tensors
        assert len(rec) == 1 and rec[0].data_ptr() == x.data_ptr()          # x itself


def test_chain_front_end_builtin_and_compiled():
    n = 50_001
    x = inputs.to_storage(np.clip(inputs.gaussian(n, 2.0, 8300), -9, 9), "f32")
    x64 = inputs.storage_to_f64(x)
    for spec, prog in (("tanhshrink", "x x tanh -"), ("x sigmoid x tanh *", "x sigmoid x tanh *")):
        xd = x.to(DEV).requires_grad_(True)
        y = A.chain(xd, spec)
        y.sum().backward()
        y_ref, d_ref = ochain.eval_chain(prog, x64)
        compare(y.detach(), y_ref, torch.float32, f"chain {spec} y", extra_tol=chain_allowance(x64, y_ref))
        compare(xd.grad, d_ref, torch.float32, f"chain {spec} grad", extra_tol=chain_allowance(x64, d_ref))


def test_module_in_a_small_network_trains_a_step():
    torch.manual_seed(0)
    net = torch.nn.Sequential(torch.nn.Linear(64, 256), A.Activation("mish"), torch.nn.Linear(256, 8)).to(DEV)
    x = torch.randn(32, 64, device=DEV)
    loss = net(x).square().mean()
    loss.backward()
    assert all(p.grad is not None and bool(torch.isfinite(p.grad).all()) for p in net.parameters())
    # same network with torch's own Mish gives the same gradients to fp32 accuracy
    ref = torch.nn.Sequential(torch.nn.Linear(64, 256), torch.nn.Mish(), torch.nn.Linear(256, 8)).to(DEV)
    ref.load_state_dict({k.replace("1.", "1."): v for k, v in net.state_dict().items()})
    ref(x).square().mean().backward()
    for p, q in zip(net.parameters(), ref.parameters()):
        assert torch.allclose(p.grad, q.grad, rtol=2e-4, atol=2e-6)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_non_contiguous_and_16bit_inputs(dtype):
    td = inputs.TORCH_DTYPE[dtype]
    a = inputs.to_storage(inputs.gaussian(64 * 48, 1.5, 8400), dtype).view(64, 48)
    xt = a.to(DEV).t()                                  # a non-contiguous view, logical shape (48, 64)
    assert not xt.is_contiguous()
    xd = xt.detach().requires_grad_(True)
    y = A.mish(xd)
    assert y.shape == xd.shape
    gy = inputs.to_storage(inputs.gaussian(48 * 64, 1.0, 8401), dtype).view(48, 64).to(DEV)
    y.backward(gy)
    x64 = inputs.storage_to_f64(a.t().contiguous())
    y_ref, d_ref = oracle.fwd(oracle.MISH, x64)
    compare(y.detach().contiguous(), y_ref, td, f"non-contiguous y {dtype}")
    gy64 = inputs.storage_to_f64(gy.cpu()).reshape(-1)
    g_ref = gy64 * d_ref
    assert xd.grad.shape == xd.shape
    # two roundings (dydx, then the product), scaled by |gy|
    compare(xd.grad.contiguous(), g_ref, td, f"non-contiguous grad {dtype}",
            extra_tol=two_stage_budget(gy64, d_ref, g_ref, td))


def test_compiled_chain_cache_is_bounded(monkeypatch):
    """Chains that bake in a changing constant must not accumulate kernels without limit: the
    front end keeps the most recently used programs and releases the rest."""
    import paper_2209_10778_amd as nfad
    import collections
    monkeypatch.setattr(A, "_compiled", collections.OrderedDict())     # a fresh table for this test
    monkeypatch.setattr(A, "MAX_COMPILED", 3)
    x = torch.randn(1000, device=DEV)
    ids = []
    for k in range(6):
        prog = f"x {1.5 + k} * tanh x *"
        y = A.chain(x, prog)
        ids.append(A._compiled[prog])
        assert torch.allclose(y, torch.tanh(x * (1.5 + k)) * x, rtol=1e-5, atol=1e-6)
    assert len(A._compiled) <= A.MAX_COMPILED
    live = set(A._compiled.values())
    assert len(live) == 3 and all(nfad.nfad_chain_name(i) is not None for i in live)
    assert len(set(ids)) < len(ids)                                     # released ids were handed out again
    assert len({nfad.nfad_chain_kernel(i) for i in live}) == 1          # one kernel serves every constant
    y = A.chain(x, "x 1.5 * tanh x *")                                  # an evicted program is accepted again
    assert torch.allclose(y, torch.tanh(x * 1.5) * x, rtol=1e-5, atol=1e-6)

"""Full-size parity on the five benchmark configurations, in the launch configuration bench.py
times: every element of every output is compared with the fp64 oracle (OpenMP makes the full
tensors affordable), and the outlier configuration must produce no NaN/Inf anywhere."""
import numpy as np
import pytest
import torch

import oracle
import paper_2209_10778_amd as nfad
from paper_2209_10778_amd import inputs
from parity import compare, tolerance

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _fwd_bwd_case(cfg, spec, kind, dtype, flat_abs=None, baselines=False):
    td = inputs.TORCH_DTYPE[dtype]
    tag = f"{cfg.name} / {nfad.KIND_NAMES[kind]} / {dtype} / {list(spec.shape)}"
    print(f"\n[case] {tag}", flush=True)
    x = inputs.make_x(cfg, spec, dtype)
    gy = inputs.make_gy(cfg, spec, dtype)
    x64 = inputs.storage_to_f64(x)
    gy64 = inputs.storage_to_f64(gy)
    y_ref, d_ref = oracle.fwd(kind, x64)

    xd, gyd = x.to(DEV), gy.to(DEV)
    y = torch.empty_like(xd)
    d = torch.empty_like(xd)
    gx = torch.empty_like(xd)
    nfad.nfad_fwd(kind, xd, y, d)
    sy = compare(y, y_ref, td, f"{tag} y", flat_abs=flat_abs)
    sd = compare(d, d_ref, td, f"{tag} dydx", flat_abs=flat_abs)

    # backward, stage-wise: both sides consume the oracle's derivative rounded to storage
    dydx_st = inputs.to_storage(d_ref.astype(np.float32), dtype)
    gx_ref = oracle.bwd(gy64, inputs.storage_to_f64(dydx_st))
    nfad.nfad_bwd(gyd, dydx_st.to(DEV), gx)
    sg = compare(gx, gx_ref, td, f"{tag} gx", flat_abs=flat_abs)
    print(f"  y {sy}\n  dydx {sd}\n  gx {sg}", flush=True)

    # end to end (GPU fwd feeding GPU bwd): finite everywhere, and within the two-rounding budget
    nfad.nfad_bwd(gyd, d, gx)
    assert bool(torch.isfinite(gx.float()).all())
    g_e2e = torch.from_numpy(oracle.bwd(gy64, d_ref)).to(DEV)
    err = (gx.double() - g_e2e).abs()
    budget = gyd.double().abs() * tolerance(torch.from_numpy(d_ref).to(DEV), td) + tolerance(g_e2e, td)
    assert bool((err <= budget).all()), f"{tag}: end-to-end gx out of budget"
    del err, budget, g_e2e

    if baselines:
        k = nfad.nfad_saveall_num_saved(kind)
        yb = torch.empty_like(xd)
        nfad.nfad_recompute_fwd(kind, xd, yb)
        compare(yb, y_ref, td, f"{tag} recompute y")
        nfad.nfad_recompute_bwd(kind, gyd, xd, gx)
        rb_ref = oracle.recompute_bwd(kind, gy64, x64)
        rb_tol = np.abs(gy64) * tolerance(torch.from_numpy(d_ref), torch.float32).numpy() \
            + tolerance(torch.from_numpy(rb_ref), td).numpy()
        assert np.all(np.abs(gx.double().cpu().numpy() - rb_ref) <= rb_tol), f"{tag}: recompute gx"
        y_sa, saved_ref = oracle.saveall_fwd(kind, x64)
        saved = [xd] + [torch.empty_like(xd) for _ in range(k - 1)]
        nfad.nfad_saveall_fwd(kind, xd, yb, saved)
        compare(yb, y_sa, td, f"{tag} saveall y")
        for j in range(1, k):
            compare(saved[j], saved_ref[j], td, f"{tag} saveall saved[{j}]")
        saved_st = [x] + [inputs.to_storage(s.astype(np.float32), dtype) for s in saved_ref[1:]]
        sb_ref = oracle.saveall_bwd(kind, gy64, [inputs.storage_to_f64(s) for s in saved_st])
        nfad.nfad_saveall_bwd(kind, gyd, [s.to(DEV) for s in saved_st], gx)
        sb_tol = tolerance(torch.from_numpy(sb_ref), td).numpy() + np.abs(gy64) * 4e-6 * np.maximum(1.0, np.abs(x64))
        assert np.all(np.abs(gx.double().cpu().numpy() - sb_ref) <= sb_tol), f"{tag}: saveall gx"
    torch.cuda.synchronize()
    del xd, gyd, y, d, gx
    torch.cuda.empty_cache()


def test_c1_gelu_tanh_f32_1d():
    cfg = inputs.CONFIGS[0]
    _fwd_bwd_case(cfg, cfg.tensors[0], cfg.kinds[0], "f32", flat_abs=2e-6, baselines=True)


def test_c2_swish_f32_resnet_stage1():
    cfg = inputs.CONFIGS[1]
    _fwd_bwd_case(cfg, cfg.tensors[0], cfg.kinds[0], "f32", flat_abs=2e-6, baselines=True)


@pytest.mark.parametrize("t", [0, 1, 2])
def test_c3_mish_bf16_resnet_tensors(t):
    cfg = inputs.CONFIGS[2]
    _fwd_bwd_case(cfg, cfg.tensors[t], cfg.kinds[0], "bf16")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_c4_gelu_erf_bert_base_ffn_with_baselines(dtype):
    cfg = inputs.CONFIGS[3]
    _fwd_bwd_case(cfg, cfg.tensors[0], cfg.kinds[0], dtype, baselines=True)


@pytest.mark.parametrize("kind", nfad.KINDS)
def test_c5_outlier_stress_bert_large_ffn(kind):
    cfg = inputs.CONFIGS[4]
    _fwd_bwd_case(cfg, cfg.tensors[0], kind, "bf16")

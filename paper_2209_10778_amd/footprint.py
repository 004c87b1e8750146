"""Training-memory footprint of an activation under the three regimes the paper compares
(Sec. V-B, "maximum batch size"), on synthetic blocks shaped like BERT and ResNet-50 layers.

No dataset or trained weight is involved: random weights, random inputs.  For one forward +
backward pass of a block it reports the peak device memory above the resident weights and
input, and the step time, for

  composite : the activation written with framework primitives (the paper's baseline:
              every primitive saves what its own backward needs)
  native    : the framework's own fused activation (saves x)
  saveall / recompute / fad : the libnfad kernels behind autograd Functions
  traced    : the composite code again, unchanged, but run under the chain detector
              (trace.fuse), which finds the chains and fuses them by itself

It also reports the paper's own headline quantity, the maximum batch size under a memory
budget: total peak memory is linear in the batch (weights + a per-sample cost), so it is
measured at two batch sizes, extrapolated to the budget, and the extrapolated batch is then
run once to confirm that it fits.

Run:  python -m paper_2209_10778_amd.footprint [--dtype bf16] [--batch 32] [--time-batch 128] [--budget-gib 16]
                                                 [--whole-models bert|resnet|both]
Prints one JSON line per (block, activation).
"""
from __future__ import annotations

import argparse
import json
import math
import sys
import time

import torch
import torch.nn as nn
import torch.nn.functional as F

from . import autograd as A
from . import trace

_C = math.sqrt(2.0 / math.pi)
COMPOSITE = {
    "gelu_tanh": lambda x: 0.5 * x * (1.0 + torch.tanh(_C * (x + 0.044715 * x * x * x))),
    "gelu_erf": lambda x: 0.5 * x * (1.0 + torch.erf(x * (1.0 / math.sqrt(2.0)))),
    "swish": lambda x: x * torch.sigmoid(x),
    "mish": lambda x: x * torch.tanh(F.softplus(x)),
}
NATIVE = {
    "gelu_tanh": lambda x: F.gelu(x, approximate="tanh"),
    "gelu_erf": lambda x: F.gelu(x),
    "swish": F.silu,
    "mish": F.mish,
}


REGIMES = ("composite", "native", "saveall", "recompute", "fad", "traced")


class Act(nn.Module):
    def __init__(self, kind, regime):
        super().__init__()
        self.kind, self.regime = kind, regime

    def forward(self, x):
        if self.regime in ("composite", "traced"):
            return COMPOSITE[self.kind](x)
        if self.regime == "native":
            return NATIVE[self.kind](x)
        return A.activation(x, self.kind, mode=self.regime)


def bert_ffn(hidden, kind, regime):
    return nn.Sequential(nn.Linear(hidden, 4 * hidden), Act(kind, regime), nn.Linear(4 * hidden, hidden))


def resnet_bottleneck(cin, mid, kind, regime):
    return nn.Sequential(
        nn.Conv2d(cin, mid, 1, bias=False), nn.BatchNorm2d(mid), Act(kind, regime),
        nn.Conv2d(mid, mid, 3, padding=1, bias=False), nn.BatchNorm2d(mid), Act(kind, regime),
        nn.Conv2d(mid, cin, 1, bias=False), nn.BatchNorm2d(cin), Act(kind, regime))


class _Bottleneck(nn.Module):
    def __init__(self, cin, mid, stride, kind, regime):
        super().__init__()
        cout = 4 * mid
        self.body = nn.Sequential(
            nn.Conv2d(cin, mid, 1, bias=False), nn.BatchNorm2d(mid), Act(kind, regime),
            nn.Conv2d(mid, mid, 3, stride=stride, padding=1, bias=False), nn.BatchNorm2d(mid), Act(kind, regime),
            nn.Conv2d(mid, cout, 1, bias=False), nn.BatchNorm2d(cout))
        self.skip = None if (stride == 1 and cin == cout) else nn.Sequential(
            nn.Conv2d(cin, cout, 1, stride=stride, bias=False), nn.BatchNorm2d(cout))
        self.act = Act(kind, regime)

    def forward(self, x):
        return self.act(self.body(x) + (x if self.skip is None else self.skip(x)))


def resnet50(kind, regime):
    """ResNet-50 (stages of 3, 4, 6, 3 bottlenecks) with every ReLU replaced by the activation,
    as in the paper's ResNet experiments (Sec. V); random weights."""
    layers = [nn.Conv2d(3, 64, 7, stride=2, padding=3, bias=False), nn.BatchNorm2d(64), Act(kind, regime),
              nn.MaxPool2d(3, stride=2, padding=1)]
    cin = 64
    for mid, count, stride in ((64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2)):
        for i in range(count):
            layers.append(_Bottleneck(cin, mid, stride if i == 0 else 1, kind, regime))
            cin = 4 * mid
    layers += [nn.AdaptiveAvgPool2d(1), nn.Flatten(), nn.Linear(cin, 1000)]
    return nn.Sequential(*layers)


def bert_base_encoder(kind, regime):
    """Twelve BERT-base encoder layers (hidden 768, 12 heads, FFN 3072, dropout 0.1) without the
    embeddings; random weights."""
    return nn.Sequential(*[nn.TransformerEncoderLayer(768, 12, 3072, dropout=0.1, activation=Act(kind, regime),
                                                      batch_first=True) for _ in range(12)])


class Traced(nn.Module):
    """The model as the user wrote it (composite activations), run under the chain detector."""

    def __init__(self, inner):
        super().__init__()
        self.inner = inner

    def forward(self, x):
        with trace.fuse():
            y = self.inner(x)
        return y.materialize() if isinstance(y, trace.Lazy) else y


def measure(make_block, x, steps=5):
    dev = x.device
    torch.manual_seed(0)
    block = make_block().to(device=dev, dtype=x.dtype)
    if any(isinstance(m, Act) and m.regime == "traced" for m in block.modules()):
        block = Traced(block)
    x = x.clone().requires_grad_(True)
    for _ in range(2):                                   # warm up allocator, autotuners
        block(x).float().square().mean().backward()
        block.zero_grad(set_to_none=True)
        x.grad = None
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    base = torch.cuda.memory_allocated()
    y = block(x)
    torch.cuda.synchronize()
    held = torch.cuda.memory_allocated() - base          # kept alive for backward (incl. the output)
    y.float().square().mean().backward()
    torch.cuda.synchronize()
    peak = torch.cuda.max_memory_allocated() - base
    del y
    block.zero_grad(set_to_none=True)
    x.grad = None
    rounds = []
    for _ in range(3 if steps else 0):                   # median of three rounds of `steps` steps
        t0 = time.perf_counter()
        for _ in range(steps):
            block(x).float().square().mean().backward()
            block.zero_grad(set_to_none=True)
            x.grad = None
        torch.cuda.synchronize()
        rounds.append((time.perf_counter() - t0) / steps * 1e3)
    del block
    return held, peak, sorted(rounds)[1] if rounds else 0.0, base + peak


def _progress(msg):
    print(f"[footprint] {msg}", file=sys.stderr, flush=True)


def total_peak(make_block, x):
    """Peak device memory of one forward + backward, everything included (weights, input, grads)."""
    p = measure(make_block, x, steps=0)[3]
    _progress(f"  batch {x.shape[0]}: total peak {p / 2 ** 30:.2f} GiB")
    return p


def max_batch(make_block, make_x, batch, budget_bytes):
    """Largest batch whose forward + backward fits in budget_bytes: linear model through the
    peaks measured at batch/2 and batch, then one confirming run at the answer."""
    lo, hi = max(1, batch // 2), batch
    p_lo, p_hi = total_peak(make_block, make_x(lo)), total_peak(make_block, make_x(hi))
    per_sample = (p_hi - p_lo) / (hi - lo)
    fixed = p_hi - per_sample * hi
    b = int((budget_bytes - fixed) // per_sample)
    while b > 1 and total_peak(make_block, make_x(b)) > budget_bytes:    # allocator rounding: step down
        b -= max(1, b // 200)
    return b, per_sample


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="bf16", choices=["f32", "f16", "bf16"])
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--whole-models", choices=("bert", "resnet", "both"), default=None,
                    help="BERT-base encoder (12 layers) and/or ResNet-50 instead of single blocks")
    ap.add_argument("--time-batch", type=int, default=0,
                    help="also time one step at this (larger) batch, where the GPU and not the interpreter sets the pace")
    ap.add_argument("--budget-gib", type=float, default=16.0,
                    help="memory budget of the maximum-batch-size figure (0 = skip it)")
    args = ap.parse_args()
    td = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[args.dtype]
    dev = torch.device("cuda:0")
    torch.manual_seed(1)
    budget = int(args.budget_gib * 2 ** 30)
    cases = [
        ("bert_base_ffn seq128", lambda k, r: (lambda: bert_ffn(768, k, r)),
         lambda b: torch.randn(b * 128, 768, device=dev, dtype=td), ("gelu_tanh", "gelu_erf")),
        ("resnet50_bottleneck 56x56", lambda k, r: (lambda: resnet_bottleneck(256, 64, k, r)),
         lambda b: torch.randn(b, 256, 56, 56, device=dev, dtype=td), ("swish", "mish", "gelu_tanh")),
    ]
    if args.whole_models:
        cases = [c for c in [
            ("bert_base_encoder 12 layers seq128", lambda k, r: (lambda: bert_base_encoder(k, r)),
             lambda b: torch.randn(b, 128, 768, device=dev, dtype=td), ("gelu_tanh", "gelu_erf")),
            ("resnet50 224x224", lambda k, r: (lambda: resnet50(k, r)),
             lambda b: torch.randn(b, 3, 224, 224, device=dev, dtype=td), ("swish", "mish", "gelu_tanh")),
        ] if args.whole_models == "both" or c[0].startswith(args.whole_models)]
    for name, maker, make_x, kinds in cases:
        rows = []
        x = make_x(args.batch)
        for kind in kinds:
            row = {"block": name, "activation": kind, "dtype": args.dtype, "batch": args.batch, "regimes": {}}
            for regime in REGIMES:
                held, peak, ms, _ = measure(maker(kind, regime), x)
                _progress(f"{name} {kind} {regime}: batch {args.batch} measured, {ms:.2f} ms/step")
                row["regimes"][regime] = {"held_after_fwd_MiB": round(held / 2 ** 20, 1),
                                          "peak_MiB": round(peak / 2 ** 20, 1), "ms_per_step": round(ms, 3)}
            if args.time_batch:
                xl = make_x(args.time_batch)
                for regime in REGIMES:
                    ms = measure(maker(kind, regime), xl)[2]
                    _progress(f"{name} {kind} {regime}: batch {args.time_batch} timed, {ms:.2f} ms/step")
                    row["regimes"][regime][f"ms_per_step_batch{args.time_batch}"] = round(ms, 3)
                del xl
            r = row["regimes"]
            row["held_composite_over_fad"] = round(r["composite"]["held_after_fwd_MiB"] / r["fad"]["held_after_fwd_MiB"], 3)
            row["held_native_over_fad"] = round(r["native"]["held_after_fwd_MiB"] / r["fad"]["held_after_fwd_MiB"], 3)
            row["time_recompute_over_fad"] = round(r["recompute"]["ms_per_step"] / r["fad"]["ms_per_step"], 3)
            rows.append(row)
        del x
        torch.cuda.empty_cache()
        for row in rows:
            if args.budget_gib > 0:          # nothing else resident while the budget is probed
                mb = {}
                for regime in REGIMES:
                    b, per_sample = max_batch(maker(row["activation"], regime), make_x, args.batch, budget)
                    _progress(f"{name} {row['activation']} {regime}: max batch {b}")
                    mb[regime] = {"max_batch": b, "MiB_per_sample": round(per_sample / 2 ** 20, 3)}
                    torch.cuda.empty_cache()
                row["max_batch"] = {"budget_GiB": args.budget_gib, **mb,
                                    "fad_over_composite": round(mb["fad"]["max_batch"] / mb["composite"]["max_batch"], 3)}
            print(json.dumps(row), flush=True)


if __name__ == "__main__":
    main()

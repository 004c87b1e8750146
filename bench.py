#!/usr/bin/env python3
"""Benchmark of the libnfad hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic activations of the chosen
configuration: the method's fused forward (y, dydx) and its backward gx = gy*dydx, then the
two baselines the paper compares against (recomputation fwd/bwd, save-all fwd/bwd), each a
single fused kernel.  Inputs are resident in HBM before the timed region starts.  Buffer
sets are rotated so that successive launches do not hit in the 256 MB last-level cache.

Prints ONE JSON line.  `value` is algorithmic HBM bytes of a step / step time.  `roofline`
describes the method's forward kernel (nfad_fwd), its launch duration measured with events
on the launch stream over a region of back-to-back launches (for tensors so small that a
launch is shorter than a Python call, the launches are replayed from a HIP graph).  `cpu_baseline` is the fp64
oracle timed on the host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="index into the benchmark configs (0..4)")
    ap.add_argument("--tensor", type=int, default=0, help="which tensor of a multi-tensor config")
    ap.add_argument("--kind", type=int, default=None, help="activation of a multi-activation config")
    ap.add_argument("--dtype", type=str, default=None, help="dtype of a multi-dtype config")
    ap.add_argument("--sets", type=int, default=0, help="rotating buffer sets (0 = enough for > 1 GiB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stream-reference", action="store_true",
                    help="skip the no-arithmetic streams (read, write, copy and the two kernels' patterns)")
    ap.add_argument("--calib-copy", type=int, default=0,
                    help="also launch this many plain device copies of x (n elements read, n written): the "
                         "known-size kernel that rocprofv3 FETCH_SIZE/WRITE_SIZE readings are scaled by")
    ap.add_argument("--prewarm-s", type=float, default=0.25,
                    help="seconds of untimed steps before the warm-up steps (reaches steady clocks)")
    ap.add_argument("--kernel-rounds", type=int, default=3,
                    help="rounds over the list of kernels; the median round of each kernel is reported")
    ap.add_argument("--kernel-warm-s", type=float, default=0.3,
                    help="seconds of untimed launches of a kernel before its launch duration is measured: the "
                         "duration keeps settling (by 2-4 %%) for a few hundred ms after the kernel mix changes")
    ap.add_argument("--chains", action="store_true",
                    help="also time the fused forward kernel of every composed chain on the same tensor")
    ap.add_argument("--cpu-sample", type=int, default=1 << 25, help="max elements the oracle is timed on")
    ap.add_argument("--launch", choices=("auto", "direct", "graph"), default="auto",
                    help="how timed launches are issued: one C-ABI call each from Python (direct), or captured "
                         "once into a HIP graph and replayed (graph); auto = graph when a launch moves less "
                         "than 64 MB, i.e. when it is shorter than the interpreter's launch rate")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path is element-wise and shards without "
              "any exchange); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2209_10778_amd as nfad
    from paper_2209_10778_amd import inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    nfad.lib()  # no fallback: raises if libnfad.so is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = inputs.CONFIGS[args.config]
    spec = cfg.tensors[args.tensor]
    kind = cfg.kinds[0] if args.kind is None else args.kind
    dtype = cfg.dtypes[0] if args.dtype is None else args.dtype
    assert kind in cfg.kinds and dtype in cfg.dtypes
    td = inputs.TORCH_DTYPE[dtype]
    n = spec.n
    es = 2 if dtype != "f32" else 4
    k_saved = nfad.nfad_saveall_num_saved(kind)

    # ---- inputs of record: seeded, storage-rounded on the host, then made resident
    x_host = inputs.make_x(cfg, spec, dtype)
    gy_host = inputs.make_gy(cfg, spec, dtype)
    per_set_bytes = (5 + (k_saved - 1)) * n * es
    nsets = args.sets or max(2, -(-(1 << 30) // per_set_bytes) + 1)
    sets = []
    for _ in range(nsets):
        s = {"x": x_host.to(dev), "gy": gy_host.to(dev)}
        for name in ("y", "dydx", "gx"):
            s[name] = torch.empty(n, dtype=td, device=dev)
        s["saved"] = [s["x"]] + [torch.empty(n, dtype=td, device=dev) for _ in range(k_saved - 1)]
        sets.append(s)
    stream = torch.cuda.current_stream()

    kernels = {
        "nfad_fwd": (lambda s, st: nfad.nfad_fwd(kind, s["x"], s["y"], s["dydx"], st), 3),
        "nfad_bwd": (lambda s, st: nfad.nfad_bwd(s["gy"], s["dydx"], s["gx"], st), 3),
        "recompute_fwd": (lambda s, st: nfad.nfad_recompute_fwd(kind, s["x"], s["y"], st), 2),
        "recompute_bwd": (lambda s, st: nfad.nfad_recompute_bwd(kind, s["gy"], s["x"], s["gx"], st), 3),
        "saveall_fwd": (lambda s, st: nfad.nfad_saveall_fwd(kind, s["x"], s["y"], s["saved"], st), 1 + k_saved),
        "saveall_bwd": (lambda s, st: nfad.nfad_saveall_bwd(kind, s["gy"], s["saved"], s["gx"], st), 2 + k_saved),
    }
    words_per_step = sum(w for _, w in kernels.values())
    bytes_per_step = words_per_step * n * es
    use_graph = args.launch == "graph" or (args.launch == "auto" and 3 * n * es < 64e6)

    def runner(fns, count):
        """A callable that enqueues `count` rounds of `fns` (buffer sets rotating) on the current
        stream: launch by launch from Python, or as one replay of a HIP graph captured here (the
        library's calls are capturable: no allocation, no synchronisation, no memset)."""
        def enqueue():
            st = torch.cuda.current_stream()
            for i in range(count):
                s = sets[i % nsets]
                for fn in fns:
                    fn(s, st)
        if not use_graph:
            return enqueue
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            enqueue()
        return g.replay

    step_fns = [fn for fn, _ in kernels.values()]

    # Untimed pre-warm: kernel times on this part settle ~3 % lower after a few tens of ms of
    # sustained streaming (clocks, TLBs), so reach steady state before the W warm-up steps.
    warm_steps = runner(step_fns, max(1, args.warmup))
    timed_steps = runner(step_fns, args.steps)
    t_pre = time.perf_counter()
    i_pre = 0
    while time.perf_counter() - t_pre < args.prewarm_s:
        warm_steps()
        i_pre += 1
        if i_pre % 4 == 0:
            torch.cuda.synchronize()
    if args.warmup > 0:
        warm_steps()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    timed_steps()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = bytes_per_step / (ms_per_step * 1e-3) / 1e9

    # ---- per-kernel launch duration: events on the launch stream around back-to-back launches.
    # The part adapts to the traffic pattern over a few hundred ms (a kernel measured right after
    # a different kernel mix reads 2-4 % slower than in steady state), so each kernel first runs
    # alone for kernel_warm_s; the last warm-up launches are queued right in front of the timed
    # region (no idle gap).
    def time_kernels(fns):
        """{name: launch duration in us}: every kernel is measured in `--kernel-rounds` rounds over the
        whole list and the median round is reported, so that no kernel owes its figure to its
        place in the process (the first seconds of a process read 1-3 % slow on some parts)."""
        timed = {name: runner([fn], args.steps) for name, fn in fns.items()}
        samples = {name: [] for name in fns}
        for _ in range(max(1, args.kernel_rounds)):
            for name, run in timed.items():
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                t_w = time.perf_counter()
                while time.perf_counter() - t_w < args.kernel_warm_s:   # sustained launches of THIS kernel
                    for _ in range(4):
                        run()
                    torch.cuda.synchronize()
                for _ in range(-(-max(300, args.warmup) // args.steps)):
                    run()
                e0.record(stream)
                run()
                e1.record(stream)
                torch.cuda.synchronize()
                samples[name].append(e0.elapsed_time(e1) * 1e3 / args.steps)
        return {name: sorted(v)[len(v) // 2] for name, v in samples.items()}

    per_kernel = {}
    launch_us = time_kernels({name: fn for name, (fn, _) in kernels.items()})
    for name, (fn, words) in kernels.items():
        us = launch_us[name]
        gbps = words * n * es / (us * 1e-6) / 1e9
        per_kernel[name] = {"us": round(us, 2), "bytes_per_elem": words * es, "GB/s": round(gbps, 1),
                            "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4),
                            "Gelem/s": round(n / (us * 1e-6) / 1e9, 1)}

    # ---- what the memory system gives each traffic pattern on THIS part: the library's launch
    # shape with the arithmetic taken out (nfad_probe_stream), same tensors, same protocol.  A
    # reference, not a bound: a ratio above 1 means the kernel with arithmetic is the faster one.
    stream_reference = None
    if not args.no_stream_reference:
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        probes = {
            "read_1": (lambda s, st: nfad.nfad_probe_stream([s["x"]], [], stream=st, sink=sink), 1),
            "write_1": (lambda s, st: nfad.nfad_probe_stream([], [s["y"]], stream=st), 1),
            "read_1_write_1": (lambda s, st: nfad.nfad_probe_stream([s["x"]], [s["y"]], stream=st), 2),
            "read_1_write_2 (pattern of nfad_fwd)":
                (lambda s, st: nfad.nfad_probe_stream([s["x"]], [s["y"], s["dydx"]], stream=st), 3),
            "read_2_write_1 (pattern of nfad_bwd)":
                (lambda s, st: nfad.nfad_probe_stream([s["gy"], s["dydx"]], [s["gx"]], stream=st), 3),
        }
        probe_us = time_kernels({k: f for k, (f, _) in probes.items()})
        stream_reference = {k: {"us": round(probe_us[k], 2),
                               "GB/s": round(w * n * es / (probe_us[k] * 1e-6) / 1e9, 1)}
                           for k, (_, w) in probes.items()}
        stream_reference["nfad_fwd_speed_vs_plain_stream"] = round(
            probe_us["read_1_write_2 (pattern of nfad_fwd)"] / per_kernel["nfad_fwd"]["us"], 4)
        stream_reference["nfad_bwd_speed_vs_plain_stream"] = round(
            probe_us["read_2_write_1 (pattern of nfad_bwd)"] / per_kernel["nfad_bwd"]["us"], 4)

    # ---- context: the runtime's own device-to-device copy of the same tensor (n read + n written)
    for i in range(3):
        sets[i % nsets]["y"].copy_(sets[i % nsets]["x"])
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    for i in range(args.steps):
        sets[i % nsets]["y"].copy_(sets[i % nsets]["x"])
    e1.record(stream)
    torch.cuda.synchronize()
    copy_us = e0.elapsed_time(e1) * 1e3 / args.steps
    reference_copy = {"what": "runtime device-to-device copy of x (hipMemcpyAsync via torch copy_)",
                      "us": round(copy_us, 2), "GB/s": round(2 * n * es / (copy_us * 1e-6) / 1e9, 1)}

    for i in range(args.calib_copy):      # plain copy of known size, for counter calibration only
        sets[i % nsets]["y"].copy_(sets[i % nsets]["x"])
    torch.cuda.synchronize()

    chains = None
    if args.chains:   # composed chains: same contract and traffic as nfad_fwd (3 words per element)
        chains = {}
        t_c = time.perf_counter()
        jit_id = nfad.nfad_chain_compile("x x softplus tanh *")    # Mish again, compiled at run time
        jit_compile_s = time.perf_counter() - t_c
        ids = list(range(nfad.nfad_chain_count())) + [jit_id]
        label = lambda cid: nfad.nfad_chain_name(cid) if cid != jit_id else "runtime-compiled mish"
        chain_us = time_kernels({label(cid): (lambda s, st, cid=cid: nfad.nfad_chain_fwd(cid, s["x"], s["y"], s["dydx"], st))
                                 for cid in ids})
        for key, us in chain_us.items():
            gbps = 3 * n * es / (us * 1e-6) / 1e9
            chains[key] = {"us": round(us, 2), "GB/s": round(gbps, 1),
                           "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4)}
        chains["runtime-compiled mish"]["compile_s"] = round(jit_compile_s, 2)
        nfad.nfad_chain_release(jit_id)

        # one source, two outputs (R^1 -> R^2): the fused multi-output forward and the merged backward
        # against the same work done chain by chain
        progs = ["x tanh x *", "x tanh sigmoid"]
        mid = nfad.nfad_chain_compile_multi(progs)
        sids = [nfad.nfad_chain_compile(p) for p in progs]
        for s in sets:
            s["y2"], s["d2"] = torch.empty_like(s["y"]), torch.empty_like(s["dydx"])

        def fwd_separate(s, st):
            nfad.nfad_chain_fwd(sids[0], s["x"], s["y"], s["dydx"], st)
            nfad.nfad_chain_fwd(sids[1], s["x"], s["y2"], s["d2"], st)

        multi_us = time_kernels({
            "fwd_multi": lambda s, st: nfad.nfad_chain_fwd_multi(mid, s["x"], [s["y"], s["y2"]], [s["dydx"], s["d2"]], st),
            "fwd_separate": fwd_separate,
            "bwd_multi": lambda s, st: nfad.nfad_bwd_multi([s["gy"], s["y"]], [s["dydx"], s["d2"]], s["gx"], st),
        })
        chains["two_outputs"] = {
            "programs": progs,
            "fwd_multi": {"us": round(multi_us["fwd_multi"], 2), "bytes_per_elem": 5 * es,
                          "GB/s": round(5 * n * es / (multi_us["fwd_multi"] * 1e-6) / 1e9, 1)},
            "fwd_chain_by_chain": {"us": round(multi_us["fwd_separate"], 2), "bytes_per_elem": 6 * es},
            "bwd_multi": {"us": round(multi_us["bwd_multi"], 2), "bytes_per_elem": 5 * es,
                          "GB/s": round(5 * n * es / (multi_us["bwd_multi"] * 1e-6) / 1e9, 1)},
        }
        for cid in [mid] + sids:
            nfad.nfad_chain_release(cid)

    fwd = per_kernel["nfad_fwd"]
    roofline = {"kernel": "nfad_fwd", "bound": "hbm", "achieved": fwd["GB/s"], "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(fwd["GB/s"] / HBM_PEAK_GBPS, 4), "traffic": None,
                "algorithmic_bytes_per_launch": 3 * n * es, "avg_launch_us": fwd["us"]}
    traffic_file = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "traffic.json")
    if os.path.exists(traffic_file):  # HBM bytes per launch from committed rocprofv3 --pmc runs
        try:
            tr = json.load(open(traffic_file))
            key = f"nfad_fwd/{nfad.KIND_NAMES[kind]}/{dtype}/{n}"
            if key in tr:
                roofline["traffic"] = tr[key]
        except Exception:
            pass

    fad_us = per_kernel["nfad_fwd"]["us"] + per_kernel["nfad_bwd"]["us"]
    rec_us = per_kernel["recompute_fwd"]["us"] + per_kernel["recompute_bwd"]["us"]
    sav_us = per_kernel["saveall_fwd"]["us"] + per_kernel["saveall_bwd"]["us"]
    summary = {
        "fad_fwd_bwd_GB/s": round(6 * n * es / (fad_us * 1e-6) / 1e9, 1),
        "fad_fwd_bwd_Gelem/s": round(n / (fad_us * 1e-6) / 1e9, 1),
        "retained_bytes_per_elem": {"fad": es, "recompute": es, "saveall": k_saved * es},
        "bytes_saved_per_elem_vs_saveall": (k_saved - 1) * es,
        "time_fad_over_recompute": round(fad_us / rec_us, 4),
        "time_fad_over_saveall": round(fad_us / sav_us, 4),
        "bwd_time_fad_over_recompute": round(per_kernel["nfad_bwd"]["us"] / per_kernel["recompute_bwd"]["us"], 4),
    }

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        ns = min(n, args.cpu_sample)
        x64 = inputs.storage_to_f64(x_host[:ns])
        gy64 = inputs.storage_to_f64(gy_host[:ns])
        threads = oracle.max_threads()
        oracle.fwd(kind, x64[: 1 << 16])          # warm the library, untimed
        def one_step_on_cpu():
            c0 = time.perf_counter()
            y64, d64 = oracle.fwd(kind, x64)
            oracle.bwd(gy64, d64)
            oracle.recompute_fwd(kind, x64)
            oracle.recompute_bwd(kind, gy64, x64)
            _, saved64 = oracle.saveall_fwd(kind, x64)
            oracle.saveall_bwd(kind, gy64, saved64)
            return time.perf_counter() - c0
        walls = [one_step_on_cpu()]
        # whole steps until about a second of wall time (10-20 s of CPU time on 16 threads), at least 3
        while len(walls) < 3 or (sum(walls) < 1.0 and len(walls) < 50):
            walls.append(one_step_on_cpu())
        wall = sorted(walls)[len(walls) // 2]
        c0, c1 = 0.0, wall
        # once single-threaded, on a sixteenth of the sample
        n1 = max(1, ns // 16)
        s0 = time.perf_counter()
        y1, d1 = oracle.fwd(kind, x64[:n1], threads=1)
        oracle.bwd(gy64[:n1], d1, threads=1)
        s1 = time.perf_counter()
        cpu_baseline = {
            "value": round(words_per_step * ns * es / (c1 - c0) / 1e9, 3), "unit": "GB/s",
            "single_thread_fwd_bwd_Gelem/s": round(n1 / (s1 - s0) / 1e9, 4),
            "cores": threads, "kind": "oracle",
            "sample": f"first {ns} of {n} elements, one step (all six passes) in fp64 with OpenMP, median of {len(walls)} steps, "
                      f"{c1 - c0:.2f} s wall; bytes counted as for the {dtype}-storage GPU step",
            "Gelem/s_per_pass": round(6 * ns / (c1 - c0) / 1e9, 4),
        }
        del x64, gy64

    out = {
        "metric": "achieved HBM GB/s (% of peak) for fused fwd+dydx and bwd; Gelem/s",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",   # arithmetic is fp32 for every storage type
        "config": {"workload": cfg.name, "activation": nfad.KIND_NAMES[kind], "shape": list(spec.shape),
                   "elements": n, "storage": dtype, "step": list(kernels.keys()),
                   "bytes_per_step": bytes_per_step, "buffer_sets": nsets,
                   "launch": "hip graph replay" if use_graph else "direct"},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "Gelem/s": round(6 * n / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": roofline, "cpu_baseline": cpu_baseline, "kernels": per_kernel, "summary": summary,
        "stream_reference": stream_reference, "reference_copy": reference_copy, "chains": chains,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()

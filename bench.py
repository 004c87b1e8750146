#!/usr/bin/env python3
"""Benchmark of the libnfad hot path on one MI355X.

A step is one pass of the method over one batch of synthetic activations of the chosen
configuration: for every activation the configuration names, the fused forward kernel
(y and dydx in one pass over x) and then the backward kernel gx = gy * dydx.  `value` is the
algorithmic HBM bytes of a step divided by its time: the metric's "fused fwd+dydx and bwd".
Inputs are resident in HBM before the timed region starts, and every launch works on COLD
data: buffer sets rotate beyond the 256 MB last-level cache and the backward kernel of a step
reads the tangent of another set (in a network the backward pass runs long after the forward
pass), so nothing a kernel reads was just written or read by its predecessor.

The default configuration is the largest one (the BERT-large-shaped stress tensor, all four
activations).  Besides the headline the same JSON line carries
  per_config   nfad_fwd / nfad_bwd launch durations on EVERY benchmark configuration,
  kernels      all six kernels (the method and the two baselines it is compared with) per
               activation of the chosen configuration, and `summary` derived from them,
  roofline     the slowest forward kernel of the chosen configuration against the HBM peak,
  stream_reference  what the memory system gives each traffic pattern without arithmetic, in
               the best launch shape found among a list of candidates (libnfad_sweep.so),
  cpu_baseline the fp64 oracle timed on the host cores on a bounded sample of the same step.
Per-kernel durations are measured with events on the launch stream around back-to-back
launches (for tensors so small that a launch is shorter than a Python call, the launches are
replayed from a HIP graph).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

HBM_PEAK_GBPS = 8000.0
ROOT = os.path.dirname(os.path.abspath(__file__))
# A launch that moves less than this is shorter than the interpreter's launch rate: graph replay.
GRAPH_BELOW_BYTES = 64e6
# time = T0 + bytes / BW fitted through the 308 MB and 805 MB forward launches (ramp-up and drain
# plus streaming at the large-tensor rate): what a small launch would take if it streamed like a
# large one.  Small launches are reported next to it.
FLOOR_T0_US, FLOOR_GBPS = 1.4, 6650.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="index into the benchmark configs (0..4); default: the largest")
    ap.add_argument("--tensor", type=int, default=0, help="which tensor of a multi-tensor config")
    ap.add_argument("--dtype", type=str, default=None, help="dtype of a multi-dtype config")
    ap.add_argument("--sets", type=int, default=0, help="rotating buffer sets (0 = enough for > 1 GiB, at least 3)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stream-reference", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="skip the sweep over all benchmark configurations")
    ap.add_argument("--no-baselines", action="store_true", help="time only nfad_fwd and nfad_bwd")
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
    ap.add_argument("--cpu-sample", type=int, default=1 << 24, help="max elements the oracle is timed on")
    ap.add_argument("--launch", choices=("auto", "direct", "graph"), default="auto",
                    help="how timed launches are issued: one C-ABI call each from Python (direct), or captured "
                         "once into a HIP graph and replayed (graph); auto = graph when a launch moves less "
                         "than 64 MB, i.e. when it is shorter than the interpreter's launch rate")
    return ap.parse_args()


def source_hash() -> str:
    """Hash of the kernel sources: measured-traffic records are only valid for the code they were taken from."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2209_10778_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hpp", ".hip", ".inc")) and name != "nfad_embedded.inc" and name != "nfad_sweep.hip":
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


class Bench:
    """Buffers of one tensor of one configuration, and the timing protocol."""

    def __init__(self, args, torch, nfad, inputs, cfg, spec, dtype, with_saved):
        self.args, self.torch, self.nfad = args, torch, nfad
        self.cfg, self.spec, self.dtype = cfg, spec, dtype
        self.td = inputs.TORCH_DTYPE[dtype]
        self.n = spec.n
        self.es = 2 if dtype != "f32" else 4
        dev = torch.device("cuda:0")
        self.x_host = inputs.make_x(cfg, spec, dtype)
        self.gy_host = inputs.make_gy(cfg, spec, dtype)
        extra = max(nfad.nfad_saveall_num_saved(k) for k in cfg.kinds) - 1 if with_saved else 0
        per_set = (5 + extra) * self.n * self.es
        self.nsets = args.sets or max(3, -(-(1 << 30) // per_set) + 1)
        self.sets = []
        for _ in range(self.nsets):
            s = {"x": self.x_host.to(dev), "gy": self.gy_host.to(dev)}
            for name in ("y", "dydx", "gx"):
                s[name] = torch.empty(self.n, dtype=self.td, device=dev)
            s["extra"] = [torch.empty(self.n, dtype=self.td, device=dev) for _ in range(extra)]
            self.sets.append(s)
        # every set's tangent holds real values before anything is timed
        for s in self.sets:
            nfad.nfad_fwd(cfg.kinds[0], s["x"], s["y"], s["dydx"])
        torch.cuda.synchronize()
        self.stream = torch.cuda.current_stream()
        self.use_graph = args.launch == "graph" or (args.launch == "auto" and 3 * self.n * self.es < GRAPH_BELOW_BYTES)

    def saved(self, s, kind):
        return [s["x"]] + s["extra"][: self.nfad.nfad_saveall_num_saved(kind) - 1]

    def runner(self, fns, count):
        """A callable that enqueues `count` rounds of `fns` (buffer sets rotating) on the current
        stream: launch by launch from Python, or as one replay of a HIP graph captured here (the
        library's calls are capturable: no allocation, no synchronisation, no memset).  fn(s, t, st):
        s is the round's set, t the NEXT set (whose tangent was written a full rotation ago)."""
        torch, sets, nsets = self.torch, self.sets, self.nsets

        def enqueue():
            st = torch.cuda.current_stream()
            for i in range(count):
                for fn in fns:
                    fn(sets[i % nsets], sets[(i + 1) % nsets], st)
        if not self.use_graph:
            return enqueue
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            enqueue()
        return g.replay

    def time_kernels(self, fns, warm_s=None):
        """{name: launch duration in us}.  The part adapts to the traffic pattern over a few hundred
        ms (a kernel measured right after a different kernel mix reads 2-4 % slower than in steady
        state), so each kernel first runs alone for kernel_warm_s, the last warm-up launches are
        queued right in front of the timed region, and every kernel is measured in `--kernel-rounds`
        rounds over the whole list, the median round being reported, so that no kernel owes its
        figure to its place in the process."""
        torch, args, stream = self.torch, self.args, self.stream
        warm_s = args.kernel_warm_s if warm_s is None else min(warm_s, args.kernel_warm_s)
        timed = {name: self.runner([fn], args.steps) for name, fn in fns.items()}
        samples = {name: [] for name in fns}
        for _ in range(max(1, args.kernel_rounds)):
            for name, run in timed.items():
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                t_w = time.perf_counter()
                while time.perf_counter() - t_w < warm_s:   # sustained launches of THIS kernel
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

    def figures(self, us, words):
        gbps = words * self.n * self.es / (us * 1e-6) / 1e9
        return {"us": round(us, 2), "bytes_per_elem": words * self.es, "GB/s": round(gbps, 1),
                "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4), "Gelem/s": round(self.n / (us * 1e-6) / 1e9, 1)}

    def free(self):
        self.sets = None
        self.torch.cuda.empty_cache()


def method_kernels(nfad, kind):
    return {
        "nfad_fwd": (lambda s, t, st: nfad.nfad_fwd(kind, s["x"], s["y"], s["dydx"], st), 3),
        "nfad_bwd": (lambda s, t, st: nfad.nfad_bwd(t["gy"], t["dydx"], t["gx"], st), 3),
    }


def baseline_kernels(nfad, bench, kind):
    k = nfad.nfad_saveall_num_saved(kind)
    return {
        "recompute_fwd": (lambda s, t, st: nfad.nfad_recompute_fwd(kind, s["x"], s["y"], st), 2),
        "recompute_bwd": (lambda s, t, st: nfad.nfad_recompute_bwd(kind, t["gy"], t["x"], t["gx"], st), 3),
        "saveall_fwd": (lambda s, t, st: nfad.nfad_saveall_fwd(kind, s["x"], s["y"], bench.saved(s, kind), st), 1 + k),
        "saveall_bwd": (lambda s, t, st: nfad.nfad_saveall_bwd(kind, t["gy"], bench.saved(t, kind), t["gx"], st), 2 + k),
    }


def stream_reference(bench, nfad):
    """The ceiling of each traffic pattern on THIS part and tensor: no arithmetic, the best of a list
    of launch shapes (block size x accesses per lane x cap on resident waves), timed under the same
    protocol as the kernels.  None if the measurement library has not been built."""
    try:
        from paper_2209_10778_amd import sweep
        sweep.sweep_lib()
    except (ImportError, OSError):
        return None
    torch = bench.torch
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    patterns = {"read_1": ("r1w0", 1), "write_1": ("r0w1", 1), "read_1_write_1": ("r1w1", 2),
                "read_1_write_2 (pattern of nfad_fwd)": ("r1w2", 3), "read_2_write_1 (pattern of nfad_bwd)": ("r2w1", 3)}
    shapes = [dict(threads=th, unroll=u, adjacent=0, ntl=1, nts=1, waves=w, grid=0, chunk=0)
              for th, u, w in ((64, 1, 0), (64, 1, 21), (64, 1, 25), (128, 1, 25), (128, 2, 16), (128, 2, 0), (256, 2, 0),
                               (512, 2, 0), (512, 4, 12), (128, 4, 12))]
    fns = {}
    for label, (pat, _) in patterns.items():
        n_in, n_out = sweep.PATTERNS[pat][1], sweep.PATTERNS[pat][2]
        for i, sh in enumerate(shapes):
            def fn(s, t, st, pat=pat, sh=sh, n_in=n_in, n_out=n_out):
                ins = [s["x"], t["dydx"]][:n_in] if n_in < 2 else [t["gy"], t["dydx"]]
                outs = [s["y"], s["dydx"]][:n_out] if n_in < 2 else [t["gx"]]
                sweep.launch(pat, bench.dtype, sh, ins, outs if outs else [sink], bench.n, st.cuda_stream)
            fns[(label, i)] = fn
    us = bench.time_kernels(fns, warm_s=0.1)
    for s in bench.sets:     # the write patterns left bit patterns in y and dydx: put real tangents back
        nfad.nfad_fwd(bench.cfg.kinds[0], s["x"], s["y"], s["dydx"])
    torch.cuda.synchronize()
    out = {}
    for label, (pat, words) in patterns.items():
        best_i = min(range(len(shapes)), key=lambda i: us[(label, i)])
        t = us[(label, best_i)]
        sh = shapes[best_i]
        out[label] = {"us": round(t, 2), "GB/s": round(words * bench.n * bench.es / (t * 1e-6) / 1e9, 1),
                      "best_shape": f"{sh['threads']} threads x {sh['unroll']} accesses, "
                                    f"{'no cap' if not sh['waves'] else str(sh['waves']) + ' waves/CU'}",
                      "worst_of_candidates_us": round(max(us[(label, i)] for i in range(len(shapes))), 2)}
    out["candidates_per_pattern"] = len(shapes)
    return out


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
    torch.cuda.set_device(torch.device("cuda:0"))

    cfg = inputs.CONFIGS[args.config]
    spec = cfg.tensors[args.tensor]
    dtype = cfg.dtypes[0] if args.dtype is None else args.dtype
    assert dtype in cfg.dtypes
    kinds = list(cfg.kinds)
    B = Bench(args, torch, nfad, inputs, cfg, spec, dtype, with_saved=not args.no_baselines)
    n, es = B.n, B.es

    # ---- the step: for every activation of the configuration, fused forward then backward
    step_fns = []
    for kind in kinds:
        mk = method_kernels(nfad, kind)
        step_fns += [mk["nfad_fwd"][0], mk["nfad_bwd"][0]]
    bytes_per_step = len(kinds) * 6 * n * es

    # Untimed pre-warm: kernel times on this part settle ~3 % lower after a few tens of ms of
    # sustained streaming (clocks, TLBs), so reach steady state before the W warm-up steps.
    warm_steps = B.runner(step_fns, max(1, args.warmup))
    timed_steps = B.runner(step_fns, args.steps)
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

    # ---- per-kernel launch durations on the chosen configuration, per activation
    per_kind, summary = {}, {}
    for kind in kinds:
        ks = dict(method_kernels(nfad, kind))
        if not args.no_baselines:
            ks.update(baseline_kernels(nfad, B, kind))
        us = B.time_kernels({name: fn for name, (fn, _) in ks.items()})
        name_k = nfad.KIND_NAMES[kind]
        per_kind[name_k] = {name: B.figures(us[name], words) for name, (_, words) in ks.items()}
        fad_us = us["nfad_fwd"] + us["nfad_bwd"]
        k_saved = nfad.nfad_saveall_num_saved(kind)
        summ = {"fad_fwd_bwd_GB/s": round(6 * n * es / (fad_us * 1e-6) / 1e9, 1),
                "fad_fwd_bwd_Gelem/s": round(n / (fad_us * 1e-6) / 1e9, 1),
                "retained_bytes_per_elem": {"fad": es, "recompute": es, "saveall": k_saved * es},
                "bytes_saved_per_elem_vs_saveall": (k_saved - 1) * es}
        if not args.no_baselines:
            rec_us = us["recompute_fwd"] + us["recompute_bwd"]
            sav_us = us["saveall_fwd"] + us["saveall_bwd"]
            summ.update({"time_fad_over_recompute": round(fad_us / rec_us, 4),
                         "time_fad_over_saveall": round(fad_us / sav_us, 4),
                         "bwd_time_fad_over_recompute": round(us["nfad_bwd"] / us["recompute_bwd"], 4)})
        summary[name_k] = summ

    # ---- roofline: the slowest forward kernel of the chosen configuration
    slow = max(per_kind, key=lambda k: per_kind[k]["nfad_fwd"]["us"])
    fwd = per_kind[slow]["nfad_fwd"]
    roofline = {"kernel": f"nfad_fwd({slow})", "bound": "hbm", "achieved": fwd["GB/s"], "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(fwd["GB/s"] / HBM_PEAK_GBPS, 4), "traffic": None,
                "algorithmic_bytes_per_launch": 3 * n * es, "avg_launch_us": fwd["us"],
                "nfad_bwd": {"achieved": per_kind[slow]["nfad_bwd"]["GB/s"],
                             "frac": per_kind[slow]["nfad_bwd"]["frac_of_peak"],
                             "avg_launch_us": per_kind[slow]["nfad_bwd"]["us"]}}
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):
        # HBM bytes per launch from committed rocprofv3 --pmc runs; only valid for the kernel sources
        # they were measured on
        try:
            tr = json.load(open(traffic_file))
            if tr.get("source_hash") == source_hash():
                roofline["traffic"] = tr.get("bytes_per_launch", {}).get(f"nfad_fwd/{slow}/{dtype}/{n}")
        except Exception:
            pass

    reference = None if args.no_stream_reference else stream_reference(B, nfad)

    # ---- context: the runtime's own device-to-device copy of the same tensor (n read + n written)
    sets, nsets, stream = B.sets, B.nsets, B.stream
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

    chains = bench_chains(B, nfad) if args.chains else None

    # ---- the oracle on the host cores, on a bounded sample of the same step
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        ns = min(n, args.cpu_sample)
        x64 = inputs.storage_to_f64(B.x_host[:ns])
        gy64 = inputs.storage_to_f64(B.gy_host[:ns])
        threads = oracle.max_threads()
        oracle.fwd(kinds[0], x64[: 1 << 16])          # warm the library, untimed

        def one_step_on_cpu():
            c0 = time.perf_counter()
            for kind in kinds:
                _, d64 = oracle.fwd(kind, x64)
                oracle.bwd(gy64, d64)
            return time.perf_counter() - c0
        walls = [one_step_on_cpu()]
        # whole steps until about a second of wall time (10-20 s of CPU time on 16 threads), at least 3
        while len(walls) < 3 or (sum(walls) < 1.0 and len(walls) < 50):
            walls.append(one_step_on_cpu())
        wall = sorted(walls)[len(walls) // 2]
        n1 = max(1, ns // 16)                        # once single-threaded, on a sixteenth of the sample
        s0 = time.perf_counter()
        _, d1 = oracle.fwd(kinds[0], x64[:n1], threads=1)
        oracle.bwd(gy64[:n1], d1, threads=1)
        s1 = time.perf_counter()
        cpu_baseline = {
            "value": round(len(kinds) * 6 * ns * es / wall / 1e9, 3), "unit": "GB/s",
            "single_thread_fwd_bwd_Gelem/s": round(n1 / (s1 - s0) / 1e9, 4),
            "cores": threads, "kind": "oracle",
            "sample": f"first {ns} of {n} elements, one step (forward and backward of {len(kinds)} activation(s)) "
                      f"in fp64 with OpenMP, median of {len(walls)} steps, {wall:.2f} s wall; bytes counted as for "
                      f"the {dtype}-storage GPU step",
            "Gelem/s_per_pass": round(2 * len(kinds) * ns / wall / 1e9, 4),
        }
        del x64, gy64
    B.free()

    # ---- nfad_fwd / nfad_bwd on every benchmark configuration
    per_config = None
    if not args.no_per_config:
        per_config = []
        for ci, c in enumerate(inputs.CONFIGS):
            for ti, sp in enumerate(c.tensors):
                for dt in c.dtypes:
                    if ci == args.config and ti == args.tensor and dt == dtype:
                        src = {k: (per_kind[nfad.KIND_NAMES[k]]["nfad_fwd"]["us"],
                                   per_kind[nfad.KIND_NAMES[k]]["nfad_bwd"]["us"]) for k in c.kinds}
                        b_n, b_es, graph, nsets_c = n, es, B.use_graph, B.nsets
                    else:
                        Bc = Bench(args, torch, nfad, inputs, c, sp, dt, with_saved=False)
                        fns = {}
                        for k in c.kinds:
                            mk = method_kernels(nfad, k)
                            fns[(k, "fwd")] = mk["nfad_fwd"][0]
                            fns[(k, "bwd")] = mk["nfad_bwd"][0]
                        us = Bc.time_kernels(fns)
                        src = {k: (us[(k, "fwd")], us[(k, "bwd")]) for k in c.kinds}
                        b_n, b_es, graph, nsets_c = Bc.n, Bc.es, Bc.use_graph, Bc.nsets
                        Bc.free()
                    moved = 3 * b_n * b_es
                    floor_us = FLOOR_T0_US + moved / (FLOOR_GBPS * 1e3)
                    for k, (fu, bu) in src.items():
                        row = {"config": f"C{ci + 1}", "activation": nfad.KIND_NAMES[k], "storage": dt,
                               "shape": list(sp.shape), "elements": b_n, "MB_per_launch": round(moved / 1e6, 1),
                               "launch": "hip graph replay" if graph else "direct", "buffer_sets": nsets_c,
                               "regime": "streams from HBM" if moved > 256e6 else
                                         ("cold, but smaller than the 256 MB last-level cache: ramp-up and drain "
                                          "are a visible share of the launch"),
                               "large_launch_model_us (1.4 us + bytes / 6.65 TB/s)": round(floor_us, 2)}
                        for nm, t in (("nfad_fwd", fu), ("nfad_bwd", bu)):
                            g = moved / (t * 1e-6) / 1e9
                            row[nm] = {"us": round(t, 2), "GB/s": round(g, 1), "frac": round(g / HBM_PEAK_GBPS, 4),
                                       "over_model": round(t / floor_us, 3)}
                        per_config.append(row)

    out = {
        "metric": "achieved HBM GB/s (% of peak) for fused fwd+dydx and bwd; Gelem/s",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",   # arithmetic is fp32 for every storage type
        "config": {"workload": cfg.name, "activations": [nfad.KIND_NAMES[k] for k in kinds], "shape": list(spec.shape),
                   "elements": n, "storage": dtype,
                   "step": "for each activation: nfad_fwd (x -> y, dydx), then nfad_bwd (gy, dydx -> gx) on "
                           "another buffer set's tangent; cold inputs",
                   "kernels_per_step": 2 * len(kinds), "bytes_per_step": bytes_per_step, "buffer_sets": B.nsets,
                   "launch": "hip graph replay" if B.use_graph else "direct"},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "Gelem/s": round(len(kinds) * 2 * n / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": roofline, "cpu_baseline": cpu_baseline, "per_config": per_config, "kernels": per_kind,
        "summary": summary, "stream_reference": reference, "reference_copy": reference_copy, "chains": chains,
        "source_hash": source_hash(), "nfad_version": nfad.nfad_version(),
    }
    print(json.dumps(out))


def bench_chains(B, nfad):
    """Composed chains on the same tensor: same contract and traffic as nfad_fwd (3 words per element)."""
    torch, n, es = B.torch, B.n, B.es
    chains = {}
    t_c = time.perf_counter()
    jit_id = nfad.nfad_chain_compile("x x softplus tanh *")    # Mish again, compiled at run time
    jit_compile_s = time.perf_counter() - t_c
    ids = list(range(nfad.nfad_chain_count())) + [jit_id]
    label = lambda cid: nfad.nfad_chain_name(cid) if cid != jit_id else "runtime-compiled mish"
    chain_us = B.time_kernels({label(cid): (lambda s, t, st, cid=cid: nfad.nfad_chain_fwd(cid, s["x"], s["y"], s["dydx"], st))
                               for cid in ids})
    for key, us in chain_us.items():
        gbps = 3 * n * es / (us * 1e-6) / 1e9
        chains[key] = {"us": round(us, 2), "GB/s": round(gbps, 1), "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4)}
    chains["runtime-compiled mish"]["compile_s"] = round(jit_compile_s, 2)
    nfad.nfad_chain_release(jit_id)

    # one source, two outputs (R^1 -> R^2): the fused multi-output forward and the merged backward
    # against the same work done chain by chain
    progs = ["x tanh x *", "x tanh sigmoid"]
    mid = nfad.nfad_chain_compile_multi(progs)
    sids = [nfad.nfad_chain_compile(p) for p in progs]
    for s in B.sets:
        s["y2"], s["d2"] = torch.empty_like(s["y"]), torch.empty_like(s["dydx"])

    def fwd_separate(s, t, st):
        nfad.nfad_chain_fwd(sids[0], s["x"], s["y"], s["dydx"], st)
        nfad.nfad_chain_fwd(sids[1], s["x"], s["y2"], s["d2"], st)

    multi_us = B.time_kernels({
        "fwd_multi": lambda s, t, st: nfad.nfad_chain_fwd_multi(mid, s["x"], [s["y"], s["y2"]], [s["dydx"], s["d2"]], st),
        "fwd_separate": fwd_separate,
        "bwd_multi": lambda s, t, st: nfad.nfad_bwd_multi([t["gy"], t["y"]], [t["dydx"], t["d2"]], t["gx"], st),
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
    return chains


if __name__ == "__main__":
    main()

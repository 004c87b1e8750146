"""Launch-shape sweeps on one MI355X: what each traffic pattern of libnfad gets from the memory
system in ANY launch shape, timed next to libnfad's own kernels in the same process.

    python3 -m paper_2209_10778_amd.sweep --patterns r1w2,r2w1 --sizes c2,c5 \
        --threads 64,128,256,512,1024 --unroll 1,2,4 --waves 0,12,16,24 --lib

Every combination of the comma-separated shape arguments is one row.  Rows are timed
INTERLEAVED (round-robin over all rows, `--rounds` times; the median round is reported),
because on this part only in-process comparisons survive the 3-5 % spread between GPU
sessions.  Protocol per row and round: `--warm-ms` of sustained launches of that row, then
`--launches` back-to-back launches between two events on the launch stream; buffer sets
rotate beyond the 256 MB last-level cache; launches that move < 64 MB are replayed from a HIP
graph so that the interpreter's launch rate is not in the figure.

The shapes are launched through libnfad_sweep.so (csrc/nfad_sweep.hip: libnfad's arithmetic
and load/store helpers with the launch shape as run-time arguments); `--lib` adds libnfad's
own entry points (their built-in shape selection) as rows.  Results go to stdout as a
markdown table sorted by time and, with --out, to a JSON-lines file.

`--phased` runs the other experiment the library carries: reads and writes separated in time
across the whole chip by the constant-rate clock (nfad_sweep_launch_phased), against the same
kernels unphased and libnfad's own.

`--residency` times blocks that only wait, with a given idle LDS reservation: how many of them
the hardware keeps resident per compute unit, i.e. what a cap on resident waves really is.

`--skew` places the tensors of a buffer set inside one allocation, 256 MiB-aligned starts plus
k x SKEW bytes for the k-th tensor (one set of rows per value): whether the relative placement
of the streams in memory matters.

This is a measurement tool: nothing in libnfad or its binding depends on it.
"""
from __future__ import annotations

import argparse
import ctypes
import itertools
import json
import os
import sys
import time

import torch

from . import binding as B

_HERE = os.path.dirname(os.path.abspath(__file__))
_SWEEP_LIB = os.path.join(_HERE, "libnfad_sweep.so")
_SKEW_ALIGN = 1 << 28

# pattern name -> (code, tensors read, tensors written, has arithmetic)
PATTERNS = {
    "r1w2": (0, 1, 2, False), "r2w1": (1, 2, 1, False), "r1w1": (2, 1, 1, False), "r1w0": (3, 1, 0, False),
    "r0w1": (4, 0, 1, False), "r0w2": (5, 0, 2, False), "r2w0": (6, 2, 0, False),
    "fwd_gelu_tanh": (10, 1, 2, True), "fwd_gelu_erf": (11, 1, 2, True), "fwd_swish": (12, 1, 2, True),
    "fwd_mish": (13, 1, 2, True), "bwd": (20, 2, 1, True),
    "recompute_fwd_gelu_tanh": (30, 1, 1, True), "recompute_fwd_gelu_erf": (31, 1, 1, True),
    "recompute_fwd_swish": (32, 1, 1, True), "recompute_fwd_mish": (33, 1, 1, True),
}
# size name -> (elements, storage dtype): the tensors of the benchmark configurations
SIZES = {
    "c1": (1_048_576, "f32"), "c2": (25_690_112, "f32"), "c3a": (51_380_224, "bf16"),
    "c3b": (25_690_112, "bf16"), "c3c": (6_422_528, "bf16"), "c4": (50_331_648, "bf16"),
    "c4h": (50_331_648, "f16"), "c5": (134_217_728, "bf16"),
}
_TD = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
_DT = {"f32": B.F32, "f16": B.F16, "bf16": B.BF16}
_sweep_lib = None


def sweep_lib() -> ctypes.CDLL:
    global _sweep_lib
    if _sweep_lib is None:
        if not os.path.exists(_SWEEP_LIB):
            raise ImportError(f"{_SWEEP_LIB} is missing: build it first (python -m paper_2209_10778_amd.build)")
        L = ctypes.CDLL(_SWEEP_LIB)
        ci, vp = ctypes.c_int, ctypes.c_void_p
        vpp = ctypes.POINTER(ctypes.c_void_p)
        L.nfad_sweep_launch.argtypes = [ci, ci, ci, ci, ci, ci, ci, ci, ctypes.c_longlong, ci, vpp, vpp,
                                        ctypes.c_size_t, vp]
        L.nfad_sweep_launch.restype = ci
        L.nfad_sweep_launch_phased.argtypes = [ci, ci, ci, ci, ci, ci, ci, ci, vpp, vpp, ctypes.c_size_t, vp]
        L.nfad_sweep_launch_phased.restype = ci
        L.nfad_sweep_residency.argtypes = [ci, ctypes.c_uint, ctypes.c_uint, ctypes.c_uint, vp, vp]
        L.nfad_sweep_residency.restype = ci
        L.nfad_sweep_lds_for_cap.argtypes = [ci, ci]
        L.nfad_sweep_lds_for_cap.restype = ctypes.c_uint
        _sweep_lib = L
    return _sweep_lib


def launch(pattern: str, dtype: str, shape: dict, ins, outs, n: int, stream=None) -> None:
    """One launch of `pattern` in `shape` (keys: threads, unroll, adjacent, ntl, nts, waves, grid, chunk)."""
    code = PATTERNS[pattern][0]
    a_in = (ctypes.c_void_p * max(1, len(ins)))(*[t.data_ptr() for t in ins])
    a_out = (ctypes.c_void_p * max(1, len(outs)))(*[t.data_ptr() for t in outs])
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    rc = sweep_lib().nfad_sweep_launch(code, _DT[dtype], shape["threads"], shape["unroll"], shape["adjacent"],
                                       shape["ntl"], shape["nts"], shape["waves"], shape["grid"], shape["chunk"],
                                       a_in, a_out, n, st)
    if rc != 0:
        raise B.NfadError(rc, f"nfad_sweep_launch({pattern}, {shape})")


def launch_phased(pattern: str, dtype: str, unroll: int, waves: int, persistent: bool, period_ticks: int,
                  read_ticks: int, ins, outs, n: int, stream=None) -> None:
    """One launch of an arithmetic pattern with its loads and stores confined to alternating phases of
    the chip-wide 100 MHz clock (period_ticks = 0: no phasing).  One-wave blocks, `waves` of them
    resident per compute unit, `unroll` 16-byte vectors per lane and tensor per period."""
    a_in = (ctypes.c_void_p * len(ins))(*[t.data_ptr() for t in ins])
    a_out = (ctypes.c_void_p * len(outs))(*[t.data_ptr() for t in outs])
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    rc = sweep_lib().nfad_sweep_launch_phased(PATTERNS[pattern][0], _DT[dtype], unroll, 1, waves, int(persistent),
                                              period_ticks, read_ticks, a_in, a_out, n, st)
    if rc != 0:
        raise B.NfadError(rc, f"nfad_sweep_launch_phased({pattern})")


def residency(threads: int, lds_bytes: int, per_cu: int = 1600, ticks: int = 5000, rounds: int = 3) -> float:
    """Blocks of `threads` threads with `lds_bytes` of idle dynamic LDS that are resident per compute
    unit at a time: `per_cu` blocks per compute unit, each waiting `ticks` x 10 ns, timed."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    grid = cus * per_cu
    out = torch.zeros(grid, dtype=torch.int32, device="cuda:0")
    stream = torch.cuda.current_stream()
    best = None
    for _ in range(rounds + 1):                      # first launch: warm-up
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        st = sweep_lib().nfad_sweep_residency(threads, lds_bytes, grid, ticks, out.data_ptr(), stream.cuda_stream)
        if st != 0:
            raise B.NfadError(st, "nfad_sweep_residency")
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3
        best = us if best is None else min(best, us)
    assert bool((out == torch.arange(grid, dtype=torch.int32, device="cuda:0")).all()), "a block did not run"
    return per_cu * ticks * 0.01 / best


def _ints(s: str):
    return [int(v) for v in s.split(",") if v != ""]


def parse_args(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--patterns", default="r1w2,r2w1")
    ap.add_argument("--sizes", default="c2", help="names of benchmark tensors (c1, c2, c3a, c3b, c3c, c4, c4h, c5) "
                                                  "or ELEMENTS:DTYPE, e.g. 100663296:bf16")
    ap.add_argument("--threads", default="128")
    ap.add_argument("--unroll", default="2")
    ap.add_argument("--adjacent", default="0")
    ap.add_argument("--ntl", default="0", help="nontemporal loads: 0, 1 or 0,1")
    ap.add_argument("--nts", default="1", help="nontemporal stores")
    ap.add_argument("--waves", default="0", help="cap on resident waves per compute unit (0 = none); the hardware can express "
                                               "32, 25, 21, 18, 16, 14, 12, 11, ... blocks: a value in between gives the next lower")
    ap.add_argument("--grid", default="0", help="0 = one block per tile; N = persistent grid of N blocks; "
                                                "cN = N blocks per compute unit")
    ap.add_argument("--chunk", default="0", help="tiles per compute die run (0 = identity order)")
    ap.add_argument("--lib", action="store_true", help="add libnfad's own kernels of the same pattern as rows")
    ap.add_argument("--rounds", type=int, default=3)
    ap.add_argument("--launches", type=int, default=60)
    ap.add_argument("--warm-ms", type=float, default=25.0)
    ap.add_argument("--sets", type=int, default=0, help="rotating buffer sets (0 = enough for > 1 GiB)")
    ap.add_argument("--skew", default="", help="byte offsets (multiples of 16) of successive tensors beyond "
                                               "256 MiB-aligned starts; empty = separate allocations")
    ap.add_argument("--top", type=int, default=0, help="print only the best N rows per (size, pattern)")
    ap.add_argument("--out", default=None, help="append one JSON line per row to this file")
    ap.add_argument("--no-verify", action="store_true")
    ap.add_argument("--phased", action="store_true",
                    help="the read/write phasing experiment on the arithmetic patterns given (fwd_*, bwd): --waves = "
                         "resident one-wave blocks per compute unit, --unroll = vectors per lane per period (2,4,8,16), "
                         "--grid 0 = one block per tile / c1 = persistent; phases sized for --phase-scale x "
                         "(7.1 TB/s reads, 6.9 TB/s writes)")
    ap.add_argument("--phase-scale", default="0.9,1.0,1.1")
    ap.add_argument("--residency", action="store_true",
                    help="measure how many blocks of --threads threads are resident per compute unit for each idle "
                         "LDS reservation in --lds (bytes) and for each cap in --waves as libnfad reserves for it")
    ap.add_argument("--lds", default="", help="dynamic LDS bytes per block for --residency")
    return ap.parse_args(argv)


def _grid_of(spec: str, cus: int) -> int:
    return int(spec[1:]) * cus if spec.startswith("c") else int(spec)


def _verify(pattern, dtype, ins, outs, n):
    """What a row wrote is what its pattern says (streams), or what libnfad writes (arithmetic)."""
    code, n_in, n_out, arith = PATTERNS[pattern]
    torch.cuda.synchronize()
    if not arith:
        i32 = [t.view(torch.int32) for t in ins]
        o32 = [t.view(torch.int32) for t in outs]
        if n_in and n_out:
            src = i32[0] if n_in == 1 else i32[0] ^ i32[1]
            assert torch.equal(o32[0], src), f"{pattern}: out[0] wrong"
            if n_out > 1:
                assert torch.equal(o32[1], ~src), f"{pattern}: out[1] wrong"
        return
    ref = [torch.empty_like(o) for o in outs]
    if pattern.startswith("fwd_"):
        B.nfad_fwd(code - 10, ins[0], ref[0], ref[1])
    elif pattern == "bwd":
        B.nfad_bwd(ins[0], ins[1], ref[0])
    else:
        B.nfad_recompute_fwd(code - 30, ins[0], ref[0])
    torch.cuda.synchronize()
    for o, r in zip(outs, ref):
        assert torch.equal(o.view(torch.int16 if o.element_size() == 2 else torch.int32),
                           r.view(torch.int16 if r.element_size() == 2 else torch.int32)), f"{pattern}: differs from libnfad"


def main(argv=None):
    args = parse_args(argv)
    assert torch.cuda.is_available(), "sweep needs a GPU"
    B.lib()
    sweep_lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    stream = torch.cuda.current_stream()
    if args.residency:
        print("| threads per block | idle LDS per block, bytes | resident blocks per compute unit (two settings) | resident waves |")
        print("|---|---|---|---|")
        for th in _ints(args.threads):
            cases = [(str(lds), lds) for lds in _ints(args.lds)]
            cases += [(f"{sweep_lib().nfad_sweep_lds_for_cap(w, th)} (libnfad's reservation for a cap of {w} waves)",
                       sweep_lib().nfad_sweep_lds_for_cap(w, th)) for w in _ints(args.waves) if w > 0]
            for label, lds in cases:
                r = [residency(th, lds, 1600, 5000), residency(th, lds, 800, 10000)]
                print(f"| {th} | {label} | {r[0]:.2f} / {r[1]:.2f} | {max(r) * th / 64:.1f} |", flush=True)
        return
    results = []
    for size in args.sizes.split(","):
        n, dtype = SIZES[size] if size in SIZES else (int(size.split(":")[0]), size.split(":")[1])
        td = _TD[dtype]
        es = 2 if dtype != "f32" else 4
        nbytes = n * es
        nsets = args.sets or max(2, -(-(1 << 30) // (4 * nbytes)) + 1)
        g = torch.Generator(device="cpu").manual_seed(1234)
        host = [torch.randn(n, generator=g, dtype=torch.float32).to(td) for _ in range(2)]
        host[1].mul_(0.1)
        placements = {}
        if not args.skew:
            placements[None] = [{"in": [h.to(dev) for h in host],
                                 "out": [torch.empty(n, dtype=td, device=dev) for _ in range(2)]} for _ in range(nsets)]
        else:
            skews = _ints(args.skew)
            assert all(k >= 0 and k % 16 == 0 for k in skews), "--skew: non-negative multiples of 16"
            span = -(-nbytes // _SKEW_ALIGN) * _SKEW_ALIGN
            arenas = [torch.empty(4 * span + 3 * max(skews) + _SKEW_ALIGN, dtype=torch.uint8, device=dev)
                      for _ in range(nsets * len(skews))]
            for j, skew in enumerate(skews):
                placements[skew] = []
                for arena in arenas[j * nsets:(j + 1) * nsets]:
                    first = (-arena.data_ptr()) % _SKEW_ALIGN
                    t = [arena[first + k * (span + skew):first + k * (span + skew) + nbytes].view(td) for k in range(4)]
                    t[0].copy_(host[0])
                    t[1].copy_(host[1])
                    placements[skew].append({"in": t[:2], "out": t[2:]})
        sets = next(iter(placements.values()))
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        for pattern in args.patterns.split(","):
            code, n_in, n_out, arith = PATTERNS[pattern]
            moved = (n_in + n_out) * nbytes
            use_graph = moved < 64e6
            rows = []
            if args.phased:
                assert arith and pattern in ("bwd",) + tuple(k for k in PATTERNS if k.startswith("fwd_")) and dtype != "f16"
                for wv, u, gr in itertools.product(_ints(args.waves), _ints(args.unroll), args.grid.split(",")):
                    persistent = gr != "0"
                    variants = [("unphased", 0, 0)]
                    chunk = cus * wv * u * 1024           # bytes per tensor per period, chip-wide
                    for sc in [float(v) for v in args.phase_scale.split(",")]:
                        read = int(n_in * chunk / (7.1e12 * sc) * 1e8)
                        variants.append((f"phased x{sc}: period {10 * (read + int(n_out * chunk / (6.9e12 * sc) * 1e8))} ns, "
                                         f"reads in the first {10 * read} ns", read + int(n_out * chunk / (6.9e12 * sc) * 1e8), read))
                    for label, period, read in variants:
                        def fn(s, st, wv=wv, u=u, persistent=persistent, period=period, read=read):
                            launch_phased(pattern, dtype, u, wv, persistent, period, read, s["in"][:n_in],
                                          s["out"][:n_out], n, st)
                        rows.append({"size": size, "pattern": pattern, "fn": fn, "shape": {"waves": wv, "unroll": u, "persistent": persistent, "period": period, "read": read},
                                     "label": f"T64 U{u} w{wv} {'persistent' if persistent else 'one block per tile'} {label}"})
            for th, u, adj, ntl, nts, wv, gr, ch, skew in ([] if args.phased else itertools.product(
                    _ints(args.threads), _ints(args.unroll), _ints(args.adjacent), _ints(args.ntl),
                    _ints(args.nts), _ints(args.waves), args.grid.split(","), _ints(args.chunk), list(placements))):
                if arith and (nts == 0 or adj or ch or u > 4 or th > 512):
                    continue    # the arithmetic patterns are libnfad's own kernel template: fewer knobs
                shape = {"threads": th, "unroll": u, "adjacent": adj, "ntl": ntl, "nts": nts, "waves": wv,
                         "grid": _grid_of(gr, cus), "chunk": ch}

                def fn(s, st, shape=shape):
                    launch(pattern, dtype, shape, s["in"][:n_in], s["out"][:n_out] if n_out else [sink], n, st)
                rows.append({"size": size, "pattern": pattern, "shape": shape, "fn": fn, "skew": skew,
                             "sets": placements[skew], "label":
                             f"T{th} U{u}{' adj' if adj else ''} ntl{ntl} nts{nts} w{wv} g{gr} c{ch}"
                             + ("" if skew is None else f" skew {skew}")})
            if args.lib:
                lib_fn = None
                if pattern in ("r1w2",) or pattern.startswith("fwd_"):
                    kind = code - 10 if arith else B.SWISH
                    lib_fn = (lambda s, st, kind=kind: B.nfad_fwd(kind, s["in"][0], s["out"][0], s["out"][1], st))
                    name = f"libnfad nfad_fwd({B.KIND_NAMES[kind]})"
                elif pattern in ("r2w1", "bwd"):
                    lib_fn = (lambda s, st: B.nfad_bwd(s["in"][0], s["in"][1], s["out"][0], st))
                    name = "libnfad nfad_bwd"
                elif pattern == "r1w1" or pattern.startswith("recompute_fwd_"):
                    kind = code - 30 if arith else B.SWISH
                    lib_fn = (lambda s, st, kind=kind: B.nfad_recompute_fwd(kind, s["in"][0], s["out"][0], st))
                    name = f"libnfad nfad_recompute_fwd({B.KIND_NAMES[kind]})"
                if lib_fn is not None:
                    for skew in placements:
                        rows.append({"size": size, "pattern": pattern, "shape": None, "fn": lib_fn, "skew": skew,
                                     "sets": placements[skew],
                                     "label": name + ("" if skew is None else f" skew {skew}")})

            if not args.no_verify:
                for r in rows:
                    if r["shape"] is not None:
                        first = r.get("sets", sets)[0]
                        for o in first["out"]:
                            o.zero_()
                        r["fn"](first, stream.cuda_stream)
                        _verify(pattern, dtype, first["in"][:n_in], first["out"][:n_out], n)

            def runner(fn, count, own):
                def enqueue():
                    st = torch.cuda.current_stream().cuda_stream
                    for i in range(count):
                        fn(own[i % nsets], st)
                if not use_graph:
                    return enqueue
                gph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gph):
                    enqueue()
                return gph.replay

            for r in rows:
                r["run"] = runner(r["fn"], args.launches, r.pop("sets", sets))
                r["us"] = []
            for rnd in range(args.rounds):
                for r in rows:
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    while (time.perf_counter() - t0) * 1e3 < args.warm_ms:
                        r["run"]()
                        torch.cuda.synchronize()
                    r["run"]()
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    r["run"]()
                    e1.record(stream)
                    torch.cuda.synchronize()
                    r["us"].append(e0.elapsed_time(e1) * 1e3 / args.launches)
                print(f"# {size} {pattern}: round {rnd + 1}/{args.rounds} done ({len(rows)} rows)", file=sys.stderr,
                      flush=True)
            for r in rows:
                us = sorted(r["us"])[len(r["us"]) // 2]
                r["med_us"] = us
                r["GB/s"] = moved / (us * 1e-6) / 1e9
                del r["run"], r["fn"]
            rows.sort(key=lambda r: r["med_us"])
            print(f"\n### {size} ({n} x {dtype}) {pattern}: {moved / 1e6:.1f} MB per launch, "
                  f"{'graph replay' if use_graph else 'direct launches'}, {nsets} buffer sets\n")
            print("| shape | us (median of rounds) | GB/s | of 8 TB/s | rounds, us |")
            print("|---|---|---|---|---|")
            shown = rows if not args.top else rows[:args.top] + [r for r in rows[args.top:] if r["shape"] is None]
            for r in shown:
                print(f"| {r['label']} | {r['med_us']:.2f} | {r['GB/s']:.0f} | {r['GB/s'] / 8000:.3f} | "
                      f"{' '.join(f'{v:.2f}' for v in r['us'])} |")
            sys.stdout.flush()
            results += rows
        del sets, placements
        torch.cuda.empty_cache()
    if args.out:
        os.makedirs(os.path.dirname(os.path.abspath(args.out)), exist_ok=True)
        with open(args.out, "a") as f:
            for r in results:
                f.write(json.dumps({k: v for k, v in r.items()}) + "\n")


if __name__ == "__main__":
    main()

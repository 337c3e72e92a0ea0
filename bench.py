#!/usr/bin/env python3
"""Benchmark of the Tesseract per-processor linear hot path on one MI355X.

A step is one pass of the whole hot path over one processor's share of a
workload: for every linear layer of the workload, forward (bias/GELU epilogue
fused), input gradient and the depth-slice weight gradient accumulated into an
fp32 buffer.  Inputs are seeded synthetic panels, resident in HBM before the
timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, the published figure (256 CU x 4096 flop/clk x 2.4 GHz = 2516.6)
PEAK_FP32_VECTOR_TFLOPS = 157.3   # MI355X fp32 vector ALU (the plain fp32 kernel of configuration 1)
DEFAULT_WORKLOAD = "cfg4_q4d4_bf16_attn_h8192"   # the largest per-processor block shapes


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-sustained", action="store_true", help="skip the 3-second sustained loop")
    ap.add_argument("--no-others", action="store_true", help="skip the other configurations")
    ap.add_argument("--graph", action="store_true",
                    help="with --sweep: record one step (all calls of all layers) into a HIP graph "
                         "after the warm-up and time replays of it, which removes the per-launch host "
                         "cost that dominates the small strong-scaling shapes")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: one JSON line per grid of the paper's own "
                         "experiment tables (QKV, attention output and the two MLP layers at the "
                         "per-processor block shapes), inputs drawn on the device")
    ap.add_argument("--layernorm", action="store_true",
                    help="instead of the benchmark line: time the local layer-normalisation kernels "
                         "(row sums, normalise) on the workload's first layer's X block, in GB/s")
    ap.add_argument("--mlp-chain", action="store_true",
                    help="for a workload with an up and a down layer: also time the two layers as one "
                         "dependent chain (pre-activation kept, GELU' and bias gradients fused)")
    ap.add_argument("--epilogues", action="store_true",
                    help="also time dX through GELU' and dW with the bias gradient beside the plain calls")
    ap.add_argument("--compare-vendor", action="store_true",
                    help="diagnostic only: launch this library's input-gradient kernel (q = 1) and the vendor GEMM "
                         "behind torch.matmul on the same 8192^3 NT problem, a few times each, and print both "
                         "timings; meant to be run under rocprofv3 counters")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    return ap.parse_args()


class LayerState:
    """Device buffers of one layer of one processor's share (packed panels)."""

    def __init__(self, torch, tess, B, wl, w, L, seed, sets, on_device=False):
        self.L = L
        self.q, self.d = w.q, w.d
        self.desc = B.make_desc(w.q, w.d, 0, 0, 0, L.a, L.b, L.c, B.BF16, B.BF16)
        self.act = {"none": B.ACT_NONE, "gelu_erf": B.ACT_GELU_ERF}[L.act]
        self.flops_call = 2.0 * L.m * L.kb * L.n * w.q          # 2abc/p
        self.sets = []
        self.host = None
        for s in range(sets):
            if on_device:
                # shape sweeps: same distributions, drawn by the device generator (seconds
                # instead of minutes for the multi-GB panel sets); no host copy is kept
                g = torch.Generator(device="cuda:0")
                g.manual_seed(seed + s)
                rn = lambda shape, std: (torch.randn(shape, generator=g, device="cuda:0") * std).to(torch.bfloat16)
                inp = {"x": rn((w.q, L.m, L.kb), 1.0), "w": rn((w.q, L.kb, L.n), 0.02),
                       "bias": rn((L.n,), L.bias_std), "dy": rn((w.q, L.m, L.n), 1.0)}
            else:
                inp = wl.share_inputs(w.q, L.m, L.kb, L.n, dtype="bf16", seed=seed + s,
                                      bias_std=L.bias_std)
            if s == 0 and not on_device:
                self.host = inp
            dev = {k: v.to("cuda:0") for k, v in inp.items()}
            dev["y"] = torch.empty((L.m, L.n), dtype=torch.bfloat16, device="cuda:0")
            dev["dx"] = torch.empty((L.m, L.kb), dtype=torch.bfloat16, device="cuda:0")
            dev["dw"] = torch.zeros((L.kb, L.n), dtype=torch.float32, device="cuda:0")
            dev["xl"], dev["wl"], dev["dyl"] = list(dev["x"]), list(dev["w"]), list(dev["dy"])
            self.sets.append(dev)
        nbytes = max(tess.workspace_bytes(self.desc, op) for op in (0, 1, 2))
        self.ws = torch.empty(max(nbytes, 4) // 4, dtype=torch.float32, device="cuda:0")
        self.tess = tess

    def fwd(self, s):
        b = self.sets[s % len(self.sets)]
        self.tess.linear_fwd(self.desc, b["xl"], b["wl"], b["bias"], self.act, b["y"],
                             workspace=self.ws)

    def dx(self, s):
        b = self.sets[s % len(self.sets)]
        self.tess.linear_bwd_dx(self.desc, b["dyl"], b["wl"], b["dx"], workspace=self.ws)

    def dw(self, s):
        b = self.sets[s % len(self.sets)]
        self.tess.linear_bwd_dw(self.desc, b["xl"], b["dyl"], b["dw"], accumulate=True,
                                workspace=self.ws)

    # the backward epilogues next to the path (timed by --epilogues only)
    def dx_act(self, s):
        b = self.sets[s % len(self.sets)]
        if "z" not in b:
            import torch
            b["z"] = torch.randn((self.L.m, self.L.kb), device="cuda:0").to(torch.bfloat16)
        self.tess.linear_bwd_dx_act(self.desc, b["dyl"], b["wl"], b["z"], 1, b["dx"], workspace=self.ws)

    def dw_bias(self, s):
        b = self.sets[s % len(self.sets)]
        if "db" not in b:
            import torch
            b["db"] = torch.zeros((self.L.n,), dtype=torch.float32, device="cuda:0")
        self.tess.linear_bwd_dw_bias(self.desc, b["xl"], b["dyl"], b["dw"], b["db"], accumulate=True,
                                     workspace=self.ws)


def time_workload(torch, tess, B, wl, w, steps, warmup, on_device=False, graph=False):
    layers = []
    for li, L in enumerate(w.layers):
        per_set = 2 * w.q * (L.m * L.kb + L.kb * L.n + L.m * L.n) + 2 * (L.m * L.n + L.m * L.kb) \
            + 4 * L.kb * L.n
        sets = 1 if per_set >= 400e6 else max(2, int(600e6 // per_set))
        layers.append(LayerState(torch, tess, B, wl, w, L, seed=1000 * li, sets=min(sets, 8),
                                 on_device=on_device))

    names = ("fwd", "dx", "dw")

    def step(s, marks=None):
        for st in layers:
            for name in names:
                if marks is not None:
                    e = torch.cuda.Event(enable_timing=True)
                    e.record()
                    marks.append(e)
                getattr(st, name)(s)
        if marks is not None:
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            marks.append(e)

    for s in range(warmup):
        step(s)
    torch.cuda.synchronize()
    if graph:
        # the library only enqueues kernels on the given stream (no allocation, no memset, no
        # synchronisation), so a step can be recorded as it is; buffer set 0 is replayed
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(0)
        torch.cuda.current_stream().wait_stream(side)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step(0)
        for _ in range(max(1, warmup)):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        flops_step = sum(3.0 * st.flops_call for st in layers)
        ms_step = dt / steps * 1e3
        return {"ms_per_step": ms_step, "tflops": flops_step / ms_step / 1e9, "calls": {},
                "flops_step": flops_step, "layers": layers}
    # the timed region: exactly K steps between two synchronisations, nothing else enqueued
    t0 = time.perf_counter()
    for s in range(steps):
        step(s)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    flops_step = sum(3.0 * st.flops_call for st in layers)
    ms_step = dt / steps * 1e3
    # the same K steps once more with one HIP event on the launch stream at every call
    # boundary: each call's average duration (an event between 20-microsecond kernels would
    # distort the step time above, so the two passes are kept apart)
    marks = [[] for _ in range(steps)]
    for s in range(steps):
        step(s, marks[s])
    torch.cuda.synchronize()

    calls = {}
    ci = 0
    for st in layers:
        for name in names:
            per_step = sorted(m[ci].elapsed_time(m[ci + 1]) for m in marks)
            ms = sum(per_step) / steps
            ms_median, ms_min = per_step[len(per_step) // 2], per_step[0]
            ci += 1
            M, N, K = {"fwd": (st.L.m, st.L.n, st.L.kb * w.q), "dx": (st.L.m, st.L.kb, st.L.n * w.q),
                       "dw": (st.L.kb, st.L.n, st.L.m * w.q)}[name]
            tm, tn, ks = tess.plan(st.desc, {"fwd": B.OP_FWD, "dx": B.OP_BWD_DX, "dw": B.OP_BWD_DW}[name])
            calls[f"{st.L.name}.{name}"] = {"MxNxK": f"{M}x{N}x{K}", "tile": f"{tm}x{tn}", "k_splits": ks,
                                            "ms": round(ms, 4), "ms_median": round(ms_median, 4),
                                            "ms_min": round(ms_min, 4),
                                            "tflops": round(st.flops_call / ms / 1e9, 1),
                                            "frac_peak": round(st.flops_call / ms / 1e9 / PEAK_BF16_TFLOPS, 4)}
    return {"ms_per_step": ms_step, "tflops": flops_step / ms_step / 1e9, "calls": calls,
            "flops_step": flops_step, "layers": layers, "step": step}


def cpu_baseline(torch, w, layer_state, budget_s=24.0):
    """The fp64 oracle as it stands, on a bounded sample of the first layer's calls:
    a subset of output rows (and, for dW, a window of columns) of the same panels."""
    import numpy as np
    from oracle import tess_oracle as orc
    L, q = layer_state.L, w.q
    host = layer_state.host

    def f64(t):
        return t.to(torch.float64).numpy()

    cols = min(L.n, 1024)
    ws = [f64(host["w"][t]) for t in range(q)]
    dyw = [f64(host["dy"][t][:, :cols]) for t in range(q)]

    def run(rows_fwd, rows_dx, rows_dw):
        rf = np.linspace(0, L.m - 1, rows_fwd).astype(np.int64)
        rx = np.linspace(0, L.m - 1, rows_dx).astype(np.int64)
        rw = np.linspace(0, L.kb - 1, rows_dw).astype(np.int64)
        xs = [f64(host["x"][t][rf]) for t in range(q)]
        dys = [f64(host["dy"][t][rx]) for t in range(q)]
        xcols = [np.ascontiguousarray(f64(host["x"][t][:, rw])) for t in range(q)]
        t0 = time.perf_counter()
        orc.fwd_panels(xs, ws, bias=f64(host["bias"]), act=orc.ACT_GELU_ERF if L.act == "gelu_erf" else 0)
        orc.bwd_dx_panels(dys, ws)
        orc.bwd_dw_panels(xcols, dyw)
        dt = time.perf_counter() - t0
        fl = 2.0 * q * L.kb * L.n * (rows_fwd + rows_dx) + 2.0 * q * L.m * cols * rows_dw
        return fl, dt

    fl, dt = run(64, 64, 64)                   # calibration (every thread gets rows)
    rate = fl / dt
    per_row = 2.0 * q * L.kb * L.n
    rows = int(max(8, min(L.m, budget_s / 3 * rate / per_row)))
    rows_dw = int(max(8, min(L.kb, budget_s / 3 * rate / (2.0 * q * L.m * cols))))
    fl, dt = run(rows, rows, rows_dw)
    return {"value": round(fl / dt / 1e12, 6), "unit": "TFLOP/s", "cores": orc.num_threads(),
            "kind": "oracle",
            "sample": f"{w.name}/{L.name}: fwd and dX on {rows} evenly spaced output rows "
                      f"(all columns), dW on {rows_dw} output rows x first {cols} columns; "
                      f"{fl / 1e9:.1f} GFLOP in {dt:.1f} s, fp64"}


def time_config1(torch, tess, B, wl, steps, warmup):
    """Configuration 1: the whole [2,2,1] grid in fp32 on the plain fp32-FMA kernel, one
    processor after the other on strided views of the global matrices (12 calls per step)."""
    import itertools
    from paper_2105_14500_amd import partition as P
    w = wl.WORKLOADS[0]
    L = w.layers[0]
    q, d, a, b, c = w.q, w.d, L.a, L.b, L.c
    X, W, bias, dY = (t.to("cuda:0") for t in wl.full_grid_inputs(a, b, c, dtype="f32", seed=0, bias_std=0.0))
    Y = torch.empty((a, c), device="cuda:0")
    dX = torch.empty((a, b), device="cuda:0")
    dW = torch.zeros((b, c), device="cuda:0")
    n = c // q
    procs = []
    for i, j, k in itertools.product(range(q), range(q), range(d)):
        desc = B.make_desc(q, d, i, j, k, a, b, c, B.F32, B.F32)
        procs.append((desc, P.fwd_panels(X, W, q, d, i, j, k), bias[j * n:(j + 1) * n], P.out_block(Y, q, d, i, j, k),
                      P.dx_panels(dY, W, q, d, i, j, k), P.out_block(dX, q, d, i, j, k),
                      P.dw_panels(X, dY, q, d, i, j, k), P.weight_block(dW, q, i, j)))

    def step():
        for desc, (ap, bp), bs, yo, (dyp, wp), dxo, (xp, dy2p), dwo in procs:
            tess.linear_fwd(desc, ap, bp, bs, B.ACT_NONE, yo)
            tess.linear_bwd_dx(desc, dyp, wp, dxo)
            tess.linear_bwd_dw(desc, xp, dy2p, dwo, accumulate=True)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    flops = 6.0 * a * b * c
    # the same step replayed from a HIP graph (no host cost per call)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(max(1, warmup)):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_graph = (time.perf_counter() - t0) / steps * 1e3
    return {"tflops": round(flops / ms / 1e9, 3), "ms_per_step": round(ms, 4), "dtype": "f32",
            "calls_per_step": 3 * len(procs), "kernel": "tess_generic_kernel (fp32 FMA)",
            "graph_replay": {"tflops": round(flops / ms_graph / 1e9, 3), "ms_per_step": round(ms_graph, 4)},
            "roofline": {"bound": "alu", "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(flops / ms_graph / 1e9 / PEAK_FP32_VECTOR_TFLOPS, 5),
                         "note": "fraction from the graph replay"},
            "note": "34 MFLOP per call on 16-64 workgroups: bound by the latency of each thread's dependent chain and by launch latency, not by the ALUs"}


def sustained(torch, step, flops_step, seconds=3.0):
    """The same step looped for `seconds`: ms/step over the last second, with the shader clock
    that rocm-smi reports sampled beside it (short bursts run at a higher clock than a
    sustained load under the board's power limit)."""
    import re
    import subprocess
    import threading
    clocks, stop = [], threading.Event()

    def sample():
        while not stop.is_set():
            try:
                r = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=5)
                m = re.search(r"sclk clock level:\s*\d+:?\s*\((\d+)Mhz\)", r.stdout)
                if m:
                    clocks.append((time.perf_counter(), int(m.group(1))))
            except Exception:
                pass
            stop.wait(0.25)

    th = threading.Thread(target=sample, daemon=True)
    th.start()
    chunks, n = [], 0
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    while time.perf_counter() - t_start < seconds:
        t0 = time.perf_counter()
        for _ in range(20):
            step(n)
            n += 1
        torch.cuda.synchronize()
        chunks.append((time.perf_counter(), (time.perf_counter() - t0) / 20 * 1e3))
    t_end = time.perf_counter()
    stop.set()
    th.join(timeout=6)
    last = [ms for t, ms in chunks if t >= t_end - 1.0] or [chunks[-1][1]]
    first = chunks[0][1]
    ms_last = sum(last) / len(last)
    sclk = [c for t, c in clocks if t >= t_end - 1.5 and t <= t_end]
    return {"seconds": round(t_end - t_start, 2), "steps": n, "ms_per_step_first_chunk": round(first, 4),
            "ms_per_step_last_second": round(ms_last, 4), "tflops_last_second": round(flops_step / ms_last / 1e9, 1),
            "sclk_mhz_last_second": (round(sum(sclk) / len(sclk)) if sclk else None),
            "sclk_source": "rocm-smi --showclocks, sampled every 0.25 s"}


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one processor's share on ONE GPU; "
              "--gpus N with N > 1 is not supported (no collectives are part of it).",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import tess_workloads as wl
    import paper_2105_14500_amd as tess
    from paper_2105_14500_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    if args.calibrate_copy:
        n = 1 << 30
        src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": n, "launches": 3}))
        return
    tess.binding.lib()   # fail loudly when the HIP library is missing
    if args.compare_vendor:
        # C[M,N] = A[M,K] B[N,K]^T, both operands K-contiguous: the input-gradient orientation
        M = N = K = 8192
        g = torch.Generator(device="cuda:0")
        g.manual_seed(0)
        a = torch.randn((M, K), generator=g, device="cuda:0").to(torch.bfloat16)
        b = (torch.randn((N, K), generator=g, device="cuda:0") * 0.02).to(torch.bfloat16)
        desc = B.make_desc(1, 1, 0, 0, 0, M, N, K, B.BF16, B.BF16)      # dX[m, kb] = dY[m, n] W[kb, n]^T
        out = torch.empty((M, N), dtype=torch.bfloat16, device="cuda:0")
        nbytes = tess.workspace_bytes(desc, B.OP_BWD_DX)
        ws = torch.empty(max(nbytes, 4) // 4, dtype=torch.float32, device="cuda:0")
        res = {}
        for name, fn in (("tess_linear_bwd_dx", lambda: tess.linear_bwd_dx(desc, [a], [b], out, workspace=ws)),
                         ("torch.matmul", lambda: torch.matmul(a, b.t()))):
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(6):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 6
            res[name] = {"ms": round(ms, 4), "tflops": round(2.0 * M * N * K / ms / 1e9, 1)}
        ref = torch.matmul(a, b.t())
        res["max_abs_difference"] = float((out.float() - ref.float()).abs().max())
        print(json.dumps({"compare_vendor": res, "MxNxK": f"{M}x{N}x{K}", "layout": "NT", "dtype": "bf16"}))
        return
    w = wl.workload_by_name(args.workload)
    if w is None or w.dtype != "bf16":
        print(f"unknown bf16 workload {args.workload}", file=sys.stderr)
        sys.exit(2)

    if args.layernorm:
        L = w.layers[0]
        # rotate over enough blocks that the working set exceeds the 256 MiB last-level cache
        nbuf = max(2, int(1.2e9 // (L.m * L.kb * 4)))
        xs = [torch.randn((L.m, L.kb), device="cuda:0").to(torch.bfloat16) for _ in range(nbuf)]
        outs = [torch.empty_like(xs[0]) for _ in range(nbuf)]
        x = xs[0]
        sums = torch.empty((L.m, 2), dtype=torch.float32, device="cuda:0")
        res = {}
        for name, fn, nbytes in (("row_sums", lambda i: B.layernorm_row_sums(xs[i % nbuf], sums),
                                  x.numel() * 2 + L.m * 8),
                                 ("normalize", lambda i: B.layernorm_normalize(xs[i % nbuf], sums, L.kb * w.q,
                                                                               1e-5, outs[i % nbuf]),
                                  x.numel() * 4 + L.m * 8)):
            for i in range(args.warmup):
                fn(i)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(args.steps):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            res[name] = {"ms": round(ms, 4), "GBps": round(nbytes / ms / 1e6, 1),
                         "frac_of_8TBps": round(nbytes / ms / 1e6 / 8000.0, 3), "bytes": nbytes}
        print(json.dumps({"layernorm": res, "block": [L.m, L.kb], "dtype": "bf16", "workload": w.name}))
        return
    if args.sweep:
        for ow in wl.PAPER_TABLE_WORKLOADS:
            torch.cuda.empty_cache()
            r = time_workload(torch, tess, B, wl, ow, args.steps, args.warmup, on_device=True,
                              graph=args.graph)
            print(json.dumps({"workload": ow.name, "grid": [ow.q, ow.q, ow.d], "graph_replay": args.graph,
                              "tflops": round(r["tflops"], 1), "ms_per_step": round(r["ms_per_step"], 4),
                              "calls": {k: {"MxNxK": v["MxNxK"], "tile": v["tile"], "k_splits": v["k_splits"],
                                            "ms": v["ms"], "tflops": v["tflops"]}
                                        for k, v in r["calls"].items()}}), flush=True)
            del r
        return
    # what the matrix cores sustain on this device at its actual clock (no memory traffic):
    # with operands of small integers, and with operands distributed like the workload's --
    # under the board's power limit the sustained clock depends on how much the operands switch
    sink = torch.empty(256 * 256, dtype=torch.float32, device="cuda:0")

    def probe(real):
        B.probe_mfma_rate(sink, 256, 1000, real_data=real)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flop = sum(B.probe_mfma_rate(sink, 256, 10000, real_data=real) for _ in range(3))
        e1.record()
        torch.cuda.synchronize()
        return flop / e0.elapsed_time(e1) / 1e9

    mfma_only = probe(False)
    mfma_only_real = probe(True)

    res = time_workload(torch, tess, B, wl, w, args.steps, args.warmup)
    # dominant kernel = the call with the most flops that is ONE launch of the MFMA kernel
    # (calls with K splits also run a reduction kernel, so their event time covers two
    # kernels); among equals the first listed, i.e. the forward call, whose launch shape is
    # unique in a kernel trace
    single = {k: v for k, v in res["calls"].items() if v["k_splits"] == 1} or res["calls"]
    layer_of = lambda name: next(st for st in res["layers"] if name.startswith(st.L.name + "."))
    dom_name = max(single, key=lambda name: layer_of(name).flops_call)
    dom, dom_layer = single[dom_name], layer_of(dom_name)
    # HBM-side bytes per launch of that call: from the committed rocprofv3 counter summary (two
    # --pmc runs of this script; counters cannot be read from inside the run)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_cfg4.txt")
    if os.path.exists(tpath):
        rows = [l for l in open(tpath) if l.strip() and not l.startswith("#")]
        if rows:
            entry = json.loads(rows[-1]).get(f"{w.name}/{dom_name}")
            traffic = entry["bytes"] if entry else None
    out = {
        "metric": "TFLOP/s and % of bf16 MFMA peak, Tesseract linear fwd+bwd, 1 MI355X",
        "value": round(res["tflops"], 2),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(res["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "pct_of_bf16_mfma_peak": round(100.0 * res["tflops"] / PEAK_BF16_TFLOPS, 2),
        "mfma_only_loop_tflops": round(mfma_only, 1),
        "mfma_only_loop_workload_like_operands_tflops": round(mfma_only_real, 1),
        "pct_of_mfma_only_loop": round(100.0 * res["tflops"] / mfma_only, 2),
        "pct_of_mfma_only_loop_workload_like_operands": round(100.0 * res["tflops"] / mfma_only_real, 2),
        "config": {"workload": w.name, "grid": [w.q, w.q, w.d], "processor": [0, 0, 0],
                   "layers": {L.name: {"a": L.a, "b": L.b, "c": L.c, "block": [L.m, L.kb, L.n],
                                       "epilogue": L.act} for L in w.layers},
                   "step": "per layer: fwd + dX + dW(accumulate fp32)",
                   "flop_per_step": res["flops_step"]},
        "calls": res["calls"],
        "roofline": {"bound": "mfma", "kernel": "tess_mfma_kernel, call " + dom_name + " " + dom["MxNxK"],
                     "achieved": dom["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(dom["tflops"] / PEAK_BF16_TFLOPS, 4),
                     "flop_per_launch": dom_layer.flops_call, "avg_ms": dom["ms"],
                     "avg_ms_median": dom["ms_median"], "avg_ms_min": dom["ms_min"],
                     "traffic": traffic, "traffic_source": "profiles/hbm_traffic_cfg4.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)",
                     # context: what a register-resident MFMA-only loop (no data movement at all)
                     # reached in this run, on small-integer operands and on operands distributed
                     # like the workload's: the second is the ceiling that the board's power
                     # limit leaves to ANY kernel on this data
                     "mfma_only_loop": round(mfma_only, 1),
                     "mfma_only_loop_workload_like_operands": round(mfma_only_real, 1),
                     "frac_of_mfma_only_loop": round(dom["tflops"] / mfma_only, 4),
                     "frac_of_mfma_only_loop_workload_like_operands": round(dom["tflops"] / mfma_only_real, 4)},
    }
    if not args.no_sustained:
        out["sustained"] = sustained(torch, res["step"], res["flops_step"], seconds=3.0)
        out["sustained"]["pct_of_bf16_mfma_peak"] = round(100.0 * out["sustained"]["tflops_last_second"] / PEAK_BF16_TFLOPS, 2)
    if args.mlp_chain:
        by_name = {L.name: L for L in w.layers}
        if "up" not in by_name or "down" not in by_name:
            raise SystemExit("--mlp-chain needs a workload with an 'up' and a 'down' layer")
        from paper_2105_14500_amd.mlp import MlpShare
        up = by_name["up"]
        mlp = MlpShare(w.q, w.d, up.m, up.kb, up.n)
        sup = next(st for st in res["layers"] if st.L.name == "up").sets[0]
        sdn = next(st for st in res["layers"] if st.L.name == "down").sets[0]
        # peers' blocks: the down layer's X panels stand for H, the up layer's dY panels for dZ1
        fw = lambda: mlp.forward(sup["xl"], sup["wl"], sup["bias"], sdn["xl"], sdn["wl"], sdn["bias"])
        bw = lambda: mlp.backward(sup["xl"], sup["wl"], sdn["xl"], sdn["wl"], sdn["dyl"], sup["dyl"])
        for _ in range(args.warmup):
            fw(); bw()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fw(); bw()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / args.steps * 1e3
        out["mlp_chain"] = {"ms_per_step": round(ms, 4), "tflops": round(mlp.flops() / ms / 1e9, 1),
                            "calls": "fwd(up, preact kept) fwd(down) dw_bias(down) dx_act(down) dw_bias(up) dx(up)"}
    if args.epilogues:
        ep = {}
        for st in res["layers"]:
            for plain, fused in (("dx", "dx_act"), ("dw", "dw_bias")):
                # alternate the two variants launch by launch so that both see the same clocks
                fp, ff = getattr(st, plain), getattr(st, fused)
                fp(0); ff(0)
                torch.cuda.synchronize()
                marks = []
                for s_ in range(args.steps):
                    for fn in (fp, ff):
                        e = torch.cuda.Event(enable_timing=True)
                        e.record()
                        marks.append(e)
                        fn(s_)
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                marks.append(e)
                torch.cuda.synchronize()
                tp = sum(marks[2 * i].elapsed_time(marks[2 * i + 1]) for i in range(args.steps)) / args.steps
                tf = sum(marks[2 * i + 1].elapsed_time(marks[2 * i + 2]) for i in range(args.steps)) / args.steps
                ep[f"{st.L.name}.{fused}"] = {plain + "_ms": round(tp, 4), fused + "_ms": round(tf, 4)}
        out["backward_epilogues"] = ep
    layers0 = res["layers"]
    if w.name == DEFAULT_WORKLOAD and not args.no_others:
        # every other configuration rides along (per-call figures; panels drawn on the device
        # with the same distributions, which takes seconds instead of minutes)
        others = {}
        res = None
        for ow in wl.WORKLOADS:
            if ow.dtype != "bf16" or ow.name == w.name:
                continue
            torch.cuda.empty_cache()
            r = time_workload(torch, tess, B, wl, ow, args.steps, args.warmup, on_device=True)
            others[ow.name] = {"tflops": round(r["tflops"], 2),
                               "pct_peak": round(100.0 * r["tflops"] / PEAK_BF16_TFLOPS, 2),
                               "ms_per_step": round(r["ms_per_step"], 4), "calls": r["calls"]}
            del r
        # the small MLP up-projection replayed from a HIP graph: what is left once the
        # per-launch host cost is gone
        ow = wl.workload_by_name("cfg2_q2d2_bf16_mlp_up_h1024")
        rg = time_workload(torch, tess, B, wl, ow, args.steps, args.warmup, on_device=True, graph=True)
        others[ow.name]["graph_replay"] = {"tflops": round(rg["tflops"], 2), "ms_per_step": round(rg["ms_per_step"], 4)}
        del rg
        others[wl.WORKLOADS[0].name] = time_config1(torch, tess, B, wl, max(args.steps, 20), args.warmup)
        out["other_workloads"] = others
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(torch, w, layers0[0])
    print(json.dumps(out))


if __name__ == "__main__":
    main()

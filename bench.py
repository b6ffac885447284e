#!/usr/bin/env python3
"""Benchmark of the BLR linear forward path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C1] [--sweep] [--no-cpu]

A step is one forward call of the workload's layer (every kernel of the call) on inputs that are
already resident in HBM. The default (headline) workload is the largest Llama-7B-shaped layer of the
token sweep the metric is quoted on: Monarch 4096 -> 11008, nblocks = 4, r = 1024, T = 8192, bf16.
Prints ONE JSON line on stdout; by default the line also carries `sweep`: the ViT-B-width BLAST
layer and the four Llama-7B-shaped layers at T = 1 ... 8192, each with its time (median of graph
replays), tokens/s, roofline bound and fraction, the same-shape dense GEMM, the cold-cache time for
T <= 128 and a short run of the CPU oracle (`--no-sweep` leaves it out). `--sweep` widens that to
the low-rank layers and to the forced executions of every call and also writes the table to
sweep.json in the results folder (OUT_DIR below).

Static factors are re-laid out once before the timed region (the paper's offline weight
re-layout); the timed call receives the packed factors.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
OUT_DIR = "gpurun_out"          # where the tables of --sweep and --table3 are written
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

import blr_inputs as bi  # noqa: E402
from paper_2512_20861_amd import roofline as rf  # noqa: E402


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def to_dev(ht):
    import torch
    if ht.dtype == "bf16":
        return torch.from_numpy(ht.bits.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(ht.bits.copy()).cuda()


class GpuLayer:
    """Device-resident factors of one layer plus a closure that enqueues its forward."""

    def __init__(self, cfg, T, seed=bi.BASE_SEED, random_x=True, host=None):
        import torch
        from paper_2512_20861_amd import binding as B
        self.B, self.cfg, self.T = B, cfg, T
        self.op, self.n_in, self.n_out = cfg["op"], cfg["n_in"], cfg["n_out"]
        self.dtype = cfg["dtype"]
        td = torch.bfloat16 if self.dtype == "bf16" else torch.float32
        lay = host if host is not None else bi.make_layer(cfg, seed)
        self.host = lay
        # activations: values do not affect run time; draw them on the device for the big sweeps
        if random_x:
            self.X = (torch.randn((T, self.n_in), device="cuda", dtype=torch.float32) * cfg["x_scale"]).to(td)
        self.Y = torch.empty((T, self.n_out), device="cuda", dtype=td)
        dt = B.BF16 if self.dtype == "bf16" else B.F32
        if self.op == "monarch":
            self.R, self.L = to_dev(lay.R), to_dev(lay.L)
            self.nb, self.r = cfg["nblocks"], cfg["r"]
            self.ws = torch.empty(max(B.monarch_workspace_bytes(T, self.n_in, self.n_out, self.nb, self.r, dt), 16),
                                  dtype=torch.uint8, device="cuda")
            self.flags = 0
        elif self.op == "lowrank":
            self.V, self.U, self.r = to_dev(lay.V), to_dev(lay.U), cfg["r"]
            self.ws = torch.empty(max(B.lowrank_workspace_bytes(T, self.n_in, self.n_out, self.r, dt), 16), dtype=torch.uint8, device="cuda")
            self.flags = 0
        else:
            self.U, self.S, self.V = to_dev(lay.U), to_dev(lay.S), to_dev(lay.V)
            self.b, self.r = cfg["b"], cfg["r"]
            self.flags = 0
            if B.blast_packed_bytes(self.n_in, self.n_out, self.b, self.r, dt) > 0:
                self.packed = B.blast_pack(self.U, self.S, self.V, self.n_in, self.n_out, self.b, self.r)
                self.flags = B.BLAST_PACKED
            self.ws = torch.empty(max(B.blast_workspace_bytes(T, self.n_in, self.n_out, self.b, self.r, dt, self.flags), 16),
                                  dtype=torch.uint8, device="cuda")

    def set_x(self, X):
        self.X = X

    def call_args(self, extra_flags=0):
        B = self.B
        if self.op == "monarch":
            return (B.monarch_forward, self.X, self.R, self.L, self.Y, self.nb, self.r, self.flags | extra_flags, self.ws)
        if self.op == "lowrank":
            return (B.lowrank_forward, self.X, self.V, self.U, self.Y, self.flags | extra_flags, self.ws)
        if self.flags & B.BLAST_PACKED:
            return (B.blast_forward, self.X, self.U, None, self.packed, self.Y, self.b, self.r, self.flags | extra_flags, self.ws)
        return (B.blast_forward, self.X, self.U, self.S, self.V, self.Y, self.b, self.r, self.flags | extra_flags, self.ws)

    def forward(self, extra_flags=0):
        a = self.call_args(extra_flags)
        a[0](*a[1:])

    def prepared(self, extra_flags=0):
        """Zero-argument callable that re-issues the C call with pre-marshalled arguments on the
        stream that is current now."""
        return self.B.prepared(*self.call_args(extra_flags))

    def shape_args(self):
        c = self.cfg
        return dict(n_in=c["n_in"], n_out=c["n_out"], r=c["r"], b=c.get("b", c.get("nblocks", 1)))


def time_calls(fn, steps, warmup):
    """Mean milliseconds per call over `steps` back-to-back calls, HIP events on the launch stream."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def time_graph(make_call, steps, warmup, replays=5):
    """Milliseconds per call with the `steps` calls captured once into a HIP graph and replayed: the
    host enqueues one graph launch, so the figure is the GPU's own back-to-back rate rather than the
    speed of the Python launch loop. Every replay is exactly `steps` calls between two events on the
    launch stream; the MEDIAN replay is reported. `make_call()` is evaluated on the capture stream."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call = make_call()
        for _ in range(max(warmup, 1)):
            call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        call = make_call()
        for _ in range(steps):
            call()
    g.replay()
    torch.cuda.synchronize()
    times = []
    for _ in range(replays):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) / steps)
    times.sort()
    return times[len(times) // 2]


def stage_times(layer, steps, warmup):
    """Per-stage mean launch duration (ms): (first, last), or None if the call is a single kernel."""
    B = layer.B
    try:
        t1 = time_graph(lambda: layer.prepared(B.ONLY_FIRST_STAGE), steps, warmup, 1)
        t2 = time_graph(lambda: layer.prepared(B.ONLY_LAST_STAGE), steps, warmup, 1)
        return t1, t2
    except B.BlrError as e:
        if e.status == B.ERR_UNSUPPORTED:
            return None
        raise


def cpu_baseline(cfg, T_cpu, seconds=10.0, lay=None):
    """The fp64 oracle as it stands, timed on this machine's host cores (baseline only): about `seconds`
    of repeated passes over the first T_cpu tokens of the workload."""
    import oracle
    lay = lay if lay is not None else bi.make_layer(cfg)
    X = bi.activations(T_cpu, cfg["n_in"], cfg["dtype"], scale=cfg["x_scale"])
    nthreads = oracle.binding.default_threads()
    if cfg["op"] == "monarch":
        fn = lambda: oracle.monarch_forward(X.f64, lay.R.f64, lay.L.f64, nthreads=nthreads)
    elif cfg["op"] == "lowrank":
        fn = lambda: oracle.lowrank_forward(X.f64, lay.V.f64, lay.U.f64, nthreads=nthreads)
    else:
        fn = lambda: oracle.blast_forward(X.f64, lay.U.f64, lay.S.f64, lay.V.f64, nthreads=nthreads)
    fn()                                                 # warm-up
    passes, t_start = 0, time.perf_counter()
    while True:                                          # about `seconds` of CPU work
        fn()
        passes += 1
        elapsed = time.perf_counter() - t_start
        if (elapsed >= seconds and passes >= min(3, seconds)) or elapsed >= 3 * seconds:
            break
    return {"value": T_cpu * passes / elapsed, "unit": "tokens/s", "cores": min(nthreads, T_cpu), "kind": "oracle",
            "sample": f"{passes} passes over {T_cpu} of the workload's tokens ({elapsed:.1f} s of fp64 oracle time "
                      f"after one warm-up pass), std::thread over tokens"}


def dominant_roofline(layer, ms_total, stages):
    """Roofline entry of the kernel that takes the most time in the call.

    The bytes/FLOPs are the ALGORITHMIC ones of the part of the path that kernel covers:
    inputs + factors it reads + outputs it writes, each once."""
    cfg, T = layer.cfg, layer.T
    sa = layer.shape_args()
    n_in, n_out, r, b = sa["n_in"], sa["n_out"], sa["r"], sa["b"]
    es = 2 if cfg["dtype"] == "bf16" else 4
    if stages is None:
        kern, ms = "whole call (one kernel)", ms_total
        byt = rf.algorithmic_bytes(cfg["op"], T, n_in, n_out, r, b, es)
        flo = rf.flops(cfg["op"], T, n_in, n_out, r, b)
    else:
        first_dom = stages[0] >= stages[1]
        ms = stages[0] if first_dom else stages[1]
        inter = T * b * r * es                       # Z' (Monarch), A (BLAST) or Z (low-rank, b = 1), written by the first, read by the last
        if cfg["op"] == "lowrank":
            if first_dom:
                kern, byt, flo = "stage 1 (X V^T)", es * (T * n_in + r * n_in) + inter, 2 * T * r * n_in
            else:
                kern, byt, flo = "stage 2 (Z U^T)", inter + es * (r * n_out + T * n_out), 2 * T * r * n_out
        elif cfg["op"] == "monarch":
            if first_dom:
                kern, byt, flo = "stage 1 (block-diagonal R + permutation)", es * (T * n_in + r * n_in) + inter, 2 * T * r * n_in
            else:
                kern, byt, flo = "stage 2 (block-diagonal L)", inter + es * (r * n_out + T * n_out), 2 * T * r * n_out
        else:
            if first_dom:
                kern, byt, flo = "stage 1+2 (X V and coupling)", es * (T * n_in + r * n_in + r * b * b) + inter, 2 * T * r * (n_in + b * b)
            else:
                kern, byt, flo = "stage 3 (A U^T)", inter + es * (r * n_out + T * n_out), 2 * T * r * n_out
    t = ms * 1e-3
    if byt / rf.HBM_PEAK >= flo / rf.MFMA_BF16_PEAK or cfg["dtype"] != "bf16":
        ach = byt / t / 1e9
        return {"bound": "hbm", "achieved": ach, "peak": rf.HBM_PEAK / 1e9, "unit": "GB/s", "frac": ach / (rf.HBM_PEAK / 1e9),
                "traffic": None, "kernel": kern, "kernel_ms": ms, "algorithmic_bytes": byt}
    ach = flo / t / 1e12
    return {"bound": "mfma", "achieved": ach, "peak": rf.MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s", "frac": ach / (rf.MFMA_BF16_PEAK / 1e12),
            "traffic": None, "kernel": kern, "kernel_ms": ms, "algorithmic_flops": flo}


def cold_copies(layer, min_bytes=512 << 20, with_io=False):
    """Shallow copies of `layer` whose factor tensors (with_io: also X and Y) are distinct device buffers,
    enough of them that one round over all copies streams at least `min_bytes` (far beyond every cache)."""
    import copy
    names = [n for n in ("R", "L", "U", "S", "V", "packed") + (("X", "Y") if with_io else ()) if getattr(layer, n, None) is not None]
    per = sum(getattr(layer, n).numel() * getattr(layer, n).element_size() for n in names)
    out = []
    for _ in range(max(2, -(-min_bytes // per))):
        c = copy.copy(layer)
        for n in names:
            setattr(c, n, getattr(layer, n).clone())
        out.append(c)
    return out


def time_cold(make_calls, steps, warmup):
    """Like time_graph, but step i uses the i-th (mod n) of the prepared calls `make_calls()` returns."""
    def make_call():
        calls = make_calls()
        state = {"i": 0}
        def step():
            calls[state["i"] % len(calls)]()
            state["i"] += 1
        return step
    return time_graph(make_call, steps, warmup)


DEFAULT_SWEEP = ("C1", "C2a", "C2b", "C3a", "C3b")      # what the default line carries
FULL_SWEEP = DEFAULT_SWEEP + ("LRa", "LRb")


def run_sweep(steps, warmup, names, variants=False, cpu_seconds=0.0, write=False):
    """Every configuration of `names` at every T of its sweep: time of the call (median of graph
    replays), its stages, the same-shape dense GEMM, roofline floor and fraction (algorithmic bytes or
    FLOPs of the whole call / time / peak), cold-cache time for T <= 128 (factors rotated through
    >= 512 MB of distinct copies), and the CPU oracle over a few tokens. `variants` adds the forced
    executions (blocked Monarch output, both large-rank BLAST executions)."""
    import torch
    from paper_2512_20861_amd import binding as B
    rows = []
    for name in names:
        cfg = bi.CONFIGS[name]
        host = bi.make_layer(cfg)
        W = to_dev(bi.dense_weight(cfg["n_in"], cfg["n_out"], cfg["dtype"]))
        for T in cfg["T"]:
            layer = GpuLayer(cfg, T, host=host)
            ms = time_graph(layer.prepared, steps, warmup)
            st = stage_times(layer, steps, warmup)
            Yd = torch.empty_like(layer.Y)
            ms_dense = time_graph(lambda: B.prepared(B.dense_reference_forward, layer.X, W, Yd), steps, warmup)
            # context only: the vendor library's GEMM on the same operands (never a denominator of a reported speed-up)
            ms_vendor = time_graph(lambda: (lambda: torch.matmul(layer.X, W.t(), out=Yd)), steps, warmup) if variants else None
            sa = layer.shape_args()
            mem, mfma = rf.floors(cfg["op"], T, **sa)
            dmem, dmfma = rf.floors("dense", T, cfg["n_in"], cfg["n_out"])
            ms_alt = {}
            if cfg["op"] == "monarch":                      # the paper's optimisation 3: blocked output order, no final permutation
                ms_alt["blocked_output"] = time_graph(lambda: layer.prepared(B.MONARCH_OUT_BLOCKED), steps, warmup)
            if variants and cfg["op"] == "blast" and st is not None:     # both executions for large ranks, forced
                for key, fl in (("fused_stage12", B.BLAST_FUSED_STAGE12), ("three_kernels", B.BLAST_THREE_KERNELS),
                                ("three_kernels_z_fp8", B.BLAST_Z_FP8)):
                    ws_alt = torch.empty(max(B.blast_workspace_bytes(T, cfg["n_in"], cfg["n_out"], cfg["b"], cfg["r"], B.BF16,
                                                                     layer.flags | fl), 16), dtype=torch.uint8, device="cuda")
                    mk = lambda: B.prepared(B.blast_forward, layer.X, layer.U, None, layer.packed, layer.Y, layer.b, layer.r,
                                            layer.flags | fl, ws_alt)
                    ms_alt[key] = time_graph(mk, steps, warmup)
            cold = None
            if T <= 128 or name == "C1":                    # HBM-bound rows: also with cold caches
                # few tokens: the factors are the stream, rotate them; C1: activations are the stream, rotate X, Y and factors
                io = name == "C1"
                copies = cold_copies(layer, with_io=io)
                n_cold = max(steps, len(copies))
                ms_cold = time_cold(lambda: [c.prepared() for c in copies], n_cold, min(warmup, 3))
                per_dense = W.numel() * W.element_size() + (2 * layer.X.numel() * layer.X.element_size() if io else 0)
                nW = max(2, -(-(512 << 20) // per_dense))
                Ws = [W.clone() for _ in range(nW)]
                Xs = [layer.X.clone() if io else layer.X for _ in range(nW)]
                Ys = [torch.empty_like(Yd) if io else Yd for _ in range(nW)]
                dense_cold = time_cold(lambda: [B.prepared(B.dense_reference_forward, x, w, y) for x, w, y in zip(Xs, Ws, Ys)],
                                       max(steps, nW), min(warmup, 3))
                cold = {"ms": ms_cold, "dense_ms": dense_cold, "frac_of_floor": max(mem, mfma) / (ms_cold * 1e-3),
                        "dense_frac_of_floor": max(dmem, dmfma) / (dense_cold * 1e-3), "factor_copies": len(copies),
                        "rotated": "X, Y and factors" if io else "factors"}
                del copies, Ws, Xs, Ys
            row = {"config": name, "op": cfg["op"], "T": T, "ms": ms, "tokens_per_s": T / (ms * 1e-3),
                   "bound": "hbm" if mem >= mfma else "mfma", "frac": max(mem, mfma) / (ms * 1e-3),
                   "floor_hbm_us": mem * 1e6, "floor_mfma_us": mfma * 1e6, "stage_ms": st,
                   "dense_ms": ms_dense, "dense_frac": max(dmem, dmfma) / (ms_dense * 1e-3),
                   "speedup_vs_dense": ms_dense / ms, "ms_variants": ms_alt, "cold": cold}
            if ms_vendor is not None:
                row["vendor_dense_ms"] = ms_vendor
            if cpu_seconds > 0:
                cb = cpu_baseline(cfg, min(T, 64), cpu_seconds, host)
                row["cpu_baseline"] = {"tokens_per_s": cb["value"], "cores": cb["cores"], "T_cpu": min(T, 64)}
            rows.append(row)
            log(f"{name:4s} {cfg['op']:7s} T={T:5d}  {ms*1e3:9.1f} us  stages={None if st is None else [round(x*1e3,1) for x in st]}  "
                f"floor {max(mem, mfma)*1e6:7.1f} us ({row['bound']}) frac {row['frac']:.3f} | "
                f"dense {ms_dense*1e3:9.1f} us frac {row['dense_frac']:.3f} | speedup {row['speedup_vs_dense']:.2f}x"
                + "".join(f" | {k} {v*1e3:.1f} us" for k, v in ms_alt.items())
                + (f" | cold {cold['ms']*1e3:.1f} us (frac {cold['frac_of_floor']:.3f}), dense cold {cold['dense_ms']*1e3:.1f} us" if cold else ""))
            del layer, Yd
        del W
        torch.cuda.empty_cache()
    if write:
        os.makedirs(os.path.join(ROOT, OUT_DIR), exist_ok=True)
        with open(os.path.join(ROOT, OUT_DIR, "sweep.json"), "w") as f:
            json.dump(rows, f, indent=1)
    return rows


def run_table3(steps, warmup, scale=1):
    """Every layer shape of the paper's Table 3 (Appendix, Layer Details) with every method, against the
    same-shape dense GEMM; rows go to table3.json in the results folder and to stderr."""
    import torch
    from paper_2512_20861_amd import binding as B
    rows = []
    for t3 in bi.TABLE3:
        model, lname, n_in, n_out, n, methods = t3
        n *= scale                                           # `scale` sequences (or images) per call
        W = to_dev(bi.dense_weight(n_in, n_out, "bf16"))
        X = torch.randn((n, n_in), device="cuda", dtype=torch.float32).to(torch.bfloat16)
        Yd = torch.empty((n, n_out), device="cuda", dtype=torch.bfloat16)
        ms_dense = time_graph(lambda: B.prepared(B.dense_reference_forward, X, W, Yd), steps, warmup)
        for method in methods:
            cfg = bi.table3_cfg(t3, method)
            cfg["T"] = (n,)
            layer = GpuLayer(cfg, n, random_x=False)
            layer.set_x(X)
            ms = time_graph(layer.prepared, steps, warmup)
            sa = layer.shape_args()
            mem, mfma = rf.floors(method, n, **sa)
            row = {"model": model, "layer": lname, "n_in": n_in, "n_out": n_out, "T": n, "method": method, "r": sa["r"], "b": sa["b"],
                   "ms": ms, "dense_ms": ms_dense, "speedup_vs_dense": ms_dense / ms, "tokens_per_s": n / (ms * 1e-3),
                   "floor_us": max(mem, mfma) * 1e6, "bound": "hbm" if mem >= mfma else "mfma", "frac_of_floor": max(mem, mfma) / (ms * 1e-3),
                   "compression": rf.params("dense", n_in, n_out) / rf.params(method, n_in, n_out, sa["r"], sa["b"])}
            rows.append(row)
            log(f"{model:13s} {lname:13s} {n_in:5d}->{n_out:5d} T={n:4d} {method:8s} (r,b)=({sa['r']},{sa['b']})  {ms*1e3:8.1f} us | dense {ms_dense*1e3:8.1f} us | "
                f"speedup {row['speedup_vs_dense']:.2f}x | floor {row['floor_us']:.1f} us ({row['bound']}) frac {row['frac_of_floor']:.3f} | CF {row['compression']:.2f}")
            del layer
        del W, X, Yd
        torch.cuda.empty_cache()
    os.makedirs(os.path.join(ROOT, OUT_DIR), exist_ok=True)
    with open(os.path.join(ROOT, OUT_DIR, "table3.json" if scale == 1 else f"table3_x{scale}.json"), "w") as f:
        json.dump(rows, f, indent=1)
    return rows


def chain_linear_cfg(op, name):
    """Benchmark-style configuration of one linear of the chain."""
    c = bi.CHAIN
    n_in, n_out = bi.chain_linear_shape(name, c["hidden"], c["mlp"])
    prm = c[op]
    r = prm["r_square"] if n_in == n_out else prm["r_mlp"]
    cfg = dict(op=op, n_in=n_in, n_out=n_out, r=r, dtype=c["dtype"], T=(c["T"],), x_scale=1.0)
    cfg["nblocks" if op == "monarch" else "b"] = prm["nblocks"] if op == "monarch" else prm["b"]
    return cfg


def run_chain(args, op):
    """One step = one forward pass of the 16-layer chain (x0 copied into the residual stream, then
    7 BLR linears + 4 glue kernels per layer), all steps captured in one HIP graph."""
    import torch
    from paper_2512_20861_amd import binding as B
    from paper_2512_20861_amd.chain import DeviceChain
    c = bi.CHAIN
    T = args.tokens or c["T"]
    layers = bi.chain_layers(op)
    chain = DeviceChain(layers, T)
    x0 = to_dev(bi.activations(T, c["hidden"], c["dtype"]))
    steps, warmup = min(args.steps, 20), min(args.warmup, 3)

    def make_call():
        calls = chain.prepared()
        def step():
            chain.h.copy_(x0)
            for f in calls:
                f()
        return step

    torch.cuda.synchronize()
    ms_eager = time_calls(make_call(), steps, warmup)
    ms = ms_eager if args.eager else time_graph(make_call, steps, warmup)

    # per-shape break-down, each linear timed alone in the chain's launch configuration
    parts, blr_ms, dense_ms, flops = [], 0.0, 0.0, 0.0
    dominant = None
    # (linear, calls per layer, flags it runs with inside the chain); a blocked-input call is timed with
    # the canonical first factor, which has the same shape (values do not matter for the timing)
    OB, IB = B.MONARCH_OUT_BLOCKED, B.MONARCH_IN_BLOCKED
    plan = ([("q", 3, OB), ("o", 1, IB), ("gate", 2, OB), ("down", 1, IB)] if chain.blocked
            else [("q", 3, 0), ("o", 1, 0), ("gate", 2, 0), ("down", 1, 0)] if chain.grouped
            else [("q", 4, 0), ("gate", 2, 0), ("down", 1, 0)])
    for name, count, fl in plan:
        cfg = chain_linear_cfg(op, name)
        layer = GpuLayer(cfg, T)
        t = time_graph(lambda: layer.prepared(fl), 50, 5)
        try:
            st = (time_graph(lambda: layer.prepared(fl | B.ONLY_FIRST_STAGE), 50, 5, 1),
                  time_graph(lambda: layer.prepared(fl | B.ONLY_LAST_STAGE), 50, 5, 1))
        except B.BlrError:
            st = None
        W = to_dev(bi.dense_weight(cfg["n_in"], cfg["n_out"], cfg["dtype"]))
        Yd = torch.empty_like(layer.Y)
        td = time_graph(lambda: B.prepared(B.dense_reference_forward, layer.X, W, Yd), 50, 5)
        sa = layer.shape_args()
        fl_ops = rf.flops(op, T, sa["n_in"], sa["n_out"], sa["r"], sa["b"])
        n_calls = count * c["n_layers"]
        parts.append({"linear": f"{name}: {cfg['n_in']}->{cfg['n_out']} r={cfg['r']}"
                                + (" (blocked output)" if fl & OB else "") + (" (blocked input)" if fl & IB else ""),
                      "calls_per_step": n_calls, "ms": t, "stage_ms": st, "dense_ms": td,
                      "frac_mfma": fl_ops / (t * 1e-3) / rf.MFMA_BF16_PEAK})
        grp = {"q": "qkv", "gate": "gu"}.get(name) if chain.grouped else None
        if grp:     # the chain runs these `count` linears as one call: that call, timed alone on the chain's buffers
            g = chain.groups[0][grp]
            tg = time_graph(lambda: B.prepared(*g.call_args(chain.n, chain.qkv if grp == "qkv" else chain.gu, chain.ws)), 50, 5)
            parts[-1].update({"grouped_call_of": count, "grouped_call_ms": tg})
            blr_ms += c["n_layers"] * tg
        else:
            blr_ms += n_calls * t
        dense_ms += n_calls * td
        flops += n_calls * fl_ops
        worst = n_calls * (max(st) if st else t)
        if dominant is None or worst > dominant[0]:
            dominant = (worst, layer, t, st)
        del W, Yd
    roof = dominant_roofline(dominant[1], dominant[2], dominant[3])
    roof["kernel"] += f" of the {dominant[1].n_in}->{dominant[1].n_out} linear"
    sa = c[op]
    out = {
        "metric": "BLR linear tokens/s", "value": T / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": c["dtype"], "data": "synthetic",
        "config": {"workload": f"C4: {c['n_layers']}-layer decoder linear chain, all-{op} "
                               f"({', '.join(f'{k}={v}' for k, v in sa.items())}), hidden {c['hidden']}, mlp {c['mlp']}, "
                               f"T={T}, 7 linears + glue per layer, no attention",
                   "factors": "packed once before timing" if op == "blast" else "canonical"},
        "launch": "eager loop" if args.eager else "hip graph of the K steps, replayed", "ms_per_step_eager": ms_eager,
        "roofline": roof,
        "chain": {"linears": parts, "linears_ms_sum": blr_ms, "glue_and_gaps_ms": ms - blr_ms,
                  "frac_mfma_whole_chain": flops / (ms * 1e-3) / rf.MFMA_BF16_PEAK},
        "dense_same_shape": {"ms_per_step": dense_ms, "note": "the 112 linears as dense GEMMs, glue excluded",
                             "speedup_of_blr_linears": dense_ms / blr_ms},
    }
    if not args.no_cpu:
        import oracle
        from oracle import chain as oc
        T_cpu = 16
        xs = bi.activations(T, c["hidden"], c["dtype"], rows=np.arange(T_cpu))
        nthreads = oracle.binding.default_threads()
        if op == "monarch":
            lin = lambda x, f: oracle.monarch_forward(x, f.R.f64, f.L.f64, nthreads=nthreads)
        else:
            lin = lambda x, f: oracle.blast_forward(x, f.U.f64, f.S.f64, f.V.f64, nthreads=nthreads)
        t0 = time.perf_counter()
        passes = 0
        while passes < 1 or time.perf_counter() - t0 < 10.0:
            oc.chain_forward(xs.f64, layers, lin)
            passes += 1
        el = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": T_cpu * passes / el, "unit": "tokens/s", "cores": min(nthreads, T_cpu), "kind": "oracle",
                               "sample": f"{passes} passes of the whole chain over the first {T_cpu} tokens ({el:.1f} s of fp64 oracle time)"}
    return out


HEADLINE = "C2b"        # Monarch 4096 -> 11008 at the last T of its sweep (8192): the largest layer of the sweep


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=HEADLINE, choices=sorted(bi.CONFIGS) + ["C4-monarch", "C4-blast"])
    ap.add_argument("--tokens", type=int, default=0, help="override T of the workload")
    ap.add_argument("--sweep", action="store_true", help="the wider sweep (low-rank layers, forced executions); also written to sweep.json")
    ap.add_argument("--no-sweep", action="store_true", help="headline workload only")
    ap.add_argument("--table3", action="store_true", help="also time every layer shape of the paper's Table 3")
    ap.add_argument("--table3-scale", type=int, default=1, help="sequences per call for --table3 (token count x this)")
    ap.add_argument("--sweep-configs", default="", help="comma-separated subset of the configurations for --sweep")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run an elementwise pass over 64 MiB in / 64 MiB out (scales the HBM byte counters)")
    ap.add_argument("--eager", action="store_true", help="report the eager Python launch loop instead of the graph replay")
    ap.add_argument("--profile-part", default="", choices=["", "call", "first", "last", "dense", "copy"],
                    help="for runs under rocprofv3: enqueue ONLY this part of the workload (a HIP graph of --steps launches, replayed 4 times) and exit "
                         "(call = the whole forward; first / last = the kernels up to / after the workspace intermediate; "
                         "dense = the same-shape dense GEMM; copy = an elementwise pass over 64 MiB in / 64 MiB out that "
                         "calibrates the HBM byte counters), so that every kernel row of the profile has one role")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (token-parallel sharding needs no exchange and is not "
              "implemented); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_20861_amd import binding as B
    B.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.manual_seed(0)
    if args.workload.startswith("C4-"):
        print(json.dumps(run_chain(args, args.workload[3:])), flush=True)
        return
    cfg = bi.CONFIGS[args.workload]
    T = args.tokens or cfg["T"][-1]
    layer = GpuLayer(cfg, T)
    layer.set_x(to_dev(bi.activations(T, cfg["n_in"], cfg["dtype"], scale=cfg["x_scale"])))
    if args.profile_part:
        if args.profile_part == "copy":
            src = torch.ones(32 << 20, dtype=torch.bfloat16, device="cuda")
            dst = torch.empty_like(src)
            fn = lambda: torch.mul(src, 2.0, out=dst)
        elif args.profile_part == "dense":
            Wp = to_dev(bi.dense_weight(cfg["n_in"], cfg["n_out"], cfg["dtype"]))
            Yp = torch.empty_like(layer.Y)
            fn = B.prepared(B.dense_reference_forward, layer.X, Wp, Yp)
        else:
            layer.forward()                             # the workspace holds an intermediate for a last-stage-only call
            fn = layer.prepared({"call": 0, "first": B.ONLY_FIRST_STAGE, "last": B.ONLY_LAST_STAGE}[args.profile_part])
        # the same launch configuration as the timed runs: the steps captured once in a HIP graph, replayed;
        # with --eager a loop of separate launches instead (the profiler records every one of those, of a graph
        # only one pass), four rounds of `steps` so that the clocks have settled
        torch.cuda.synchronize()
        if args.eager:
            ms = [time_calls(fn, args.steps, 2) for _ in range(4)][-1]
        else:
            ms = time_graph(lambda: fn, args.steps, 2, replays=3)
        print(json.dumps({"profile_part": args.profile_part, "workload": args.workload, "T": T,
                          "launches": f"{args.steps} per round, 4 rounds + warm-up calls, " + ("separate launches" if args.eager else "one HIP graph per round"),
                          "ms_per_launch": ms}), flush=True)
        return

    # timed region: exactly `steps` forward calls, inputs resident, synchronised on both sides.
    # eager = a Python loop of C calls (host-launch-bound for microsecond kernels);
    # graph = the same `steps` calls captured once in a HIP graph and replayed (the reported value).
    torch.cuda.synchronize()
    ms_eager = time_calls(layer.prepared(), args.steps, args.warmup)
    torch.cuda.synchronize()
    ms = ms_eager if args.eager else time_graph(layer.prepared, args.steps, args.warmup)
    torch.cuda.synchronize()
    stages = stage_times(layer, args.steps, args.warmup)
    roof = dominant_roofline(layer, ms, stages)
    try:                                                 # HBM bytes per launch of that kernel from the committed counter runs
        with open(os.path.join(ROOT, "paper_2512_20861_amd", "measured_traffic.json")) as f:
            entry = json.load(f).get(f"{args.workload}:{T}")
        if entry:
            roof["traffic"] = entry["bytes"]
            roof["traffic_source"] = entry["profile"]
            roof["traffic_kernel"] = entry["kernel"]
            roof["traffic_commit"] = entry.get("commit")
    except OSError:
        pass

    W = to_dev(bi.dense_weight(cfg["n_in"], cfg["n_out"], cfg["dtype"]))
    Yd = torch.empty_like(layer.Y)
    ms_dense = time_graph(lambda: B.prepared(B.dense_reference_forward, layer.X, W, Yd), args.steps, args.warmup)

    sa = layer.shape_args()
    out = {
        "metric": "BLR linear tokens/s", "value": T / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": f"{args.workload}: {cfg['op']} linear {cfg['n_in']}->{cfg['n_out']}, "
                               f"b={sa['b']}, r={sa['r']}, T={T}, {cfg['dtype']} storage / fp32 accumulate",
                   "factors": "packed once before timing" if getattr(layer, "flags", 0) & B.BLAST_PACKED else "canonical"},
        "launch": "eager loop" if args.eager else "hip graph of the K steps, replayed", "ms_per_step_eager": ms_eager,
        "roofline": roof,
        "dense_same_shape": {"ms_per_step": ms_dense, "tokens_per_s": T / (ms_dense * 1e-3), "speedup_of_blr": ms_dense / ms},
    }
    if args.copy_calibration:
        # a kernel whose HBM traffic is known: reads 64 MiB, writes 64 MiB (far beyond every cache)
        src = torch.ones(32 << 20, dtype=torch.bfloat16, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 2.0, out=dst)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"read_bytes": src.numel() * 2, "write_bytes": dst.numel() * 2, "launches": 5}
    if not args.no_cpu:
        T_cpu = min(T, {"C1": 6304, "C0": 8}.get(args.workload, 512))
        out["cpu_baseline"] = cpu_baseline(cfg, T_cpu, lay=layer.host)
    if args.table3:
        out["table3"] = run_table3(max(args.steps // 4, 20), max(args.warmup // 2, 5), max(args.table3_scale, 1))
    if not args.no_sweep:
        only = set(filter(None, args.sweep_configs.split(",")))
        names = [n for n in (FULL_SWEEP if args.sweep else DEFAULT_SWEEP) if not only or n in only]
        out["sweep"] = run_sweep(max(args.steps // 4, 20), max(args.warmup // 2, 5), names, variants=args.sweep,
                                 cpu_seconds=0.0 if args.no_cpu else 0.7, write=args.sweep)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

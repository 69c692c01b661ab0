#!/usr/bin/env python3
"""Benchmark of the forward-convolution hot path on one MI355X.

A step is one forward convolution of the headline layer on blocked tensors that are already
resident in HBM: the region the paper times (its Fig. 4 loop nest runs on blocked arrays, Section 5)
and the one the metric 2*N*K*P*Q*C*R*S / t is defined on.  The layout transforms are one-off per
network input / per layer; their bandwidth is reported beside the headline, not inside it.

Prints ONE JSON line.  Extra keys: ``roofline`` (dominant kernel against the fp32 MFMA peak, timed
with HIP events on the launch stream), ``cpu_baseline`` (the CPU oracle on the host cores),
``layers`` (every ResNet-50-shaped layer with the tile model's pick), ``transforms``, ``bf16`` (the same layers with
bf16 inputs), ``via_select`` and ``api_call_host_us`` (the call that picks its own tile against an explicit tile).
"""
from __future__ import annotations

import argparse
import hashlib
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}   # MI355X dense MFMA peaks
HBM_PEAK_GBS = 8000.0


def kernel_source_digest(dtype: str) -> str:
    """Digest of the kernel sources of `dtype`: the stored HBM-traffic counters only describe the kernel they were
    taken on."""
    h = hashlib.sha256()
    files = ["conv_fwd_kernel.h", f"conv_fwd_{dtype}.hip"] + (["conv_fwd_bf16_halo.h", "conv_fwd_bf16_shape.h", "conv_fwd_bf16_packed.hip"] if dtype == "bf16" else
                                                            ["conv_fwd_f32_n16.h", "conv_fwd_f32_n16_kloop.h", "conv_fwd_f32_packed.hip"])
    for f in files:
        with open(os.path.join(ROOT, "paper_2002_02145_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def _precondition(fn, min_ms: float = 80.0) -> float:
    """Runs fn() back to back for at least min_ms of GPU time and returns the milliseconds spent.  The shader clock
    needs tens of milliseconds of load to settle at the level it sustains; launches timed before that read 10-15 %
    slower than the same kernel in steady state, whatever the counted warm-up is."""
    import torch
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    spent, chunk = 0.0, 50
    while spent < min_ms:
        for _ in range(chunk):
            fn()
        e1.record(stream)
        e1.synchronize()
        spent = e0.elapsed_time(e1)
        chunk = min(2000, chunk * 2)
    return spent


def _time_steps(fn, steps: int, warmup: int):
    """(wall ms per step, event ms per step) for `steps` back-to-back launches of fn()."""
    import torch
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(steps):
        fn()
    e1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


class _GraphTimer:
    """`per_graph` launches of fn() captured into one HIP graph and replayed: what a caller does with a launch-bound
    loop.  A convolution of 7-12 us is shorter than one call through the Python binding (about 7 us of host time), so
    a Python loop of eager calls would time the interpreter; the graph keeps the launches back to back on the device
    (between two dependent kernels of a graph lies the same gap as between two eager ones whose queue is full)."""

    def __init__(self, fn, per_graph: int = 40):
        import torch
        self.per_graph = per_graph
        self.side = torch.cuda.Stream()
        self.graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.stream(self.side):
            with torch.cuda.graph(self.graph, stream=self.side):
                for _ in range(per_graph):
                    fn()
        torch.cuda.synchronize()

    def replay(self):
        self.graph.replay()

    def time_us(self, min_ms: float = 100.0) -> float:
        """Microseconds per launch over at least min_ms of replays (events around all of them)."""
        import torch
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        self.graph.replay()                      # sizes the run: one replay timed on its own
        e0.record(stream)
        self.graph.replay()
        e1.record(stream)
        torch.cuda.synchronize()
        n = max(3, int(min_ms / max(e0.elapsed_time(e1), 1e-3)) + 1)
        e0.record(stream)
        for _ in range(n):
            self.graph.replay()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (n * self.per_graph)


def _launch_us(fn, precondition_ms: float, min_ms: float = 100.0):
    """(microseconds per launch, how it was timed): graph replay, or, should capture fail on this runtime, an eager
    loop (which reads high for launches shorter than a call through the binding)."""
    import torch
    try:
        gt = _GraphTimer(fn)
        _precondition(gt.replay, precondition_ms)
        return gt.time_us(min_ms), "graph replay"
    except Exception as e:   # never lose the bench line over the timing method
        torch.cuda.synchronize()
        _precondition(fn, precondition_ms)
        _, ms = _time_steps(fn, 2000, 20)
        return ms * 1e3, f"eager loop (graph capture failed: {type(e).__name__})"


def _time_each(fn, launches: int):
    """Mean duration in ms of single launches, each bracketed by its own pair of HIP events on the launch
    stream.  The event records between launches keep consecutive launches from overlapping and add a few
    microseconds of their own, so this reads higher than a kernel trace; it is reported beside the
    region-based figure, not used for the roofline."""
    import torch
    stream = torch.cuda.current_stream()
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(launches)]
    torch.cuda.synchronize()
    for e0, e1 in pairs:
        e0.record(stream)
        fn()
        e1.record(stream)
    torch.cuda.synchronize()
    return sum(e0.elapsed_time(e1) for e0, e1 in pairs) / launches


# HBM-side bytes per launch of the headline kernel from rocprofv3 counter runs (FETCH_SIZE + WRITE_SIZE, each
# scaled by a reference copy; see profiles/), keyed by a digest of the kernel sources they were taken with.
# A different digest, a different tile picked by the model or a different inner loop means the launch is not the one the counters were
# taken on: traffic is then reported as null.
MEASURED_TRAFFIC = {"f32": ("9875042ee13446c2", (64, 176, 2, 1, 0), 3, 46593629),
                    "bf16": ("5f9c8b5a490f0680", (64, 256, 2, 1, 0), 9, 34631516)}


def _layer_rows(ps, wl, torch, dtype_name: str, workspace, ws_cap: int):
    """Every ResNet-50-shaped layer with the library's own pick: microseconds per launch (launches replayed from a HIP
    graph, see _GraphTimer), TFLOP/s, fractions of the MFMA peak and of min(MFMA, HBM).  Device-side random tensors
    (timing only)."""
    dtype = ps.PS_F32 if dtype_name == "f32" else ps.PS_BF16
    tdt = torch.float32 if dtype_name == "f32" else torch.bfloat16
    es = 4 if dtype_name == "f32" else 2
    dev = "cuda:0"
    g = torch.Generator(device=dev).manual_seed(7)
    rows = []
    base = wl.resnet50_layers()
    for L in base + [wl.CFG3B]:
        dl = ps.ConvDesc.of(L, dtype)
        xi = torch.rand(ps.ps_blocked_in_bytes(dl) // es, device=dev, generator=g).to(tdt)
        wi = ((torch.rand(ps.ps_blocked_wt_bytes(dl) // es, device=dev, generator=g) - 0.5) * 0.1).to(tdt)
        oi = torch.empty(ps.ps_blocked_out_bytes(dl) // 4, device=dev, dtype=torch.float32)
        t = ps.ps_tile_pick(dl, True, ws_cap)
        fn = lambda: ps.ps_conv2d_fwd_ws(dl, None, xi, wi, oi, workspace, ws_cap)   # the library picks (cached)
        us, how = _launch_us(fn, 60.0)
        tf = L.flops / (us * 1e-6) * 1e-12
        t_roof = max(L.flops / (PEAK_TFLOPS[dtype_name] * 1e12), L.algorithmic_bytes(es) / (HBM_PEAK_GBS * 1e9))
        row = {"layer": L.name, "us": round(us, 2), "TFLOP/s": round(tf, 2),
               "frac_mfma_peak": round(tf / PEAK_TFLOPS[dtype_name], 4),
               "frac_min_mfma_hbm_roofline": round(t_roof / (us * 1e-6), 4),
               "tile": list(t.as_tuple()), "kernel": ps.KERNEL_NAMES[ps.ps_tile_kernel(dl, t)]}
        if how != "graph replay":
            row["timing"] = how
        # the paper's protocol with k = 3 (Section 4.2): the library runs its three best-ranked tiles and keeps the
        # fastest; the same call is then timed again (the figures above are k = 1, the paper's own setting)
        t3, _, _ = ps.ps_tile_autotune(dl, 3, xi, wi, oi, workspace, ws_cap)
        if t3.as_tuple() != t.as_tuple():
            us3, _ = _launch_us(fn, 20.0)        # captured anew: the call now launches the tile the library kept
            row["top3"] = {"tile": list(t3.as_tuple()), "us": round(us3, 2)}
        rows.append(row)
        del xi, wi, oi
    n = len(base)
    tot_flop = sum(L.flops for L in base)
    tot_s = sum(r["us"] for r in rows[:n]) * 1e-6
    agg = {"flop_weighted_TFLOP/s": round(tot_flop / tot_s * 1e-12, 2),
           "geomean_TFLOP/s": round(math.exp(sum(math.log(r["TFLOP/s"]) for r in rows[:n - 1]) / (n - 1)), 2),
           "geomean_covers": "the 12 layers whose channel counts are multiples of 16 (the paper's selection, Section 5.1)"}
    return rows, agg


class _Headline:
    """Blocked tensors of one seeded layer resident on the device, and the calls that are timed on them."""

    def __init__(self, ps, wl, torch, shape, dtype_name: str, workspace, ws_cap: int):
        self.ps, self.shape, self.dtype_name = ps, shape, dtype_name
        dev = "cuda:0"
        self.dtype = ps.PS_F32 if dtype_name == "f32" else ps.PS_BF16
        self.tdt = torch.float32 if dtype_name == "f32" else torch.bfloat16
        self.es = 4 if dtype_name == "f32" else 2
        x, w = wl.relu_like(shape, 2)
        if dtype_name == "bf16":
            x, w = wl.round_to_bf16(x), wl.round_to_bf16(w)
        self.x, self.w = x, w
        d = self.d = ps.ConvDesc.of(shape, self.dtype)
        self.xd = torch.from_numpy(x).to(self.tdt).to(dev)
        self.wd = torch.from_numpy(w).to(self.tdt).to(dev)
        self.xb = torch.empty(ps.ps_blocked_in_bytes(d) // self.es, dtype=self.tdt, device=dev)
        self.wb = torch.empty(ps.ps_blocked_wt_bytes(d) // self.es, dtype=self.tdt, device=dev)
        self.ob = torch.empty(ps.ps_blocked_out_bytes(d) // 4, dtype=torch.float32, device=dev)
        self.y = torch.empty((shape.N, shape.K, shape.P, shape.Q), dtype=torch.float32, device=dev)
        ps.ps_nchw_to_blocked(d, self.xd, self.xb)
        ps.ps_kcrs_to_blocked(d, self.wd, self.wb)
        # ranking cost, first and steady (host only; the first call prices every candidate, later ones are lookups)
        t0 = time.perf_counter()
        self.tile = ps.ps_tile_pick(d, True, ws_cap)
        t1 = time.perf_counter()
        for _ in range(1000):
            ps.ps_tile_pick(d, True, ws_cap)
        t2 = time.perf_counter()
        self.pick_first_us, self.pick_steady_us = (t1 - t0) * 1e6, (t2 - t1) / 1000 * 1e6
        _, self.model_us = ps.ps_tile_select_ws(d, ws_cap)
        self.ws_bytes = ps.ps_workspace_bytes(d, self.tile)
        self.ws = workspace
        # the timed step: explicit tile (what the sweeps time); and the same launch with the library choosing
        self.step = lambda: ps.ps_conv2d_fwd_ws(d, self.tile, self.xb, self.wb, self.ob, self.ws, self.ws_bytes)
        self.step_select = lambda: ps.ps_conv2d_fwd_ws(d, None, self.xb, self.wb, self.ob, self.ws, ws_cap)

    def host_call_us(self, fn, calls: int = 300) -> float:
        """Host time of one call (argument marshalling, pick and plan lookup, kernel launch), queue not full."""
        import torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(calls):
            fn()
        dt = time.perf_counter() - t0
        torch.cuda.synchronize()
        return dt / calls * 1e6

    def check(self, oracle):
        import torch
        ps = self.ps
        ps.ps_blocked_to_nkpq(self.d, self.ob, self.y)
        torch.cuda.synchronize()
        got = self.y.cpu().numpy()
        out, mag = oracle.conv2d_fwd(self.shape, self.x, self.w)
        err = oracle.normalised_error(got, out, mag)
        tol = 1e-4 if self.dtype_name == "f32" else 2e-2
        return {"max_normalised_error": err, "tolerance": tol, "pass": bool(err <= tol)}


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3000)
    ap.add_argument("--warmup", type=int, default=1000, help="untimed steps before the timed ones")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--no-layers", action="store_true", help="skip the per-layer sweeps")
    ap.add_argument("--no-bf16", action="store_true", help="skip the bf16 section of an fp32 run")
    ap.add_argument("--layer", default=None,
                    help="time this layer of the ResNet-50-shaped sweep instead of the headline one (for profiling a "
                         "kernel the headline does not use; the default run is the benchmark)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ref-copy-mib", type=int, default=0,
                    help="also run 3 plain device-to-device copies of this many MiB (reference dispatches of known "
                         "size for scaling FETCH_SIZE / WRITE_SIZE counter runs)")
    a = ap.parse_args(argv)
    if a.gpus != 1:
        print("bench.py: this library runs on one GPU only (forward convolution shards over images with no exchange "
              "between GPUs, so several GPUs are several independent runs); rerun with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2002_02145_amd import binding as ps
    from paper_2002_02145_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    es = 4 if a.dtype == "f32" else 2

    # ---- headline workload: ResNet-50-shaped 3x3, N=28, C=K=64, 56x56 -------------------------
    shape = wl.CFG2
    if a.layer is not None:
        named = {L.name: L for L in wl.resnet50_layers() + [wl.CFG3B]}
        if a.layer not in named:
            print(f"bench.py: unknown layer {a.layer}; one of {sorted(named)}", file=sys.stderr)
            return 2
        shape = named[a.layer]
    WS_CAP = 256 << 20   # workspace the caller is willing to lend for split reductions
    workspace = torch.empty(WS_CAP // 4, dtype=torch.float32, device=dev)
    hl = _Headline(ps, wl, torch, shape, a.dtype, workspace, WS_CAP)
    d, tile, step = hl.d, hl.tile, hl.step
    xb, wb, ob, y, xd, wd, ws, ws_bytes = hl.xb, hl.wb, hl.ob, hl.y, hl.xd, hl.wd, hl.ws, hl.ws_bytes

    # the clocks settle under load first (time-based, not counted in --warmup), then W untimed and K timed steps
    precond_ms = _precondition(step)
    wall_ms, ev_ms = _time_steps(step, a.steps, a.warmup)
    gflops = shape.flops / (wall_ms * 1e-3) * 1e-9
    # the same launch when the library picks the tile itself (cached ranking): must cost the same
    _, sel_ms = _time_steps(hl.step_select, max(a.steps, 200), max(a.warmup, 20))
    _, exp_ms = _time_steps(step, max(a.steps, 200), max(a.warmup, 20))
    host_select_us = hl.host_call_us(hl.step_select)
    host_explicit_us = hl.host_call_us(step)
    each_ms = _time_each(step, min(500, max(20, a.steps)))
    # cold regime: rotate through enough distinct input/output pairs (> 512 MB) that no launch finds its
    # tensors in the Infinity Cache
    pair_bytes = xb.numel() * es + ob.numel() * 4
    n_sets = max(2, -(-(600 << 20) // pair_bytes))
    xs = [xb.clone() for _ in range(n_sets)]
    os_ = [torch.empty_like(ob) for _ in range(n_sets)]
    turn = [0]

    def cold_step():
        i = turn[0] = (turn[0] + 1) % n_sets
        ps.ps_conv2d_fwd_ws(d, tile, xs[i], wb, os_[i], ws, ws_bytes)
    _, cold_ms = _time_steps(cold_step, max(200, a.steps // 3), 200)
    del xs, os_
    # average duration of the dominant kernel: with an unsplit tile a step is exactly one launch, so the HIP
    # events around the timed region give it directly (this is what a kernel trace averages to); a split tile
    # adds the plane-adding pass to every step, and its time is charged to the convolution kernel as well
    kernel_ms = ev_ms
    digest, ttile, tvariant, tbytes = MEASURED_TRAFFIC.get(a.dtype, (None, None, None, None))
    same_launch = (a.layer is None and digest == kernel_source_digest(a.dtype) and ttile == tile.as_tuple()
                   and tvariant == ps.ps_tile_kernel(d, tile))
    traffic = tbytes if same_launch else None

    # transforms: bytes moved (plain tensor + blocked tensor; they differ where channels are padded) per call; warm
    # (same buffers every call) and cold (rotating through more than 600 MB of source/destination pairs)
    tr = {}
    for name, fn, src, dst in (
            ("nchw_to_blocked", ps.ps_nchw_to_blocked, xd, xb),
            ("blocked_to_nkpq", ps.ps_blocked_to_nkpq, ob, y),
            ("kcrs_to_blocked", ps.ps_kcrs_to_blocked, wd, wb)):
        nbytes = src.numel() * src.element_size() + dst.numel() * dst.element_size()
        _, ms = _time_steps(lambda: fn(d, src, dst), 50, 5)
        tr[name] = {"us": round(ms * 1e3, 2), "GB/s": round(nbytes / (ms * 1e-3) * 1e-9, 1), "bytes": nbytes}
        if name != "kcrs_to_blocked":
            k = max(2, -(-(600 << 20) // nbytes))
            srcs, dsts = [src.clone() for _ in range(k)], [torch.empty_like(dst) for _ in range(k)]
            turn[0] = 0

            def cold_tr():
                i = turn[0] = (turn[0] + 1) % k
                fn(d, srcs[i], dsts[i])
            _, cms = _time_steps(cold_tr, 60, 10)
            tr[name].update({"cold_us": round(cms * 1e3, 2), "cold_GB/s": round(nbytes / (cms * 1e-3) * 1e-9, 1)})
            del srcs, dsts
    _, e2e_ms = _time_steps(lambda: (ps.ps_nchw_to_blocked(d, xd, xb), step(),
                                     ps.ps_blocked_to_nkpq(d, ob, y)), 50, 5)

    if a.ref_copy_mib > 0:
        src = torch.ones(a.ref_copy_mib << 18, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- correctness of what was timed, and the CPU baseline, on the same inputs ----------------
    cpu = None
    checked = None
    oracle = None
    if not a.no_cpu_baseline:
        import oracle
        oracle.build()
        step()
        checked = hl.check(oracle)
        reps, t0 = 0, time.perf_counter()
        while True:
            oracle.conv2d_fwd(shape, hl.x, hl.w)
            reps += 1
            if time.perf_counter() - t0 >= 8.0 or reps >= 200:
                break
        dt = (time.perf_counter() - t0) / reps
        cpu = {"value": round(shape.flops / dt * 1e-9, 3), "unit": "GFLOP/s", "cores": oracle.threads(),
               "kind": "oracle", "sample": f"whole layer {shape.name} (all {shape.N} images), {reps} repetitions of "
                                          f"{dt:.2f} s each; fp64 seven-loop definition, OpenMP over (n, k)"}

    # ---- every ResNet-50-shaped layer with the model's pick --------------------------------------
    layers, agg = ([], None) if a.no_layers else _layer_rows(ps, wl, torch, a.dtype, workspace, WS_CAP)

    # ---- the 16-bit configuration (same layers, bf16 inputs and filters, fp32 accumulation and output) -------
    bf16 = None
    if a.dtype == "f32" and not a.no_bf16 and a.layer is None:
        hb = _Headline(ps, wl, torch, wl.CFG2, "bf16", workspace, WS_CAP)
        _precondition(hb.step)
        _, b_eager_ms = _time_steps(hb.step, max(a.steps, 1000), max(a.warmup, 100))
        # the launch takes about as long as one call through the Python binding costs the host: the figure of record is
        # the same launch replayed from a HIP graph (see _GraphTimer), the eager loop's is reported beside it
        b_us, b_how = _launch_us(hb.step, 40.0)
        b_ms = b_us * 1e-3
        b_alg = wl.CFG2.algorithmic_bytes(2)
        b_tf = wl.CFG2.flops / (b_ms * 1e-3) * 1e-12
        bf16 = {"workload": "same layer, inputs and filters rounded to bf16 (nearest even), fp32 accumulate and output",
                "us": round(b_ms * 1e3, 2), "timing": b_how, "eager_python_loop_us": round(b_eager_ms * 1e3, 2),
                "TFLOP/s": round(b_tf, 1), "frac_mfma_peak": round(b_tf / PEAK_TFLOPS["bf16"], 4),
                "roofline": {"bound": "hbm", "achieved": round(b_alg / (b_ms * 1e-3) * 1e-9, 1), "peak": HBM_PEAK_GBS,
                             "unit": "GB/s", "frac": round(b_alg / (b_ms * 1e-3) * 1e-9 / HBM_PEAK_GBS, 4),
                             "algorithmic_bytes": b_alg},
                "tile": list(hb.tile.as_tuple()), "kernel": ps.KERNEL_NAMES[ps.ps_tile_kernel(hb.d, hb.tile)],
                "checked_against_oracle": hb.check(oracle) if oracle is not None else None}
        # the epilogue fused into the store (bias, max(., 0)) and, for 16-bit inputs, a 16-bit output that the next
        # layer reads as its blocked input: same layers, same tiles, graph replay
        bias = torch.zeros(wl.CFG2.K, dtype=torch.float32, device=dev)
        ob16 = torch.empty(ps.ps_blocked_out_bytes(hb.d) // 4, dtype=torch.bfloat16, device=dev)
        fused = {}
        for name, H, out, odt in (("f32_bias_relu_us", hl, hl.ob, ps.PS_F32), ("bf16_bias_relu_us", hb, hb.ob, ps.PS_F32),
                                  ("bf16_bias_relu_bf16_out_us", hb, ob16, ps.PS_BF16)):
            if H.shape is not wl.CFG2:
                continue
            fn = (lambda H=H, out=out, odt=odt: ps.ps_conv2d_fwd_fused(H.d, None, H.xb, H.wb, out, workspace, WS_CAP,
                                                                       bias=bias, relu=True, out_dtype=odt))
            fused[name] = round(_launch_us(fn, 40.0)[0], 2)
        bf16["fused_epilogue"] = fused
        if not a.no_layers:
            bf16["layers"], bf16["layers_aggregate"] = _layer_rows(ps, wl, torch, "bf16", workspace, WS_CAP)
        del hb, ob16

    peak = PEAK_TFLOPS[a.dtype]
    alg_bytes = shape.algorithmic_bytes(es)
    if shape.flops / (peak * 1e12) >= alg_bytes / (HBM_PEAK_GBS * 1e9):
        achieved = shape.flops / (kernel_ms * 1e-3) * 1e-12
        roof = {"bound": "mfma", "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved / peak, 4)}
    else:   # below the ridge: the layer cannot keep the matrix cores busy even at full HBM bandwidth
        achieved = alg_bytes / (kernel_ms * 1e-3) * 1e-9
        roof = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4)}
    roof.update({"traffic": traffic, "traffic_unit": "bytes per launch (HBM side)", "algorithmic_bytes": alg_bytes,
                 "kernel": "conv_fwd_%s %s loop <kt=%d,mt=%d,ring=%d>" % (a.dtype, ps.KERNEL_NAMES[ps.ps_tile_kernel(d, tile)],
                                                                           tile.kt, tile.mt, tile.ring),
                 "kernel_us": round(kernel_ms * 1e3, 2), "isolated_launch_us": round(each_ms * 1e3, 2),
                 "launches_per_step": 1 if tile.c_split == 1 else 2, "flop_per_launch": shape.flops})
    # what the matrix cores of this device sustain with no operand traffic at all (context for the published peak)
    sink = torch.zeros(1024, dtype=torch.float32, device=dev)
    probe_iters = 2000 if a.dtype == "f32" else 4000
    for _ in range(3):
        probe_flop = ps.ps_probe_mfma(hl.dtype, probe_iters, sink)
    torch.cuda.synchronize()
    pe0, pe1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    pe0.record(torch.cuda.current_stream())
    for _ in range(10):
        ps.ps_probe_mfma(hl.dtype, probe_iters, sink)
    pe1.record(torch.cuda.current_stream())
    torch.cuda.synchronize()
    probe_tflops = probe_flop * 10 / (pe0.elapsed_time(pe1) * 1e-3) * 1e-12
    line = {
        "metric": "conv fwd GFLOP/s (2*N*K*P*Q*C*R*S/t), 1 GPU",
        "value": round(gflops, 1),
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": a.dtype,
        "data": "synthetic (seeded: input U[0,1), filter N(0, sqrt(2/(C*R*S))))",
        "config": {"workload": f"ResNet-50-shaped {shape.R}x{shape.S} conv fwd ({shape.name}): N={shape.N} C={shape.C} "
                               f"K={shape.K} H=W={shape.H} R=S={shape.R} stride {shape.stride} pad {shape.pad}, "
                               f"blocked 16c layouts, tensors resident in HBM",
                   "tile": list(tile.as_tuple()), "tile_model_us": round(hl.model_us, 2),
                   "timing": "warm (same buffers every step)"},
        "preconditioning_ms": round(precond_ms, 1),
        "via_select": {"us": round(sel_ms * 1e3, 2), "explicit_tile_us": round(exp_ms * 1e3, 2),
                       "ratio": round(sel_ms / exp_ms, 4),
                       "what": "ps_conv2d_fwd_ws with tile = NULL (library picks, cached) against the same launch with "
                               "the tile passed in"},
        "api_call_host_us": {"pick_first": round(hl.pick_first_us, 2), "pick_steady": round(hl.pick_steady_us, 2),
                             "call_with_select": round(host_select_us, 2), "call_with_explicit_tile": round(host_explicit_us, 2),
                             "what": "host time through the Python binding: ps_tile_pick alone (first call ranks every "
                                     "candidate, later calls are lookups), and one whole ps_conv2d_fwd_ws call "
                                     "including the kernel launch"},
        "cold": {"us": round(cold_ms * 1e3, 2), "GFLOP/s": round(shape.flops / (cold_ms * 1e-3) * 1e-9, 1),
                 "buffer_sets": n_sets, "bytes_rotated": n_sets * pair_bytes},
        "frac_mfma_peak": round(gflops * 1e-3 / peak, 4),
        "mfma_only_loop_TFLOP/s": round(probe_tflops, 1),   # ps_probe_mfma: no LDS or memory traffic
        "roofline": roof,
        "cpu_baseline": cpu,
        "checked_against_oracle": checked,
        "transforms": tr,
        "with_layout_transforms_GFLOP/s": round(shape.flops / (e2e_ms * 1e-3) * 1e-9, 1),
        "layers": layers,
        "layers_timing": "each layer's launch replayed from a HIP graph (40 per graph), library's own pick",
        "layers_aggregate": agg,
        "bf16": bf16,
        "paper_context": "paper: 2448 GFLOP/s geomean on ResNet-50 layers, 28-core Xeon 8280, fp32 (Table 1)",
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())

"""Exhaustive sweep over the tile enumerator's candidates, timed on the GPU.

The paper runs its top-k ranked variants on the target and keeps the fastest, and reports, per
layer, the slowest and fastest variant next to the one its model picked (Section 5.2, the
"performance distribution" figures).  This module produces the same three numbers for the GPU
variant space: every candidate of ``ps_tile_get`` is timed, and the model's pick
(``ps_tile_select``) is located in that distribution.

Timing uses HIP events on the launch stream; torch supplies memory and events only.
"""
from __future__ import annotations

import argparse
import json
import sys

import torch

from . import binding as ps
from . import workloads as wl


def _buffers(desc: ps.ConvDesc, es: int, copies: int = 1):
    tdt = torch.float32 if es == 4 else torch.bfloat16
    g = torch.Generator(device="cuda").manual_seed(1)
    sets = []
    for _ in range(copies):
        xb = torch.rand(ps.ps_blocked_in_bytes(desc) // es, device="cuda", generator=g).to(tdt)
        wb = (torch.rand(ps.ps_blocked_wt_bytes(desc) // es, device="cuda", generator=g) - 0.5).to(tdt)
        ob = torch.empty(ps.ps_blocked_out_bytes(desc) // 4, device="cuda", dtype=torch.float32)
        sets.append((xb, wb, ob))
    return sets


_SIDE = None   # the stream launches are captured on (one per process)


def time_tile(desc: ps.ConvDesc, tile: ps.Tile | None, sets, warmup: int = 5, min_ms: float = 20.0,
              max_iters: int = 2000, workspace=None, per_graph: int = 20) -> float:
    """Mean microseconds per launch of one tile (None = the library's own pick).  With a workspace tensor
    the call goes through ps_conv2d_fwd_ws (split reductions use partial planes instead of atomics).
    The launches are captured into a HIP graph (`per_graph` of them, rotating through `sets`) and the graph is
    replayed: many layers take 4-12 us per launch, about what one call through the Python binding costs the host, so a
    loop of eager calls would time the interpreter.  Between dependent kernels of a graph lies the same gap as between
    eager launches whose queue is full."""
    global _SIDE
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()

    def launch(i):   # on the current stream (the capturing one during capture)
        xb, wb, ob = sets[i % len(sets)]
        if workspace is not None:
            ps.ps_conv2d_fwd_ws(desc, tile, xb, wb, ob, workspace, ws_bytes)
        elif tile is None:
            ps.ps_conv2d_fwd(desc, xb, wb, ob)
        else:
            ps.ps_conv2d_fwd_tile(desc, tile, xb, wb, ob)

    for i in range(warmup):
        launch(i)
    torch.cuda.synchronize()
    per_graph = -(-per_graph // len(sets)) * len(sets)
    if _SIDE is None:
        _SIDE = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(_SIDE):
        with torch.cuda.graph(graph, stream=_SIDE):
            for i in range(per_graph):
                launch(i)
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    # size the repetition count from a first timed batch
    reps = 1
    while True:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            graph.replay()
        e1.record(stream)
        e1.synchronize()
        ms = e0.elapsed_time(e1)
        if ms >= min_ms or reps * per_graph >= max_iters:
            return ms * 1e3 / (reps * per_graph)
        reps = min(-(-max_iters // per_graph), max(reps * 2, int(reps * min_ms / max(ms, 1e-3)) + 1))


def sweep(shape: wl.ConvShape, dtype: int = ps.PS_F32, min_ms: float = 20.0, cold: bool = False,
          use_ws: bool = True) -> dict:
    desc = ps.ConvDesc.of(shape, dtype)
    es = 4 if dtype == ps.PS_F32 else 2
    per_set = ps.ps_blocked_in_bytes(desc) + ps.ps_blocked_wt_bytes(desc) + ps.ps_blocked_out_bytes(desc)
    copies = max(1, -(-(600 << 20) // per_set)) if cold else 1
    sets = _buffers(desc, es, copies)
    rows = []
    tiles = [ps.ps_tile_get(desc, i) for i in range(ps.ps_tile_count(desc))]
    workspace = None
    if use_ws:
        need = max([ps.ps_workspace_bytes(desc, t) for t in tiles] + [16])
        workspace = torch.empty(need // 4, device="cuda", dtype=torch.float32)
    cost = ps.ps_tile_cost_ws_us if use_ws else ps.ps_tile_cost_us
    for t in tiles:
        us = time_tile(desc, t, sets, min_ms=min_ms, workspace=workspace)
        rows.append({"tile": t.as_tuple(), "us": us, "model_us": cost(desc, t)})
    pick, model_us = ps.ps_tile_select_ws(desc, need) if use_ws else ps.ps_tile_select(desc)
    best = min(rows, key=lambda r: r["us"])
    worst = max(rows, key=lambda r: r["us"])
    mine = next(r for r in rows if r["tile"] == pick.as_tuple())
    gf = lambda us: shape.flops / us * 1e-3
    return {
        "layer": shape.name, "dtype": "f32" if dtype == ps.PS_F32 else "bf16", "candidates": len(rows),
        "split_reduction": "workspace" if use_ws else "atomics",
        "pick": pick.as_tuple(), "pick_us": mine["us"], "pick_model_us": model_us, "pick_gflops": gf(mine["us"]),
        "best": best["tile"], "best_us": best["us"], "best_gflops": gf(best["us"]),
        "worst": worst["tile"], "worst_us": worst["us"], "worst_gflops": gf(worst["us"]),
        "pick_vs_best": best["us"] / mine["us"],
        "rank_of_pick": sorted(r["us"] for r in rows).index(mine["us"]) + 1,
        "rows": rows,
    }


def run_top_k(desc: ps.ConvDesc, k: int, workspace: torch.Tensor, sets=None, min_ms: float = 5.0):
    """The paper's selection protocol (Section 4.2): the model ranks all variants, the best k are run on the target
    and the fastest is kept.  Returns (tile, measured us, [(tile, modelled us, measured us), ...]); k = 1 is the
    library's own pick.  `workspace` is what the caller lends for split reductions (may be a 4-element tensor)."""
    es = 4 if desc.dtype == ps.PS_F32 else 2
    sets = sets or _buffers(desc, es)
    ws_bytes = workspace.numel() * workspace.element_size()
    ranked = ps.ps_tile_rank_ws(desc, ws_bytes, k)
    rows = [(t, model_us, time_tile(desc, t, sets, min_ms=min_ms, workspace=workspace)) for t, model_us in ranked]
    best = min(rows, key=lambda r: r[2])
    return best[0], best[2], rows


def stored_row(result: dict, N: int) -> dict:
    """The compact form sweeps are kept in under data/: one line per layer, a row [kt, mt, ring, c_split, raster, us]
    per candidate."""
    return {"layer": result["layer"], "N": N, "dtype": result["dtype"],
            "rows": [list(r["tile"]) + [round(r["us"], 3)] for r in result["rows"]]}


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--layers", default="sweep",
                    help="sweep (the ResNet-50-shaped set) | heldout | validation | first (the out-of-sample sets) | cfg1 | cfg2 | cfg3a | cfg3b | "
                         "comma list of layer names")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--batch", type=int, default=wl.MINIBATCH, help="mini-batch size of the named layer sets")
    ap.add_argument("--min-ms", type=float, default=20.0)
    ap.add_argument("--cold", action="store_true", help="rotate buffers so every launch streams from HBM")
    ap.add_argument("--rows", action="store_true", help="include every candidate's time in the output")
    ap.add_argument("--atomics", action="store_true",
                    help="time split reductions through ps_conv2d_fwd_tile (clear + atomics) instead of the workspace path")
    ap.add_argument("--out", default=None)
    ap.add_argument("--store", default=None,
                    help="append each layer's sweep in the compact stored form to this file; layers already in the file "
                         "are skipped, so an interrupted sweep resumes where it stopped")
    a = ap.parse_args(argv)
    N = a.batch
    rebatch = lambda L: wl.ConvShape(N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad, L.name)
    named = {"cfg1": wl.CFG1, "cfg2": wl.CFG2, "cfg3a": wl.CFG3A, "cfg3b": wl.CFG3B}
    named.update({l.name: l for l in wl.resnet50_layers(N) + wl.heldout_layers(N) + wl.validation_layers(N) + wl.first_layers(N) + [rebatch(wl.CFG3B)]})
    if a.layers == "sweep":
        layers = wl.resnet50_layers(N) + [rebatch(wl.CFG3B)]
    elif a.layers == "heldout":
        layers = wl.heldout_layers(N)
    elif a.layers == "validation":
        layers = wl.validation_layers(N)
    elif a.layers == "first":
        layers = wl.first_layers(N)
    else:
        layers = [named[n] for n in a.layers.split(",")]
    dtype = ps.PS_F32 if a.dtype == "f32" else ps.PS_BF16
    done = set()
    if a.store:
        try:
            done = {json.loads(l)["layer"] for l in open(a.store) if l.strip()}
        except FileNotFoundError:
            pass
    out = open(a.out, "w") if a.out else sys.stdout
    for shape in layers:
        if shape.name in done:
            print(f"{shape.name}: already stored, skipped", file=sys.stderr, flush=True)
            continue
        r = sweep(shape, dtype, a.min_ms, a.cold, use_ws=not a.atomics)
        if a.store:
            with open(a.store, "a") as f:
                f.write(json.dumps(stored_row(r, shape.N), separators=(",", ":")) + "\n")
        if not a.rows:
            r.pop("rows")
        print(json.dumps(r), file=out, flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())

"""Pairwise neural ranking of candidate tiles (Section 4.2.2 of the paper): training and use.

The network and its tournament run in the GPU library (``ps_ranker_play``, ``ps_tile_rank_dnn``); the statistics of
a tile come from the library's host calls.  This module only

* trains the network's parameters from exhaustive sweeps (``train``; PyTorch autograd on the CPU, which is all a
  3338-parameter network needs) and stores them as JSON under ``data/``,
* loads stored parameters (``load_params``), gathers the statistics of a descriptor's candidates (``tile_stats``),
* reports how the network's picks compare with the sweep's best (``evaluate``; needs the GPU).

Two kinds of statistics feed the same network:

* ``PS_RANKER_WORKING_SETS`` -- the paper's own input: the working-set sizes Algorithm 2 assigns to the three cache
  levels and to memory, here for the workgroup-level loop nest of a tile;
* ``PS_RANKER_LEVEL_TIMES`` -- the four parts of this library's tile model, i.e. the time each level of the machine
  is busy.  Occupancy, wave quantisation and launch cost decide between tiles on a GPU and none of them is visible
  in working-set sizes, so this is the variant that is useful for picking tiles.

Training follows the paper: the network sees two variants, their eight statistics divided by the common sum, and
learns which of the two ran faster (cross-entropy over the two outputs).  Pairs whose measured times differ by less
than 2 % are left out, since their order is measurement noise.

    python -m paper_2002_02145_amd.ranker train --dtype f32 --kind level_times
    python -m paper_2002_02145_amd.ranker evaluate --dtype f32 --kind level_times      # on the GPU
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

from . import binding as ps
from . import workloads as wl

DATA = os.path.join(os.path.dirname(os.path.abspath(__file__)), "data")
KINDS = {"working_sets": ps.PS_RANKER_WORKING_SETS, "level_times": ps.PS_RANKER_LEVEL_TIMES}
WIDTHS = (2 * ps.PS_RANKER_STATS, 64, 32, 16, 8, 2)
THETA = 0.6                      # Section 4.2.2
SWEEPS = {"f32": ("sweep_f32_N28.jsonl", "sweep_f32_N8.jsonl", "sweep_f32_N1.jsonl"), "bf16": ("sweep_bf16_N28.jsonl", "sweep_bf16_N8.jsonl", "sweep_bf16_N1.jsonl")}
NOISE = 0.02                     # pairs closer than this are not used for training


def _kind_name(kind: int) -> str:
    return {v: k for k, v in KINDS.items()}[kind]


def params_path(kind: int, dtype: str) -> str:
    return os.path.join(DATA, f"ranker_{dtype}_{_kind_name(kind)}.json")


def held_out_params_path(kind: int, dtype: str) -> str:
    """Parameters of the leave-one-layer-out networks (one float32 [PS_RANKER_PARAMS] array per batch-28 layer)."""
    return os.path.join(DATA, f"ranker_{dtype}_{_kind_name(kind)}_leave_one_out.npz")


def load_params(kind: int, dtype: str = "f32") -> np.ndarray:
    """Stored parameters as float32 [PS_RANKER_PARAMS] in the library's flat layout."""
    with open(params_path(kind, dtype)) as f:
        blob = json.load(f)
    p = np.asarray(blob["params"], dtype=np.float32)
    if p.shape != (ps.PS_RANKER_PARAMS,):
        raise ValueError(f"{params_path(kind, dtype)} holds {p.size} parameters, expected {ps.PS_RANKER_PARAMS}")
    return p


def tile_stats(desc: ps.ConvDesc, kind: int, workspace_bytes: int = 1 << 62, tiles=None):
    """(tiles, float32 [n][4]) of the candidates the ranking call considers, in enumeration order: those whose
    split-reduction workspace fits and that have statistics of this kind."""
    if tiles is None:
        tiles = [ps.ps_tile_get(desc, i) for i in range(ps.ps_tile_count(desc))]
    kept, rows = [], []
    for t in tiles:
        if t.c_split > 1 and ps.ps_workspace_bytes(desc, t) > workspace_bytes:
            continue
        if kind == ps.PS_RANKER_WORKING_SETS:
            try:
                level, mem = ps.ps_tile_reuse_levels(desc, t)
            except ps.PsError as e:
                if e.status == ps.PS_EUNSUPPORTED:
                    continue
                raise
            rows.append(level + [mem])
        else:
            rows.append(ps.ps_tile_level_times_ws(desc, t))
        kept.append(t)
    return kept, np.asarray(rows, dtype=np.float32).reshape(len(kept), ps.PS_RANKER_STATS)


def _named_layers(N: int):
    named = {l.name: l for l in wl.resnet50_layers(N) + wl.heldout_layers(N) + wl.validation_layers(N) + wl.first_layers(N)}
    b = wl.CFG3B
    named[b.name] = wl.ConvShape(N, b.C, b.H, b.W, b.K, b.R, b.S, b.stride, b.pad, b.name)
    return named


def load_sweeps(dtype: str, kind: int):
    """[(layer name, N, tiles, stats float64 [n][4], measured us [n])] from the sweeps stored under data/."""
    out = []
    dt = ps.PS_F32 if dtype == "f32" else ps.PS_BF16
    for fname in SWEEPS[dtype]:
        for line in open(os.path.join(DATA, fname)):
            r = json.loads(line)
            L = _named_layers(r["N"])[r["layer"]]
            d = ps.ConvDesc.of(L, dt)
            us = {tuple(row[:5]): row[5] for row in r["rows"]}
            tiles, stats = tile_stats(d, kind, tiles=[ps.Tile(*t) for t in us])
            out.append((r["layer"], r["N"], tiles, stats.astype(np.float64),
                        np.array([us[t.as_tuple()] for t in tiles])))
    return out


def _pairs(stats, us, limit, rng):
    n = len(us)
    i, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    i, j = i.ravel(), j.ravel()
    keep = (i != j) & (np.abs(us[i] / us[j] - 1.0) > NOISE)
    i, j = i[keep], j[keep]
    if len(i) > limit:
        sel = rng.choice(len(i), limit, replace=False)
        i, j = i[sel], j[sel]
    x = np.concatenate([stats[i], stats[j]], axis=1)
    total = x.sum(axis=1, keepdims=True)
    x = np.divide(x, total, out=np.zeros_like(x), where=total != 0)
    return x, (us[j] < us[i]).astype(np.int64)      # label 0: the first variant is faster


def _fit(sweeps, epochs: int, seed: int, pairs_per_layer: int = 20000):
    import torch
    nn = torch.nn
    rng = np.random.default_rng(seed)
    torch.manual_seed(seed)
    xs, ys = zip(*[_pairs(s, u, pairs_per_layer, rng) for _, _, _, s, u in sweeps])
    x = torch.tensor(np.concatenate(xs), dtype=torch.float32)
    y = torch.tensor(np.concatenate(ys))
    acts = (nn.ReLU, nn.ReLU, nn.Softsign, nn.ReLU)
    layers = []
    for k, (a, b) in enumerate(zip(WIDTHS[:-1], WIDTHS[1:])):
        layers.append(nn.Linear(a, b))
        if k < 4:
            layers.append(acts[k]())
    net = nn.Sequential(*layers)
    opt = torch.optim.Adam(net.parameters(), lr=2e-3)
    for _ in range(epochs):
        perm = torch.randperm(len(x))
        for b in range(0, len(x), 4096):
            idx = perm[b:b + 4096]
            loss = nn.functional.cross_entropy(net(x[idx]), y[idx])
            opt.zero_grad()
            loss.backward()
            opt.step()
    with torch.no_grad():
        acc = float((net(x).argmax(1) == y).float().mean())
    flat = []
    for m in net:
        if isinstance(m, nn.Linear):                 # torch keeps [units][inputs]; the library wants [inputs][units]
            flat.append(m.weight.detach().numpy().T.ravel())
            flat.append(m.bias.detach().numpy().ravel())
    return np.concatenate(flat).astype(np.float32), acc, net


def _pick_loss_cpu(net, stats, us):
    """Held-out check during training: the tournament with torch's own forward pass (float32, CPU)."""
    import torch
    n = len(us)
    i, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    i, j = i.ravel(), j.ravel()
    k = i != j
    i, j = i[k], j[k]
    x = np.concatenate([stats[i], stats[j]], axis=1)
    total = x.sum(axis=1, keepdims=True)
    x = np.divide(x, total, out=np.zeros_like(x), where=total != 0)
    with torch.no_grad():
        p = torch.softmax(net(torch.tensor(x, dtype=torch.float32)), 1).numpy()
    wins = np.zeros(n, dtype=np.int64)
    np.add.at(wins, i[p[:, 0] > THETA], 1)
    np.add.at(wins, j[p[:, 1] > THETA], 1)
    return float(us[int(np.argmax(wins))] / us.min() - 1.0)


def train(dtype: str, kind: int, epochs: int = 40, seed: int = 0, held_out: bool = True, out=sys.stdout) -> dict:
    """Fits the network on every stored sweep of this dtype and writes data/ranker_<dtype>_<kind>.json.  With
    held_out, each layer of the batch-28 sweep is first ranked by a network that never saw that layer (at any batch
    size); those losses are stored beside the parameters."""
    sweeps = load_sweeps(dtype, kind)
    report = {}
    if held_out:
        loo = {}
        for name, N, _, stats, us in sweeps:
            if N != wl.MINIBATCH:
                continue
            loo[name], _, net = _fit([s for s in sweeps if s[0] != name], epochs, seed)
            report[name] = round(_pick_loss_cpu(net, stats, us), 4)
            print(json.dumps({"held_out_layer": name, "pick_vs_best": report[name]}), file=out, flush=True)
        # kept so that `evaluate --held-out` can play these networks' tournaments in the GPU library
        np.savez_compressed(held_out_params_path(kind, dtype), **loo)
    params, acc, _ = _fit(sweeps, epochs, seed)
    blob = {"kind": _kind_name(kind), "dtype": dtype, "theta": THETA, "widths": list(WIDTHS),
            "layout": "per layer: weights [inputs][units] row-major, then bias",
            "trained_on": list(SWEEPS[dtype]), "epochs": epochs, "seed": seed,
            "pair_accuracy_on_training_pairs": round(acc, 4), "held_out_pick_vs_best": report,
            "params": [float(f"{v:.8g}") for v in params]}
    with open(params_path(kind, dtype), "w") as f:
        json.dump(blob, f, separators=(",", ":"))
        f.write("\n")
    print(json.dumps({"written": params_path(kind, dtype), "pair_accuracy": round(acc, 4)}), file=out)
    return blob


def evaluate(dtype: str, kind: int, out=sys.stdout, held_out: bool = False) -> dict:
    """Ranks every stored batch-28 layer with ps_tile_rank_dnn (GPU) and compares the pick with the sweep's best and
    with the tile model's pick.  held_out: each layer is ranked by the network that was trained without that layer (at
    any batch size) instead of the shipped one -- the same library call, other parameters."""
    import torch
    dt = ps.PS_F32 if dtype == "f32" else ps.PS_BF16
    params = torch.from_numpy(load_params(kind, dtype)).to("cuda:0")
    loo = np.load(held_out_params_path(kind, dtype)) if held_out else None
    worst = worst_model = 0.0
    rows = []
    for line in open(os.path.join(DATA, SWEEPS[dtype][0])):
        r = json.loads(line)
        L = _named_layers(r["N"])[r["layer"]]
        d = ps.ConvDesc.of(L, dt)
        us = {tuple(row[:5]): row[5] for row in r["rows"]}
        best = min(us.values())
        scratch = torch.empty(ps.ps_tile_rank_dnn_scratch_bytes(d), dtype=torch.uint8, device="cuda:0")
        if loo is not None:
            params = torch.from_numpy(np.ascontiguousarray(loo[r["layer"]], dtype=np.float32)).to("cuda:0")
        t0 = time.perf_counter()
        ranked = ps.ps_tile_rank_dnn(d, 1 << 40, kind, params, THETA, scratch, scratch.numel(), 3)
        rank_ms = (time.perf_counter() - t0) * 1e3          # statistics on the host, copies, tournament, sort
        # the tournament alone, on statistics already in device memory
        tiles, stats = tile_stats(d, kind)
        sd = torch.from_numpy(stats).to("cuda:0")
        wins = torch.empty(len(tiles), dtype=torch.int32, device="cuda:0")
        ps.ps_ranker_play(sd, len(tiles), params, THETA, wins)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            ps.ps_ranker_play(sd, len(tiles), params, THETA, wins)
        e1.record()
        torch.cuda.synchronize()
        play_us = e0.elapsed_time(e1) * 1e3 / 20
        ranked = [(t.as_tuple(), w) for t, w in ranked if t.as_tuple() in us]
        model_pick, _ = ps.ps_tile_select_ws(d, 1 << 40)
        row = {"layer": r["layer"], "pick": list(ranked[0][0]), "wins": ranked[0][1],
               "pick_vs_best": round(us[ranked[0][0]] / best - 1.0, 4),
               "top3_vs_best": round(min(us[t] for t, _ in ranked) / best - 1.0, 4),
               "model_pick_vs_best": round(us.get(model_pick.as_tuple(), float("nan")) / best - 1.0, 4),
               "candidates": len(tiles), "rank_call_ms": round(rank_ms, 2), "tournament_us": round(play_us, 1),
               # n (n - 1) games, 2 flop per parameter each
               "tournament_gflops": round(len(tiles) * (len(tiles) - 1) * 2.0 * ps.PS_RANKER_PARAMS / play_us / 1e3, 1)}
        worst, worst_model = max(worst, row["pick_vs_best"]), max(worst_model, row["model_pick_vs_best"])
        rows.append(row)
        print(json.dumps(row), file=out)
    summary = {"dtype": dtype, "kind": _kind_name(kind), "networks": "leave-one-layer-out" if held_out else "shipped",
               "layers": len(rows), "worst_pick_vs_best": worst,
               "mean_pick_vs_best": round(sum(r["pick_vs_best"] for r in rows) / len(rows), 4),
               "worst_model_pick_vs_best": worst_model}
    print(json.dumps({"summary": summary}), file=out)
    return summary


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("command", choices=["train", "evaluate"])
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--kind", default="level_times", choices=sorted(KINDS))
    ap.add_argument("--epochs", type=int, default=40)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-held-out", action="store_true", help="train: skip the leave-one-layer-out networks")
    ap.add_argument("--held-out", action="store_true",
                    help="evaluate: rank each layer with the network trained without it (GPU tournament as always)")
    a = ap.parse_args(argv)
    if a.command == "train":
        train(a.dtype, KINDS[a.kind], a.epochs, a.seed, not a.no_held_out)
    else:
        evaluate(a.dtype, KINDS[a.kind], held_out=a.held_out)
    return 0


if __name__ == "__main__":
    sys.exit(main())

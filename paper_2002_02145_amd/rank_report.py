"""Ranking report over an exhaustive sweep (output of ``autotune --rows --out FILE`` or a stored sweep of ``data/``); runs
on the host.

Two questions, both from Section 4.2 of the paper:

* top-k: the paper ranks n variants and runs the best k (it uses k = 1).  For k = 1, 2, 3, 5 this prints how far
  the best of the tile model's top k is from the sweep's best, and where the model's first pick ranks.
* does the paper's own cost function transfer?  Every candidate tile is written as a loop nest at workgroup
  granularity -- (pixel tile, channel tile) in launch order, then the split, then the batch-reduce loop -- whose
  array elements are the blocks a workgroup moves (its input pixels for one c-block, one filter slice, its output
  tile), weighted by their size in bytes.  ``ps_reuse_working_sets`` (Algorithm 1), ``ps_reuse_assign``
  (Algorithm 2 with registers+LDS, L2, Infinity Cache as the hierarchy) and ``ps_reuse_cost`` (Eq. 1) then give a
  cost per candidate, and its ranking is compared with the measured one.  The nest is the sequential one the
  paper analyses; nothing in it knows about 256 compute units, wave quantisation or the matrix cores.
"""
from __future__ import annotations

import argparse
import json
import math
import sys

from . import binding as ps
from . import workloads as wl

# latency (s) / bandwidth (B/s) of the levels a reuse can be served from, fastest first, plus memory: registers+LDS
# of one compute unit, all L2 slices, Infinity Cache, HBM (their capacities are ps_tile_reuse_levels')
LATENCY = [0.1e-6, 0.5e-6, 0.8e-6, 1.2e-6]
BANDWIDTH = [100e12, 14e12, 9e12, 5e12]


def _spearman(a, b):
    def ranks(v):
        order = sorted(range(len(v)), key=lambda i: v[i])
        r = [0.0] * len(v)
        i = 0
        while i < len(order):
            j = i
            while j + 1 < len(order) and v[order[j + 1]] == v[order[i]]:
                j += 1
            for k in range(i, j + 1):
                r[order[k]] = (i + j) / 2.0
            i = j + 1
        return r
    ra, rb = ranks(a), ranks(b)
    ma, mb = sum(ra) / len(ra), sum(rb) / len(rb)
    num = sum((x - ma) * (y - mb) for x, y in zip(ra, rb))
    den = math.sqrt(sum((x - ma) ** 2 for x in ra) * sum((y - mb) ** 2 for y in rb))
    return num / den if den > 0 else float("nan")


def paper_cost(desc: ps.ConvDesc, tile) -> float | None:
    """Eq. 1 for one candidate tile, or None where the workgroup-level nest is not rectangular (a split that cuts
    through a c-block's taps)."""
    try:
        level, mem = ps.ps_tile_reuse_levels(desc, ps.Tile(*tile))
    except ps.PsError as e:
        if e.status == ps.PS_EUNSUPPORTED:
            return None
        raise
    return ps.ps_reuse_cost(level, mem, LATENCY, BANDWIDTH)


def report(path: str, dtype: str, with_paper_cost: bool = True, out=sys.stdout) -> dict:
    named = {l.name: l for l in wl.resnet50_layers()}
    named[wl.CFG3B.name] = wl.CFG3B
    named[wl.CFG1.name] = wl.CFG1
    dt, es = (ps.PS_F32, 4) if dtype == "f32" else (ps.PS_BF16, 2)
    ks = (1, 2, 3, 5)
    worst = {k: 0.0 for k in ks}
    rows = []
    for line in open(path):
        r = json.loads(line)
        L = named[r["layer"]]
        d = ps.ConvDesc.of(L, dt)
        # rows as autotune --rows writes them ({"tile": [...], "us": ...}) or in the compact stored form ([kt, mt, ring, split, order, us])
        meas = {(tuple(x["tile"]) if isinstance(x, dict) else tuple(x[:5])): (x["us"] if isinstance(x, dict) else x[5]) for x in r["rows"]}
        use_ws = r.get("split_reduction", "workspace") == "workspace"
        model = {t: (ps.ps_tile_cost_ws_us if use_ws else ps.ps_tile_cost_us)(d, ps.Tile(*t)) for t in meas}
        model = {t: c for t, c in model.items() if c > 0}
        best = min(meas.values())
        order = sorted(model, key=model.get)
        by_meas = sorted(meas, key=meas.get)
        row = {"layer": r["layer"], "candidates": len(meas), "rank_of_pick": by_meas.index(order[0]) + 1,
               "spearman_model": round(_spearman([model[t] for t in model], [meas[t] for t in model]), 3)}
        for k in ks:
            loss = min(meas[t] for t in order[:k]) / best - 1.0
            row[f"top{k}_loss"] = round(loss, 4)
            worst[k] = max(worst[k], loss)
        if with_paper_cost:
            pc = {t: paper_cost(d, t) for t in meas}
            pc = {t: c for t, c in pc.items() if c is not None}
            if pc:
                pick = min(pc, key=pc.get)
                row["eq1_candidates"] = len(pc)
                row["eq1_pick_loss"] = round(meas[pick] / best - 1.0, 4)
                row["eq1_spearman"] = round(_spearman([pc[t] for t in pc], [meas[t] for t in pc]), 3)
        rows.append(row)
        print(json.dumps(row), file=out)
    summary = {"layers": len(rows), **{f"worst_top{k}_loss": round(worst[k], 4) for k in ks},
               "picks_ranked_first": sum(r["rank_of_pick"] == 1 for r in rows),
               "picks_in_top3": sum(r["rank_of_pick"] <= 3 for r in rows)}
    if with_paper_cost and any("eq1_pick_loss" in r for r in rows):
        e = [r for r in rows if "eq1_pick_loss" in r]
        summary["eq1_worst_pick_loss"] = max(r["eq1_pick_loss"] for r in e)
        summary["eq1_median_spearman"] = sorted(r["eq1_spearman"] for r in e)[len(e) // 2]
        summary["model_median_spearman"] = sorted(r["spearman_model"] for r in rows)[len(rows) // 2]
    print(json.dumps({"summary": summary}), file=out)
    return summary


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("sweep", help="JSON-lines file written by autotune --rows --out, or a stored sweep (data/sweep_*_N28.jsonl)")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--no-paper-cost", action="store_true")
    a = ap.parse_args(argv)
    report(a.sweep, a.dtype, not a.no_paper_cost)
    return 0


if __name__ == "__main__":
    sys.exit(main())

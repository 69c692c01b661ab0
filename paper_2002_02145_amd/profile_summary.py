"""Turns the CSV output of rocprofv3 runs of bench.py into a short text summary.

Expects a directory with the sub-folders written by four separate runs of the same command:
``trace/`` (--kernel-trace --stats), ``fetch/`` (--pmc FETCH_SIZE), ``write/`` (--pmc WRITE_SIZE) and
optionally ``sq/`` (SQ_* / GRBM_* counters).  FETCH_SIZE and WRITE_SIZE (KiB per dispatch) are scaled by what
the same counter reads for the plain device-to-device copies of known size that ``bench.py --ref-copy-mib``
issues in the same process.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))


def kernel_source_digest(dtype: str = "f32") -> str:
    """Digest of the kernel sources of `dtype` ("f32" or "bf16"); which tile and which inner loop run is recorded
    beside it."""
    h = hashlib.sha256()
    files = ["conv_fwd_kernel.h", f"conv_fwd_{dtype}.hip"] + (["conv_fwd_bf16_halo.h"] if dtype == "bf16" else
                                                            ["conv_fwd_f32_n16.h", "conv_fwd_f32_n16_kloop.h"])
    for f in files:
        with open(os.path.join(HERE, "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def _one(pattern: str) -> str | None:
    g = glob.glob(pattern)
    return g[0] if g else None


def _counters(path: str):
    per = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        per[r["Kernel_Name"]][r["Counter_Name"]].append((float(r["Counter_Value"]), int(r["Grid_Size"])))
    return per


def _ref_scale(per, counter: str, ref_mib: int) -> float | None:
    """known KiB / counted KiB over the reference copies (the largest copyBuffer dispatches)."""
    vals = []
    for k, c in per.items():
        if "copyBuffer" in k:
            vals += [v for v, _ in c.get(counter, [])]
    vals = sorted(vals)[-3:]
    if not vals or min(vals) <= 0:
        return None
    return ref_mib * 1024.0 / (sum(vals) / len(vals))


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("dir")
    ap.add_argument("--ref-copy-mib", type=int, default=256)
    ap.add_argument("--kernel", default="conv_fwd", help="substring of the kernel of interest")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"], help="which kernel sources the digest covers")
    a = ap.parse_args(argv)
    out = []
    stats = _one(os.path.join(a.dir, "trace", "*kernel_stats.csv"))
    if stats:
        out.append("kernel-trace --stats (per kernel: calls, average ns, share of GPU time)")
        for r in list(csv.DictReader(open(stats)))[:8]:
            out.append(f"  {r['Name'][:90]:90s} calls {r['Calls']:>5s}  avg {float(r['AverageNs']):10.0f} ns  "
                       f"min {r['MinNs']:>8s}  max {r['MaxNs']:>8s}  {float(r['Percentage']):5.1f} %")
    traffic = {}
    for sub, counter in (("fetch", "FETCH_SIZE"), ("write", "WRITE_SIZE")):
        f = _one(os.path.join(a.dir, sub, "*counter_collection.csv"))
        if not f:
            continue
        per = _counters(f)
        scale = _ref_scale(per, counter, a.ref_copy_mib)
        out.append(f"{counter} (KiB per dispatch); reference {a.ref_copy_mib} MiB copy -> scale factor "
                   f"{scale if scale is None else round(scale, 4)}")
        for k, c in per.items():
            vals = [v for v, _ in c.get(counter, [])]
            if not vals or ("ps::" not in k):
                continue
            mean = sum(vals) / len(vals)
            scaled = mean * (scale or 1.0)
            out.append(f"  {k[:90]:90s} n {len(vals):4d}  raw {mean:12.1f} KiB  scaled {scaled * 1024 / 1e6:9.2f} MB")
            if a.kernel in k:
                traffic[counter] = scaled * 1024
    f = _one(os.path.join(a.dir, "sq", "*counter_collection.csv"))
    if f:
        per = _counters(f)
        for k, c in per.items():
            if a.kernel not in k:
                continue
            m = {n: sum(v for v, _ in vs) / len(vs) for n, vs in c.items()}
            out.append(f"SQ counters, mean per dispatch of {k[:80]}")
            for n, v in sorted(m.items()):
                out.append(f"  {n:32s} {v:16.1f}")
            if "SQ_VALU_MFMA_BUSY_CYCLES" in m and "GRBM_GUI_ACTIVE" in m and m["GRBM_GUI_ACTIVE"] > 0:
                # MFMA busy cycles are summed over 1024 SIMDs, GRBM_GUI_ACTIVE over 8 XCDs
                util = (m["SQ_VALU_MFMA_BUSY_CYCLES"] / 1024.0) / (m["GRBM_GUI_ACTIVE"] / 8.0)
                out.append(f"  -> matrix-core busy fraction while the kernel runs: {util:.3f}")
            if m.get("SQ_LDS_IDX_ACTIVE", 0) > 0:
                out.append(f"  -> LDS bank-conflict cycles / LDS active cycles: "
                           f"{m.get('SQ_LDS_BANK_CONFLICT', 0) / m['SQ_LDS_IDX_ACTIVE']:.3f}")
    if traffic:
        tot = sum(traffic.values())
        out.append(f"HBM-side traffic of {a.kernel} per launch: fetch {traffic.get('FETCH_SIZE', 0) / 1e6:.2f} MB + "
                   f"write {traffic.get('WRITE_SIZE', 0) / 1e6:.2f} MB = {tot / 1e6:.2f} MB")
        out.append(f"kernel source digest ({a.dtype}): {kernel_source_digest(a.dtype)}")
        out.append(f"bench.py constant: ({kernel_source_digest(a.dtype)!r}, <tile the trace names>, {int(tot)})")
    print("\n".join(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

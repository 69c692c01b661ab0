"""Static check of the generated gfx950 code for a hardware hazard the compiler does not guard against.

A vector-ALU instruction that writes the data registers of a multi-dword buffer/global store (the form with a scalar
offset) right behind that store can overtake the store's read of them: a few lanes of a few stores then carry the new
value.  The kernels avoid it (stores straight from accumulator registers, or a short s_nop that keeps the stored
registers live); this test recompiles the kernel sources to assembly and fails if any such store is followed, within
three instructions and without an s_nop in between, by a write to one of its data registers.  Host only (hipcc
cross-compiles); it takes a minute or two."""
import os
import re
import shutil
import subprocess

import pytest

from paper_2002_02145_amd import build as psbuild

WINDOW = 3


def _regs(tok):
    m = re.match(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def _scan(asm_path):
    kernel, ins = None, []
    for line in open(asm_path):
        m = re.match(r"^([A-Za-z_][A-Za-z0-9_]*):", line)
        if m:
            kernel = m.group(1)
        t = line.strip()
        if line.startswith("\t") and t and not t.startswith((".", ";")):
            ins.append((kernel, t))
    hits, stores = [], 0
    for i, (k, t) in enumerate(ins):
        m = re.match(r"(buffer_store_dwordx[34]|global_store_dwordx[34]|flat_store_dwordx[34])\s+(.*)", t)
        if not m:
            continue
        ops = [o.strip() for o in m.group(2).split(",")]
        data = _regs(ops[0] if m.group(1).startswith("buffer") else ops[1])
        if not data:
            continue                       # data in accumulator registers
        stores += 1
        for j in range(i + 1, min(i + 1 + WINDOW, len(ins))):
            kj, tj = ins[j]
            op = tj.split()[0]
            if kj != k or op.startswith("s_nop"):
                break
            if op.startswith(("v_", "ds_read", "buffer_load", "global_load")) and not op.startswith("v_cmp"):
                dst = tj.split(None, 1)[1].split(",")[0].strip() if " " in tj else ""
                if _regs(dst) & data:
                    hits.append((k, t, tj))
                    break
    return stores, hits


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not installed")
@pytest.mark.parametrize("src", ["conv_fwd_f32.hip", "conv_fwd_bf16.hip"])
def test_no_vector_write_behind_a_wide_store(src, tmp_path):
    out = tmp_path / (src + ".s")
    flags = [f for f in psbuild.HIP_FLAGS if f != "-fPIC"]
    cmd = ["hipcc", "-x", "hip", "-S", "--cuda-device-only", os.path.join(psbuild.CSRC, src), "-o", str(out)] + flags
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    stores, hits = _scan(out)
    assert stores > 100, "the scan found no stores with vector-register data: has the assembly syntax changed?"
    assert not hits, "\n".join(f"{k}: {a} -> {b}" for k, a, b in hits[:10])


def test_scan_flags_a_planted_hazard(tmp_path):
    good = "k1:\n\tbuffer_store_dwordx4 v[8:11], v12, s[20:23], s10 offen\n\ts_nop 1\n\tv_add_f32_e32 v8, v0, v18\n"
    bad = "k2:\n\tbuffer_store_dwordx4 v[8:11], v12, s[20:23], s10 offen\n\tv_add_f32_e32 v9, v0, v18\n"
    agpr = "k3:\n\tbuffer_store_dwordx4 a[8:11], v12, s[20:23], s10 offen\n\tv_add_f32_e32 v9, v0, v18\n"
    p = tmp_path / "x.s"
    p.write_text(good + bad + agpr)
    stores, hits = _scan(p)
    assert stores == 2 and [h[0] for h in hits] == ["k2"]

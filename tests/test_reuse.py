"""The library's host-side reuse analysis (Section 4 of the paper: Algorithm 1, Algorithm 2, Eq. 1) against the
brute-force oracle and the paper's worked example.  No GPU needed."""
import os
import random

import pytest

from oracle import reuse_oracle as ro

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    rows = []
    for line in open(os.path.join(HERE, "golden", "reuse_matmul_worked_example.txt")):
        if line.strip() and not line.startswith("#"):
            rows.append(tuple(int(v) for v in line.split()))
    return rows


def _dep(deps, a, b):
    (hit,) = [d for d in deps if d[0] == a and d[1] == b]
    return hit[2], hit[3]


# ---- the library against the oracle -------------------------------------------------------------------------
@pytest.fixture(scope="module")
def ps():
    from paper_2002_02145_amd import binding
    return binding


def _to_lib(ps, refs, weight=None):
    weight = weight or {}
    return [ps.ArrayRef.of(r.array, r.coef, r.offset, r.is_write, weight.get(r.array, 1)) for r in refs]


@pytest.mark.parametrize("M,N,K,ws_min,ws_max", _golden())
def test_library_reproduces_the_papers_worked_example(ps, M, N, K, ws_min, ws_max):
    deps = ps.ps_reuse_working_sets((M, N, K), _to_lib(ps, ro.matmul_refs()))
    assert _dep(deps, 2, 2) == (ws_min, ws_max)


def test_library_matches_oracle_on_random_nests(ps):
    rng = random.Random(5)
    for case in range(40):
        n_loops = rng.randint(1, 4)
        extents = tuple(rng.randint(1, 4) for _ in range(n_loops))
        refs = []
        dims = {}
        for _ in range(rng.randint(1, 5)):
            arr = rng.randint(0, 2)
            nd = dims.setdefault(arr, rng.randint(1, 3))
            coef = tuple(tuple(rng.choice([0, 0, 1, 1, 2, -1]) for _ in range(n_loops)) for _ in range(nd))
            off = tuple(rng.randint(-1, 2) for _ in range(nd))
            refs.append(ro.Ref(arr, coef, off, rng.random() < 0.3))
        weight = {0: 1, 1: rng.randint(1, 3), 2: rng.randint(1, 8)}
        want = sorted(ro.working_set_sizes(extents, refs, weight))
        got = sorted(ps.ps_reuse_working_sets(extents, _to_lib(ps, refs, weight)))
        assert got == want, (case, extents, refs)


def test_library_conv_loop_nest_matches_oracle(ps):
    """The convolution of Fig. 4 without the GEMM loops: (img, ofm_tile, ifm_tile, oj, oi, kj, ki), blocks as elements."""
    N, Kb, Cb, P, Q, R, S = 2, 2, 2, 2, 3, 2, 2
    ext = (N, Kb, Cb, P, Q, R, S)
    #                 img ofm ifm oj oi kj ki
    out = ro.Ref(0, ((1, 0, 0, 0, 0, 0, 0), (0, 1, 0, 0, 0, 0, 0), (0, 0, 0, 1, 0, 0, 0), (0, 0, 0, 0, 1, 0, 0)), (0,) * 4, True)
    inp = ro.Ref(1, ((1, 0, 0, 0, 0, 0, 0), (0, 0, 1, 0, 0, 0, 0), (0, 0, 0, 1, 0, 1, 0), (0, 0, 0, 0, 1, 0, 1)), (0,) * 4)
    flt = ro.Ref(2, ((0, 1, 0, 0, 0, 0, 0), (0, 0, 1, 0, 0, 0, 0), (0, 0, 0, 0, 0, 1, 0), (0, 0, 0, 0, 0, 0, 1)), (0,) * 4)
    refs = [out, inp, flt]
    assert sorted(ps.ps_reuse_working_sets(ext, _to_lib(ps, refs))) == sorted(ro.working_set_sizes(ext, refs))


def test_library_algorithm_2_and_eq1(ps):
    assert ps.ps_reuse_assign([40, 4, 16, 8], [10, 30]) == ([4, 24], 40)
    assert ps.ps_reuse_assign([8, 8, 8], [10, 30]) == ([8, 0], 0)          # WS_all is a set
    rng = random.Random(2)
    for _ in range(50):
        ws = [rng.randint(1, 60) for _ in range(rng.randint(0, 8))]
        sizes = sorted(rng.randint(1, 80) for _ in range(rng.randint(0, 3)))
        assert ps.ps_reuse_assign(ws, sizes) == ro.assign_to_caches(set(ws), sizes)
        lvl, mem = ro.assign_to_caches(set(ws), sizes)
        lat = [rng.uniform(1, 100) for _ in range(len(sizes) + 1)]
        bw = [rng.uniform(1, 100) for _ in range(len(sizes) + 1)]
        assert ps.ps_reuse_cost(lvl, mem, lat, bw) == pytest.approx(ro.cost(lvl, mem, lat, bw), rel=1e-12)


def test_library_rejects_bad_arguments(ps):
    with pytest.raises(ps.PsError):
        ps.ps_reuse_working_sets((0, 2), _to_lib(ps, ro.matmul_refs()))
    with pytest.raises(ps.PsError):
        ps.ps_reuse_working_sets((4096, 4096, 4096), _to_lib(ps, ro.matmul_refs()))   # too many iterations
    with pytest.raises(ps.PsError):
        ps.ps_reuse_cost([1], 1, [1.0, 1.0], [1.0, 0.0])


def test_rank_report_on_a_synthetic_sweep(ps, tmp_path):
    """The report runs on the host from a sweep file; times here are made up (the tile model's own cost plus a
    deterministic wobble), so only the mechanics are checked."""
    import io
    import json
    from paper_2002_02145_amd import rank_report, workloads as wl
    L = wl.resnet50_layers()[5]                      # a 1x1 layer
    d = ps.ConvDesc.of(L)
    rows = []
    for i in range(ps.ps_tile_count(d)):
        t = ps.ps_tile_get(d, i)
        rows.append({"tile": list(t.as_tuple()), "us": ps.ps_tile_cost_ws_us(d, t) * (1.0 + 0.03 * ((i * 7) % 5))})
    f = tmp_path / "sweep.jsonl"
    f.write_text(json.dumps({"layer": L.name, "split_reduction": "workspace", "rows": rows}) + "\n")
    out = io.StringIO()
    s = rank_report.report(str(f), "f32", True, out)
    assert s["layers"] == 1 and 0.0 <= s["worst_top5_loss"] <= s["worst_top1_loss"] <= 0.13
    row = json.loads(out.getvalue().splitlines()[0])
    assert row["eq1_candidates"] == len(rows) and -1.0 <= row["eq1_spearman"] <= 1.0
    # Eq. 1 prefers fewer bytes through the slow levels: a larger tile of the same shape family never costs more
    small = rank_report.paper_cost(d, (64, 64, 4, 1, 0))
    large = rank_report.paper_cost(d, (64, 128, 4, 1, 0))
    assert small is not None and large is not None and small > 0 and large > 0

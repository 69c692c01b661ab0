"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared
symbol, validates descriptors, and the tile enumerator/model behave sanely."""
import ctypes
import os
import re

import pytest

from paper_2002_02145_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ps():
    from paper_2002_02145_amd import binding
    return binding


def test_every_declared_symbol_is_exported(ps):
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in os.listdir(inc):
        text = open(os.path.join(inc, f)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(ps_[a-z0-9_]+)\s*\(", text))
    assert len(names) >= 17
    raw = ctypes.CDLL(ps.LIB_PATH)
    for n in sorted(names):
        assert hasattr(raw, n), f"{n} declared in include/ but not exported"
        assert hasattr(ps, n) or n == "ps_strerror", f"{n} has no Python binding of the same name"


def test_sizes_and_dims(ps):
    d = ps.ConvDesc.of(wl.CFG3B)
    assert ps.ps_out_dims(d) == (14, 14)
    assert ps.ps_blocked_in_bytes(d) == 28 * 512 * 28 * 28 * 4
    assert ps.ps_blocked_wt_bytes(d) == 1024 * 512 * 4
    assert ps.ps_blocked_out_bytes(d) == 28 * 1024 * 14 * 14 * 4
    stem = wl.resnet50_layers()[-1]
    d = ps.ConvDesc.of(stem)
    assert ps.ps_out_dims(d) == (112, 112)
    assert ps.ps_blocked_in_bytes(d) == 28 * 16 * 224 * 224 * 4          # C = 3 padded to one block
    assert ps.ps_blocked_wt_bytes(d) == 64 * 16 * 49 * 4
    d = ps.ConvDesc.of(stem, ps.PS_BF16)
    assert ps.ps_blocked_in_bytes(d) == 28 * 16 * 224 * 224 * 2
    assert ps.ps_blocked_out_bytes(d) == 28 * 64 * 112 * 112 * 4         # output stays fp32


def test_descriptor_validation(ps):
    ok = wl.ConvShape(1, 16, 8, 8, 16, 3, 3, 1, 1)
    for field, val, status in [("N", 0, ps.PS_EINVAL), ("C", -1, ps.PS_EINVAL), ("stride", 0, ps.PS_EINVAL),
                               ("pad", -1, ps.PS_EINVAL), ("R", 11, ps.PS_EINVAL), ("K", 24, ps.PS_EUNSUPPORTED)]:
        d = ps.ConvDesc.of(ok)
        setattr(d, field, val)
        with pytest.raises(ps.PsError) as e:
            ps.ps_out_dims(d)
        assert e.value.status == status, field
        assert ps.ps_blocked_in_bytes(d) == 0
    d = ps.ConvDesc.of(ok, 7)
    with pytest.raises(ps.PsError) as e:
        ps.ps_out_dims(d)
    assert e.value.status == ps.PS_EUNSUPPORTED
    huge = ps.ConvDesc.of(wl.ConvShape(512, 1024, 224, 224, 16, 1, 1, 1, 0))     # > 2 GiB input
    with pytest.raises(ps.PsError) as e:
        ps.ps_out_dims(huge)
    assert e.value.status == ps.PS_EUNSUPPORTED
    assert "unsupported" in ps.strerror(ps.PS_EUNSUPPORTED)
    assert ps.strerror(ps.PS_OK) == "ok"


def test_tile_enumerator_and_model(ps):
    from shapes import EDGE_SHAPES
    for shape, dtype in [(s, t) for s in wl.resnet50_layers() + [wl.CFG1, wl.CFG3B] + EDGE_SHAPES
                         for t in (ps.PS_F32, ps.PS_BF16)]:
        d = ps.ConvDesc.of(shape, dtype)
        n = ps.ps_tile_count(d)
        assert n > 0
        tiles = [ps.ps_tile_get(d, i) for i in range(n)]
        assert len({t.as_tuple() for t in tiles}) == n, "duplicate candidates"
        nb = -(-shape.C // 16) * shape.R * shape.S
        for t in tiles:
            assert ps.ps_tile_valid(d, t)
            assert nb % t.c_split == 0
            assert ps.ps_tile_cost_us(d, t) > 0
        for t in tiles:
            assert ps.ps_workspace_bytes(d, t) == (0 if t.c_split == 1 else t.c_split * shape.N * shape.K * shape.P * shape.Q * 4)
            assert ps.ps_tile_cost_ws_us(d, t) > 0
        bw, usw = ps.ps_tile_select_ws(d, 0)
        assert bw.c_split == 1                       # no workspace: only unsplit tiles compete
        bw, usw = ps.ps_tile_select_ws(d, 1 << 40)
        assert usw == pytest.approx(min(ps.ps_tile_cost_ws_us(d, t) for t in tiles))
        # rank n, run top k: the k lowest modelled times, best first, the first being the k = 1 pick
        ranked = ps.ps_tile_rank_ws(d, 1 << 40, 5)
        assert len(ranked) == min(5, n) and ranked[0][0].as_tuple() == bw.as_tuple()
        assert [u for _, u in ranked] == sorted(u for _, u in ranked)
        assert [u for _, u in ranked] == pytest.approx(sorted(ps.ps_tile_cost_ws_us(d, t) for t in tiles)[:len(ranked)])
        assert all(u == pytest.approx(ps.ps_tile_cost_ws_us(d, t)) for t, u in ranked)
        assert len(ps.ps_tile_rank_ws(d, 1 << 40, n + 7)) == n
        assert all(t.c_split == 1 for t, _ in ps.ps_tile_rank_ws(d, 0, 3))
        best, us = ps.ps_tile_select(d)
        costs = [ps.ps_tile_cost_us(d, t) for t in tiles]
        assert us == pytest.approx(min(costs))
        assert best.as_tuple() in {t.as_tuple() for t in tiles}
        # no variant can be modelled faster than the matrix cores allow
        assert us * 1e-6 >= shape.flops / (157.3e12 if dtype == ps.PS_F32 else 2.5e15) * 0.999
        with pytest.raises(ps.PsError):
            ps.ps_tile_get(d, n)
    assert not ps.ps_tile_valid(ps.ConvDesc.of(wl.CFG1), ps.Tile(128, 128, 2, 1, 0))   # K = 64 < kt
    assert ps.ps_tile_cost_us(ps.ConvDesc.of(wl.CFG1), ps.Tile(128, 128, 2, 1, 0)) < 0


def test_specialised_shapes_are_refused_where_they_do_not_apply(ps):
    """The 16x16-tile kernels have no loop for a runtime filter size and no atomic epilogue, the pixel-stationary ones
    only serve 1x1 filters over exactly 64 channels: the validity call is what keeps them from being launched on
    anything else."""
    def valid(shape, tile, dtype=None):
        return ps.ps_tile_valid(ps.ConvDesc.of(shape, ps.PS_F32 if dtype is None else dtype), ps.Tile(*tile))
    S = wl.ConvShape
    stationary, n16 = (256, 176, 2, 1, 0), (64, 176, 2, 1, 0)
    assert valid(S(2, 64, 8, 8, 256, 1, 1, 1, 0), stationary)
    assert not valid(S(2, 128, 8, 8, 256, 1, 1, 1, 0), stationary)          # 8 c-blocks
    assert not valid(S(2, 48, 8, 8, 256, 1, 1, 1, 0), stationary)           # 3 c-blocks
    assert not valid(S(2, 64, 8, 8, 256, 3, 3, 1, 1), stationary)           # not 1x1
    assert not valid(S(2, 64, 3, 3, 256, 1, 1, 1, 0), stationary)           # images of fewer than 16 pixels
    assert not valid(S(2, 64, 8, 8, 256, 1, 1, 1, 0), (256, 176, 2, 2, 0))  # no split reduction
    assert not valid(S(2, 64, 8, 8, 256, 1, 1, 1, 0), stationary, ps.PS_BF16)
    assert valid(S(2, 64, 8, 8, 64, 3, 3, 1, 1), n16) and valid(S(2, 64, 8, 8, 64, 1, 1, 2, 0), n16)
    assert valid(S(2, 64, 8, 8, 64, 5, 5, 1, 2), n16)                       # 5x5 has a baked loop too
    assert not valid(S(2, 64, 8, 8, 64, 4, 4, 1, 2), n16)                   # no baked 4x4 loop
    assert not valid(S(2, 64, 8, 8, 64, 3, 3, 1, 1), (64, 176, 2, 2, 0))    # no atomic epilogue
    assert valid(S(2, 3, 20, 20, 64, 7, 7, 2, 3), n16)                      # tap-packed stem, 3 channels
    assert not valid(S(2, 4, 20, 20, 64, 7, 7, 2, 3), n16)                  # 4 channels: only the 32x32 kernels
    assert valid(S(2, 4, 20, 20, 64, 7, 7, 2, 3), (64, 128, 2, 1, 0))
    # and the variant report names them
    d = ps.ConvDesc.of(S(2, 64, 8, 8, 256, 1, 1, 1, 0))
    assert ps.KERNEL_NAMES[ps.ps_tile_kernel(d, ps.Tile(*stationary))] == "1x1 pixel-stationary"
    assert ps.KERNEL_NAMES[ps.ps_tile_kernel(ps.ConvDesc.of(S(2, 3, 20, 20, 64, 7, 7, 2, 3)), ps.Tile(*n16))] == "tap-packed"
    # the tap-packed loops of the other first-layer filter sizes: 3x3, 5x5, 11x11 over at most 3 channels in fp32
    # (16x16- and 32x32-tile kernels), over at most 8 in 16 bits; never for a split range
    kernel = lambda shape, tile, dtype=ps.PS_F32: ps.KERNEL_NAMES[ps.ps_tile_kernel(ps.ConvDesc.of(shape, dtype), ps.Tile(*tile))]
    for F, stride, pad in ((3, 2, 1), (5, 1, 2), (11, 4, 0)):
        first = S(2, 3, 40, 40, 64, F, F, stride, pad)
        assert kernel(first, n16) == "tap-packed" and kernel(first, (64, 128, 2, 1, 0)) == "tap-packed"
        assert kernel(first, (64, 128, 2, 1, 0), ps.PS_BF16) == "tap-packed"
        assert kernel(S(2, 8, 40, 40, 64, F, F, stride, pad), (64, 128, 2, 1, 0), ps.PS_BF16) == "tap-packed"
        assert kernel(S(2, 9, 40, 40, 64, F, F, stride, pad), (64, 128, 2, 1, 0), ps.PS_BF16) != "tap-packed"
        four = S(2, 4, 40, 40, 64, F, F, stride, pad)
        assert kernel(four, (64, 128, 2, 1, 0)) != "tap-packed"       # fp32 packs four channels for 7x7 only
        assert valid(four, n16) == (F in (3, 5)) and (F not in (3, 5) or kernel(four, n16) == f"{F}x{F} baked")
    assert kernel(S(2, 3, 40, 40, 64, 3, 3, 1, 1), (64, 128, 2, 3, 0)) == "general"        # split range: not packed
    assert kernel(S(2, 3, 40, 40, 64, 9, 9, 1, 4), (64, 128, 2, 1, 0)) == "general"        # no packed loop for 9x9
    assert kernel(S(2, 3, 12, 12, 64, 3, 3, 1, 1), (64, 128, 2, 1, 0), ps.PS_BF16) == "3x3 patch"   # the patch loop keeps its layers


def test_tile_cache_matches_uncached_selection_under_threads(ps):
    """ps_tile_pick serves the convolution calls' tile from the per-process table; 8 threads asking for a mix of
    descriptors, modes and workspace sizes at once must all see what the uncached ranking returns, and asking again
    must add no entries."""
    import threading
    from shapes import EDGE_SHAPES
    shapes = wl.resnet50_layers() + [wl.CFG1, wl.CFG3B] + EDGE_SHAPES
    jobs = []
    for s in shapes:
        for dtype in (ps.PS_F32, ps.PS_BF16):
            out_bytes = s.N * s.K * s.P * s.Q * 4
            for with_ws, ws_bytes in ((0, 0), (1, 0), (1, 3 * out_bytes + 5), (1, 1 << 40)):
                jobs.append((s, dtype, with_ws, ws_bytes))
    expect = {}
    for s, dtype, with_ws, ws_bytes in jobs:
        d = ps.ConvDesc.of(s, dtype)
        t = ps.ps_tile_select_ws(d, ws_bytes)[0] if with_ws else ps.ps_tile_select(d)[0]
        expect[(s.name, dtype, with_ws, ws_bytes)] = t.as_tuple()
    errors = []

    def worker(k):
        order = jobs[k::3] + jobs            # every thread starts elsewhere, then walks the whole list
        for s, dtype, with_ws, ws_bytes in order:
            got = ps.ps_tile_pick(ps.ConvDesc.of(s, dtype), with_ws, ws_bytes).as_tuple()
            if got != expect[(s.name, dtype, with_ws, ws_bytes)]:
                errors.append((s.name, dtype, with_ws, ws_bytes, got))

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(8)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors[:3]
    filled = ps.ps_tile_cache_entries()
    assert 0 < filled <= len(jobs)
    worker(0)
    assert ps.ps_tile_cache_entries() == filled
    # workspace sizes that admit the same number of partial planes share an entry
    d = ps.ConvDesc.of(wl.CFG1)
    out_bytes = wl.CFG1.N * wl.CFG1.K * wl.CFG1.P * wl.CFG1.Q * 4
    ps.ps_tile_pick(d, 1, 9 * out_bytes)
    n = ps.ps_tile_cache_entries()
    assert ps.ps_tile_pick(d, 1, 9 * out_bytes + 100).as_tuple() == ps.ps_tile_select_ws(d, 9 * out_bytes + 100)[0].as_tuple()
    assert ps.ps_tile_cache_entries() == n
    with pytest.raises(ps.PsError):
        ps.ps_tile_pick(ps.ConvDesc.of(wl.ConvShape(1, 16, 8, 8, 24, 3, 3, 1, 1)))


def test_steady_state_pick_is_a_lookup(ps):
    """After the first call the pick costs a table lookup: far below the microseconds the ranking itself takes."""
    import time
    worst = 0.0
    for s in wl.resnet50_layers():
        for dtype in (ps.PS_F32, ps.PS_BF16):
            d = ps.ConvDesc.of(s, dtype)
            ps.ps_tile_pick(d, 1, 256 << 20)
            t0 = time.perf_counter()
            for _ in range(2000):
                ps.lib.ps_tile_pick(ctypes.byref(d), 1, 256 << 20, ctypes.byref(ps.Tile()))
            worst = max(worst, (time.perf_counter() - t0) / 2000)
    assert worst < 5e-6, f"steady pick costs {worst * 1e6:.2f} us per call (ctypes overhead included)"

"""Host side of the pairwise ranker (Section 4.2.2 of the paper): the statistics of a candidate tile against the
brute-force working-set oracle, the tile model's level times against its total, and argument checks of the device
entry points that return before anything is launched."""
import ctypes

import numpy as np
import pytest

from oracle import reuse_oracle as ro
from paper_2002_02145_amd import binding as ps
from paper_2002_02145_amd import workloads as wl

LEVELS = [(160 + 512) * 1024, 32 * 1024 * 1024, 256 * 1024 * 1024]


def _oracle_levels(shape, es, kt, mt, c_split, raster):
    """The nest the header describes, written for the enumerating oracle: loops (tile, tile, split, c-block, tap),
    arrays 0 = output tile (read and written), 1 = input pixels of one c-block, 2 = one filter tap."""
    M = shape.N * shape.P * shape.Q
    n_mt, n_kt = -(-M // mt), -(-shape.K // kt)
    cbs, taps = -(-shape.C // 16) // c_split, shape.R * shape.S
    lm, lk = (0, 1) if raster == 0 else (1, 0)
    ext = [0] * 5
    ext[lm], ext[lk], ext[2], ext[3], ext[4] = n_mt, n_kt, c_split, cbs, taps

    def row(**kw):
        r = [0] * 5
        for name, v in kw.items():
            r[{"m": lm, "k": lk, "s": 2, "c": 3, "t": 4}[name]] = v
        return tuple(r)
    refs = [
        ro.Ref(0, (row(m=1), row(k=1), row(s=1)), (0, 0, 0), False),
        ro.Ref(0, (row(m=1), row(k=1), row(s=1)), (0, 0, 0), True),
        ro.Ref(1, (row(m=1), row(s=cbs, c=1)), (0, 0), False),
        ro.Ref(2, (row(k=1), row(s=cbs, c=1), row(t=1)), (0, 0, 0), False),
    ]
    weight = {0: min(mt, M) * min(kt, shape.K) * 4, 1: min(mt, M) * 16 * es, 2: min(kt, shape.K) * 16 * es}
    return ro.assign_to_caches(ro.ws_all(ext, refs, weight), LEVELS)


@pytest.mark.parametrize("shape,dtype,tile", [
    (wl.ConvShape(1, 32, 4, 4, 64, 3, 3, 1, 1, "t0"), ps.PS_F32, (32, 8, 2, 1, 0)),
    (wl.ConvShape(1, 32, 4, 4, 64, 3, 3, 1, 1, "t0"), ps.PS_F32, (32, 8, 2, 2, 1)),
    (wl.ConvShape(2, 64, 3, 3, 32, 1, 1, 1, 0, "t1"), ps.PS_BF16, (32, 16, 2, 2, 0)),
    (wl.ConvShape(1, 48, 5, 5, 96, 1, 1, 2, 0, "t2"), ps.PS_F32, (32, 4, 4, 3, 1)),
])
def test_tile_statistics_match_the_enumerating_oracle(shape, dtype, tile):
    d = ps.ConvDesc.of(shape, dtype)
    kt, mt, _ring, c_split, raster = tile
    got = ps.ps_tile_reuse_levels(d, ps.Tile(*tile))
    want = _oracle_levels(shape, 4 if dtype == ps.PS_F32 else 2, kt, mt, c_split, raster)
    assert got == (list(want[0]), want[1])
    assert sum(got[0]) + got[1] > 0


def test_tile_statistics_refuse_a_split_that_cuts_channel_blocks():
    d = ps.ConvDesc.of(wl.ConvShape(1, 64, 4, 4, 64, 3, 3, 1, 1, "t"))
    with pytest.raises(ps.PsError) as e:
        ps.ps_tile_reuse_levels(d, ps.Tile(64, 64, 2, 3, 0))      # 4 channel blocks, split 3
    assert e.value.status == ps.PS_EUNSUPPORTED
    with pytest.raises(ps.PsError) as e:
        ps.ps_tile_reuse_levels(d, ps.Tile(64, 0, 2, 1, 0))
    assert e.value.status == ps.PS_EINVAL


def test_level_times_add_up_to_the_tile_models_cost():
    """Without a split the total is (max + 0.12 min) of matrix-core time and the slower of the two traffic terms,
    times a launch-order factor of 1 or 1.02, plus the fixed part."""
    for L in (wl.CFG2, wl.CFG3A, wl.resnet50_layers()[3]):
        d = ps.ConvDesc.of(L)
        checked = 0
        for i in range(ps.ps_tile_count(d)):
            t = ps.ps_tile_get(d, i)
            if t.c_split != 1:
                continue
            t0, t1, t2, t3 = ps.ps_tile_level_times_ws(d, t)
            assert min(t0, t1, t2, t3) >= 0.0
            body = max(t0, max(t1, t2)) + 0.12 * min(t0, max(t1, t2))
            total = ps.ps_tile_cost_ws_us(d, t)
            assert any(abs(body * f + t3 - total) <= 1e-9 * total for f in (1.0, 1.02)), (L.name, t)
            checked += 1
        assert checked > 5
    with pytest.raises(ps.PsError) as e:
        ps.ps_tile_level_times_ws(ps.ConvDesc.of(wl.CFG2), ps.Tile(64, 100, 2, 1, 0))
    assert e.value.status == ps.PS_EUNSUPPORTED


def test_device_entry_points_check_their_arguments_before_launching():
    # none of these reaches the GPU: the pointers are never dereferenced
    fake = 0x1000
    ok = dict(stats=fake, n=4, params=fake, theta=0.6, wins=fake, probs=None, stream=0)

    def status(**kw):
        a = {**ok, **kw}
        try:
            ps.ps_ranker_play(a["stats"], a["n"], a["params"], a["theta"], a["wins"], a["probs"], a["stream"])
        except ps.PsError as e:
            return e.status
        return ps.PS_OK
    assert status(n=0, stats=None, params=None, wins=None) == ps.PS_OK          # nothing to do
    assert status(n=-1) == ps.PS_EINVAL
    assert status(theta=0.4) == ps.PS_EINVAL and status(theta=1.0) == ps.PS_EINVAL
    assert status(theta=float("nan")) == ps.PS_EINVAL
    assert status(stats=None) == ps.PS_EINVAL and status(params=None) == ps.PS_EINVAL and status(wins=None) == ps.PS_EINVAL
    assert status(stats=fake + 4) == ps.PS_EINVAL                                 # rows are read 16 bytes at a time
    assert status(probs=fake + 4) == ps.PS_EINVAL
    assert status(n=ps.PS_RANKER_MAX_VARIANTS + 1) == ps.PS_EUNSUPPORTED

    d = ps.ConvDesc.of(wl.CFG2)
    need = ps.ps_tile_rank_dnn_scratch_bytes(d)
    assert need == ps.ps_tile_count(d) * 20

    def rank_status(**kw):
        a = dict(ws=1 << 30, kind=ps.PS_RANKER_LEVEL_TIMES, params=fake, theta=0.6, scratch=fake, sb=need, k=3)
        a.update(kw)
        try:
            ps.ps_tile_rank_dnn(d, a["ws"], a["kind"], a["params"], a["theta"], a["scratch"], a["sb"], a["k"], stream=0)
        except ps.PsError as e:
            return e.status
        return ps.PS_OK
    assert rank_status(k=0) == ps.PS_EINVAL
    assert rank_status(kind=2) == ps.PS_EINVAL
    assert rank_status(params=None) == ps.PS_EINVAL and rank_status(scratch=None) == ps.PS_EINVAL
    assert rank_status(theta=0.2) == ps.PS_EINVAL
    assert rank_status(scratch=fake + 8) == ps.PS_EINVAL
    assert rank_status(sb=need - 1) == ps.PS_EINVAL                               # found before anything is copied


def test_seeded_ranker_inputs_are_reproducible():
    assert np.array_equal(wl.ranker_params(3), wl.ranker_params(3))
    assert wl.ranker_params(3).shape == (ps.PS_RANKER_PARAMS,) and wl.ranker_params(3).dtype == np.float32
    s = wl.ranker_stats(40, 5, duplicates=3)
    assert s.shape == (40, 4) and s.dtype == np.float32 and (s >= 0).all() and (s == 0).any()
    assert np.array_equal(s[39], s[0]) and np.array_equal(s[37], s[2])

"""Seeded random convolution shapes through the C ABI against the CPU oracle: the model's pick and a few other
candidate tiles per shape, in fp32 and bf16.  Small integer inputs make every sum exact, so the comparison is for
equality and a misplaced tap, pixel or channel cannot hide inside a tolerance; one pass with real values checks the
tolerances on the same shapes."""
import zlib

import numpy as np
import pytest

import oracle
from paper_2002_02145_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = {0: 1e-4, 1: 2e-2}
SHAPES = wl.random_shapes(36, seed=2024)


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
def test_random_shape_is_exact_on_integers_and_within_tolerance_on_reals(shape):
    from gpu_util import run_conv, all_tiles
    rng = np.random.default_rng(zlib.crc32(shape.name.encode()))   # which candidates: fixed per shape
    xi, wi = wl.small_integers(shape, 11)
    exact, _ = oracle.conv2d_fwd(shape, xi, wi)
    xr, wr = wl.uniform_pm1(shape, 12)
    for dtype in (0, 1):
        tiles = all_tiles(shape, dtype)
        assert tiles, f"no candidate tile for {shape}"
        some = [tiles[i] for i in sorted(rng.choice(len(tiles), size=min(4, len(tiles)), replace=False))]
        for t in [None] + some:
            got = run_conv(shape, xi, wi, dtype, t, ws=t is not None and t.c_split > 1)
            assert np.array_equal(got.astype(np.float64), exact), f"{shape} dtype={dtype} tile={t}"
        x, w = (xr, wr) if dtype == 0 else (wl.round_to_bf16(xr), wl.round_to_bf16(wr))
        out, mag = oracle.conv2d_fwd(shape, x, w)
        err = oracle.normalised_error(run_conv(shape, x, w, dtype), out, mag)
        assert err <= TOL[dtype], f"{shape} dtype={dtype}: err {err}"


@pytest.mark.parametrize("shape", wl.random_first_layer_shapes(16, seed=77), ids=lambda s: s.name)
def test_random_first_layer_shape_every_tile_is_exact_on_integers(shape):
    """Few input channels and square filters of side 3, 5, 7, 11: the layers the tap-packed loops take (where channel
    count and element type allow; the others run the ordinary loops).  Every candidate tile, both element types,
    integer inputs, equality with the oracle."""
    from gpu_util import run_conv, all_tiles
    xi, wi = wl.small_integers(shape, 13)
    exact, _ = oracle.conv2d_fwd(shape, xi, wi)
    for dtype in (0, 1):
        tiles = all_tiles(shape, dtype)
        assert tiles, f"no candidate tile for {shape}"
        for t in [None] + tiles:
            got = run_conv(shape, xi, wi, dtype, t, ws=t is not None and t.c_split > 1)
            assert np.array_equal(got.astype(np.float64), exact), f"{shape} dtype={dtype} tile={t and t.as_tuple()}"

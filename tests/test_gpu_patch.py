"""3x3 / stride 1 / pad 1 on bf16 inputs: the kernel that stages the input patch once per c-block, on shapes that
stress its row bookkeeping (tiles that span many small images, ragged pixel and channel tails, split ranges) and on
shapes whose patch does not fit, where the gathering kernel must take over.  Integer tensors: exact comparison."""
import numpy as np
import pytest

from paper_2002_02145_amd import binding as ps
from paper_2002_02145_amd import workloads as wl
from tests.gpu_util import all_tiles, run_conv

pytestmark = pytest.mark.gpu

SHAPES = [
    wl.ConvShape(9, 32, 7, 7, 64, 3, 3, 1, 1, "many_7x7_images"),
    wl.ConvShape(37, 40, 5, 3, 16, 3, 3, 1, 1, "tiny_5x3_images_K16"),
    wl.ConvShape(3, 48, 14, 14, 96, 3, 3, 1, 1, "14x14_K96"),
    wl.ConvShape(2, 16, 56, 56, 64, 3, 3, 1, 1, "56x56_one_cblock"),
    wl.ConvShape(1, 144, 28, 28, 128, 3, 3, 1, 1, "28x28_9_cblocks"),
    wl.ConvShape(1, 16, 9, 300, 32, 3, 3, 1, 1, "wide_rows_patch_does_not_fit"),
    wl.ConvShape(2, 32, 1, 1, 32, 3, 3, 1, 1, "1x1_images"),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
def test_patch_kernel_exact_on_integers(oracle_lib, shape):
    x, w = wl.small_integers(shape, 17)
    want, _ = oracle_lib.conv2d_fwd(shape, x, w)
    tiles = [t for t in all_tiles(shape, ps.PS_BF16) if t.ring == 2]      # the rows that may run the patch kernel
    assert tiles
    d = ps.ConvDesc.of(shape, ps.PS_BF16)
    variants = {ps.ps_tile_kernel(d, t) for t in tiles}
    if "does_not_fit" in shape.name:
        assert 9 not in variants and 3 in variants          # the gathering 3x3 loop takes over
    else:
        assert 9 in variants
    for t in tiles:
        for use_ws in (True, False):
            got = run_conv(shape, x, w, ps.PS_BF16, t, ws=use_ws)
            assert np.array_equal(got.astype(np.float64), want), (t, use_ws)


def test_patch_kernel_within_tolerance_on_real_values(oracle_lib):
    shape = wl.ConvShape(4, 128, 14, 14, 128, 3, 3, 1, 1, "14x14_128")
    x, w = wl.relu_like(shape, 23)
    x, w = wl.round_to_bf16(x), wl.round_to_bf16(w)
    want, mag = oracle_lib.conv2d_fwd(shape, x, w)
    for t in [t for t in all_tiles(shape, ps.PS_BF16) if t.ring == 2]:
        got = run_conv(shape, x, w, ps.PS_BF16, t, ws=True)
        assert oracle_lib.normalised_error(got, want, mag) <= 2e-2, t

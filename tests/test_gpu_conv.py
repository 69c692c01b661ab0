"""GPU forward convolution (through the C ABI) against the CPU oracle, element by element.

Tolerances: max |gpu - oracle| / sum|x*w| <= 1e-4 for fp32
inputs and <= 2e-2 for bf16 inputs with fp32 accumulation; outputs whose magnitude sum is zero must
be exactly zero; integer-valued inputs must reproduce the exact result."""
import numpy as np
import pytest

import oracle
from paper_2002_02145_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {0: 1e-4, 1: 2e-2}


def _prep(shape, gen, seed, dtype):
    x, w = gen(shape, seed)
    if dtype == 1:
        x, w = wl.round_to_bf16(x), wl.round_to_bf16(w)
    return x, w


def _dtypes():
    return [0, 1]


from shapes import EDGE_SHAPES


@pytest.mark.parametrize("shape", EDGE_SHAPES, ids=lambda s: s.name)
def test_every_candidate_tile_matches_oracle(shape):
    """Each tile the enumerator can emit must itself be correct (edge tiles, ragged tails, splits)."""
    from gpu_util import run_conv, all_tiles
    for dtype in _dtypes():
        x, w = _prep(shape, wl.uniform_pm1, 1, dtype)
        out, mag = oracle.conv2d_fwd(shape, x, w)
        tiles = all_tiles(shape, dtype)
        assert tiles, "enumerator produced no candidate"
        for t in tiles:
            got = run_conv(shape, x, w, dtype, t)
            err = oracle.normalised_error(got, out, mag)
            assert err <= TOL[dtype], f"{shape.name} dtype={dtype} {t}: err {err}"
            if t.c_split > 1:                       # same split through the workspace path
                got = run_conv(shape, x, w, dtype, t, ws=True)
                err = oracle.normalised_error(got, out, mag)
                assert err <= TOL[dtype], f"{shape.name} dtype={dtype} {t} (workspace): err {err}"
        got = run_conv(shape, x, w, dtype)          # the model's pick through ps_conv2d_fwd
        assert oracle.normalised_error(got, out, mag) <= TOL[dtype]
        got = run_conv(shape, x, w, dtype, ws=True)  # the model's pick through ps_conv2d_fwd_ws
        assert oracle.normalised_error(got, out, mag) <= TOL[dtype]


@pytest.mark.parametrize("shape", EDGE_SHAPES[:5] + [s for s in EDGE_SHAPES if s.name.startswith(("1x1_64to256", "stem_like_K64"))],
                         ids=lambda s: s.name)
def test_integer_inputs_reproduce_exact_result(shape):
    from gpu_util import run_conv, all_tiles
    for dtype in _dtypes():
        x, w = wl.small_integers(shape, 7)
        out, _ = oracle.conv2d_fwd(shape, x, w)
        for t in all_tiles(shape, dtype):
            got = run_conv(shape, x, w, dtype, t)
            assert np.array_equal(got.astype(np.float64), out), f"{shape.name} dtype={dtype} {t}"


def test_zero_magnitude_outputs_are_exact_zero():
    from gpu_util import run_conv
    shape = wl.ConvShape(2, 32, 10, 10, 32, 3, 3, 1, 1)
    x, w = wl.uniform_pm1(shape, 3)
    x[1] = 0.0                      # a whole image of zeros
    w[5] = 0.0                      # a whole output channel of zeros
    out, mag = oracle.conv2d_fwd(shape, x, w)
    got = run_conv(shape, x, w)
    assert not got[1].any() and not got[:, 5].any()
    assert oracle.normalised_error(got, out, mag) <= 1e-4


def test_output_is_overwritten_not_accumulated():
    from gpu_util import run_conv
    shape = wl.CFG1
    x, w = wl.uniform_pm1(shape, 1)
    out, mag = oracle.conv2d_fwd(shape, x, w)
    for poison in (1e30, float("nan")):
        got = run_conv(shape, x, w, poison=poison)
        assert oracle.normalised_error(got, out, mag) <= 1e-4


FULL = [(wl.CFG2, 2), (wl.CFG3A, 3), (wl.CFG3B, 4)]


@pytest.mark.parametrize("shape,seed", FULL, ids=lambda v: getattr(v, "name", str(v)))
def test_full_size_configs_fp32(shape, seed):
    """Benchmark sizes, launch configuration the benchmark times (the model's pick): two whole images
    plus random samples of the rest against the oracle."""
    from gpu_util import run_conv
    x, w = wl.relu_like(shape, seed)
    got = run_conv(shape, x, w)
    out, mag = oracle.conv2d_fwd(shape, x, w, images=(0, 1))
    assert oracle.normalised_error(got[:1], out[:1], mag[:1]) <= 1e-4
    n = shape.N - 1
    out, mag = oracle.conv2d_fwd(shape, x, w, images=(n, n + 1))
    assert oracle.normalised_error(got[n:], out[n:], mag[n:]) <= 1e-4
    rng = np.random.default_rng(seed)
    for _ in range(300):
        n, k, p, q = (int(rng.integers(v)) for v in (shape.N, shape.K, shape.P, shape.Q))
        o, m = oracle.conv2d_fwd_point(shape, x, w, n, k, p, q)
        assert abs(got[n, k, p, q] - o) <= 1e-4 * m


@pytest.mark.parametrize("dtype", [0, 1], ids=["fp32", "bf16"])
def test_resnet50_sweep(dtype):
    """Every layer of the ResNet-50-shaped sweep at N = 28 with the model's pick, every output element against the
    oracle (a fault that hits a few lanes of a few stores now and then does not show in one sampled image).
    bf16: inputs and filters rounded to bf16 first, oracle on the same values."""
    from gpu_util import run_conv
    for i, shape in enumerate(wl.resnet50_layers()):
        x, w = _prep(shape, wl.relu_like, wl.sweep_seed(i), dtype)
        got = run_conv(shape, x, w, dtype, ws=True)      # the configuration bench.py times
        out, mag = oracle.conv2d_fwd(shape, x, w)
        err = oracle.normalised_error(got, out, mag)
        assert err <= TOL[dtype], f"{shape.name}: {err}"
        rng = np.random.default_rng(i)
        for _ in range(20):                              # the point-wise oracle agrees with the bulk one
            nn, k, p, q = (int(rng.integers(v)) for v in (shape.N, shape.K, shape.P, shape.Q))
            o, m = oracle.conv2d_fwd_point(shape, x, w, nn, k, p, q)
            assert abs(got[nn, k, p, q] - o) <= TOL[dtype] * m, shape.name


@pytest.mark.parametrize("dtype", [0, 1], ids=["fp32", "bf16"])
def test_out_of_sample_layer_sets(dtype):
    """The layers of the out-of-sample sets (other widths, 5x5 and 11x11 filters, strided 3x3, a 96-channel stem, first
    layers with three input channels) at N = 28 with the library's pick: every output element against the oracle."""
    from gpu_util import run_conv
    for i, shape in enumerate(wl.heldout_layers() + wl.validation_layers() + wl.first_layers()):
        x, w = _prep(shape, wl.relu_like, 200 + i, dtype)
        got = run_conv(shape, x, w, dtype, ws=True)
        out, mag = oracle.conv2d_fwd(shape, x, w)
        err = oracle.normalised_error(got, out, mag)
        assert err <= TOL[dtype], f"{shape.name}: {err}"


@pytest.mark.parametrize("shape", [
    # blocked input of 2 * 4 * 2040 * 2040 * 64 B = 0.992 * 2^31 bytes: the largest byte offsets the kernels form
    wl.ConvShape(2, 64, 2040, 2040, 16, 1, 1, 2, 0, "input_near_2GiB"),
    # output of 4 * 512 * 510 * 510 * 4 B = 0.992 * 2^31 bytes
    wl.ConvShape(4, 16, 510, 510, 512, 1, 1, 1, 0, "output_near_2GiB"),
], ids=lambda s: s.name)
def test_tensors_near_the_size_limit(shape):
    """32-bit byte offsets up to the documented limit of 2 GiB per tensor: every output element against the oracle;
    one element more per side is refused."""
    from gpu_util import run_conv
    x, w = wl.relu_like(shape, 77)
    got = run_conv(shape, x, w, 0, ws=True)
    out, mag = oracle.conv2d_fwd(shape, x, w)
    assert oracle.normalised_error(got, out, mag) <= TOL[0]
    del got, out, mag
    too_big = wl.ConvShape(shape.N, shape.C, shape.H + 32, shape.W + 32, shape.K, 1, 1, shape.stride, 0)
    from paper_2002_02145_amd import binding as ps
    with pytest.raises(ps.PsError) as e:
        ps.ps_out_dims(ps.ConvDesc.of(too_big))
    assert e.value.status == ps.PS_EUNSUPPORTED


@pytest.mark.parametrize("dtype", [0, 1], ids=["fp32", "bf16"])
def test_every_candidate_tile_at_full_size(dtype):
    """Every tile the enumerator offers for every layer of the sweep, at N = 28: the oracle checks the first image of
    the model's pick (the sweep test above checks all of it), and every other candidate must agree with the pick on
    every output element up to the reordering of fp32 additions (compared on the device in blocked order; the data
    are the library's outputs on both sides, so no reference arithmetic is involved).  Covers the kernels the model
    does not pick (32x32- against 16x16-tile, gathering against patch loop, split reductions) at their real grids."""
    import torch
    from gpu_util import DEV, all_tiles, blocked_inputs
    from paper_2002_02145_amd import binding as ps
    for i, shape in enumerate(wl.resnet50_layers() + [wl.CFG3B] + wl.heldout_layers()):
        x, w = _prep(shape, wl.relu_like, wl.sweep_seed(i), dtype)
        d, xb, wb = blocked_inputs(shape, x, w, dtype)
        n_out = ps.ps_blocked_out_bytes(d) // 4
        ws = torch.empty((256 << 20) // 4, dtype=torch.float32, device=DEV)
        ref = torch.full((n_out,), float("nan"), dtype=torch.float32, device=DEV)
        ps.ps_conv2d_fwd_ws(d, None, xb, wb, ref, ws, ws.numel() * 4)
        P, Q = ps.ps_out_dims(d)
        first = ref.view(shape.N, shape.K // 16, P, Q, 16)[0].permute(0, 3, 1, 2).reshape(shape.K, P, Q).cpu().numpy()
        out, mag = oracle.conv2d_fwd(shape, x, w, images=(0, 1))
        assert oracle.normalised_error(first[None], out[:1], mag[:1]) <= TOL[dtype], shape.name
        scale = float(ref.abs().max())
        # the K-dimension of a sum is at most 4608 terms: reordering moves a result by a few units in the last place
        # of its largest partial sum; 1e-5 (fp32) of the layer's largest output is far above that and far below any
        # misplaced or missing term
        bound = (1e-5 if dtype == 0 else 1e-5) * scale
        got = torch.empty_like(ref)
        for t in all_tiles(shape, dtype):
            need = ps.ps_workspace_bytes(d, t)
            if need > ws.numel() * 4:
                continue
            got.fill_(float("nan"))
            ps.ps_conv2d_fwd_ws(d, t, xb, wb, got, ws if need else None, need)
            diff = float((got - ref).abs().max())            # NaN if anything was left unwritten
            assert diff <= bound, f"{shape.name} dtype={dtype} {t}: max |diff| {diff} against {bound}"
        del ws, ref, got, xb, wb

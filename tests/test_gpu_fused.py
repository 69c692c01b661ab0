"""Fused epilogue (bias, max(., 0), bf16 output) and chaining of layers with no transform in between, through the
C ABI against the oracle."""
import numpy as np
import pytest
import torch

from paper_2002_02145_amd import binding as ps
from paper_2002_02145_amd import workloads as wl
from tests.gpu_util import DEV, all_tiles, blocked_inputs

pytestmark = pytest.mark.gpu

TOL = {ps.PS_F32: 1e-4, ps.PS_BF16: 2e-2}


def _unblock(ob: torch.Tensor, shape, P, Q) -> np.ndarray:
    """[N][Kb][P][Q][16] (any element type) -> NKPQ float64 on the host (plain index shuffle, as oracle/layout.py)."""
    a = ob.to(torch.float32).cpu().numpy().astype(np.float64).reshape(shape.N, shape.K // 16, P, Q, 16)
    return a.transpose(0, 1, 4, 2, 3).reshape(shape.N, shape.K, P, Q)


def _run(shape, x, w, dtype, tile, bias, relu, out_dtype):
    d, xb, wb = blocked_inputs(shape, x, w, dtype)
    P, Q = ps.ps_out_dims(d)
    n_out = shape.N * shape.K * P * Q
    odt = torch.float32 if out_dtype == ps.PS_F32 else torch.bfloat16
    ob = torch.full((n_out,), float("nan"), dtype=odt, device=DEV)
    need = ps.ps_workspace_bytes(d, tile) if tile is not None else 64 << 20
    ws = torch.full((max(need, 16) // 4,), float("nan"), dtype=torch.float32, device=DEV)
    bd = None if bias is None else torch.from_numpy(bias).to(DEV)
    ps.ps_conv2d_fwd_fused(d, tile, xb, wb, ob, ws if need else None, need, bias=bd, relu=relu, out_dtype=out_dtype)
    torch.cuda.synchronize()
    return _unblock(ob, shape, P, Q), ob, d


def _check(oracle, got, shape, x, w, bias, relu, out_dtype, tol):
    want, mag, exact = oracle.conv2d_fwd_fused(shape, x, w, bias, relu, out_dtype == ps.PS_BF16)
    # accumulation error against the unrounded result, plus (bf16 output) one rounding of the stored value
    slack = tol * mag + (np.abs(exact) * 2.0 ** -8 if out_dtype == ps.PS_BF16 else 0.0)
    bad = np.abs(got - (exact if out_dtype == ps.PS_BF16 else want)) > slack + 1e-30 * (mag == 0)
    assert not bad.any(), (int(bad.sum()), float(np.abs(got - want).max()))
    if relu:
        assert got.min() >= 0.0
    return want


SHAPES = [wl.ConvShape(3, 40, 9, 11, 48, 3, 3, 1, 1, "3x3_C40_K48"), wl.ConvShape(2, 64, 14, 14, 128, 1, 1, 1, 0, "1x1_64to128"),
          wl.ConvShape(2, 256, 7, 7, 64, 3, 3, 1, 1, "3x3_256to64_7"), wl.ConvShape(1, 3, 30, 30, 32, 7, 7, 2, 3, "stem_like")]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("dtype", [ps.PS_F32, ps.PS_BF16], ids=["fp32", "bf16"])
@pytest.mark.parametrize("out_dtype", [ps.PS_F32, ps.PS_BF16], ids=["out_fp32", "out_bf16"])
def test_fused_matches_oracle_on_every_tile(oracle_lib, shape, dtype, out_dtype):
    x, w = wl.uniform_pm1(shape, 21)
    if dtype == ps.PS_BF16:
        x, w = wl.round_to_bf16(x), wl.round_to_bf16(w)
    bias = np.random.default_rng(4).standard_normal(shape.K).astype(np.float32)
    tiles = all_tiles(shape, dtype)
    assert any(t.c_split > 1 for t in tiles) or shape.C <= 16
    tiles = tiles[::max(1, len(tiles) // 40)]                  # a spread of at most ~40 candidates per case
    assert any(t.c_split > 1 for t in tiles) or shape.C <= 16
    for i, t in enumerate(tiles):
        relu, b = bool(i % 2), (bias if i % 3 else None)      # rotate through the combinations
        got, _, _ = _run(shape, x, w, dtype, t, b, relu, out_dtype)
        _check(oracle_lib, got, shape, x, w, b, relu, out_dtype, TOL[dtype])


@pytest.mark.parametrize("out_dtype", [ps.PS_F32, ps.PS_BF16], ids=["out_fp32", "out_bf16"])
def test_fused_pixel_stationary_tiles(oracle_lib, out_dtype):
    """The kernels that keep a tile's pixels in LDS and walk over four output tiles have their own fused stores."""
    shape = wl.ConvShape(3, 64, 9, 7, 512, 1, 1, 1, 0, "1x1_64to512")
    x, w = wl.uniform_pm1(shape, 22)
    bias = np.random.default_rng(5).standard_normal(shape.K).astype(np.float32)
    tiles = [t for t in all_tiles(shape, ps.PS_F32) if ps.KERNEL_NAMES[ps.ps_tile_kernel(ps.ConvDesc.of(shape), t)] == "1x1 pixel-stationary"]
    assert len(tiles) >= 3
    for i, t in enumerate(tiles):
        relu, b = bool(i % 2), (bias if i % 3 != 1 else None)
        got, _, _ = _run(shape, x, w, ps.PS_F32, t, b, relu, out_dtype)
        _check(oracle_lib, got, shape, x, w, b, relu, out_dtype, TOL[ps.PS_F32])


@pytest.mark.parametrize("dtype", [ps.PS_F32, ps.PS_BF16], ids=["fp32", "bf16"])
def test_fused_bf16_output_is_exact_on_integers(oracle_lib, dtype):
    """Small-integer tensors make every sum exact, so the stored bf16 must be the correctly rounded value (many sums
    here are exact ties between two bf16 values)."""
    shape = wl.ConvShape(2, 64, 10, 10, 64, 3, 3, 1, 1)
    x, w = wl.small_integers(shape, 5, -8, 8)
    bias = np.arange(shape.K, dtype=np.float32) - 31.0
    for t in (None, all_tiles(shape, dtype)[0], [t for t in all_tiles(shape, dtype) if t.c_split > 1][0]):
        got, _, _ = _run(shape, x, w, dtype, t, bias, True, ps.PS_BF16)
        want, _, exact = oracle_lib.conv2d_fwd_fused(shape, x, w, bias, True, True)
        assert np.abs(exact).max() > 300 and (want != exact).any()     # rounding really happens
        assert np.array_equal(got, want)


def test_layers_chain_without_transforms(oracle_lib):
    """3x3 (+bias, max(., 0)) -> 1x1: the first output buffer is the second layer's blocked input, in fp32 and, with
    bf16 output, for a bf16 second layer."""
    s1 = wl.ConvShape(2, 32, 12, 12, 64, 3, 3, 1, 1)
    s2 = wl.ConvShape(2, 64, 12, 12, 32, 1, 1, 1, 0)
    x, w1 = wl.small_integers(s1, 8)
    _, w2 = wl.small_integers(s2, 9)
    bias = (np.arange(s1.K, dtype=np.float32) % 7) - 3.0
    for mid in (ps.PS_F32, ps.PS_BF16):
        _, ob1, _ = _run(s1, x, w1, ps.PS_F32, None, bias, True, mid)
        y1, _, _ = oracle_lib.conv2d_fwd_fused(s1, x, w1, bias, True, mid == ps.PS_BF16)
        d2 = ps.ConvDesc.of(s2, mid)
        tdt = torch.float32 if mid == ps.PS_F32 else torch.bfloat16
        w2d = torch.from_numpy(w2).to(tdt).to(DEV)
        wb2 = torch.empty(ps.ps_blocked_wt_bytes(d2) // (4 if mid == ps.PS_F32 else 2), dtype=tdt, device=DEV)
        ps.ps_kcrs_to_blocked(d2, w2d, wb2)
        ob2 = torch.full((ps.ps_blocked_out_bytes(d2) // 4,), float("nan"), dtype=torch.float32, device=DEV)
        ps.ps_conv2d_fwd(d2, ob1, wb2, ob2)
        torch.cuda.synchronize()
        got = _unblock(ob2, s2, 12, 12)
        want, mag = oracle_lib.conv2d_fwd(s2, y1.astype(np.float32), w2)
        assert oracle_lib.normalised_error(got, want, mag) <= 1e-6   # integers: exact up to fp32 sums of large values


def test_fused_rejects_bad_arguments():
    shape = wl.ConvShape(1, 64, 7, 7, 64, 3, 3, 1, 1)
    x, w = wl.uniform_pm1(shape, 1)
    d, xb, wb = blocked_inputs(shape, x, w)
    ob = torch.empty(ps.ps_blocked_out_bytes(d) // 4, dtype=torch.float32, device=DEV)
    split = [t for t in all_tiles(shape) if t.c_split > 1][0]
    with pytest.raises(ps.PsError) as e:
        ps.ps_conv2d_fwd_fused(d, split, xb, wb, ob, None, 0, relu=True)       # split tile without its workspace
    assert e.value.status == ps.PS_EINVAL
    with pytest.raises(ps.PsError) as e:
        ps.ps_conv2d_fwd_fused(d, None, xb, wb, ob, None, 0, out_dtype=5)
    assert e.value.status == ps.PS_EUNSUPPORTED
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype", [ps.PS_F32, ps.PS_BF16], ids=["fp32", "bf16"])
def test_fused_every_candidate_tile_at_full_size(dtype):
    """Every tile of every layer of the sweep at N = 28 with bias and max(., 0), fp32 and bf16 output, against the same
    two elementwise steps applied (torch, on the device) to the unfused output of the model's pick, which
    tests/test_gpu_conv.py checks against the oracle.  The fused kernels are separate instances with their own
    instruction schedules; this runs each of them at its real grid."""
    for i, shape in enumerate(wl.resnet50_layers() + [wl.CFG3B]):
        x, w = wl.relu_like(shape, 200 + i)
        if dtype == ps.PS_BF16:
            x, w = wl.round_to_bf16(x), wl.round_to_bf16(w)
        d, xb, wb = blocked_inputs(shape, x, w, dtype)
        P, Q = ps.ps_out_dims(d)
        n_out = shape.N * shape.K * P * Q
        ws = torch.empty((256 << 20) // 4, dtype=torch.float32, device=DEV)
        ref = torch.empty(n_out, dtype=torch.float32, device=DEV)
        ps.ps_conv2d_fwd_ws(d, None, xb, wb, ref, ws, ws.numel() * 4)
        bias = torch.from_numpy(np.random.default_rng(i).standard_normal(shape.K).astype(np.float32)).to(DEV)
        want = torch.clamp(ref.view(shape.N, shape.K // 16, P, Q, 16) + bias.view(1, shape.K // 16, 1, 1, 16), min=0).reshape(-1)
        scale = float(want.abs().max())
        for out_dtype, odt in ((ps.PS_F32, torch.float32), (ps.PS_BF16, torch.bfloat16)):
            # reordered fp32 additions, plus one bf16 rounding (2^-8 relative) of the stored value
            bound = 1e-5 * scale + (scale * 2.0 ** -8 if out_dtype == ps.PS_BF16 else 0.0)
            got = torch.empty(n_out, dtype=odt, device=DEV)
            for t in all_tiles(shape, dtype):
                need = ps.ps_workspace_bytes(d, t)
                if need > ws.numel() * 4:
                    continue
                got.fill_(float("nan"))
                ps.ps_conv2d_fwd_fused(d, t, xb, wb, got, ws if need else None, need, bias=bias, relu=True, out_dtype=out_dtype)
                diff = float((got.float() - want).abs().max())
                assert diff <= bound, f"{shape.name} dtype={dtype} out={out_dtype} {t}: {diff} against {bound}"
        del ws, ref, got, xb, wb, want

"""GPU layout transforms against the numpy index identities: bit for bit."""
import numpy as np
import pytest
import torch

from oracle import layout
from paper_2002_02145_amd import workloads as wl

pytestmark = pytest.mark.gpu

SHAPES = [
    wl.ConvShape(2, 35, 9, 13, 32, 3, 2, 1, 1),       # ragged channel count, odd sizes
    wl.ConvShape(1, 3, 40, 37, 16, 7, 7, 2, 3),       # stem-like: C = 3 padded to 16, HW > one pixel tile
    wl.ConvShape(3, 64, 14, 14, 64, 3, 3, 1, 1),
    wl.ConvShape(2, 16, 1, 1, 48, 1, 1, 1, 0),        # single pixel
    wl.ConvShape(1, 128, 28, 28, 16, 1, 1, 2, 0),     # strided: output smaller than input
    wl.ConvShape(300, 4096, 2, 2, 16, 1, 1, 1, 0),    # 76800 (image, channel block) pairs: more than one grid dimension holds
    wl.ConvShape(2, 24, 16, 24, 32, 1, 1, 1, 0),      # pixel count a multiple of 8: 16-byte blocks in both element sizes, ragged C
]


def _bits(t, np_dtype):
    return t.cpu().contiguous().view(torch.int32 if np_dtype == np.uint32 else torch.int16).numpy().view(np_dtype)


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: f"N{s.N}C{s.C}H{s.H}W{s.W}K{s.K}R{s.R}S{s.S}")
@pytest.mark.parametrize("es", [4, 2])
def test_transforms_bit_exact(shape, es):
    from paper_2002_02145_amd import binding as ps
    rng = np.random.default_rng(shape.C * 7 + es)
    npdt, tdt = (np.uint32, torch.int32) if es == 4 else (np.uint16, torch.int16)
    dtype = ps.PS_F32 if es == 4 else ps.PS_BF16
    d = ps.ConvDesc.of(shape, dtype)
    # arbitrary bit patterns (NaNs, infinities, denormals included): a permutation must keep them all
    x = rng.integers(0, 2 ** (8 * es), size=(shape.N, shape.C, shape.H, shape.W), dtype=np.uint64).astype(npdt)
    w = rng.integers(0, 2 ** (8 * es), size=(shape.K, shape.C, shape.R, shape.S), dtype=np.uint64).astype(npdt)
    xd = torch.from_numpy(x.view(np.int32 if es == 4 else np.int16)).to("cuda:0")
    wd = torch.from_numpy(w.view(np.int32 if es == 4 else np.int16)).to("cuda:0")
    xb = torch.full((ps.ps_blocked_in_bytes(d) // es,), -1, dtype=tdt, device="cuda:0")
    wb = torch.full((ps.ps_blocked_wt_bytes(d) // es,), -1, dtype=tdt, device="cuda:0")
    ps.ps_nchw_to_blocked(d, xd, xb)
    ps.ps_kcrs_to_blocked(d, wd, wb)
    np.testing.assert_array_equal(_bits(xb, npdt), layout.act_to_blocked(x).ravel())
    want_w = layout.filt_to_blocked(w) if es == 4 else layout.filt_to_blocked_packed8(w)
    np.testing.assert_array_equal(_bits(wb, npdt), want_w.ravel())
    # inverses
    x2 = torch.full_like(xd, -1)
    w2 = torch.full_like(wd, -1)
    ps.ps_blocked_to_nchw(d, xb, x2)
    ps.ps_blocked_to_kcrs(d, wb, w2)
    np.testing.assert_array_equal(_bits(x2, npdt).reshape(x.shape), x)
    np.testing.assert_array_equal(_bits(w2, npdt).reshape(w.shape), w)
    if es == 4:
        P, Q = ps.ps_out_dims(d)
        y = rng.integers(0, 2 ** 32, size=(shape.N, shape.K, P, Q), dtype=np.uint64).astype(np.uint32)
        yb = torch.from_numpy(layout.out_to_blocked(y).view(np.int32)).to("cuda:0")
        yo = torch.full((y.size,), -1, dtype=torch.int32, device="cuda:0")
        ps.ps_blocked_to_nkpq(d, yb, yo)
        np.testing.assert_array_equal(_bits(yo, np.uint32).reshape(y.shape), y)


def test_transform_rejects_bad_arguments():
    from paper_2002_02145_amd import binding as ps
    d = ps.ConvDesc.of(wl.CFG1)
    t = torch.zeros(64 * 14 * 14 + 8, device="cuda:0")
    with pytest.raises(ps.PsError) as e:
        ps.ps_nchw_to_blocked(d, 0, t)
    assert e.value.status == ps.PS_EINVAL
    with pytest.raises(ps.PsError) as e:
        ps.ps_nchw_to_blocked(d, t.data_ptr() + 4, t)       # misaligned
    assert e.value.status == ps.PS_EINVAL
    bad = ps.ConvDesc.of(wl.ConvShape(1, 16, 8, 8, 24, 3, 3, 1, 1))
    with pytest.raises(ps.PsError) as e:
        ps.ps_kcrs_to_blocked(bad, t, t)
    assert e.value.status == ps.PS_EUNSUPPORTED

"""Helpers for the GPU parity tests: move seeded numpy tensors through the C ABI."""
import numpy as np
import torch

from paper_2002_02145_amd import binding as ps
from paper_2002_02145_amd import workloads as wl

DEV = "cuda:0"


def to_dev(a: np.ndarray, dtype: int) -> torch.Tensor:
    """fp32 numpy -> device tensor of the path's element type (bf16 values must be pre-rounded)."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype == ps.PS_BF16:
        t = t.to(torch.bfloat16)
    return t.to(DEV)


def blocked_inputs(shape, x: np.ndarray, w: np.ndarray, dtype: int = ps.PS_F32):
    """NCHW/KCRS numpy -> blocked device tensors, using the library's own transforms."""
    d = ps.ConvDesc.of(shape, dtype)
    tdt = torch.float32 if dtype == ps.PS_F32 else torch.bfloat16
    es = 4 if dtype == ps.PS_F32 else 2
    xd, wd = to_dev(x, dtype), to_dev(w, dtype)
    xb = torch.empty(ps.ps_blocked_in_bytes(d) // es, dtype=tdt, device=DEV)
    wb = torch.empty(ps.ps_blocked_wt_bytes(d) // es, dtype=tdt, device=DEV)
    ps.ps_nchw_to_blocked(d, xd, xb)
    ps.ps_kcrs_to_blocked(d, wd, wb)
    return d, xb, wb


def run_conv(shape, x, w, dtype: int = ps.PS_F32, tile=None, poison: float = float("nan"), ws: bool = False) -> np.ndarray:
    """Full path through the C ABI: transforms, convolution, inverse transform.  Returns NKPQ fp32.
    The blocked output buffer is pre-filled with `poison` so that unwritten elements show.
    ws=True goes through ps_conv2d_fwd_ws with a poisoned workspace of exactly the needed size."""
    d, xb, wb = blocked_inputs(shape, x, w, dtype)
    ob = torch.full((ps.ps_blocked_out_bytes(d) // 4,), poison, dtype=torch.float32, device=DEV)
    if ws:
        need = ps.ps_workspace_bytes(d, tile) if tile is not None else 64 << 20
        buf = torch.full((max(need, 16) // 4,), poison, dtype=torch.float32, device=DEV)
        ps.ps_conv2d_fwd_ws(d, tile, xb, wb, ob, buf if need else None, need)
    elif tile is None:
        ps.ps_conv2d_fwd(d, xb, wb, ob)
    else:
        ps.ps_conv2d_fwd_tile(d, tile, xb, wb, ob)
    P, Q = ps.ps_out_dims(d)
    y = torch.empty((shape.N, shape.K, P, Q), dtype=torch.float32, device=DEV)
    ps.ps_blocked_to_nkpq(d, ob, y)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def all_tiles(shape, dtype: int = ps.PS_F32):
    d = ps.ConvDesc.of(shape, dtype)
    return [ps.ps_tile_get(d, i) for i in range(ps.ps_tile_count(d))]

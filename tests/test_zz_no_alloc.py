"""ps_conv2d_fwd_static: the convolution on the library's static scratch array (for callers that cannot allocate),
against ps_conv2d_fwd_ws with a caller's workspace and against the CPU oracle.

Two calls in a row share the array, the second on a smaller input, so what the first call leaves behind in the array
must not show in the second one's result."""
import numpy as np
import pytest
import torch

import oracle
from paper_2002_02145_amd import binding as ps
from paper_2002_02145_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _split_tile(d):
    """The candidate with the deepest split of the reduction (the most partial planes in the scratch array)."""
    tiles = [ps.ps_tile_get(d, i) for i in range(ps.ps_tile_count(d))]
    split = [t for t in tiles if t.c_split > 1 and ps.ps_workspace_bytes(d, t) <= ps.PS_STATIC_SCRATCH_BYTES]
    assert split, "no split candidate for this shape"
    return max(split, key=lambda t: (t.c_split, t.mt))


def _both_paths(shape, seed, dtype, tile_of):
    from gpu_util import blocked_inputs, DEV
    x, w = wl.uniform_pm1(shape, seed)
    if dtype == ps.PS_BF16:
        x, w = wl.round_to_bf16(x), wl.round_to_bf16(w)
    d, xb, wb = blocked_inputs(shape, x, w, dtype)
    tile = tile_of(d)
    n = ps.ps_blocked_out_bytes(d) // 4
    got = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    ref = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    print(f"static-scratch call: {shape.name} dtype={dtype} tile={tile}", flush=True)
    ps.ps_conv2d_fwd_static(d, tile, xb, wb, got)
    if tile is None:
        tile = ps.ps_tile_pick(d, True, ps.PS_STATIC_SCRATCH_BYTES)
    need = ps.ps_workspace_bytes(d, tile)
    buf = torch.full((max(need, 16) // 4,), float("nan"), dtype=torch.float32, device=DEV)
    ps.ps_conv2d_fwd_ws(d, tile, xb, wb, ref, buf if need else None, need)
    y = torch.empty((shape.N, shape.K, shape.P, shape.Q), dtype=torch.float32, device=DEV)
    ps.ps_blocked_to_nkpq(d, got, y)
    torch.cuda.synchronize()
    out, mag = oracle.conv2d_fwd(shape, x, w)
    return got.cpu().numpy(), ref.cpu().numpy(), oracle.normalised_error(y.cpu().numpy(), out, mag), tile


@pytest.mark.parametrize("dtype", [ps.PS_F32, ps.PS_BF16])
def test_two_calls_in_a_row_second_one_smaller(dtype):
    big = wl.ConvShape(4, 64, 14, 14, 64, 3, 3, 1, 1, "static_3x3_64_14_N4")
    small = wl.ConvShape(1, 48, 7, 9, 32, 3, 3, 1, 1, "static_3x3_48to32_7x9_N1")
    tol = 1e-4 if dtype == ps.PS_F32 else 2e-2
    for shape, seed in ((big, 11), (small, 12)):
        got, ref, err, tile = _both_paths(shape, seed, dtype, _split_tile)
        assert tile.c_split > 1
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), f"{shape.name}: differs from ps_conv2d_fwd_ws"
        assert err <= tol, f"{shape.name}: normalised error {err}"


def test_library_pick_and_unsplit_tiles():
    """t = NULL (the pick among tiles whose planes fit the array) and a tile that needs no scratch at all."""
    for shape, seed in ((wl.CFG1, 1), (wl.ConvShape(2, 32, 9, 9, 64, 1, 1, 1, 0, "static_1x1"), 5)):
        got, ref, err, tile = _both_paths(shape, seed, ps.PS_F32, lambda d: None)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
        assert err <= 1e-4


def test_tile_beyond_the_array_is_refused_and_nothing_runs():
    from gpu_util import DEV
    shape = wl.ConvShape(56, 512, 7, 7, 512, 3, 3, 1, 1, "static_too_big")
    d = ps.ConvDesc.of(shape)
    tiles = [ps.ps_tile_get(d, i) for i in range(ps.ps_tile_count(d))]
    too_big = [t for t in tiles if ps.ps_workspace_bytes(d, t) > ps.PS_STATIC_SCRATCH_BYTES]
    assert too_big, "expected a candidate whose partial planes exceed the static scratch"
    xb = torch.zeros(ps.ps_blocked_in_bytes(d) // 4, device=DEV)
    wb = torch.zeros(ps.ps_blocked_wt_bytes(d) // 4, device=DEV)
    ob = torch.full((ps.ps_blocked_out_bytes(d) // 4,), 7.0, device=DEV)
    with pytest.raises(ps.PsError) as e:
        ps.ps_conv2d_fwd_static(d, too_big[0], xb, wb, ob)
    assert e.value.status == ps.PS_ESCRATCH
    torch.cuda.synchronize()
    assert bool((ob == 7.0).all())
    # the library's own pick stays within the array
    ps.ps_conv2d_fwd_static(d, None, xb, wb, ob)
    torch.cuda.synchronize()
    assert ps.ps_workspace_bytes(d, ps.ps_tile_pick(d, True, ps.PS_STATIC_SCRATCH_BYTES)) <= ps.PS_STATIC_SCRATCH_BYTES
    assert not bool(ob.any())


def test_static_scratch_calls_replay_from_a_captured_graph():
    """What the entry point is for: a chain of two convolutions (a split 3x3, then a 1x1 on its output, no transform in
    between) captured into a HIP graph and replayed.  Capture must find nothing to allocate; every replay, with eager
    work and synchronisations in between, must reproduce the eager result bit for bit."""
    from gpu_util import blocked_inputs, DEV
    s1 = wl.ConvShape(2, 64, 14, 14, 64, 3, 3, 1, 1, "graph_3x3")
    s2 = wl.ConvShape(2, 64, 14, 14, 128, 1, 1, 1, 0, "graph_1x1")
    x, w1 = wl.uniform_pm1(s1, 31)
    _, w2 = wl.uniform_pm1(s2, 32)
    d1, xb, w1b = blocked_inputs(s1, x, w1)
    d2, _, w2b = blocked_inputs(s2, np.zeros((s2.N, s2.C, s2.H, s2.W), np.float32), w2)
    t1 = _split_tile(d1)
    mid = torch.empty(ps.ps_blocked_out_bytes(d1) // 4, device=DEV)      # blocked output of layer 1 = blocked input of layer 2
    out = torch.empty(ps.ps_blocked_out_bytes(d2) // 4, device=DEV)

    def chain():
        ps.ps_conv2d_fwd_static(d1, t1, xb, w1b, mid)
        ps.ps_conv2d_fwd_static(d2, None, mid, w2b, out)

    chain()                                  # eager: also the first call on the device (looks the array's address up)
    torch.cuda.synchronize()
    want_mid, want_out = mid.clone(), out.clone()
    # against the oracle, layer by layer
    y1 = torch.empty((s1.N, s1.K, s1.P, s1.Q), device=DEV)
    ps.ps_blocked_to_nkpq(d1, mid, y1)
    o1, m1 = oracle.conv2d_fwd(s1, x, w1)
    assert oracle.normalised_error(y1.cpu().numpy(), o1, m1) <= 1e-4
    y2 = torch.empty((s2.N, s2.K, s2.P, s2.Q), device=DEV)
    ps.ps_blocked_to_nkpq(d2, out, y2)
    o2, m2 = oracle.conv2d_fwd(s2, y1.cpu().numpy(), w2)
    assert oracle.normalised_error(y2.cpu().numpy(), o2, m2) <= 1e-4

    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            chain()
    for replay in range(3):
        mid.fill_(float("nan"))
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(mid.view(torch.int32), want_mid.view(torch.int32)), f"replay {replay}: first layer differs"
        assert torch.equal(out.view(torch.int32), want_out.view(torch.int32)), f"replay {replay}: second layer differs"
        # eager work between replays, on the same scratch array
        ps.ps_conv2d_fwd_static(d1, t1, xb, w1b, mid)
        torch.cuda.synchronize()

"""The tile model's pick against an exhaustive sweep of the enumerator's candidates (the paper's protocol:
rank n variants analytically, run the top k = 1, compare with the best variant found empirically,
Section 5.2).  Target: the pick is within 10 % of the fastest candidate."""
import pytest

from paper_2002_02145_amd import workloads as wl

pytestmark = pytest.mark.gpu

LAYERS = ["3x3_64_56", "3x3_256_14", "1x1_256to64_56", "1x1_2048to512_7", "1x1_128to512_28"]


@pytest.mark.parametrize("name", LAYERS)
def test_model_pick_within_ten_percent_of_sweep_best_fp32(name):
    import torch
    from paper_2002_02145_amd import autotune, binding as ps
    shape = {l.name: l for l in wl.resnet50_layers()}[name]
    r = autotune.sweep(shape, ps.PS_F32, min_ms=5.0)
    assert r["candidates"] >= 8
    pick_us, best_us = r["pick_us"], r["best_us"]
    if pick_us > 1.10 * best_us:
        # timing noise: measure the two contenders again, longer
        desc = ps.ConvDesc.of(shape)
        sets = autotune._buffers(desc, 4)
        tiles = [ps.Tile(*r["pick"]), ps.Tile(*r["best"])]
        need = max(ps.ps_workspace_bytes(desc, t) for t in tiles)
        ws = torch.empty(max(need, 16) // 4, device="cuda")
        pick_us, best_us = (autotune.time_tile(desc, t, sets, min_ms=40.0, workspace=ws) for t in tiles)
    assert pick_us <= 1.10 * best_us, f"{name}: pick {r['pick']} {pick_us:.1f} us vs best {r['best']} {best_us:.1f} us"
    # sanity of the distribution the paper plots: the worst variant is clearly slower than the best
    assert r["worst_us"] >= best_us

"""The seeded workload module: shapes, reproducibility, and the bf16 input rounding."""
import numpy as np
import pytest

from paper_2002_02145_amd import workloads as wl


def test_shapes_and_flops():
    assert (wl.CFG3B.P, wl.CFG3B.Q) == (14, 14)
    layers = wl.resnet50_layers()
    assert len(layers) == 13
    stem = layers[-1]
    assert (stem.P, stem.Q) == (112, 112)
    assert stem.flops == 2 * 28 * 64 * 112 * 112 * 3 * 49
    assert stem.flops_issued == stem.flops // 3 * 16
    assert wl.CFG2.flops == 2 * 28 * 64 * 56 * 56 * 64 * 9
    assert all(l.K % 16 == 0 for l in layers)
    assert wl.CFG2.algorithmic_bytes(4) == 4 * (28 * 64 * 56 * 56 * 2 + 64 * 64 * 9)


def test_generators_are_seeded():
    a = wl.relu_like(wl.CFG1, 2)
    b = wl.relu_like(wl.CFG1, 2)
    c = wl.relu_like(wl.CFG1, 3)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
    assert not np.array_equal(a[0], c[0])
    x, w = a
    assert x.dtype == np.float32 and x.min() >= 0 and x.max() < 1
    assert abs(w.std() - np.sqrt(2 / (64 * 9))) < 0.1 * np.sqrt(2 / (64 * 9))
    x, w = wl.uniform_pm1(wl.CFG1, 1)
    assert x.min() >= -1 and x.max() < 1 and x.min() < -0.9
    x, w = wl.small_integers(wl.CFG1, 1)
    assert set(np.unique(x)) <= {-2.0, -1.0, 0.0, 1.0, 2.0}


def test_bf16_rounding_matches_torch_and_ties_to_even():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 10.0 ** rng.integers(-20, 20, 4096),
                        np.array([0.0, -0.0, 1.0, np.inf, -np.inf, 3.3895314e38], np.float32)]).astype(np.float32)
    # exact ties: bit patterns xxxx8000 must round to the even neighbour
    ties = np.array([0x3F808000, 0x3F818000, 0xBF808000, 0x3F80FFFF, 0x3F807FFF], np.uint32).view(np.float32)
    a = np.concatenate([a, ties])
    got = wl.round_to_bf16(a)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32))
    assert got.view(np.uint32)[-5] == 0x3F800000 and got.view(np.uint32)[-4] == 0x3F820000
    assert np.all(wl.bf16_bits(got).astype(np.uint32) << 16 == got.view(np.uint32))
    assert np.isnan(wl.round_to_bf16(np.array([np.nan], np.float32)))[0]


def test_random_shapes_are_seeded_and_valid():
    a, b = wl.random_shapes(20, 5), wl.random_shapes(20, 5)
    assert a == b and a != wl.random_shapes(20, 6)
    for s in a:
        assert s.K % 16 == 0 and s.P >= 1 and s.Q >= 1 and 1 <= s.stride <= 3 and 0 <= s.pad <= 3

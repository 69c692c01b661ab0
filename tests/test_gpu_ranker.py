"""GPU parity of the pairwise ranker's tournament (Section 4.2.2 of the paper) against the float64 oracle.

The network's outputs are compared value by value.  Tolerance: single precision, five layers of at most 64 products
each on inputs that sum to one; with weights of unit scale the logits carry an absolute error of a few 1e-6 and the
two-way softmax at most a quarter of that, so 5e-5 leaves an order of magnitude of room.  A win is decided by comparing
an output with theta in single precision; games whose float64 output lies within 1e-4 of theta may fall either way,
so the win count of a variant must lie between its sure wins and its sure-plus-undecided wins, and must equal the
oracle's count when no game of that variant is that close."""
import math

import numpy as np
import pytest
import torch

from oracle import ranker_oracle as ro
from paper_2002_02145_amd import binding as ps
from paper_2002_02145_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
PROB_TOL = 5e-5
MARGIN = 1e-4


def _play(stats: np.ndarray, params: np.ndarray, theta: float, want_probs: bool = True):
    n = stats.shape[0]
    s = torch.from_numpy(np.ascontiguousarray(stats, dtype=np.float32)).to(DEV)
    p = torch.from_numpy(np.ascontiguousarray(params, dtype=np.float32)).to(DEV)
    wins = torch.full((max(n, 1),), -7, dtype=torch.int32, device=DEV)
    probs = torch.full((max(n * n, 1), 2), float("nan"), dtype=torch.float32, device=DEV) if want_probs else None
    ps.ps_ranker_play(s, n, p, theta, wins, probs)
    torch.cuda.synchronize()
    assert torch.equal(s.cpu(), torch.from_numpy(np.ascontiguousarray(stats, dtype=np.float32)))   # inputs untouched
    return wins.cpu().numpy()[:n], (probs.cpu().numpy().reshape(n, n, 2) if want_probs and n else None)


def _check_against_oracle(stats, params, theta):
    n = stats.shape[0]
    wins, probs = _play(stats, params, theta)
    o_wins, o_probs = ro.tournament(stats.astype(np.float64), ro.unpack(params), theta)
    assert np.abs(probs - o_probs).max() <= PROB_TOL
    off = ~np.eye(n, dtype=bool)
    sure = np.zeros(n, dtype=np.int64)
    maybe = np.zeros(n, dtype=np.int64)
    first, second = o_probs[:, :, 0], o_probs[:, :, 1]
    sure += ((first > theta + MARGIN) & off).sum(axis=1) + ((second > theta + MARGIN) & off).sum(axis=0)
    maybe += ((np.abs(first - theta) <= MARGIN) & off).sum(axis=1) + ((np.abs(second - theta) <= MARGIN) & off).sum(axis=0)
    assert np.all(wins >= sure) and np.all(wins <= sure + maybe)
    clear = maybe == 0
    assert np.array_equal(wins[clear], o_wins[clear])
    return wins, o_wins, int((~clear).sum())


@pytest.mark.parametrize("n,seed,theta,scale,dups", [
    (1, 11, 0.6, 3.0, 0), (2, 12, 0.6, 3.0, 0), (7, 13, 0.5, 3.0, 0), (64, 14, 0.6, 4.0, 4),
    (257, 15, 0.6, 3.0, 0), (300, 16, 0.55, 5.0, 20),
])
def test_tournament_matches_the_oracle(n, seed, theta, scale, dups):
    stats = wl.ranker_stats(n, seed, duplicates=dups)
    params = wl.ranker_params(seed + 100, scale)
    wins, o_wins, undecided = _check_against_oracle(stats, params, theta)
    assert undecided <= max(1, n // 10)
    if n >= 64:
        assert o_wins.max() > 0 and len(set(o_wins.tolist())) > 3      # the case decides something


def test_empty_and_all_zero_statistics():
    params = wl.ranker_params(5, 3.0)
    wins, probs = _play(np.zeros((0, 4), dtype=np.float32), params, 0.6)
    assert wins.size == 0
    _check_against_oracle(np.zeros((5, 4), dtype=np.float32), params, 0.6)   # nothing to divide by: inputs stay zero


def _zeros():
    return [(np.zeros((a, b)), np.zeros(b)) for a, b in zip(ro.WIDTHS[:-1], ro.WIDTHS[1:])]


def test_hand_set_comparator_gives_the_sorted_order():
    # the network of the oracle's pins: the smaller memory size wins once the sizes differ enough (relative
    # difference above 0.14); sizes in a geometric sequence of ratio 1.5 differ by 0.2 or more
    p = _zeros()
    p[0][0][7, 0], p[0][0][3, 0] = 1.0, -1.0
    p[0][0][3, 1], p[0][0][7, 1] = 1.0, -1.0
    p[1][0][0, 0] = p[1][0][1, 1] = 1.0
    p[2][0][0, 0] = p[2][0][1, 1] = 1.0
    p[3][0][0, 0] = p[3][0][1, 1] = 1.0
    p[4][0][0, 0] = p[4][0][1, 1] = 3.0 * math.log(3.0)
    params = ro.pack(p).astype(np.float32)
    n = 150
    order = np.random.default_rng(3).permutation(n)
    stats = np.zeros((n, 4), dtype=np.float32)
    stats[:, 3] = (1.5 ** order).astype(np.float32)
    wins, _ = _play(stats, params, 0.6)
    assert np.array_equal(wins, 2 * (n - 1 - order))        # two seatings against every larger size


def test_largest_tournament_counts_every_game():
    # all weights zero and a last bias of (ln 4, 0): the first seat wins every game, n - 1 wins each
    p = _zeros()
    p[4][1][0] = math.log(4.0)
    n = ps.PS_RANKER_MAX_VARIANTS
    wins, _ = _play(wl.ranker_stats(n, 9), ro.pack(p).astype(np.float32), 0.6, want_probs=False)
    assert np.array_equal(wins, np.full(n, n - 1))


def test_two_runs_agree_bit_for_bit():
    stats, params = wl.ranker_stats(200, 21), wl.ranker_params(22, 4.0)
    a = _play(stats, params, 0.6)
    b = _play(stats, params, 0.6)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


@pytest.mark.parametrize("kind", [ps.PS_RANKER_WORKING_SETS, ps.PS_RANKER_LEVEL_TIMES])
@pytest.mark.parametrize("layer", [0, 5, 10])
def test_ranking_of_a_layers_tiles_matches_the_oracle(kind, layer):
    """ps_tile_rank_dnn end to end: statistics of every candidate, tournament, order by wins."""
    from paper_2002_02145_amd import ranker
    L = wl.resnet50_layers()[layer]
    d = ps.ConvDesc.of(L)
    params = ranker.load_params(kind, "f32")
    tiles, stats = ranker.tile_stats(d, kind, workspace_bytes=1 << 30)
    n = len(tiles)
    pd = torch.from_numpy(params).to(DEV)
    scratch = torch.empty(ps.ps_tile_rank_dnn_scratch_bytes(d), dtype=torch.uint8, device=DEV)
    got = ps.ps_tile_rank_dnn(d, 1 << 30, kind, pd, ro.THETA, scratch, scratch.numel(), n)
    assert [t.as_tuple() for t, _ in got] != [] and len(got) == n
    wins_by_tile = {t.as_tuple(): w for t, w in got}
    wins = np.array([wins_by_tile[t.as_tuple()] for t in tiles])
    # the same counts as the tournament entry point on the same statistics, and as the oracle
    direct, o_wins, _ = _check_against_oracle(stats, params, ro.THETA)
    assert np.array_equal(wins, direct)
    # order: most wins first, equal counts in enumeration order
    assert [t.as_tuple() for t, _ in got] == [tiles[i].as_tuple() for i in ro.ranking(wins)]
    top3 = ps.ps_tile_rank_dnn(d, 1 << 30, kind, pd, ro.THETA, scratch, scratch.numel(), 3)
    assert [(t.as_tuple(), w) for t, w in top3] == [(t.as_tuple(), w) for t, w in got[:3]]


def test_tournament_replays_correctly_from_a_captured_graph():
    """The call enqueues two kernels and no memset; captured once and replayed on changing statistics it must give
    what the eager call gives, on every replay."""
    n = 200
    params = torch.from_numpy(wl.ranker_params(31, 4.0)).to(DEV)
    stats = torch.from_numpy(wl.ranker_stats(n, 32)).to(DEV)
    wins = torch.zeros(n, dtype=torch.int32, device=DEV)
    eager = torch.zeros(n, dtype=torch.int32, device=DEV)
    ps.ps_ranker_play(stats, n, params, 0.6, wins)            # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ps.ps_ranker_play(stats, n, params, 0.6, wins)
    for replay in range(4):
        stats.copy_(torch.from_numpy(wl.ranker_stats(n, 40 + replay)).to(DEV))
        wins.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        ps.ps_ranker_play(stats, n, params, 0.6, eager)
        torch.cuda.synchronize()
        assert torch.equal(wins, eager), f"replay {replay}"
        assert int(eager.max()) > 0


def test_ranking_respects_the_workspace_limit_and_runs_in_bf16():
    """With no workspace only unsplit tiles may be ranked; the statistics of both kinds exist for 16-bit descriptors."""
    from paper_2002_02145_amd import ranker
    L = wl.resnet50_layers()[3]                               # 3x3, 512 channels, 7x7: many split candidates
    d = ps.ConvDesc.of(L, ps.PS_BF16)
    for kind in (ps.PS_RANKER_LEVEL_TIMES, ps.PS_RANKER_WORKING_SETS):
        params = torch.from_numpy(ranker.load_params(kind, "bf16")).to(DEV)
        scratch = torch.empty(ps.ps_tile_rank_dnn_scratch_bytes(d), dtype=torch.uint8, device=DEV)
        everything = ps.ps_tile_rank_dnn(d, 1 << 40, kind, params, ro.THETA, scratch, scratch.numel(), 10000)
        unsplit = ps.ps_tile_rank_dnn(d, 0, kind, params, ro.THETA, scratch, scratch.numel(), 10000)
        assert any(t.c_split > 1 for t, _ in everything)
        assert unsplit and all(t.c_split == 1 for t, _ in unsplit) and len(unsplit) < len(everything)
        tiles, stats = ranker.tile_stats(d, kind, workspace_bytes=0)
        assert sorted(t.as_tuple() for t, _ in unsplit) == sorted(t.as_tuple() for t in tiles)
        o_wins, _ = ro.tournament(stats.astype(np.float64), ro.unpack(params.cpu().numpy()), ro.THETA)
        got = {t.as_tuple(): w for t, w in unsplit}
        close = sum(abs(got[t.as_tuple()] - int(w)) for t, w in zip(tiles, o_wins))
        assert close <= max(2, len(tiles) // 20)              # games within rounding of the threshold may fall either way

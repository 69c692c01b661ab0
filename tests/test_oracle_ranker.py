"""Pins of the float64 pairwise-ranking oracle (Section 4.2.2 of the paper): closed forms worked out by hand for
networks whose weights are set by hand, the normalisation on a numeric example, and a cross-check of the layer
arithmetic against torch's float64 library routines."""
import math

import numpy as np
import pytest

from oracle import ranker_oracle as ro


def _zeros():
    return [(np.zeros((a, b)), np.zeros(b)) for a, b in zip(ro.WIDTHS[:-1], ro.WIDTHS[1:])]


def _memory_comparator(gain: float, through_negative_softsign: bool = False):
    """Unit 0 carries relu(x7 - x3), unit 1 carries relu(x3 - x7) through all hidden layers (x3, x7: the memory
    statistics of the first and second variant after normalisation); the outputs are gain times the two."""
    p = _zeros()
    p[0][0][7, 0], p[0][0][3, 0] = 1.0, -1.0
    p[0][0][3, 1], p[0][0][7, 1] = 1.0, -1.0
    p[1][0][0, 0] = p[1][0][1, 1] = 1.0
    s = -1.0 if through_negative_softsign else 1.0
    p[2][0][0, 0] = p[2][0][1, 1] = s      # softsign sees -h when s = -1 ...
    p[3][0][0, 0] = p[3][0][1, 1] = s      # ... and the next layer flips the sign back before its relu
    p[4][0][0, 0] = p[4][0][1, 1] = gain
    return p


def test_parameter_count_and_layout():
    assert ro.n_params() == 8 * 64 + 64 + 64 * 32 + 32 + 32 * 16 + 16 + 16 * 8 + 8 + 8 * 2 + 2 == 3338
    flat = np.arange(ro.n_params(), dtype=np.float64)
    params = ro.unpack(flat)
    assert [W.shape for W, _ in params] == [(8, 64), (64, 32), (32, 16), (16, 8), (8, 2)]
    assert params[0][0][1, 0] == 64.0                       # row-major (inputs, units): second input's first weight
    assert params[0][1][0] == 8 * 64                        # the bias follows its matrix
    assert params[1][0][0, 0] == 8 * 64 + 64
    assert np.array_equal(ro.pack(params), flat)


def test_pair_input_divides_by_the_common_sum():
    x = ro.pair_input((1, 2, 3, 4), (5, 6, 7, 12))          # sum = 40
    assert np.allclose(x, [0.025, 0.05, 0.075, 0.1, 0.125, 0.15, 0.175, 0.3], rtol=0, atol=1e-15)
    assert abs(x.sum() - 1.0) < 1e-15
    # scaling both variants by the same factor changes nothing; scaling one of them does
    assert np.allclose(ro.pair_input((10, 20, 30, 40), (50, 60, 70, 120)), x, rtol=0, atol=1e-15)
    assert not np.allclose(ro.pair_input((2, 4, 6, 8), (5, 6, 7, 12)), x)
    assert np.array_equal(ro.pair_input((0, 0, 0, 0), (0, 0, 0, 0)), np.zeros(8))


@pytest.mark.parametrize("negative_path", [False, True])
def test_forward_closed_form_of_a_hand_set_network(negative_path):
    # memory sizes 1 and 3: x3 = 1/4, x7 = 3/4; unit 0 = 1/2, softsign(1/2) = 1/3 (softsign(-1/2) = -1/3 on the
    # negative path); outputs (gain / 3, 0); with gain = 3 ln 3 the softmax is (3, 1) / 4
    params = _memory_comparator(3.0 * math.log(3.0), negative_path)
    p = ro.forward(ro.pair_input((0, 0, 0, 1), (0, 0, 0, 3)), params)
    assert np.allclose(p, [0.75, 0.25], rtol=0, atol=1e-14)
    p = ro.forward(ro.pair_input((0, 0, 0, 3), (0, 0, 0, 1)), params)
    assert np.allclose(p, [0.25, 0.75], rtol=0, atol=1e-14)
    assert ro.play((0, 0, 0, 1), (0, 0, 0, 3), params) == 1
    assert ro.play((0, 0, 0, 3), (0, 0, 0, 1), params) == 2


def test_biases_reach_the_output():
    # all weights zero, last bias (ln 4, 0): softmax = (0.8, 0.2) whatever the input
    params = _zeros()
    params[4][1][0] = math.log(4.0)
    assert np.allclose(ro.forward(np.full(8, 0.125), params), [0.8, 0.2], rtol=0, atol=1e-15)
    # a hidden bias travels the same way: unit 5 of the last hidden layer gets bias 2, the first output reads it
    params = _zeros()
    params[3][1][5] = 2.0
    params[4][0][5, 0] = math.log(3.0) / 2.0                # z = (ln 3, 0): softmax (0.75, 0.25)
    assert np.allclose(ro.forward(np.zeros(8), params), [0.75, 0.25], rtol=0, atol=1e-15)
    # first seat always wins: n - 1 wins for every variant
    params = _zeros()
    params[4][1][0] = math.log(4.0)
    wins, _ = ro.tournament(np.arange(20.0).reshape(5, 4) + 1.0, params)
    assert list(wins) == [4] * 5


def test_threshold_decides_win_or_draw():
    params = _zeros()
    params[4][1][0] = math.log(1.4)                         # softmax = (1.4, 1) / 2.4 = (0.5833, 0.4167): below 0.6
    assert ro.play((1, 1, 1, 1), (1, 1, 1, 1), params) == 0
    assert ro.play((1, 1, 1, 1), (1, 1, 1, 1), params, theta=0.58) == 1
    params[4][1][0] = -math.log(1.6)                        # (1, 1.6) / 2.6 = (0.3846, 0.6154)
    assert ro.play((1, 1, 1, 1), (1, 1, 1, 1), params) == 2
    assert ro.play((1, 1, 1, 1), (1, 1, 1, 1), params, theta=0.62) == 0


def test_tournament_counts_both_seatings_and_draws():
    # With gain 3 ln 3 the smaller memory size wins iff (m_big - m_small) / (m_big + m_small) = a satisfies
    # 3 ln 3 * a / (1 + a) > ln 1.5, i.e. a > 0.1403.  Sizes 1 and 1.02 draw (a = 0.0099); every other pair is
    # decided, and is decided the same way in both seatings, so the smaller size collects two wins per pair.
    mem = [5.0, 1.0, 3.0, 1.02, 9.0]
    stats = np.array([[0.0, 0.0, 0.0, m] for m in mem])
    wins, probs = ro.tournament(stats, _memory_comparator(3.0 * math.log(3.0)))
    assert list(wins) == [2, 6, 4, 6, 0]
    assert ro.ranking(wins) == [1, 3, 2, 0, 4]
    # game (0, 1): sizes 5 and 1, a = 2/3, softsign 2/5: the second unit gets exp(1.2 ln 3) against 1
    e = 3.0 ** 1.2
    assert np.allclose(probs[0, 1], [1.0 / (1.0 + e), e / (1.0 + e)], rtol=0, atol=1e-14)
    assert np.allclose(probs[1, 0], [e / (1.0 + e), 1.0 / (1.0 + e)], rtol=0, atol=1e-14)
    assert np.array_equal(probs[2, 2], [0.0, 0.0])
    assert np.allclose(probs.sum(axis=2)[~np.eye(5, dtype=bool)], 1.0, rtol=0, atol=1e-15)


def test_ranking_is_stable_for_equal_wins():
    assert ro.ranking([3, 5, 3, 0, 5]) == [1, 4, 0, 2, 3]


def test_layers_agree_with_library_routines():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = np.random.default_rng(7)
    flat = rng.normal(0.0, 0.5, ro.n_params())
    params = ro.unpack(flat)
    for _ in range(5):
        v1, v2 = rng.uniform(0, 1e6, 4), rng.uniform(0, 1e6, 4)
        x = torch.tensor(np.concatenate([v1, v2]) / (v1.sum() + v2.sum()), dtype=torch.float64)
        h = x
        acts = (F.relu, F.relu, F.softsign, F.relu)
        for (W, b), act in zip(params[:4], acts):
            h = act(F.linear(h, torch.tensor(W).T.contiguous(), torch.tensor(b)))
        W, b = params[4]
        want = F.softmax(F.linear(h, torch.tensor(W).T.contiguous(), torch.tensor(b)), dim=0).numpy()
        got = ro.forward(ro.pair_input(v1, v2), params)
        assert np.allclose(got, want, rtol=0, atol=1e-13)

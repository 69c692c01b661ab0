"""Pairwise neural ranking of code variants, by its definition in float64.  TEST INFRASTRUCTURE ONLY.

Follows Section 4.2.2 of the paper ("DNN-based ranking algorithm") step by step:

  * pair_input   -- a variant is described by four working-set sizes (what Algorithm 2 assigns to L1, L2, L3
    and memory).  The eight numbers of two variants are divided by their common sum, first variant first.
  * forward      -- fully connected layers of 64, 32, 16 and 8 units with relu, relu, softsign, relu, then
    two output units through softmax.
  * play         -- an output above the threshold theta (0.6 in the paper) counts as fired; the first unit firing
    makes the first variant the winner, the second unit the second variant, neither a draw.
  * tournament   -- every variant plays every other one; wins are counted.
  * ranking      -- more wins rank higher.

Readings where the paper leaves room:
  * "Plays against every other variant": every ordered pair (i, j), i != j, is one game with variant i presented
    first, so a pair meets twice, once in each seating.  The network is not symmetric in its two halves, and with
    both seatings the tally does not depend on the order in which variants are listed.
  * Two statistics vectors that are all zero have no common sum to divide by: their input is all zeros.
  * Equal win counts keep the order in which the variants were listed.
  * A layer computes act(x W + b) with W of shape (inputs, units); the softsign is x / (1 + |x|); the softmax
    is taken over the two output units.

Parameters are a list of five (W, b) pairs.  ``unpack`` reads them from the flat float array the GPU library
takes (for each layer W row-major as (inputs, units), then b), which is an interface both sides have to agree on.
"""
from __future__ import annotations

import numpy as np

STATS = 4                                  # working-set sizes per variant: L1, L2, L3, memory
WIDTHS = (2 * STATS, 64, 32, 16, 8, 2)     # input, four hidden layers, output
THETA = 0.6


def n_params() -> int:
    return sum(a * b + b for a, b in zip(WIDTHS[:-1], WIDTHS[1:]))


def unpack(flat) -> list:
    flat = np.asarray(flat, dtype=np.float64).ravel()
    if flat.size != n_params():
        raise ValueError(f"expected {n_params()} parameters, got {flat.size}")
    out, at = [], 0
    for a, b in zip(WIDTHS[:-1], WIDTHS[1:]):
        W = flat[at:at + a * b].reshape(a, b)
        at += a * b
        out.append((W, flat[at:at + b]))
        at += b
    return out


def pack(params) -> np.ndarray:
    return np.concatenate([np.concatenate([np.asarray(W, dtype=np.float64).ravel(),
                                           np.asarray(b, dtype=np.float64).ravel()]) for W, b in params])


def pair_input(v1, v2) -> np.ndarray:
    x = np.concatenate([np.asarray(v1, dtype=np.float64), np.asarray(v2, dtype=np.float64)])
    if x.size != 2 * STATS:
        raise ValueError("each variant has four statistics")
    total = x.sum()
    return x / total if total != 0.0 else np.zeros_like(x)


def _relu(x):
    return np.maximum(x, 0.0)


def _softsign(x):
    return x / (1.0 + np.abs(x))


_ACT = (_relu, _relu, _softsign, _relu)


def forward(x, params) -> np.ndarray:
    """The two softmax outputs for one input vector."""
    h = np.asarray(x, dtype=np.float64)
    for (W, b), act in zip(params[:4], _ACT):
        h = act(h @ W + b)
    W, b = params[4]
    z = h @ W + b
    e = np.exp(z - z.max())
    return e / e.sum()


def play(v1, v2, params, theta: float = THETA) -> int:
    """1 if the first variant wins, 2 if the second wins, 0 for a draw."""
    p = forward(pair_input(v1, v2), params)
    if p[0] > theta:
        return 1
    if p[1] > theta:
        return 2
    return 0


def tournament(stats, params, theta: float = THETA):
    """wins[i] over all games, and the (n, n, 2) array of softmax outputs (the diagonal is unused and zero)."""
    stats = np.asarray(stats, dtype=np.float64)
    n = stats.shape[0]
    wins = np.zeros(n, dtype=np.int64)
    probs = np.zeros((n, n, 2))
    for i in range(n):
        for j in range(n):
            if i == j:
                continue
            p = forward(pair_input(stats[i], stats[j]), params)
            probs[i, j] = p
            if p[0] > theta:
                wins[i] += 1
            elif p[1] > theta:
                wins[j] += 1
    return wins, probs


def ranking(wins) -> list:
    """Variant indices, most wins first; equal counts in listing order."""
    wins = list(wins)
    return sorted(range(len(wins)), key=lambda i: (-wins[i], i))

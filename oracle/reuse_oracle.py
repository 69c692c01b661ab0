"""Working-set analysis and cost ranking of a loop nest, by brute force.  TEST INFRASTRUCTURE ONLY.

Follows Section 4 of the paper for perfectly nested rectangular loops with one statement:

  * working_set_sizes  -- Algorithm 1 (Section 4.1): for every dependence (a pair of references to the same
    array that touch the same element in two different iterations), take the lexicographically first source
    iteration, its first and its last target iteration, and count the distinct array elements read or written
    by all iterations from the source up to and including that target: WS_min and WS_max.
  * assign_to_caches   -- Algorithm 2 (Section 4.2): working sets sorted ascending; each goes to the fastest
    cache whose accumulated working-set size still admits it; the rest is served from memory.
  * cost               -- Eq. 1 (Section 4.2.1): sum over levels of WS^{L_i} * lat^{L_i} / bw^{L_i}, plus the
    memory term.

Everything is enumerated: iterations are tuples walked in lexicographic order (the schedule of the written
loop nest), dependences are found by comparing accessed elements, working sets are Python sets.  Only small
nests are feasible, which is all the tests need.

Readings where the paper leaves room:
  * WS_all is a set (it is initialised to the empty set and sizes are added to it), so equal sizes coming from
    different dependences appear once.
  * A dependence between two references needs two different iterations (source strictly before target); the
    read and the write of one statement instance are not a reuse across iterations.
  * "All dependences" = every ordered pair of references to the same array (read/read, write/read, read/write,
    write/write), the same reference paired with itself included.
  * Sizes are counted in array elements, each weighted by the element size given for its array (1 by default).
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass
from typing import Sequence


@dataclass(frozen=True)
class Ref:
    """array[ sum_l coef[d][l] * iter_l + offset[d]  for each dimension d ]"""
    array: int
    coef: tuple          # one tuple of per-loop coefficients per array dimension
    offset: tuple        # one constant per array dimension
    is_write: bool = False

    def element(self, it):
        return (self.array,) + tuple(sum(c * i for c, i in zip(row, it)) + o for row, o in zip(self.coef, self.offset))


def iterations(extents: Sequence[int]):
    """The iteration space in schedule (lexicographic) order, outermost loop first."""
    return itertools.product(*[range(e) for e in extents])


def _touched(refs, its, weight):
    seen = set()
    for it in its:
        for r in refs:
            seen.add(r.element(it))
    return sum(weight.get(e[0], 1) for e in seen)


def working_set_sizes(extents: Sequence[int], refs: Sequence[Ref], weight: dict | None = None):
    """Algorithm 1.  Returns the list of (src_ref, tgt_ref, WS_min, WS_max) over all dependences that exist."""
    weight = weight or {}
    space = list(iterations(extents))
    out = []
    for a, ra in enumerate(refs):
        for b, rb in enumerate(refs):
            if ra.array != rb.array:
                continue
            # the dependence relation d: source iteration -> later iterations touching the same element
            source = None
            targets = []
            for si, s in enumerate(space):                      # lexmin of dom d
                el = ra.element(s)
                targets = [t for t in space[si + 1:] if rb.element(t) == el]
                if targets:
                    source = si
                    break
            if source is None:
                continue
            t_min, t_max = targets[0], targets[-1]              # lexmin / lexmax of d(source)
            i_min = space.index(t_min)
            i_max = space.index(t_max)
            ws_min = _touched(refs, space[source:i_min + 1], weight)   # (I <<= target) - (I << source)
            ws_max = _touched(refs, space[source:i_max + 1], weight)
            out.append((a, b, ws_min, ws_max))
    return out


def ws_all(extents, refs, weight=None):
    """WS_all of Algorithm 1: the set of all WS_min and WS_max."""
    s = set()
    for _, _, lo, hi in working_set_sizes(extents, refs, weight):
        s.add(lo)
        s.add(hi)
    return s


def assign_to_caches(ws, cache_sizes: Sequence[int]):
    """Algorithm 2.  Returns ([WS^{L_1}, ..., WS^{L_n}], WS^{mem})."""
    level = [0] * len(cache_sizes)
    mem = 0
    for w in sorted(ws):
        for i, size in enumerate(cache_sizes):
            if w + level[i] <= size:
                level[i] += w
                break
        else:
            mem += w
    return level, mem


def cost(level_ws: Sequence[int], mem_ws: int, lat: Sequence[float], bw: Sequence[float]):
    """Eq. 1; lat and bw carry one entry per cache level followed by the memory's."""
    n = len(level_ws)
    return sum(level_ws[i] * lat[i] / bw[i] for i in range(n)) + mem_ws * lat[n] / bw[n]


def matmul_refs():
    """C[i][j] += A[i][k] * B[k][j] with loops (i, j, k): the running example of Section 3."""
    return [Ref(0, ((1, 0, 0), (0, 1, 0)), (0, 0), False),   # C read
            Ref(0, ((1, 0, 0), (0, 1, 0)), (0, 0), True),    # C write
            Ref(1, ((1, 0, 0), (0, 0, 1)), (0, 0), False),   # A[i][k]
            Ref(2, ((0, 0, 1), (0, 1, 0)), (0, 0), False)]   # B[k][j]

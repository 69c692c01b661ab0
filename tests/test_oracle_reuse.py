"""Pins of the brute-force reuse-analysis oracle (Section 4 of the paper: Algorithm 1, Algorithm 2, Eq. 1): the
paper's worked example, hand-derived closed forms and small hand examples."""
import os
import pytest

from oracle import reuse_oracle as ro

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    rows = []
    for line in open(os.path.join(HERE, "golden", "reuse_matmul_worked_example.txt")):
        if line.strip() and not line.startswith("#"):
            rows.append(tuple(int(v) for v in line.split()))
    return rows


def _dep(deps, a, b):
    (hit,) = [d for d in deps if d[0] == a and d[1] == b]
    return hit[2], hit[3]


@pytest.mark.parametrize("M,N,K,ws_min,ws_max", _golden())
def test_oracle_reproduces_the_papers_worked_example(M, N, K, ws_min, ws_max):
    deps = ro.working_set_sizes((M, N, K), ro.matmul_refs())
    assert _dep(deps, 2, 2) == (ws_min, ws_max)          # A[i][k] reused along j


@pytest.mark.parametrize("M,N,K", [(2, 3, 4), (3, 2, 5), (4, 4, 3)])
def test_oracle_other_matmul_dependences_closed_forms(M, N, K):
    """Hand-derived: C[i][j] is reused along k from (0,0,0) to (0,0,1) / (0,0,K-1); B[k][j] along i from (0,0,0) to
    (1,0,0) / (M-1,0,0)."""
    deps = ro.working_set_sizes((M, N, K), ro.matmul_refs())
    for a in (0, 1):
        for b in (0, 1):                                  # read/read, read/write, write/read, write/write on C
            assert _dep(deps, a, b) == (5, 2 * K + 1)
    assert _dep(deps, 3, 3) == (K * N + (K + 1) + (N + 1), ((M - 1) * K + 1) + K * N + ((M - 1) * N + 1))
    assert len(deps) == 6


def test_oracle_no_reuse_no_dependence():
    # a[i] = b[i]: every element is touched once
    refs = [ro.Ref(0, ((1,),), (0,), True), ro.Ref(1, ((1,),), (0,), False)]
    assert ro.working_set_sizes((8,), refs) == []
    # stencil b[i] + b[i+1]: element i+1 read at iteration i (second ref) is read again at i+1 (first ref)
    refs = [ro.Ref(0, ((1,),), (0,), False), ro.Ref(0, ((1,),), (1,), False)]
    deps = ro.working_set_sizes((8,), refs)
    assert deps == [(1, 0, 3, 3)]                         # iterations 0 and 1 touch b[0], b[1], b[2]


def test_oracle_element_weights():
    deps = ro.working_set_sizes((2, 3, 4), ro.matmul_refs(), weight={0: 4, 1: 2, 2: 1})
    # d2: K elements of A (x2), K+1 of B (x1), 2 of C (x4)
    assert _dep(deps, 2, 2)[0] == 2 * 4 + 5 + 8


def test_oracle_algorithm_2_hand_example():
    assert ro.assign_to_caches([40, 4, 16, 8], [10, 30]) == ([4, 24], 40)
    assert ro.assign_to_caches([], [10]) == ([0], 0)
    assert ro.assign_to_caches([5, 5], []) == ([], 10)
    # cumulative rule: 6 fits L1 alone but not next to the 5 already there
    assert ro.assign_to_caches([5, 6], [10, 100]) == ([5, 6], 0)


def test_oracle_eq1_by_hand():
    assert ro.cost([4, 24], 40, lat=[1.0, 10.0, 100.0], bw=[2.0, 5.0, 10.0]) == pytest.approx(4 * 0.5 + 24 * 2.0 + 40 * 10.0)

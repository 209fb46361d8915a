"""Pins of the reuse-analysis oracle: the paper's printed closed forms and hand-worked cases."""
import os

import pytest

from oracle import reuse

GOLD = os.path.join(os.path.dirname(__file__), "golden", "matmul_d2_working_sets.txt")


def gold_rows():
    rows = []
    for line in open(GOLD):
        if line.strip() and not line.startswith("#"):
            rows.append(tuple(int(v) for v in line.split()))
    return rows


def dep_of(deps, array_index):
    """The merged dependence whose references are (array_index, array_index)."""
    for d in deps:
        if (array_index, array_index) in d["refs"]:
            return d
    raise AssertionError("dependence not found")


@pytest.mark.parametrize("M,N,K,ws_min,ws_max", gold_rows())
def test_matmul_d2_matches_printed_closed_forms(M, N, K, ws_min, ws_max):
    assert ws_min == 2 * K + 3 and ws_max == N * K + N + 1       # the file holds the paper's formulas
    loops, refs = reuse.matmul_nest(M, N, K)
    d2 = dep_of(reuse.working_sets(loops, refs), 1)              # reference 1 is A[i][k]
    assert d2["source"] == (0, 0, 0)
    assert d2["min_target"] == (0, 1, 0) and d2["max_target"] == (0, N - 1, 0)
    want = [ws_min] if N == 2 else [ws_min, ws_max]
    assert d2["ws"] == want


def test_matmul_has_the_three_dependences_of_the_paper():
    loops, refs = reuse.matmul_nest(3, 3, 3)
    deps = reuse.working_sets(loops, refs)
    assert len(deps) == 3
    d1, d3 = dep_of(deps, 0), dep_of(deps, 2)
    # d1: C[i][j] reused along k: between k=0 and k=1 two iterations touch C[0][0], A[0][0..1], B[0..1][0]
    assert d1["min_target"] == (0, 0, 1) and d1["ws"][0] == 5
    # d1 up to the last k: C[0][0], A[0][0..2], B[0..2][0]
    assert d1["max_target"] == (0, 0, 2) and d1["ws"][1] == 7
    # d3: B[k][j] reused along i: from (0,0,0) to (1,0,0) the whole first row block is swept:
    # C[0][0..2] + C[1][0], A[0][0..2] + A[1][0], all of B
    assert d3["min_target"] == (1, 0, 0) and d3["ws"][0] == 4 + 4 + 9


def test_parallel_dependence_uses_whole_parallel_footprint():
    # i parallel: d3 (B reused across i) spans parallel iterations -> footprint of the whole nest
    M, N, K = 2, 3, 2
    loops, refs = reuse.matmul_nest(M, N, K)
    deps = reuse.working_sets(loops, refs, parallel=("i",))
    d3 = dep_of(deps, 2)
    assert d3["parallel"] and d3["ws"] == [M * N + M * K + K * N]
    # j parallel (inner): iterators outside j (i) are held fixed: C[0][*], A[0][*], all of B
    deps = reuse.working_sets(loops, refs, parallel=("j",))
    d2 = dep_of(deps, 1)
    assert d2["parallel"] and d2["ws"] == [N + K + K * N]
    assert not dep_of(deps, 0)["parallel"]       # reuse of C along k stays inside one j iteration


def test_bucket_hand_example():
    # capacities 10 and 100: 3,4 -> L1 (7); 5 does not fit beside them -> L2; 50 -> L2 (55);
    # 60 fits neither -> memory; 200 -> memory
    levels, mem = reuse.bucket_working_sets([50, 3, 200, 5, 60, 4], [10, 100])
    assert levels == [7, 55] and mem == 260
    assert reuse.bucket_working_sets([], [10]) == ([0], 0)
    assert reuse.bucket_working_sets([10, 10], [10, 10]) == ([10, 10], 0)   # exact fit counts


def test_cost_equation():
    assert reuse.cost([7, 55], 260, [1.0, 4.0], 100.0) == 7 + 220 + 26000
    # a variant whose reuse moves from memory into a cache gets cheaper (lower cost = better rank)
    slow = reuse.cost(*reuse.bucket_working_sets([8, 80, 800], [16, 128]), [1.0, 4.0], 100.0)
    fast = reuse.cost(*reuse.bucket_working_sets([8, 80, 100], [16, 128]), [1.0, 4.0], 100.0)
    assert fast < slow

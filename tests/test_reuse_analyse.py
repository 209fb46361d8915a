"""The library's working-set analyser for small loop nests against the oracle's and against the
closed forms the paper prints for its matmul example (no GPU needed)."""
import ctypes

import pytest

from oracle import reuse
import paper_2006_02230_amd as P


def oracle_refs(refs):
    """The same affine references as Python functions of the iteration tuple."""
    out = []
    for array, coef, offset in refs:
        def f(it, coef=coef, offset=offset):
            return tuple(o + sum(c * v for c, v in zip(row, it)) for row, o in zip(coef, offset))
        out.append((array, f))
    return out


def compare(extents, refs, parallel=None):
    names = ["l%d" % i for i in range(len(extents))]
    par_names = [] if parallel is None else [n for n, f in zip(names, parallel) if f]
    want = reuse.working_sets(list(zip(names, extents)), oracle_refs(refs), par_names)
    got = P.reuse_analyse(extents, refs, parallel)
    assert len(got) == len(want)
    for g, w in zip(got, want):                      # both list dependences in order of first reference pair
        assert (g["src_ref"], g["tgt_ref"]) == w["refs"][0] and g["n_pairs"] == len(w["refs"])
        assert g["parallel"] == w["parallel"] and g["ws"] == w["ws"] and g["source"] == w["source"]
        assert g["min_target"] == w["min_target"] and g["max_target"] == w["max_target"]
    return got


def matmul(M, N, K):
    # for i, j, k: C[i][j] += A[i][k] * B[k][j]
    return [M, N, K], [(0, [[1, 0, 0], [0, 1, 0]], [0, 0]), (1, [[1, 0, 0], [0, 0, 1]], [0, 0]),
                       (2, [[0, 0, 1], [0, 1, 0]], [0, 0])]


@pytest.mark.parametrize("M,N,K", [(2, 2, 2), (3, 4, 3), (2, 5, 4), (4, 3, 6)])
def test_matmul_closed_forms_of_the_paper(M, N, K):
    extents, refs = matmul(M, N, K)
    deps = compare(extents, refs)
    assert len(deps) == 3                                           # d1 (C), d2 (A), d3 (B)
    d2 = [d for d in deps if d["src_ref"] == 1][0]
    assert d2["source"] == (0, 0, 0) and d2["min_target"] == (0, 1, 0) and d2["max_target"] == (0, N - 1, 0)
    assert d2["ws"] == ([2 * K + 3] if N == 2 else [2 * K + 3, N * K + N + 1])


def test_parallel_loops_take_the_other_branch():
    extents, refs = matmul(3, 4, 2)
    seq = compare(extents, refs)
    par = compare(extents, refs, parallel=[1, 0, 0])               # i parallel: B is reused across it
    assert [d["parallel"] for d in par] == [False, False, True]
    d3 = par[2]
    assert d3["ws"] == [3 * 4 + 3 * 2 + 2 * 4]                      # the whole nest: C, A and B
    assert seq[0]["ws"] == par[0]["ws"]
    both = compare(extents, refs, parallel=[1, 1, 0])
    assert [d["parallel"] for d in both] == [False, True, True]
    assert both[1]["ws"] == [4 + 2 + 2 * 4]                         # one i: a row of C, a row of A, all of B


def test_tiled_and_strided_nests_match_the_oracle():
    # two column tiles of a GEMM: for tn, k, i, j: C[i][2 tn + j] += A[i][k] * B[k][2 tn + j]
    refs = [(0, [[0, 0, 1, 0], [2, 0, 0, 1]], [0, 0]), (1, [[0, 0, 1, 0], [0, 1, 0, 0]], [0, 0]),
            (2, [[0, 1, 0, 0], [2, 0, 0, 1]], [0, 0])]
    compare([2, 3, 2, 2], refs)
    compare([2, 3, 2, 2], refs, parallel=[1, 0, 0, 0])
    # a 1-D convolution with stride 2 and an offset: for p, r: out[p] += in[2 p + r - 1] * w[r]
    refs = [(0, [[1, 0]], [0]), (1, [[2, 1]], [-1]), (2, [[0, 1]], [0])]
    deps = compare([5, 3], refs)
    assert any(d["src_ref"] == 1 for d in deps)                      # neighbouring windows share an input element
    # two references to the same array with identical iteration pairs are merged
    refs = [(0, [[1, 0]], [0]), (0, [[1, 0]], [0])]
    deps = compare([3, 4], refs)
    assert len(deps) == 1 and deps[0]["n_pairs"] == 4


def test_argument_errors():
    ext = (ctypes.c_int * 2)(4, 4)
    ref = (P.binding.LoopRef * 1)()
    ref[0].rank = 1
    nd = ctypes.c_int(0)
    f = P.lib.polydl_reuse_analyse
    assert f(2, ext, None, 1, ref, 0, None, ctypes.byref(nd)) == 0 and nd.value == 1
    assert f(0, ext, None, 1, ref, 0, None, ctypes.byref(nd)) == -2
    assert f(9, ext, None, 1, ref, 0, None, ctypes.byref(nd)) == -2
    assert f(2, None, None, 1, ref, 0, None, ctypes.byref(nd)) == -1
    assert f(2, ext, None, 1, ref, 4, None, ctypes.byref(nd)) == -1
    big = (ctypes.c_int * 2)(300, 300)
    assert f(2, big, None, 1, ref, 0, None, ctypes.byref(nd)) == -2
    ref[0].rank = 5
    assert f(2, ext, None, 1, ref, 0, None, ctypes.byref(nd)) == -2


def test_too_many_iteration_pairs_are_refused():
    # one reference that always touches the same element: 4096 iterations make 8 million pairs
    with pytest.raises(P.PolydlError) as e:
        P.reuse_analyse([64, 64], [(0, [[0, 0]], [0])])
    assert e.value.status == -3
    # the same nest, small: one dependence, everything is one element
    deps = P.reuse_analyse([4, 4], [(0, [[0, 0]], [0])])
    assert len(deps) == 1 and deps[0]["ws"] == [1, 1]              # WS_min and WS_max: the one element
    assert deps[0]["min_target"] == (0, 1) and deps[0]["max_target"] == (3, 3)

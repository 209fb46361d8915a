"""Pins of the matrix-product oracle."""
import numpy as np
import pytest

import oracle
import synth


def test_two_by_two_by_hand():
    A = np.array([[1, 2], [3, 4]], np.float32)
    B = np.array([[5, 6], [7, 8]], np.float32)
    C, ab = oracle.gemm(A, B)
    assert np.array_equal(C, [[19, 22], [43, 50]])
    assert np.array_equal(ab, [[19, 22], [43, 50]])
    C, ab = oracle.gemm(A, -B, C0=np.array([[1, 1], [1, 1]], np.float32))
    assert np.array_equal(C, [[-18, -21], [-42, -49]])
    assert np.array_equal(ab, [[20, 23], [44, 51]])


def test_nonsquare_operand_order():
    # A is 2x3, B is 3x1: a transposed operand or swapped index would not even give this shape/value
    A = np.array([[1, 2, 3], [4, 5, 6]], np.float32)
    B = np.array([[1], [10], [100]], np.float32)
    C, _ = oracle.gemm(A, B)
    assert np.array_equal(C, [[321], [654]])


def test_identity_and_ones():
    M, N, K = 7, 5, 5
    A, _, C0 = synth.sgemm_inputs(M, N, K, 2, c0="random")
    C, _ = oracle.gemm(A, np.eye(K, dtype=np.float32), C0)
    assert np.array_equal(C, A.astype(np.float64) + C0.astype(np.float64))
    _, B, _ = synth.sgemm_inputs(3, 9, 6, 3)
    C, _ = oracle.gemm(np.ones((3, 6), np.float32), B)
    col = np.zeros(9)
    for k in range(6):
        col = col + B[k].astype(np.float64)
    assert np.array_equal(C, np.tile(col, (3, 1)))


@pytest.mark.parametrize("M,N,K", [(5, 7, 3), (33, 17, 129), (64, 64, 64), (1, 1, 1000)])
def test_small_integers_exact(M, N, K):
    A, B, C0 = synth.sgemm_inputs(M, N, K, 8, dist="ints", c0="random")
    C, ab = oracle.gemm(A, B, C0)
    want = A.astype(np.int64) @ B.astype(np.int64) + C0.astype(np.int64)
    assert np.array_equal(C, want.astype(np.float64))
    wantab = np.abs(A.astype(np.int64)) @ np.abs(B.astype(np.int64)) + np.abs(C0.astype(np.int64))
    assert np.array_equal(ab, wantab.astype(np.float64))


def test_alpha_beta_applied_once():
    A, B, C0 = synth.sgemm_inputs(4, 6, 50, 5, dist="ints", c0="random")
    C, _ = oracle.gemm(A, B, C0, alpha=2.0, beta=-3.0)
    want = 2 * (A.astype(np.int64) @ B.astype(np.int64)) - 3 * C0.astype(np.int64)
    assert np.array_equal(C, want.astype(np.float64))


def test_random_against_library_matmul():
    A, B, C0 = synth.sgemm_inputs(40, 30, 300, 6, c0="random")
    C, ab = oracle.gemm(A, B, C0)
    lib = A.astype(np.float64) @ B.astype(np.float64) + C0
    assert np.max(np.abs(C - lib) / ab) < 1e-14


def test_sampled_elements():
    A, B, C0 = synth.sgemm_inputs(9, 8, 20, 7, c0="random")
    C, ab = oracle.gemm(A, B, C0)
    idx = np.array([0, 71, 13, 40], np.int64)
    Cs, abs_ = oracle.gemm(A, B, C0, at=idx)
    assert np.array_equal(Cs, C.ravel()[idx]) and np.array_equal(abs_, ab.ravel()[idx])


def test_scaled_error_metric():
    assert oracle.scaled_error([1.0, 2.0], [1.0, 2.5], [10.0, 5.0]) == pytest.approx(0.1)
    assert oracle.scaled_error([0.0], [0.0], [0.0]) == 0.0
    assert oracle.scaled_error([1e-30], [0.0], [0.0]) == float("inf")

"""GPU parity of polydl_sgemm against the fp64 oracle (C += A.B, row-major)."""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import FP32_TOL, dev, host, sample_indices

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2006_02230_amd as p
    yield p
    p.set_tile_override(None)


def run_sgemm(P, A, B, C0):
    C = dev(C0.copy())
    P.sgemm(dev(A), dev(B), C)
    return host(C)


def variant_ids(P):
    return [(v.bm, v.bn, v.bk, v.wm, v.wn) for v in P.variants(1)]


SHAPES = [(256, 256, 64), (200, 136, 75), (130, 260, 17), (64, 64, 8), (1, 1, 1), (33, 1000, 129),
          (300, 70, 256), (129, 127, 1)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_all_variants_random(P, M, N, K):
    A, B, C0 = synth.sgemm_inputs(M, N, K, seed=M + N + K, c0="random")
    want, ab = oracle.gemm(A, B, C0)
    for v in P.variants(1):
        for split_k, raster in ((1, 0), (3, 1)):
            v.split_k, v.raster = split_k, raster
            P.set_tile_override(v)
            got = run_sgemm(P, A, B, C0)
            err = oracle.scaled_error(got, want, ab)
            assert err <= FP32_TOL, (v, err)
    P.set_tile_override(None)


@pytest.mark.parametrize("M,N,K", [(256, 384, 512), (131, 67, 300)])
def test_all_variants_small_integers_exact(P, M, N, K):
    # |a|,|b| <= 3 and K*9 < 2^24: every partial sum is exact in fp32 in any order
    A, B, C0 = synth.sgemm_inputs(M, N, K, seed=5, dist="ints", c0="random")
    want, _ = oracle.gemm(A, B, C0)
    for v in P.variants(1):
        for split_k in (1, 2):
            v.split_k = split_k
            P.set_tile_override(v)
            got = run_sgemm(P, A, B, C0)
            assert np.array_equal(got.astype(np.float64), want), v
    P.set_tile_override(None)


@pytest.mark.parametrize("K", [2, 7, 9, 15, 16, 24, 25, 31, 32, 33, 40, 48, 56])
def test_reduction_lengths_around_stage_and_chunk_boundaries(P, K):
    # a stage is 8 or 16 reduction rows in chunks of eight; stages run in pairs with an odd one peeled
    # off, and a last chunk that lies wholly past the end is skipped: every such boundary, exactly
    M, N = 130, 200
    A, B, C0 = synth.sgemm_inputs(M, N, K, seed=40 + K, dist="ints", c0="random")
    want, _ = oracle.gemm(A, B, C0)
    for v in P.variants(1):
        for split_k in (1, 2):
            v.split_k = split_k
            P.set_tile_override(v)
            got = run_sgemm(P, A, B, C0)
            assert np.array_equal(got.astype(np.float64), want), (v, K)
    P.set_tile_override(None)


def test_identity_gives_exact_copy(P):
    M = N = K = 192
    A, _, C0 = synth.sgemm_inputs(M, N, K, seed=9, c0="random")
    got = run_sgemm(P, A, np.eye(K, dtype=np.float32), np.zeros((M, N), np.float32))
    assert np.array_equal(got, A)


def test_unaligned_base_pointers(P):
    # operands that start 4 bytes into an allocation take the dword-load paths
    import torch
    M, N, K = 96, 72, 40
    A, B, C0 = synth.sgemm_inputs(M, N, K, seed=12, c0="random")
    want, ab = oracle.gemm(A, B, C0)
    bufA = torch.zeros(M * K + 1, device="cuda"); bufA[1:] = dev(A).ravel()
    bufB = torch.zeros(K * N + 1, device="cuda"); bufB[1:] = dev(B).ravel()
    bufC = torch.zeros(M * N + 1, device="cuda"); bufC[1:] = dev(C0).ravel()
    import ctypes
    st = P.lib.polydl_sgemm(M, N, K, ctypes.c_void_p(bufA.data_ptr() + 4), ctypes.c_void_p(bufB.data_ptr() + 4),
                            ctypes.c_void_p(bufC.data_ptr() + 4), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0
    got = host(bufC)[1:].reshape(M, N)
    assert oracle.scaled_error(got, want, ab) <= FP32_TOL
    assert host(bufC)[0] == 0.0


@pytest.mark.parametrize("n", synth.SGEMM_SIZES)
def test_square_full_compare(P, n):
    # the picker's own configuration at every square size of the workload list; every element of C
    A, B, C0 = synth.sgemm_inputs(n, n, n, seed=n)
    want, ab = oracle.gemm(A, B, C0)
    got = run_sgemm(P, A, B, C0)
    assert oracle.scaled_error(got, want, ab) <= FP32_TOL, P.get_last_tile()


@pytest.mark.parametrize("M,N,K", synth.PAPER_GEMM_SIZES, ids=lambda v: str(v))
def test_paper_gemm_sizes_sampled(P, M, N, K):
    # the (M, N, K) of the paper's GEMM-size table (section "GEMM"), in the picker's own
    # configuration; operands are drawn in row chunks (one stream each) to bound host memory
    from synth import rng
    seed = (M * 31 + N) * 31 + K
    A = np.empty((M, K), np.float32)
    rows = max(1, (1 << 24) // K)
    for c, i0 in enumerate(range(0, M, rows)):
        A[i0:i0 + rows] = rng.uniform_pm1(seed, 100 + c, (min(rows, M - i0), K))
    B = rng.uniform_pm1(seed, 1, (K, N))
    C0 = rng.uniform_pm1(seed, 2, (M, N))
    got = run_sgemm(P, A, B, C0)
    idx = sample_indices(M * N, 4000, seed=seed)
    want, ab = oracle.gemm(A, B, C0, at=idx)
    assert oracle.scaled_error(got.ravel()[idx], want, ab) <= FP32_TOL


def test_split_reduction_is_reproducible(P):
    # the parts of a split reduction are summed in index order whatever order they finish in
    A, B, C0 = synth.sgemm_inputs(300, 200, 1000, seed=11, c0="random")
    want, ab = oracle.gemm(A, B, C0)
    for v in P.variants(1):
        for split_k in (2, 7):
            v.split_k = split_k
            P.set_tile_override(v)
            first = run_sgemm(P, A, B, C0)
            assert oracle.scaled_error(first, want, ab) <= FP32_TOL, v
            for _ in range(2):
                assert np.array_equal(run_sgemm(P, A, B, C0), first), v
    P.set_tile_override(None)


@pytest.mark.parametrize("alpha,beta", [(2.0, -3.0), (0.5, 0.0), (0.0, 1.5), (-1.25, 1.0)])
def test_alpha_beta(P, alpha, beta):
    # section "GEMM": C = beta*C + alpha*A*B, each scalar applied once per element
    M, N, K = 200, 136, 300
    A, B, C0 = synth.sgemm_inputs(M, N, K, seed=77, c0="random")
    want, ab = oracle.gemm(A, B, C0, alpha=alpha, beta=beta)
    for v in P.variants(1):
        for split_k in (1, 3):
            v.split_k = split_k
            P.set_tile_override(v)
            C = dev(C0.copy())
            P.sgemm(dev(A), dev(B), C, alpha=alpha, beta=beta)
            err = oracle.scaled_error(host(C), want, ab)
            assert err <= FP32_TOL, (v, err)
    P.set_tile_override(None)


def test_alpha_beta_special_cases(P):
    import torch
    M, N, K = 130, 67, 129
    A, B, C0 = synth.sgemm_inputs(M, N, K, seed=78, c0="random")
    # alpha = beta = 1 is polydl_sgemm bit for bit
    C1, C2 = dev(C0.copy()), dev(C0.copy())
    P.sgemm(dev(A), dev(B), C1)
    P.sgemm(dev(A), dev(B), C2, alpha=1.0, beta=1.0)
    assert np.array_equal(host(C1), host(C2))
    # beta = 0 does not read C: what it held, NaN included, does not reach the result
    Cn = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    P.sgemm(dev(A), dev(B), Cn, alpha=1.0, beta=0.0)
    want, ab = oracle.gemm(A, B, None)
    assert oracle.scaled_error(host(Cn), want, ab) <= FP32_TOL
    # small integers with integer scalars: exact
    Ai, Bi, Ci = synth.sgemm_inputs(M, N, K, seed=5, dist="ints", c0="random")
    C = dev(Ci.copy())
    P.sgemm(dev(Ai), dev(Bi), C, alpha=-2.0, beta=3.0)
    want, _ = oracle.gemm(Ai, Bi, Ci, alpha=-2.0, beta=3.0)
    assert np.array_equal(host(C).astype(np.float64), want)
    # an empty product scales C
    C = dev(C0.copy())
    assert P.lib.polydl_sgemm_ex(M, N, 0, 2.0, None, None, 0.5, C.data_ptr(), None) == 0
    assert np.array_equal(host(C), C0 * np.float32(0.5))


def test_argument_errors(P):
    import ctypes
    z = ctypes.c_void_p(0)
    one = ctypes.c_void_p(256)
    assert P.lib.polydl_sgemm(0, 4, 4, one, one, one, z) == -2
    assert P.lib.polydl_sgemm(4, -1, 4, one, one, one, z) == -2
    assert P.lib.polydl_sgemm(4, 4, 4, z, one, one, z) == -1
    assert P.lib.polydl_sgemm(4, 4, 4, one, one, z, z) == -1
    assert P.lib.polydl_sgemm(4, 4, 0, z, z, one, z) == 0   # K = 0: nothing to add
    assert P.lib.polydl_sgemm_ex(4, 4, 0, 2.0, z, z, 1.0, one, z) == 0   # K = 0, beta = 1: C unchanged, untouched
    assert P.lib.polydl_sgemm_ex(0, 4, 4, 1.0, one, one, 1.0, one, z) == -2
    assert P.lib.polydl_sgemm_ex(4, 4, 4, 1.0, one, z, 1.0, one, z) == -1

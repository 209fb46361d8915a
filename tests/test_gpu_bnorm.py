"""GPU parity of polydl_bnorm_fwd (inference batch normalisation with an optional activation in the
same pass) against the fp64 oracle."""
import numpy as np
import pytest

import oracle
from oracle import elementwise as ew
from synth import rng
from gpu_util import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2006_02230_amd as p
    return p


def inputs(shape, seed):
    N, K, Pq, Q = shape
    x = rng.normal(seed, 0, shape, sigma=2.0)
    gamma = rng.uniform_pm1(seed, 1, (K,)) * 1.5
    beta = rng.uniform_pm1(seed, 2, (K,))
    mean = rng.uniform_pm1(seed, 3, (K,))
    var = (rng.uniform_pm1(seed, 4, (K,)) + 1.0) * 2.0 + 0.01      # (0.01, 4.01)
    return x, gamma, beta, mean, var


def want_and_scale(x, gamma, beta, mean, var, eps, act):
    y = ew.bnorm_inference(x, gamma, beta, mean, var, eps)
    f = lambda v: np.asarray(v, np.float64)[None, :, None, None]   # noqa: E731
    scale = np.abs(f(gamma) * (x.astype(np.float64) - f(mean)) / np.sqrt(f(var) + eps)) + np.abs(f(beta)) + \
        np.abs(f(gamma) * f(mean) / np.sqrt(f(var) + eps))
    if act == "relu":
        y = ew.relu(y)
    elif act == "relu6":
        y = ew.relu6(y)
    return y, scale


# planes of 4k floats (vector path), odd planes (scalar path), one channel, one pixel, many channels
SHAPES = [(2, 16, 14, 14), (3, 5, 7, 7), (1, 1, 5, 3), (4, 7, 1, 1), (2, 130, 6, 10), (1, 3, 56, 56)]


@pytest.mark.parametrize("shape", SHAPES, ids=str)
@pytest.mark.parametrize("act", [None, "relu", "relu6"])
def test_bnorm_act_parity(P, shape, act):
    eps = 1e-5
    x, gamma, beta, mean, var = inputs(shape, seed=sum(shape))
    want, scale = want_and_scale(x, gamma, beta, mean, var, eps, act)
    got = host(P.bnorm_fwd(dev(x), dev(gamma), dev(beta), dev(mean), dev(var), eps, act=act))
    # a handful of fp32 roundings (subtract, divide, multiply, add) relative to the terms' magnitudes
    assert np.max(np.abs(got.astype(np.float64) - want) / scale) <= 1e-6


def test_in_place_equals_out_of_place_and_fused_equals_separate(P):
    shape = (3, 24, 14, 14)
    x, gamma, beta, mean, var = inputs(shape, seed=9)
    a = [dev(v) for v in (gamma, beta, mean, var)]
    fused = host(P.bnorm_fwd(dev(x), *a, 1e-3, act="relu"))
    xi = dev(x)
    P.bnorm_fwd(xi, *a, 1e-3, out=xi, act="relu")
    assert np.array_equal(host(xi), fused)
    sep = P.bnorm_fwd(dev(x), *a, 1e-3, act=None)
    P.activation(sep, "relu")
    assert np.array_equal(host(sep), fused)          # same arithmetic, one pass instead of two


def test_identity_statistics_give_the_input_back(P):
    shape = (2, 8, 6, 6)
    x = rng.small_ints(3, 0, shape)
    one, zero = np.ones(8, np.float32), np.zeros(8, np.float32)
    got = host(P.bnorm_fwd(dev(x), dev(one), dev(zero), dev(zero), dev(one), 0.0))
    assert np.array_equal(got, x)


def test_full_size_tensor_sampled(P):
    # the largest output tensor of the suite: N=32, K=256, 56x56 (102.8 MB)
    shape = (32, 256, 56, 56)
    x, gamma, beta, mean, var = inputs(shape, seed=77)
    got = host(P.bnorm_fwd(dev(x), dev(gamma), dev(beta), dev(mean), dev(var), 1e-5, act="relu"))
    sl = (slice(None, None, 7), slice(None), slice(None, None, 5), slice(None, None, 3))
    want, scale = want_and_scale(x[sl], gamma, beta, mean, var, 1e-5, "relu")
    assert np.max(np.abs(got[sl].astype(np.float64) - want) / scale) <= 1e-6


def test_argument_errors(P):
    import ctypes
    z, one = ctypes.c_void_p(0), ctypes.c_void_p(256)
    f = P.lib.polydl_bnorm_fwd
    eps = ctypes.c_float(1e-5)
    assert f(0, 1, 1, 1, one, one, one, one, one, eps, one, 0, z) == -2
    assert f(1, 1, 1, 1, z, one, one, one, one, eps, one, 0, z) == -1
    assert f(1, 1, 1, 1, one, one, one, one, one, eps, one, 7, z) == -3
    assert f(1, 1, 1, 1, one, one, one, one, one, ctypes.c_float(-1.0), one, 0, z) == -3
    assert f(1 << 10, 1 << 10, 1 << 6, 1 << 6, one, one, one, one, one, eps, one, 0, z) == -3

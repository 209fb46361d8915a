"""GPU parity of the blocked-layout transforms and the separate element-wise kernels (bit exact:
permutations, one fp32 add, max/min)."""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2006_02230_amd as p
    return p


@pytest.mark.parametrize("N,C,H,W,b", [(2, 8, 5, 7, 4), (1, 3, 30, 30, 4), (3, 10, 17, 19, 8), (2, 64, 56, 56, 16),
                                        (1, 5, 1, 1, 2), (2, 33, 14, 14, 32), (1, 7, 23, 300, 1),
                                        # planes that are a multiple of four floats: the 128-bit kernel
                                        (3, 20, 8, 6, 8), (1, 16, 40, 36, 16), (2, 5, 64, 64, 12), (1, 40, 2, 2, 20)])
def test_nchwc_roundtrip_and_parity(P, N, C, H, W, b):
    x = synth.uniform_pm1(41, 0, (N, C, H, W))
    want = oracle.nchw_to_nchwc(x, b)
    got = host(P.nchw_to_nchwc(dev(x), b))
    assert got.shape == want.shape and np.array_equal(got, want)
    back = host(P.nchwc_to_nchw(dev(want), C))
    assert np.array_equal(back, x)


@pytest.mark.parametrize("K,C,R,S,bc,bk", [(8, 8, 3, 3, 4, 4), (64, 3, 7, 7, 2, 64), (70, 12, 3, 3, 2, 64),
                                            (130, 64, 1, 1, 2, 128), (5, 9, 2, 5, 8, 2), (256, 256, 3, 3, 16, 16)])
def test_kcrsck_parity(P, K, C, R, S, bc, bk):
    w = synth.uniform_pm1(42, 0, (K, C, R, S))
    want = oracle.kcrs_to_kcrsck(w, bc, bk)
    got = host(P.kcrs_to_kcrsck(dev(w), bc, bk))
    assert got.shape == want.shape and np.array_equal(got, want)


def test_full_size_transform(P):
    # a suite-sized activation tensor: batch 32, 64 channels, 56x56
    x = synth.normal(43, 0, (32, 64, 56, 56))
    got = host(P.nchw_to_nchwc(dev(x), 8))
    assert np.array_equal(got, oracle.nchw_to_nchwc(x, 8))


@pytest.mark.parametrize("shape", [(2, 5, 3, 7), (3, 64, 14, 14), (1, 1, 1, 1), (2, 6, 5, 5)])
def test_bias_add_and_activations(P, shape):
    y = (synth.uniform_pm1(44, 0, shape).astype(np.float64) * 8.0).astype(np.float32)
    b = synth.uniform_pm1(44, 1, (shape[1],))
    got = host(P.bias_add(dev(y.copy()), dev(b)))
    want = (y + b[None, :, None, None]).astype(np.float32)       # one fp32 add per element
    assert np.array_equal(got, want)
    assert np.array_equal(got.astype(np.float64), oracle.bias_add(y, b).astype(np.float32).astype(np.float64))
    for act, ref in (("relu", oracle.relu), ("relu6", oracle.relu6)):
        g = host(P.activation(dev(want.copy()), act))
        assert np.array_equal(g.astype(np.float64), ref(want))


def test_unaligned_activation(P):
    import torch
    y = (synth.uniform_pm1(45, 0, (1001,)).astype(np.float64) * 8.0).astype(np.float32)
    buf = torch.zeros(1002, device="cuda")
    buf[1:] = dev(y)
    view = buf[1:]
    P.activation(view, "relu6")
    assert np.array_equal(host(view).astype(np.float64), oracle.relu6(y))
    assert host(buf)[0] == 0.0


def test_fused_epilogue_equals_separate_kernels(P):
    # conv + bias + ReLU in one kernel against conv, then bias_add, then activation (section
    # "Operator Fusion": fusion must not change the result); same convolution variant => same bits
    s = synth.ConvShape("f", 2, 32, 14, 14, 48, 3, 3, 1, 1)
    x, w, b = synth.conv_inputs(s, 46, "normal", bias=True)
    tile, _ = P.pick_conv2d(tuple(s)[1:])
    tile.split_k = 1   # whole reduction in one workgroup: the same launch with and without the tail
    P.set_tile_override(tile)
    fused = host(P.conv2d_fwd(dev(x), dev(w), dev(b), stride=1, pad=1, act="relu"))
    y = P.conv2d_fwd(dev(x), dev(w), None, stride=1, pad=1)
    P.bias_add(y, dev(b))
    P.activation(y, "relu")
    P.set_tile_override(None)
    assert np.array_equal(host(y), fused)
    want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=1, pad=1, act="relu")
    assert oracle.scaled_error(fused, want, ab) <= 1e-5


def test_argument_errors(P):
    import ctypes
    z, one = ctypes.c_void_p(0), ctypes.c_void_p(256)
    assert P.lib.polydl_nchw_to_nchwc(1, 4, 2, 2, 0, one, one, z) == -2
    assert P.lib.polydl_nchw_to_nchwc(1, 4, 2, 2, 64, one, one, z) == -3
    assert P.lib.polydl_nchw_to_nchwc(1, 4, 2, 2, 4, z, one, z) == -1
    assert P.lib.polydl_kcrs_to_kcrsck(4, 4, 1, 1, 0, 2, one, one, z) == -2
    assert P.lib.polydl_bias_add(1, 1, 1, 1, one, z, z) == -1
    assert P.lib.polydl_activation(4, one, 0, z) == -3
    assert P.lib.polydl_activation(0, one, 1, z) == -2

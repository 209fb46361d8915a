"""Pins of the convolution oracle: facts fixed by the paper's loop nest and by arithmetic,
none of them produced by the oracle itself or by the HIP library."""
import numpy as np
import pytest

import oracle
import synth


def test_tap_count_3x3_pad1():
    # all-ones image and filter: each output counts the filter taps that land inside the image
    x = np.ones((1, 1, 3, 3), np.float32)
    w = np.ones((1, 1, 3, 3), np.float32)
    y, ab = oracle.conv2d_fwd(x, w, stride=1, pad=1)
    want = np.array([[4, 6, 4], [6, 9, 6], [4, 6, 4]], np.float64)
    assert np.array_equal(y[0, 0], want)
    assert np.array_equal(ab[0, 0], want)


def test_tap_count_stride2_nonsquare():
    # H=4, W=5, R=2, S=3, stride 2, pad 1: rows {2p-1,2p} inside [0,4): 1,2,1;
    # cols {2q-1,2q,2q+1} inside [0,5): 2,3,2
    x = np.ones((1, 1, 4, 5), np.float32)
    w = np.ones((1, 1, 2, 3), np.float32)
    y, _ = oracle.conv2d_fwd(x, w, stride=2, pad=1)
    assert y.shape == (1, 1, 3, 3)
    assert np.array_equal(y[0, 0], np.outer([1, 2, 1], [2, 3, 2]).astype(np.float64))


def test_no_padding_output_size_floor():
    # H=W=7, R=S=3, stride 2, pad 0: P = floor(4/2)+1 = 3; H=8 also gives 3 (floor)
    for H in (7, 8):
        y, _ = oracle.conv2d_fwd(np.ones((1, 1, H, H), np.float32), np.ones((1, 1, 3, 3), np.float32),
                                 stride=2, pad=0)
        assert y.shape == (1, 1, 3, 3) and np.all(y == 9)


def test_hand_worked_2x2_filter_no_flip():
    # image rows [1 2 3; 4 5 6; 7 8 9], filter [1 10; 100 1000], no padding:
    # out[p][q] = x[p][q] + 10 x[p][q+1] + 100 x[p+1][q] + 1000 x[p+1][q+1]  (correlation)
    x = np.arange(1, 10, dtype=np.float32).reshape(1, 1, 3, 3)
    w = np.array([[1, 10], [100, 1000]], np.float32).reshape(1, 1, 2, 2)
    y, _ = oracle.conv2d_fwd(x, w)
    assert np.array_equal(y[0, 0], np.array([[5421, 6532], [8754, 9865]], np.float64))


@pytest.mark.parametrize("stride,pad", [(1, 0), (1, 1), (2, 1), (2, 3), (3, 2)])
def test_one_hot_filter_is_shifted_copy(stride, pad):
    N, C, H, W, K, R, S = 2, 3, 9, 7, 4, 3, 5
    x = synth.uniform_pm1(11, 0, (N, C, H, W))
    k0, c0, r0, s0 = 2, 1, 2, 3
    w = np.zeros((K, C, R, S), np.float32)
    w[k0, c0, r0, s0] = 1.0
    y, _ = oracle.conv2d_fwd(x, w, stride=stride, pad=pad)
    P, Q = y.shape[2:]
    assert (P, Q) == ((H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1)
    want = np.zeros((N, K, P, Q))
    for p in range(P):
        for q in range(Q):
            h, v = p * stride + r0 - pad, q * stride + s0 - pad
            if 0 <= h < H and 0 <= v < W:
                want[:, k0, p, q] = x[:, c0, h, v]
    assert np.array_equal(y, want)


def test_1x1_conv_is_matrix_product():
    # the inner three loops of the listing are a GEMM: for R=S=1, stride 1, out[n] (K x HW)
    # = wt (K x C) . in[n] (C x HW).  Same summation order in both oracles => identical bits.
    N, C, H, W, K = 2, 37, 5, 6, 11
    x = synth.uniform_pm1(3, 0, (N, C, H, W))
    w = synth.uniform_pm1(3, 1, (K, C, 1, 1))
    y, ab = oracle.conv2d_fwd(x, w)
    for n in range(N):
        g, gab = oracle.gemm(w.reshape(K, C), x[n].reshape(C, H * W))
        assert np.array_equal(y[n].reshape(K, H * W), g)
        assert np.array_equal(ab[n].reshape(K, H * W), gab)
        lib = w.reshape(K, C).astype(np.float64) @ x[n].reshape(C, H * W).astype(np.float64)
        assert np.allclose(y[n].reshape(K, H * W), lib, rtol=0, atol=1e-13)


def test_linearity_in_input_and_filter():
    shp = synth.ConvShape("t", 2, 5, 8, 9, 6, 3, 3, 2, 1)
    x1, w1, _ = synth.conv_inputs(shp, 5, "uniform")
    x2, w2, _ = synth.conv_inputs(shp, 6, "uniform")
    a, b = 2.0, -0.5  # powers of two: a*x1+b*x2 is exact in float32 for 24-bit uniforms? not always,
    xs = (a * x1.astype(np.float64) + b * x2.astype(np.float64)).astype(np.float32)
    exact = np.array_equal(xs.astype(np.float64), a * x1.astype(np.float64) + b * x2.astype(np.float64))
    y1, _ = oracle.conv2d_fwd(x1, w1, stride=2, pad=1)
    y2, _ = oracle.conv2d_fwd(x2, w1, stride=2, pad=1)
    ys, _ = oracle.conv2d_fwd(xs, w1, stride=2, pad=1)
    tol = 1e-12 if exact else 1e-5
    assert np.allclose(ys, a * y1 + b * y2, rtol=0, atol=tol)
    ws = (w1.astype(np.float64) * 4.0).astype(np.float32)
    y4, _ = oracle.conv2d_fwd(x1, ws, stride=2, pad=1)
    assert np.array_equal(y4, 4.0 * y1)


@pytest.mark.parametrize("shape", [
    synth.ConvShape("a", 2, 7, 10, 11, 5, 3, 3, 1, 1),
    synth.ConvShape("b", 1, 4, 12, 9, 6, 5, 2, 2, 2),
    synth.ConvShape("c", 3, 3, 15, 15, 8, 7, 7, 2, 3),
    synth.ConvShape("d", 1, 16, 6, 6, 16, 1, 1, 2, 0),
])
def test_small_integers_exact_against_window_sum(shape):
    # independent route: gather sliding windows of the zero-padded image with numpy and
    # contract in int64
    s = shape
    x, w, b = synth.conv_inputs(s, 21, "ints", bias=True)
    y, ab = oracle.conv2d_fwd(x, w, bias=b, stride=s.stride, pad=s.pad)
    xi = np.pad(x.astype(np.int64), ((0, 0), (0, 0), (s.pad, s.pad), (s.pad, s.pad)))
    win = np.lib.stride_tricks.sliding_window_view(xi, (s.R, s.S), axis=(2, 3))
    win = win[:, :, ::s.stride, ::s.stride]  # N C P Q R S
    want = np.einsum("ncpqrs,kcrs->nkpq", win, w.astype(np.int64)) + b.astype(np.int64)[None, :, None, None]
    assert y.shape == want.shape
    assert np.array_equal(y, want.astype(np.float64))
    wantab = np.einsum("ncpqrs,kcrs->nkpq", np.abs(win), np.abs(w.astype(np.int64)))
    wantab = wantab + np.abs(b.astype(np.int64))[None, :, None, None]
    assert np.array_equal(ab, wantab.astype(np.float64))


def test_against_library_convolution():
    torch = pytest.importorskip("torch")
    s = synth.ConvShape("lib", 2, 6, 13, 10, 7, 3, 4, 2, 2)
    x, w, b = synth.conv_inputs(s, 9, "normal", bias=True)
    y, ab = oracle.conv2d_fwd(x, w, bias=b, stride=2, pad=2)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     torch.from_numpy(b).double(), stride=2, padding=2).numpy()
    assert y.shape == ref.shape
    assert np.max(np.abs(y - ref) / ab) < 1e-14


def test_bias_relu_relu6_tail():
    # one output channel pair with known pre-activation values -2, 3, 8 (1x1 filter = scale)
    x = np.array([-2.0, 3.0, 8.0], np.float32).reshape(1, 1, 1, 3)
    w = np.ones((2, 1, 1, 1), np.float32)
    b = np.array([0.0, 1.5], np.float32)
    y, ab = oracle.conv2d_fwd(x, w, bias=b)
    assert np.array_equal(y[0, :, 0], [[-2, 3, 8], [-0.5, 4.5, 9.5]])
    assert np.array_equal(ab[0, :, 0], [[2, 3, 8], [3.5, 4.5, 9.5]])
    y, _ = oracle.conv2d_fwd(x, w, bias=b, act="relu")
    assert np.array_equal(y[0, :, 0], [[0, 3, 8], [0, 4.5, 9.5]])
    y, _ = oracle.conv2d_fwd(x, w, bias=b, act="relu6")
    assert np.array_equal(y[0, :, 0], [[0, 3, 6], [0, 4.5, 6]])
    # the separate element-wise operators give the same as the fused tail
    y0, _ = oracle.conv2d_fwd(x, w)
    assert np.array_equal(oracle.relu(oracle.bias_add(y0, b))[0, :, 0], [[0, 3, 8], [0, 4.5, 9.5]])
    assert np.array_equal(oracle.relu6(oracle.bias_add(y0, b))[0, :, 0], [[0, 3, 6], [0, 4.5, 6]])


def test_bnorm_inference_hand_values():
    x = np.array([1.0, 3.0], np.float32).reshape(1, 2, 1, 1)
    y = oracle.bnorm_inference(x, gamma=[2.0, 0.5], beta=[1.0, -1.0], mean=[1.0, 1.0],
                               var=[3.0, 15.0], eps=1.0)
    # channel 0: 2*(1-1)/2+1 = 1 ; channel 1: 0.5*(3-1)/4-1 = -0.75
    assert np.array_equal(y.ravel(), [1.0, -0.75])


def test_sampled_outputs_match_full_tensor():
    s = synth.ConvShape("s", 2, 5, 9, 8, 6, 3, 3, 2, 1)
    x, w, b = synth.conv_inputs(s, 4, "normal", bias=True)
    y, ab = oracle.conv2d_fwd(x, w, bias=b, stride=2, pad=1, act="relu")
    idx = np.array([0, 1, y.size - 1, 17, 123, 77], np.int64)
    ys, abs_ = oracle.conv2d_fwd(x, w, bias=b, stride=2, pad=1, act="relu", at=idx)
    assert np.array_equal(ys, y.ravel()[idx]) and np.array_equal(abs_, ab.ravel()[idx])
    with pytest.raises(ValueError):
        oracle.conv2d_fwd(x, w, stride=2, pad=1, at=np.array([y.size]))


def test_rejects_empty_output():
    with pytest.raises(ValueError):
        oracle.conv2d_fwd(np.ones((1, 1, 2, 2), np.float32), np.ones((1, 1, 3, 3), np.float32))


def test_suite_shapes_keep_h_over_stride():
    want = [112, 56, 56, 56, 28, 14, 7, 7]
    for s, p in zip(synth.RESNET50_SUITE(32), want):
        assert synth.out_hw(s) == (p, p)

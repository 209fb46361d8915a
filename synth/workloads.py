"""Shapes, seeds and value distributions of the synthetic workloads.

The convolution suite has the layer shapes of a ResNet-50 forward pass (stem 7x7/2, the
1x1 / 3x3 bottleneck convolutions of the four stages, and a strided 1x1 projection); inputs are
N(0,1) activations and He-normal weights, variance 2/(C*R*S).  They stand in for the CNN layer
sets the paper evaluates (section "Convolutions"); no trained weights or images are involved.
The square SGEMM sizes and the non-square sizes of the paper's GEMM table use U[-1,1) values.
"""
from collections import namedtuple
import math
import numpy as np
from . import rng

ConvShape = namedtuple("ConvShape", "name N C H W K R S stride pad")


def out_hw(shape):
    """Output height and width: floor((H + 2 pad - R)/stride) + 1, same for W with S."""
    P = (shape.H + 2 * shape.pad - shape.R) // shape.stride + 1
    Q = (shape.W + 2 * shape.pad - shape.S) // shape.stride + 1
    return P, Q


def _layer(idx, N, C, K, H, R, stride):
    return ConvShape("resnet50_l%d" % idx, N, C, H, H, K, R, R, stride, (R - 1) // 2)


_SUITE_TUPLES = [(3, 64, 224, 7, 2), (64, 64, 56, 1, 1), (64, 64, 56, 3, 1), (64, 256, 56, 1, 1),
                 (128, 128, 28, 3, 1), (256, 256, 14, 3, 1), (512, 512, 7, 3, 1),
                 (1024, 2048, 14, 1, 2)]


def RESNET50_SUITE(N=32):
    """The eight (C, K, H, R, stride) layers at batch N, pad = (R-1)/2 so P = H/stride."""
    return [_layer(i, N, C, K, H, R, st) for i, (C, K, H, R, st) in enumerate(_SUITE_TUPLES)]


CONFIG1 = ConvShape("cfg1_c64k64_56_3x3", 1, 64, 56, 56, 64, 3, 3, 1, 1)
CONFIG4 = ConvShape("cfg4_c256k256_14_3x3_bias_relu", 32, 256, 14, 14, 256, 3, 3, 1, 1)
SGEMM_SIZES = [256, 1024, 2048, 4096]
# (M, N, K) of the paper's GEMM-size table (section "GEMM")
PAPER_GEMM_SIZES = [(128, 2048, 4096), (320, 3072, 4096), (2048, 4096, 32), (1024, 16, 500000),
                    (4096, 4096, 4096), (1024, 1024, 32768), (1024, 32768, 1024),
                    (32768, 1024, 1024)]


def conv_inputs(shape, seed, dist="normal", bias=False):
    """(in NCHW, wt KCRS, bias K or None), float32, from three independent streams of ``seed``.

    dist "normal": in ~ N(0,1), wt ~ N(0, 2/(C R S)); "uniform": both U[-1,1);
    "ints": both small integers in [-3,3].  bias, when asked for, is U[-0.1, 0.1)
    (integers in [-3,3] for "ints").
    """
    s = shape
    ishape, wshape = (s.N, s.C, s.H, s.W), (s.K, s.C, s.R, s.S)
    if dist == "normal":
        x = rng.normal(seed, 0, ishape)
        w = rng.normal(seed, 1, wshape, sigma=math.sqrt(2.0 / (s.C * s.R * s.S)))
    elif dist == "uniform":
        x = rng.uniform_pm1(seed, 0, ishape)
        w = rng.uniform_pm1(seed, 1, wshape)
    elif dist == "ints":
        x = rng.small_ints(seed, 0, ishape)
        w = rng.small_ints(seed, 1, wshape)
    else:
        raise ValueError(dist)
    b = None
    if bias:
        if dist == "ints":
            b = rng.small_ints(seed, 2, (s.K,))
        else:
            b = (rng.uniform_pm1(seed, 2, (s.K,)).astype(np.float64) * 0.1).astype(np.float32)
    return x, w, b


def sgemm_inputs(M, N, K, seed, dist="uniform", c0="zero"):
    """(A MxK, B KxN, C0 MxN) float32 row-major.  c0: "zero" or "random" (U[-1,1))."""
    draw = rng.uniform_pm1 if dist == "uniform" else rng.small_ints
    A = draw(seed, 0, (M, K))
    B = draw(seed, 1, (K, N))
    C0 = np.zeros((M, N), dtype=np.float32) if c0 == "zero" else draw(seed, 2, (M, N))
    return A, B, C0

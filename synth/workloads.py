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


# Layer shapes of ResNet-50 / Inception-style networks that are NOT in the suite above: none of the
# picker's constants was fitted on them.  (C, K, H, R, stride), pad = (R-1)/2.
_HELDOUT_TUPLES = [(256, 64, 56, 1, 1), (128, 128, 56, 3, 2), (512, 128, 28, 1, 1), (256, 512, 28, 1, 2),
                   (2048, 512, 7, 1, 1), (512, 2048, 7, 1, 1), (64, 192, 56, 3, 1), (96, 208, 14, 3, 1),
                   (128, 512, 28, 1, 1), (1024, 256, 14, 1, 1), (256, 1024, 14, 1, 1), (512, 512, 14, 3, 2),
                   (3, 32, 149, 3, 2), (48, 64, 28, 5, 1)]


# A second set: the first set's sweep was looked at while the model's treatment of 1x1 layers was
# corrected; this one's misses (split reductions on small pointwise layers) set one constant.
_HELDOUT2_TUPLES = [(128, 128, 28, 1, 1), (256, 256, 14, 1, 1), (512, 512, 7, 1, 1), (512, 1024, 28, 1, 2),
                    (64, 64, 112, 3, 2), (256, 256, 28, 3, 1), (32, 64, 112, 3, 1), (160, 320, 14, 3, 1),
                    (1024, 512, 14, 1, 1), (1024, 1024, 7, 3, 1), (16, 96, 56, 1, 1), (24, 144, 56, 1, 1),
                    (320, 1280, 7, 1, 1), (80, 192, 35, 3, 1)]


# A third set (VGG-, AlexNet-, MobileNet-, SqueezeNet- and Xception-like shapes), drawn up after the
# cost of a split reduction on the two smallest gather tiles was set from the second set's misses:
# measured once, after that, and not looked at for any change.
_HELDOUT3_TUPLES = [(64, 128, 112, 3, 1), (128, 256, 56, 3, 1), (512, 512, 28, 3, 1), (192, 384, 13, 3, 1),
                    (32, 192, 28, 1, 1), (576, 96, 14, 1, 1), (960, 160, 7, 1, 1), (728, 728, 19, 1, 1),
                    (64, 16, 55, 1, 1), (16, 64, 55, 3, 1), (1536, 256, 8, 1, 1), (3, 64, 224, 3, 1),
                    (32, 96, 28, 5, 1), (128, 256, 28, 3, 2)]


def HELDOUT_SUITE(N=32, which=1):
    """Fourteen further CNN layer shapes at batch N (pick quality off the fitting set); which = 1, 2 or 3."""
    tuples = {1: _HELDOUT_TUPLES, 2: _HELDOUT2_TUPLES, 3: _HELDOUT3_TUPLES}[which]
    return [ConvShape("heldout%d_l%d" % (which, i), N, C, H, H, K, R, R, st, (R - 1) // 2)
            for i, (C, K, H, R, st) in enumerate(tuples)]


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

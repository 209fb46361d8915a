"""Element-wise operators that follow a heavy operator (sections "Operator Fusion" and
"Evaluation of Operator Fusion"), in float64 numpy.  TEST INFRASTRUCTURE ONLY.

ReLU is y = max(x, 0); ReLU6 is y = min(max(x, 0), 6).  Inference batch normalisation is the
per-channel affine map y = gamma * (x - mean) / sqrt(var + eps) + beta on an NCHW tensor.
Pinned in tests/test_oracle_conv.py by values worked by hand.
"""
import numpy as np


def bias_add(y, bias):
    """y[n][k][p][q] + bias[k]."""
    return np.asarray(y, dtype=np.float64) + np.asarray(bias, dtype=np.float64)[None, :, None, None]


def relu(y):
    return np.maximum(np.asarray(y, dtype=np.float64), 0.0)


def relu6(y):
    return np.minimum(np.maximum(np.asarray(y, dtype=np.float64), 0.0), 6.0)


def bnorm_inference(x, gamma, beta, mean, var, eps):
    f = lambda v: np.asarray(v, dtype=np.float64)[None, :, None, None]  # noqa: E731
    return f(gamma) * (np.asarray(x, dtype=np.float64) - f(mean)) / np.sqrt(f(var) + eps) + f(beta)

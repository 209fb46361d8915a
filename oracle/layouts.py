"""Blocked tensor layouts of the paper's convolution listing (figure "The 2-D Convolution code"),
written as plain numpy index permutations.  TEST INFRASTRUCTURE ONLY.

The listing indexes input[img][ifm_tile][h][w][ifm], output[img][ofm_tile][p][q][ofm] and
filter[ofm_tile][ifm_tile][kj][ki][ifm][ofm]: channels are split into tiles of GEMM_BLOCK with
the within-tile channel innermost, and in the filter the output channel is innermost.  The paper
only runs layers whose channel counts are multiples of the block; here a partial last tile is
filled with zeros so any channel count can be blocked (a reading, stated in the design notes).

Pinned by tests/test_oracle_layouts.py with explicit per-element index loops and round trips.
"""
import numpy as np


def nchw_to_nchwc(x, b):
    """[N][C][H][W] -> [N][ceil(C/b)][H][W][b], element (n, c) at tile c//b, lane c%b."""
    x = np.asarray(x)
    N, C, H, W = x.shape
    Cb = -(-C // b)
    xp = np.zeros((N, Cb * b, H, W), dtype=x.dtype)
    xp[:, :C] = x
    return np.ascontiguousarray(xp.reshape(N, Cb, b, H, W).transpose(0, 1, 3, 4, 2))


def nchwc_to_nchw(xb, C):
    """Inverse of nchw_to_nchwc, dropping the zero-filled channels beyond C."""
    xb = np.asarray(xb)
    N, Cb, H, W, b = xb.shape
    return np.ascontiguousarray(xb.transpose(0, 1, 4, 2, 3).reshape(N, Cb * b, H, W)[:, :C])


def kcrs_to_kcrsck(w, bc, bk):
    """[K][C][R][S] -> [ceil(K/bk)][ceil(C/bc)][R][S][bc][bk] (input channel, then output
    channel innermost)."""
    w = np.asarray(w)
    K, C, R, S = w.shape
    Kb, Cb = -(-K // bk), -(-C // bc)
    wp = np.zeros((Kb * bk, Cb * bc, R, S), dtype=w.dtype)
    wp[:K, :C] = w
    return np.ascontiguousarray(wp.reshape(Kb, bk, Cb, bc, R, S).transpose(0, 2, 4, 5, 3, 1))


def kcrsck_to_kcrs(wb, K, C):
    """Inverse of kcrs_to_kcrsck."""
    wb = np.asarray(wb)
    Kb, Cb, R, S, bc, bk = wb.shape
    return np.ascontiguousarray(wb.transpose(0, 5, 1, 4, 2, 3).reshape(Kb * bk, Cb * bc, R, S)[:K, :C])

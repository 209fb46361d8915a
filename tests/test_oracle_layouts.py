"""Pins of the blocked-layout definitions: explicit per-element index loops following the
array subscripts of the paper's convolution listing, and round trips."""
import numpy as np
import pytest

import oracle
import synth


@pytest.mark.parametrize("C,b", [(8, 4), (3, 4), (10, 4), (16, 16), (5, 8)])
def test_nchwc_elementwise(C, b):
    N, H, W = 2, 3, 5
    x = synth.uniform_pm1(1, 0, (N, C, H, W))
    xb = oracle.nchw_to_nchwc(x, b)
    Cb = (C + b - 1) // b
    assert xb.shape == (N, Cb, H, W, b) and xb.flags["C_CONTIGUOUS"]
    flat = xb.ravel()
    for n in range(N):
        for cp in range(Cb * b):
            for h in range(H):
                for w in range(W):
                    addr = (((n * Cb + cp // b) * H + h) * W + w) * b + cp % b
                    want = x[n, cp, h, w] if cp < C else 0.0
                    assert flat[addr] == want
    assert np.array_equal(oracle.nchwc_to_nchw(xb, C), x)


@pytest.mark.parametrize("K,C,bc,bk", [(8, 8, 4, 4), (6, 3, 4, 4), (16, 5, 4, 8), (5, 9, 8, 2)])
def test_kcrsck_elementwise(K, C, bc, bk):
    R, S = 3, 2
    w = synth.uniform_pm1(2, 0, (K, C, R, S))
    wb = oracle.kcrs_to_kcrsck(w, bc, bk)
    Kb, Cb = (K + bk - 1) // bk, (C + bc - 1) // bc
    assert wb.shape == (Kb, Cb, R, S, bc, bk) and wb.flags["C_CONTIGUOUS"]
    flat = wb.ravel()
    for k in range(Kb * bk):
        for c in range(Cb * bc):
            for r in range(R):
                for s in range(S):
                    # filter[ofm_tile][ifm_tile][kj][ki][ifm][ofm]
                    addr = ((((k // bk * Cb + c // bc) * R + r) * S + s) * bc + c % bc) * bk + k % bk
                    want = w[k, c, r, s] if (k < K and c < C) else 0.0
                    assert flat[addr] == want
    assert np.array_equal(oracle.kcrsck_to_kcrs(wb, K, C), w)

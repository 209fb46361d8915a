"""Pins of the learned-ranking oracle (section "DNN-based ranking algorithm"): the network's
layer sizes and activations, the normalisation of the two variants' statistics by their common
sum, the threshold rule and the tournament, each against values worked out by hand."""
import math

import numpy as np
import pytest

from oracle import ranker


def offsets():
    """Start of W and of b of each layer in the flat parameter vector."""
    at, out = 0, []
    for n_in, n_out, _ in ranker.LAYERS:
        out.append((at, at + n_in * n_out, n_in))
        at += n_in * n_out + n_out
    assert at == ranker.NUM_PARAMS
    return out


def hand_network(c, shift=0.0, first_bias=0.0):
    """A network whose outputs can be followed on paper.  With a (b) the sum of the first (second)
    variant's 8 inputs:
      layer 1 (relu):      h0 = a + first_bias, h1 = b + first_bias
      layer 2 (relu):      u0 = max(h0 - h1, 0), u1 = max(h1 - h0, 0)
      layer 3 (softsign):  s0 = softsign(3 u0 - 1), s1 = softsign(3 u1 - 1)
      layer 4 (relu):      v0 = max(2 s0 + 1/2, 0), v1 = max(2 s1 + 1/2, 0)
      output (softmax):    z0 = c v1 + shift, z1 = c v0 + shift
    so the variant with the smaller statistics gets the larger output."""
    p = [0.0] * ranker.NUM_PARAMS
    (w1, b1, i1), (w2, b2, i2), (w3, b3, i3), (w4, b4, i4), (w5, b5, i5) = offsets()
    for k in range(ranker.STATS):
        p[w1 + 0 * i1 + k] = 1.0
        p[w1 + 1 * i1 + ranker.STATS + k] = 1.0
    p[b1 + 0] = p[b1 + 1] = first_bias
    p[w2 + 0 * i2 + 0], p[w2 + 0 * i2 + 1] = 1.0, -1.0
    p[w2 + 1 * i2 + 0], p[w2 + 1 * i2 + 1] = -1.0, 1.0
    p[w3 + 0 * i3 + 0] = p[w3 + 1 * i3 + 1] = 3.0
    p[b3 + 0] = p[b3 + 1] = -1.0
    p[w4 + 0 * i4 + 0] = p[w4 + 1 * i4 + 1] = 2.0
    p[b4 + 0] = p[b4 + 1] = 0.5
    p[w5 + 0 * i5 + 1] = c
    p[w5 + 1 * i5 + 0] = c
    p[b5 + 0] = p[b5 + 1] = shift
    return p


SMALL = (1, 0, 0, 0, 1, 1, 0, 1)
LARGE = (3, 0, 0, 0, 3, 3, 0, 3)


def test_layer_sizes_of_the_paper():
    assert [(i, o) for i, o, _ in ranker.LAYERS] == [(16, 64), (64, 32), (32, 16), (16, 8), (8, 2)]
    assert [a for _, _, a in ranker.LAYERS] == ["relu", "relu", "softsign", "relu", "softmax"]
    assert ranker.NUM_PARAMS == 16 * 64 + 64 + 64 * 32 + 32 + 32 * 16 + 16 + 16 * 8 + 8 + 8 * 2 + 2


def test_statistics_are_divided_by_the_sum_over_both_variants():
    # sizes: 2 + 6 = 8 bytes in all; times: 2 + 6 = 8 us in all
    x = ranker.normalise(SMALL, LARGE)
    assert x == [1 / 8, 0, 0, 0, 1 / 8, 1 / 8, 0, 1 / 8, 3 / 8, 0, 0, 0, 3 / 8, 3 / 8, 0, 3 / 8]
    # each kind by its own sum: scaling all times leaves the inputs alone, and so does scaling all sizes
    s1 = (5, 1, 0, 2, 40, 7, 3, 1)
    s2 = (2, 9, 4, 0, 10, 1, 8, 6)
    t1, t2 = s1[:5] + tuple(1000 * v for v in s1[5:]), s2[:5] + tuple(1000 * v for v in s2[5:])
    assert ranker.normalise(t1, t2) == pytest.approx(ranker.normalise(s1, s2), rel=1e-15)
    x = ranker.normalise(s1, s2)
    assert sum(x[0:5]) + sum(x[8:13]) == pytest.approx(1.0) and sum(x[5:8]) + sum(x[13:16]) == pytest.approx(1.0)
    assert x[4] == 40 / 73 and x[12] == 10 / 73 and x[5] == 7 / 26 and x[14] == 8 / 26
    # nothing to compare: all inputs 0, no division by 0
    assert ranker.normalise((0,) * 8, (0,) * 8) == [0.0] * 16


def test_zero_parameters_give_a_draw():
    w, p = ranker.play([0.0] * ranker.NUM_PARAMS, SMALL, LARGE)
    assert w == 0 and p == [0.5, 0.5]
    wins, order = ranker.tournament([0.0] * ranker.NUM_PARAMS, [SMALL, LARGE, SMALL])
    assert wins == [0, 0, 0] and order == [0, 1, 2]


def test_hand_network_closed_form():
    # a = 4/8, b = 12/8: u = (0, 1); s = (softsign(-1), softsign(2)) = (-1/2, 2/3);
    # v = (max(-1/2, 0), 4/3 + 1/2) = (0, 11/6); z = (4 * 11/6, 0) = (22/3, 0)
    # p0 = 1 / (1 + e^(-22/3)) = 1 / 1.000653391976 = 0.999347035
    w, p = ranker.play(hand_network(4.0), SMALL, LARGE)
    assert w == 1
    assert p[0] == pytest.approx(0.999347035, abs=2e-9) and p[0] + p[1] == pytest.approx(1.0, abs=1e-15)
    assert p[0] == pytest.approx(1.0 / (1.0 + math.exp(-22.0 / 3.0)), rel=1e-14)
    # tanh in place of softsign would give v1 = 2 tanh(2) + 1/2 and p0 = 0.99994
    assert abs(p[0] - 1.0 / (1.0 + math.exp(-4.0 * (2 * math.tanh(2.0) + 0.5)))) > 5e-4
    # the same two the other way round: the second output fires
    w, q = ranker.play(hand_network(4.0), LARGE, SMALL)
    assert w == 2 and q[1] == pytest.approx(p[0], rel=1e-14)
    # softmax does not see a common shift of its two inputs; a - b does not see a common bias
    _, p2 = ranker.play(hand_network(4.0, shift=1.5, first_bias=0.25), SMALL, LARGE)
    assert p2[0] == pytest.approx(p[0], rel=1e-13)


def test_threshold_rule():
    # same network with output weight 0.1: z = (0.1 * 11/6, 0), p0 = 1 / (1 + e^(-11/60)) = 0.5457
    net = hand_network(0.1)
    w, p = ranker.play(net, SMALL, LARGE, theta=0.6)
    assert p[0] == pytest.approx(0.545705, abs=1e-6)
    assert w == 0                                        # neither output above 0.6: a draw
    assert ranker.play(net, SMALL, LARGE, theta=0.5)[0] == 1
    assert ranker.play(net, LARGE, SMALL, theta=0.5)[0] == 2
    assert ranker.play(net, SMALL, SMALL, theta=0.4)[0] == 1   # both at 0.5 > 0.4: the first output is looked at first


def test_tournament_ranks_by_games_won():
    # variants whose statistics are m times one base vector: in a game the hand network sees
    # a = 2 m_i / (m_i + m_j); with m a factor 2 or more apart, u >= 2/3, v >= 3/2, z >= 6, so the
    # smaller m wins with p > 0.997 whichever of the two is named first.  A variant that has
    # r smaller ones below it among n therefore wins 2 (n - 1 - r) games.
    base = (1, 2, 0, 4, 1, 3, 1, 1)
    m = [8, 1, 16, 2, 4]
    stats = [tuple(k * v for v in base) for k in m]
    wins, order = ranker.tournament(hand_network(4.0), stats)
    assert wins == [2, 8, 0, 6, 4]
    assert order == [1, 3, 4, 0, 2]
    # equal variants draw (a = b gives p = (1/2, 1/2)); equal wins keep the given order
    stats = [tuple(k * v for v in base) for k in [2, 1, 2, 1]]
    wins, order = ranker.tournament(hand_network(4.0), stats)
    assert wins == [0, 4, 0, 4] and order == [1, 3, 0, 2]


def test_forward_against_matrix_products():
    # the loops over units against numpy's matrix-vector products on random parameters
    rng = np.random.default_rng(3)
    params = rng.normal(0, 0.4, ranker.NUM_PARAMS)
    for _ in range(20):
        x = rng.uniform(0, 1, 16)
        h, at = x, 0
        for n_in, n_out, act in ranker.LAYERS:
            W = params[at:at + n_in * n_out].reshape(n_out, n_in)
            b = params[at + n_in * n_out:at + n_in * n_out + n_out]
            at += n_in * n_out + n_out
            z = W @ h + b
            if act == "relu":
                h = np.maximum(z, 0)
            elif act == "softsign":
                h = z / (1 + np.abs(z))
            else:
                h = np.exp(z - z.max()) / np.exp(z - z.max()).sum()
        assert ranker.forward(params, x) == pytest.approx(list(h), rel=1e-12, abs=1e-15)

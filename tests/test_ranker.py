"""The library's learned ranking (host code, no GPU needed) against the oracle: network outputs,
the threshold rule, the tournament and the pick among the convolution candidates."""
import ctypes
import os
import subprocess
import sys

import numpy as np
import pytest

import synth
from oracle import ranker
import paper_2006_02230_amd as P
from test_oracle_ranker import hand_network, SMALL, LARGE

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_calls_fail_until_parameters_are_loaded():
    # process-wide state: ask a fresh interpreter
    code = ("import paper_2006_02230_amd as P\n"
            "try:\n    P.ranker_play([1]*8, [2]*8)\nexcept P.PolydlError as e:\n    print('status', e.status)\n"
            "try:\n    P.pick_conv2d_learned((1, 8, 8, 8, 8, 3, 3, 1, 1))\nexcept P.PolydlError as e:\n    print('status', e.status)\n")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.stdout.split() == ["status", "-3", "status", "-3"], r.stdout + r.stderr


def test_parameter_count_and_argument_errors():
    assert P.ranker_num_params() == ranker.NUM_PARAMS and P.RANKER_STATS == ranker.STATS
    buf = (ctypes.c_double * ranker.NUM_PARAMS)()
    assert P.lib.polydl_ranker_set_params(buf, ranker.NUM_PARAMS - 1) == -2
    assert P.lib.polydl_ranker_set_params(None, ranker.NUM_PARAMS) == -1
    buf[5] = float("nan")
    assert P.lib.polydl_ranker_set_params(buf, ranker.NUM_PARAMS) == -2
    P.ranker_set_params([0.0] * ranker.NUM_PARAMS)
    with pytest.raises(P.PolydlError):
        P.ranker_play([-1.0] + [1.0] * 7, [1.0] * 8)            # negative statistic
    with pytest.raises(P.PolydlError):
        P.ranker_play([1.0] * 8, [1.0] * 8, theta=1.5)
    with pytest.raises(P.PolydlError):
        P.ranker_play([float("inf")] + [1.0] * 7, [1.0] * 8)
    assert P.lib.polydl_ranker_tournament(-1, None, 0.6, None, None) == -2
    assert P.lib.polydl_ranker_tournament(3, None, 0.6, None, None) == -1
    assert P.lib.polydl_ranker_tournament(1025, (ctypes.c_double * (1025 * 8))(), 0.6, None, None) == -2
    assert P.ranker_tournament([]) == ([], [])


def test_hand_network_through_the_library():
    P.ranker_set_params(hand_network(4.0))
    w, p = P.ranker_play(SMALL, LARGE)
    assert w == 1 and p[0] == pytest.approx(0.999347035, abs=2e-9)
    assert P.ranker_play(LARGE, SMALL)[0] == 2
    P.ranker_set_params(hand_network(0.1))
    assert P.ranker_play(SMALL, LARGE, 0.6)[0] == 0 and P.ranker_play(SMALL, LARGE, 0.5)[0] == 1
    P.ranker_set_params(hand_network(4.0))
    base = (1, 2, 0, 4, 1, 3, 1, 1)
    wins, order = P.ranker_tournament([tuple(k * v for v in base) for k in [8, 1, 16, 2, 4]])
    assert wins == [2, 8, 0, 6, 4] and order == [1, 3, 4, 0, 2]
    wins, order = P.ranker_tournament([tuple(k * v for v in base) for k in [2, 1, 2, 1]])
    assert wins == [0, 4, 0, 4] and order == [1, 3, 0, 2]
    P.ranker_set_params([0.0] * ranker.NUM_PARAMS)
    assert P.ranker_play(SMALL, LARGE) == (0, [0.5, 0.5])


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_networks_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    params = rng.normal(0, 0.6, ranker.NUM_PARAMS)
    P.ranker_set_params(params)
    decided = 0
    for _ in range(300):
        scale = 10.0 ** rng.integers(0, 9)
        a = list(rng.uniform(0, scale, 8) * (rng.random(8) < 0.8))      # some statistics exactly 0
        b = list(rng.uniform(0, scale, 8) * (rng.random(8) < 0.8))
        w, p = P.ranker_play(a, b)
        ow, op = ranker.play(params, a, b)
        assert p == pytest.approx(op, abs=1e-13)
        if min(abs(op[0] - 0.6), abs(op[1] - 0.6)) > 1e-9:             # the decision is not on the threshold
            assert w == ow
            decided += 1
    assert decided > 250
    stats = [list(rng.uniform(0, 1000, 8)) for _ in range(40)]
    assert P.ranker_tournament(stats) == ranker.tournament(params, stats)
    assert P.ranker_tournament(stats, 0.5) == ranker.tournament(params, stats, 0.5)


def test_trained_parameters_load_and_pick_a_candidate():
    assert os.path.exists(P.RANKER_PARAMS_PATH)
    P.ranker_load()
    params = [float(l) for l in open(P.RANKER_PARAMS_PATH) if l.strip() and not l.startswith("#")]
    assert len(params) == ranker.NUM_PARAMS
    for s in synth.RESNET50_SUITE(32)[1:7:2]:
        shape = tuple(s)[1:]
        cfg, rep, wins, games = P.pick_conv2d_learned(shape)
        # the library's tournament over the candidates the model ranks
        cands, stats = [], []
        for c in P.conv_candidates(shape):
            try:
                stats.append(P.ranker_stats_conv2d(shape, c))
            except P.PolydlError:
                continue
            cands.append(c)
        assert games == 2 * (len(cands) - 1) and 0 < wins <= games
        rep2 = P.model_conv2d(shape, cfg)
        assert stats[[c.as_dict() for c in cands].index(cfg.as_dict())] == \
            list(rep2.level_bytes) + [rep2.mem_bytes, rep2.mfma_us, rep2.mem_us, rep2.fixed_us]
        lwins, lorder = P.ranker_tournament(stats)
        assert cands[lorder[0]].as_dict() == cfg.as_dict() and lwins[lorder[0]] == wins
        # the oracle plays in pure Python: every sixth candidate, the same tournament both ways
        some = stats[::6]
        assert P.ranker_tournament(some) == ranker.tournament(params, some)
        assert rep.predicted_us == pytest.approx(rep2.predicted_us)

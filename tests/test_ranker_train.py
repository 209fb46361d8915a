"""Host checks of the ranker's training script: its vectorised network and normalisation against the
oracle's, its gradients against finite differences, the packed sweep file, the 70/30 split."""
import json

import numpy as np
import pytest

from oracle import ranker
import paper_2006_02230_amd as P
from paper_2006_02230_amd import ranker_train as T


def test_inputs_and_forward_match_the_oracle():
    rng = np.random.default_rng(5)
    stats = rng.uniform(0, 1000, (12, 8)) * (rng.random((12, 8)) < 0.8)
    I, J = np.array([0, 3, 7, 11, 2]), np.array([1, 4, 2, 0, 2])
    X = T.network_inputs(stats, I, J)
    for row, i, j in zip(X, I, J):
        assert list(row) == pytest.approx(ranker.normalise(list(stats[i]), list(stats[j])), rel=1e-14, abs=0)
    flat = rng.normal(0, 0.5, ranker.NUM_PARAMS)
    assert len(T.flatten(T.unflatten(flat))) == ranker.NUM_PARAMS
    assert np.array_equal(T.flatten(T.unflatten(flat)), flat)
    out = T.forward(T.unflatten(flat), X)
    for row, x in zip(out, X):
        assert list(row) == pytest.approx(ranker.forward(flat, list(x)), rel=1e-12)


def test_gradients_against_finite_differences():
    rng = np.random.default_rng(6)
    layers = T.unflatten(rng.normal(0, 0.4, ranker.NUM_PARAMS))
    X = rng.uniform(0, 0.3, (16, 16))
    Y = np.eye(2)[rng.integers(0, 2, 16)]
    loss, grads = T.loss_and_gradients(layers, X, Y)
    assert loss > 0
    eps = 1e-6
    for k in (0, 2, 4):                       # a relu, the softsign and the output layer
        for which in (0, 1):                  # weights, biases
            arr = layers[k][which]
            for _ in range(4):
                idx = tuple(rng.integers(0, n) for n in arr.shape)
                old = arr[idx]
                arr[idx] = old + eps
                up, _ = T.loss_and_gradients(layers, X, Y)
                arr[idx] = old - eps
                down, _ = T.loss_and_gradients(layers, X, Y)
                arr[idx] = old
                assert grads[k][which][idx] == pytest.approx((up - down) / (2 * eps), rel=2e-4, abs=1e-8)


def test_packed_sweep_file_round_trip(tmp_path):
    shape = [2, 64, 8, 8, 64, 3, 3, 1, 1]
    cands = []
    for us, c in zip((30.0, 20.0, 25.0), P.conv_candidates(shape)[:3]):
        cands.append({"us": us, "pred_us": 1.0, "cfg": c.as_dict()})
    src = tmp_path / "sweep.json"
    src.write_text(json.dumps([{"layer": 0, "shape": shape, "picked": cands[0]["cfg"], "picked_us": 30.0,
                                "candidates": cands}]))
    packed = tmp_path / "packed.json"
    assert T.import_sweeps([str(src)], str(packed)) == (1, 3)
    group, us, pred, stats, cfgs, shapes = T.load_table(str(packed))
    assert list(group) == [0, 0, 0] and list(us) == [30.0, 20.0, 25.0] and shapes == [tuple(shape)]
    assert [c.as_dict() for c in cfgs] == [c["cfg"] for c in cands]
    assert stats.shape == (3, 8) and (stats >= 0).all() and (pred > 0).all()
    assert list(stats[1]) == P.ranker_stats_conv2d(shape, cfgs[1])
    I, J = T.ordered_pairs(group, np.ones(3, bool))
    assert sorted(zip(I, J)) == [(0, 1), (0, 2), (1, 0), (1, 2), (2, 0), (2, 1)]


def test_split_is_seeded_and_about_seventy_percent():
    a, b = T.split_mask(5000, 0), T.split_mask(5000, 0)
    assert np.array_equal(a, b) and not np.array_equal(a, T.split_mask(5000, 1))
    assert 0.67 < a.mean() < 0.73


def test_committed_data_and_parameters_belong_together():
    data = json.load(open(T.DATA))
    assert data["fields"] == T.CFG_FIELDS + ["us"] and len(data["problems"]) >= 8
    assert all(len(p["shape"]) == 9 and len(p["rows"]) > 10 for p in data["problems"])
    assert len(T.read_params(P.RANKER_PARAMS_PATH)) == ranker.NUM_PARAMS

"""GPU parity of polydl_conv2d_fwd_tap (filter also given as [K][R][S][C], reduction walked tap by
tap in the gather kernel) against the fp64 oracle, and its fall-backs to the plain call."""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import FP32_TOL, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2006_02230_amd as p
    yield p
    p.set_tile_override(None)


# channel counts that are multiples of the stage depth (16), 2..63 taps
TAP = [
    synth.ConvShape("k3", 2, 16, 14, 14, 32, 3, 3, 1, 1),
    synth.ConvShape("k3c48", 3, 48, 13, 9, 70, 3, 3, 1, 1),      # ragged filter rows and pixels
    synth.ConvShape("s2", 2, 32, 17, 15, 70, 3, 3, 2, 1),
    synth.ConvShape("5x5", 1, 16, 12, 12, 40, 5, 5, 1, 2),
    synth.ConvShape("7x7", 2, 16, 30, 30, 64, 7, 7, 2, 3),       # 49 taps: two mask words
    synth.ConvShape("rect", 1, 32, 9, 20, 5, 2, 5, 1, 2),        # R != S, pad > (R-1)/2
    synth.ConvShape("2x2nopad", 2, 64, 8, 8, 24, 2, 2, 2, 0),
    synth.ConvShape("1x3", 1, 16, 6, 40, 33, 1, 3, 1, 1),        # pad also above and below a one-row filter
]


def gather_variants(P, layout):
    out = []
    for v in P.variants(0):
        if v.algo == 0:
            v.layout = layout
            out.append(v)
    return out


def test_filter_copy_is_the_blocked_layout(P):
    s = TAP[1]
    _, w, _ = synth.conv_inputs(s, seed=70, dist="normal")
    got = host(P.filter_tap_copy(dev(w)))
    assert got.shape == (s.K, s.R, s.S, s.C)
    assert np.array_equal(got.reshape(-1), oracle.kcrs_to_kcrsck(w, s.C, 1).reshape(-1))
    assert np.array_equal(got, w.transpose(0, 2, 3, 1))


@pytest.mark.parametrize("s", TAP, ids=lambda s: s.name)
def test_every_gather_variant_random(P, s):
    x, w, b = synth.conv_inputs(s, seed=71, dist="normal", bias=True)
    want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=s.stride, pad=s.pad, act="relu6")
    dx, dw, db = dev(x), dev(w), dev(b)
    wt = P.filter_tap_copy(dw)
    ran = 0
    for v in gather_variants(P, 2):
        for split_k, raster in ((1, 0), (1, 2), (1, 3), (3, 1)):
            v.split_k, v.raster = split_k, raster
            P.set_tile_override(v)
            got = host(P.conv2d_fwd(dx, dw, db, stride=s.stride, pad=s.pad, act="relu6", w_tap=wt))
            last = P.get_last_tile()
            assert last.layout == 2 and last.algo == 0
            err = oracle.scaled_error(got, want, ab)
            assert err <= FP32_TOL, (v, err)
            ran += 1
    P.set_tile_override(None)
    assert ran >= 3


@pytest.mark.parametrize("s", TAP, ids=lambda s: s.name)
def test_every_gather_variant_small_integers_exact(P, s):
    x, w, b = synth.conv_inputs(s, seed=72, dist="ints", bias=True)
    want, _ = oracle.conv2d_fwd(x, w, bias=b, stride=s.stride, pad=s.pad)
    dx, dw, db = dev(x), dev(w), dev(b)
    wt = P.filter_tap_copy(dw)
    for v in gather_variants(P, 2):
        for split_k in (1, 2):
            v.split_k = split_k
            P.set_tile_override(v)
            got = host(P.conv2d_fwd(dx, dw, db, stride=s.stride, pad=s.pad, w_tap=wt))
            assert np.array_equal(got.astype(np.float64), want), v
    P.set_tile_override(None)


def test_copy_ignored_where_it_does_not_apply(P):
    import torch
    # channel count not a multiple of the stage depth, and a 1x1 filter: the call is the plain one
    for s in (synth.ConvShape("c24", 2, 24, 10, 10, 40, 3, 3, 1, 1), synth.ConvShape("1x1", 2, 32, 9, 9, 40, 1, 1, 1, 0)):
        x, w, b = synth.conv_inputs(s, seed=73, dist="normal", bias=True)
        dx, dw, db = dev(x), dev(w), dev(b)
        wt = P.filter_tap_copy(dw)
        plain = host(P.conv2d_fwd(dx, dw, db, stride=s.stride, pad=s.pad, act="relu"))
        tile = P.get_last_tile()
        got = host(P.conv2d_fwd(dx, dw, db, stride=s.stride, pad=s.pad, act="relu", w_tap=wt))
        assert P.get_last_tile().layout == 0 and P.get_last_tile().as_dict() == tile.as_dict()
        assert np.array_equal(got, plain)
        # forcing the tap-major walk on it is refused
        v = gather_variants(P, 2)[0]
        P.set_tile_override(v)
        with pytest.raises(P.PolydlError) as err:
            P.conv2d_fwd(dx, dw, db, stride=s.stride, pad=s.pad, act="relu", w_tap=wt)
        assert err.value.status == -3
        P.set_tile_override(None)
    # a forced layout 2 without the copy is refused; a copy aligned to less than 16 bytes is ignored
    s = TAP[0]
    x, w, b = synth.conv_inputs(s, seed=74, dist="normal", bias=True)
    dx, dw, db = dev(x), dev(w), dev(b)
    v = gather_variants(P, 2)[0]
    P.set_tile_override(v)
    with pytest.raises(P.PolydlError) as err:
        P.conv2d_fwd(dx, dw, db, stride=s.stride, pad=s.pad)
    assert err.value.status == -3
    P.set_tile_override(None)
    plain = host(P.conv2d_fwd(dx, dw, db, stride=s.stride, pad=s.pad))
    room = torch.empty(w.size + 1, dtype=torch.float32, device="cuda")
    skew = room[1:].view(s.K, s.R, s.S, s.C)
    skew.copy_(P.filter_tap_copy(dw))
    got = host(P.conv2d_fwd(dx, dw, db, stride=s.stride, pad=s.pad, w_tap=skew))
    assert P.get_last_tile().layout == 0
    assert np.array_equal(got, plain)


def test_candidate_list_with_the_copy(P):
    s = synth.RESNET50_SUITE(32)[4]
    plain = P.conv_candidates(tuple(s)[1:])
    tap = P.conv_candidates(tuple(s)[1:], tap=True)
    assert len(plain) == len(tap)
    assert all(c.layout == 0 for c in plain)
    assert all((c.layout == 2) == (c.algo == 0) for c in tap)
    # never priced above the same tile without the copy, and below it where the gather counts
    cheaper = 0
    for a, b in zip(plain, tap):
        if a.algo == 0:
            pa, pb = P.model_conv2d(tuple(s)[1:], a).predicted_us, P.model_conv2d(tuple(s)[1:], b).predicted_us
            assert pb <= pa
            cheaper += pb < pa
    assert cheaper > 0
    # the stem has three channels: nothing changes
    stem = synth.RESNET50_SUITE(32)[0]
    assert all(c.layout == 0 for c in P.conv_candidates(tuple(stem)[1:], tap=True))


@pytest.mark.parametrize("layer", [2, 4, 5, 6])
def test_resnet_suite_full_size_with_the_copy(P, layer):
    # the configuration the benchmark times (batch 32, the picker's own choice), every output
    s = synth.RESNET50_SUITE(32)[layer]
    x, w, b = synth.conv_inputs(s, seed=100 + layer, dist="normal", bias=True)
    dx, dw, db = dev(x), dev(w), dev(b)
    wt = P.filter_tap_copy(dw)
    got = host(P.conv2d_fwd(dx, dw, db, stride=s.stride, pad=s.pad, act="relu", w_tap=wt))
    tile = P.get_last_tile()
    assert tile.layout == 2, tile
    for n0 in range(0, s.N, 16):
        want, ab = oracle.conv2d_fwd(x[n0:n0 + 16], w, bias=b, stride=s.stride, pad=s.pad, act="relu")
        assert oracle.scaled_error(got[n0:n0 + 16], want, ab) <= FP32_TOL, (tile, n0)

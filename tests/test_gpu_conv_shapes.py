"""GPU parity on the three sets of further CNN layer shapes (synth.HELDOUT_SUITE) at a small batch,
every output against the fp64 oracle, each layer run with the variant the picker chooses for it:
with the KCRS filter alone and with its [K][R][S][C] copy beside it."""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import FP32_TOL, dev, host

pytestmark = pytest.mark.gpu

SHAPES = [s for which in (1, 2, 3) for s in synth.HELDOUT_SUITE(2, which)]


@pytest.fixture(scope="module")
def P():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2006_02230_amd as p
    p.set_tile_override(None)
    return p


@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_picked_variant_matches_the_oracle(P, s):
    x, w, b = synth.conv_inputs(s, seed=500 + len(s.name) + s.C + s.K, dist="normal", bias=True)
    want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=s.stride, pad=s.pad, act="relu")
    dx, dw, db = dev(x), dev(w), dev(b)
    got = host(P.conv2d_fwd(dx, dw, db, stride=s.stride, pad=s.pad, act="relu"))
    plain = P.get_last_tile()
    assert plain.layout == 0
    assert oracle.scaled_error(got, want, ab) <= FP32_TOL, plain
    wt = P.filter_tap_copy(dw)
    got = host(P.conv2d_fwd(dx, dw, db, stride=s.stride, pad=s.pad, act="relu", w_tap=wt))
    tile = P.get_last_tile()
    # the copy is walked exactly where it applies: 2..63 taps, channels a multiple of the stage depth
    applies = tile.algo == 0 and 2 <= s.R * s.S <= 63 and s.C % tile.bk == 0
    assert (tile.layout == 2) == applies, tile
    assert oracle.scaled_error(got, want, ab) <= FP32_TOL, tile

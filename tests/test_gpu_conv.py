"""GPU parity of polydl_conv2d_fwd against the fp64 oracle."""
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


def run_conv(P, s, x, w, b=None, act=None):
    return host(P.conv2d_fwd(dev(x), dev(w), dev(b), stride=s.stride, pad=s.pad, act=act))


def try_variant(P, v, s, x, w, b=None, act=None):
    """Run one forced variant; None if that variant declares the problem outside its limits."""
    try:
        P.set_tile_override(v)
        return run_conv(P, s, x, w, b, act)
    except P.PolydlError as e:
        if e.status == -3:
            return None
        raise


SMALL = [
    synth.ConvShape("k3", 2, 8, 14, 14, 16, 3, 3, 1, 1),
    synth.ConvShape("odd", 3, 5, 13, 9, 7, 3, 3, 1, 1),        # C*R*S = 45: dword filter loads
    synth.ConvShape("s2", 2, 12, 17, 15, 70, 3, 3, 2, 1),
    synth.ConvShape("7x7", 2, 3, 30, 30, 64, 7, 7, 2, 3),      # stem-like
    synth.ConvShape("1x1", 3, 64, 7, 7, 130, 1, 1, 1, 0),      # P*Q = 49: odd pixel count
    synth.ConvShape("1x1s2", 2, 32, 14, 14, 64, 1, 1, 2, 0),
    synth.ConvShape("rect", 1, 4, 9, 20, 5, 2, 5, 1, 2),       # R != S, pad > (R-1)/2
    synth.ConvShape("nopad", 1, 16, 12, 12, 32, 5, 5, 3, 0),
    synth.ConvShape("tiny", 1, 1, 1, 1, 1, 1, 1, 1, 0),
]


@pytest.mark.parametrize("s", SMALL, ids=lambda s: s.name)
def test_all_variants_random(P, s):
    x, w, b = synth.conv_inputs(s, seed=31, dist="normal", bias=True)
    want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=s.stride, pad=s.pad, act="relu")
    ran = {0: 0, 1: 0, 2: 0}
    for v in P.variants(0):
        for raster in (0, 1):
            v.raster = raster
            got = try_variant(P, v, s, x, w, b, act="relu")
            if got is None:
                continue
            ran[v.algo] += 1
            assert got.shape == want.shape
            err = oracle.scaled_error(got, want, ab)
            assert err <= FP32_TOL, (v, err)
    P.set_tile_override(None)
    assert ran[0] > 0 and ran[1] > 0


@pytest.mark.parametrize("s", SMALL[:6], ids=lambda s: s.name)
def test_all_variants_small_integers_exact(P, s):
    x, w, b = synth.conv_inputs(s, seed=32, dist="ints", bias=True)
    want, _ = oracle.conv2d_fwd(x, w, bias=b, stride=s.stride, pad=s.pad)
    for v in P.variants(0):
        for split_k in (1, 2):
            v.split_k = split_k
            for cb in ((0, 2, 4) if v.algo == 1 else (0,)):
                v.cb = cb
                got = try_variant(P, v, s, x, w, b)
                if got is not None:
                    assert np.array_equal(got.astype(np.float64), want), v
    P.set_tile_override(None)


@pytest.mark.parametrize("s", SMALL[:7], ids=lambda s: s.name)
def test_one_hot_filter_is_exact_shifted_copy(P, s):
    x, _, _ = synth.conv_inputs(s, seed=33, dist="normal")
    w = np.zeros((s.K, s.C, s.R, s.S), np.float32)
    k0, c0, r0, s0 = s.K - 1, s.C // 2, s.R - 1, s.S // 2
    w[k0, c0, r0, s0] = 1.0
    want, _ = oracle.conv2d_fwd(x, w, stride=s.stride, pad=s.pad)
    got = run_conv(P, s, x, w)
    assert np.array_equal(got.astype(np.float64), want)
    for v in P.variants(0):
        got = try_variant(P, v, s, x, w)
        if got is not None:
            assert np.array_equal(got.astype(np.float64), want), v
    P.set_tile_override(None)


def test_activation_tails(P):
    s = synth.ConvShape("act", 2, 16, 10, 10, 24, 3, 3, 1, 1)
    x, w, b = synth.conv_inputs(s, seed=34, dist="uniform", bias=True)
    w = w * 4.0   # make some outputs exceed 6
    for act in (None, "relu", "relu6"):
        want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=1, pad=1, act=act)
        got = run_conv(P, s, x, w, b, act=act)
        assert oracle.scaled_error(got, want, ab) <= FP32_TOL
        if act == "relu6":
            assert got.max() == 6.0 and got.min() == 0.0
    # no bias pointer
    want, ab = oracle.conv2d_fwd(x, w, stride=1, pad=1, act="relu")
    assert oracle.scaled_error(run_conv(P, s, x, w, None, act="relu"), want, ab) <= FP32_TOL


def test_config1_full_compare(P):
    s = synth.CONFIG1
    x, w, _ = synth.conv_inputs(s, seed=0, dist="uniform")
    want, ab = oracle.conv2d_fwd(x, w, stride=s.stride, pad=s.pad)
    got = run_conv(P, s, x, w)
    assert oracle.scaled_error(got, want, ab) <= FP32_TOL


@pytest.mark.parametrize("layer", range(8))
def test_resnet_suite_full_size(P, layer):
    # batch 32, the picker's own configuration (what the benchmark times): EVERY output of the
    # layer against the oracle
    s = synth.RESNET50_SUITE(32)[layer]
    x, w, b = synth.conv_inputs(s, seed=100 + layer, dist="normal", bias=True)
    got = run_conv(P, s, x, w, b, act="relu")
    Pq, Qq = synth.out_hw(s)
    assert got.shape == (s.N, s.K, Pq, Qq)
    want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=s.stride, pad=s.pad, act="relu")
    assert oracle.scaled_error(got, want, ab) <= FP32_TOL, P.get_last_tile()
    # without bias and activation (another epilogue path of the same launch configuration)
    got0 = run_conv(P, s, x, w)
    want0, ab0 = oracle.conv2d_fwd(x, w, stride=s.stride, pad=s.pad)
    assert oracle.scaled_error(got0, want0, ab0) <= FP32_TOL, P.get_last_tile()


@pytest.mark.parametrize("layer", range(8))
def test_resnet_suite_batch64_full_size(P, layer):
    # batch 64: other picks than at batch 32 (leftover-tile splits, the pointwise kernel, other
    # split factors); every output against the oracle, in chunks of 16 images to bound host memory
    s = synth.RESNET50_SUITE(64)[layer]
    x, w, b = synth.conv_inputs(s, seed=100 + layer, dist="normal", bias=True)
    got = run_conv(P, s, x, w, b, act="relu")
    tile = P.get_last_tile()
    for n0 in range(0, s.N, 16):
        want, ab = oracle.conv2d_fwd(x[n0:n0 + 16], w, bias=b, stride=s.stride, pad=s.pad, act="relu")
        assert oracle.scaled_error(got[n0:n0 + 16], want, ab) <= FP32_TOL, (tile, n0)


@pytest.mark.parametrize("layer", [0, 2, 4, 7])
def test_leftover_tile_split_full_size(P, layer):
    # raster 3 (what the picker ranks: leftover tiles cut, XCD-aware order) at full size on the layers
    # where it is ranked (batch 32 and 64): the whole tiles and the tiles cut along the reduction,
    # every output
    for N in (32, 64):
        s = synth.RESNET50_SUITE(N)[layer]
        x, w, b = synth.conv_inputs(s, seed=100 + layer, dist="normal", bias=True)
        want = None
        for v in P.variants(0):
            if v.algo != 0 or v.wm * v.wn > 64 * 32:
                continue
            v.raster, v.split_k = 3, 1
            got = try_variant(P, v, s, x, w, b, act="relu")
            if got is None:
                continue
            if want is None:
                want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=s.stride, pad=s.pad, act="relu")
            assert oracle.scaled_error(got, want, ab) <= FP32_TOL, (v, N)
        assert want is not None
    P.set_tile_override(None)


def test_split_k_random(P):
    s = synth.ConvShape("split", 2, 64, 7, 7, 96, 3, 3, 1, 1)
    x, w, b = synth.conv_inputs(s, seed=35, dist="normal", bias=True)
    want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=1, pad=1)
    want_r, ab_r = oracle.conv2d_fwd(x, w, bias=b, stride=1, pad=1, act="relu")
    for v in P.variants(0):
        if v.algo == 2:
            continue            # the pointwise kernel has no split
        v.split_k = 4
        got = try_variant(P, v, s, x, w, b)
        assert got is not None and oracle.scaled_error(got, want, ab) <= FP32_TOL, v
        got = try_variant(P, v, s, x, w, b, act="relu")
        assert oracle.scaled_error(got, want_r, ab_r) <= FP32_TOL, v
        assert np.array_equal(try_variant(P, v, s, x, w, b, act="relu"), got), v   # fixed summation order
    P.set_tile_override(None)


def test_split_reduction_in_patch_kernel_is_reproducible(P):
    # the parts of a split reduction are summed in a fixed order whatever order they finish in:
    # repeated launches agree bit for bit, over many tiles, ragged tile edges and a reused scratch
    s = synth.ConvShape("split_many", 5, 48, 13, 11, 150, 3, 3, 1, 1)
    x, w, b = synth.conv_inputs(s, seed=36, dist="normal", bias=True)
    want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=1, pad=1, act="relu")
    small = synth.ConvShape("split_small", 1, 16, 6, 6, 20, 3, 3, 1, 1)
    xs, ws, bs = synth.conv_inputs(small, seed=37, dist="normal", bias=True)
    want_s, ab_s = oracle.conv2d_fwd(xs, ws, bias=bs, stride=1, pad=1, act="relu")
    ran = 0
    for v in P.variants(0):
        if v.algo != 1:
            continue
        for split_k in (2, 3, 12):
            v.split_k, v.cb = split_k, 4
            first = try_variant(P, v, s, x, w, b, act="relu")
            if first is None:
                continue
            assert oracle.scaled_error(first, want, ab) <= FP32_TOL, v
            for _ in range(3):
                assert np.array_equal(try_variant(P, v, s, x, w, b, act="relu"), first), v
            # a smaller problem next, on the same scratch memory and counters
            got_s = try_variant(P, v, small, xs, ws, bs, act="relu")
            assert got_s is not None and oracle.scaled_error(got_s, want_s, ab_s) <= FP32_TOL, v
            ran += 1
    assert ran > 0
    P.set_tile_override(None)


ROW_STAGED = [
    synth.ConvShape("rows5", 3, 10, 12, 12, 40, 5, 5, 1, 2),        # channel tail, runs crossing images
    synth.ConvShape("rows7s2", 2, 6, 32, 32, 70, 7, 7, 2, 3),       # 16x16 outputs: tiles inside one image
    synth.ConvShape("rows5x3", 1, 7, 15, 9, 33, 5, 3, 1, 1),        # R != S, pad < (R-1)/2: rows fall off both edges
    synth.ConvShape("rows9", 2, 4, 20, 20, 16, 9, 9, 1, 4),         # filter size without an unrolled instantiation
]


@pytest.mark.parametrize("s", ROW_STAGED, ids=lambda s: s.name)
def test_filter_row_staging(P, s):
    # filters of five rows or more: a stage of the patch kernel holds one filter row of its channels
    x, w, b = synth.conv_inputs(s, seed=39, dist="normal", bias=True)
    want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=s.stride, pad=s.pad, act="relu")
    xi, wi, bi = synth.conv_inputs(s, seed=40, dist="ints", bias=True)
    want_i, _ = oracle.conv2d_fwd(xi, wi, bias=bi, stride=s.stride, pad=s.pad)
    ran = 0
    for v in P.variants(0):
        if v.algo != 1:
            continue
        for cb, split_k in ((2, 1), (4, 1), (2, 5), (4, 2)):
            v.cb, v.split_k = cb, split_k
            got = try_variant(P, v, s, x, w, b, act="relu")
            if got is None:
                continue
            assert oracle.scaled_error(got, want, ab) <= FP32_TOL, (v, cb, split_k)
            got_i = try_variant(P, v, s, xi, wi, bi)
            assert np.array_equal(got_i.astype(np.float64), want_i), (v, cb, split_k)
            ran += 1
    assert ran > 0
    P.set_tile_override(None)


GATHER_MODES = [
    synth.ConvShape("taps1_pad1x1", 2, 8, 6, 6, 16, 1, 1, 1, 1),      # one tap, but padded: not the 1x1 fast path
    synth.ConvShape("taps1_31", 1, 2, 12, 40, 8, 1, 31, 1, 15),       # 31 taps: the most one register of tap bits holds
    synth.ConvShape("taps2_32", 1, 2, 12, 40, 8, 1, 32, 1, 16),       # 32 taps: first size with two registers
    synth.ConvShape("taps2_63", 1, 2, 30, 30, 8, 7, 9, 1, 3),         # 63 taps: the most two registers hold
    synth.ConvShape("masks_64", 1, 2, 30, 30, 8, 8, 8, 1, 3),         # 64 taps: row and column masks
    synth.ConvShape("masks_81s2", 2, 3, 21, 21, 16, 9, 9, 2, 4),
    synth.ConvShape("point_1x1", 3, 20, 8, 6, 70, 1, 1, 1, 0),        # 1x1 fast path, reduction shorter than two stages
    synth.ConvShape("point_1x1_big", 5, 33, 16, 12, 130, 1, 1, 1, 0),   # tiles crossing images, channel tail, ragged K
]


@pytest.mark.parametrize("s", GATHER_MODES, ids=lambda s: s.name)
def test_gather_addressing_modes(P, s):
    # the gather kernel decides tap validity in one of several ways depending on the filter size;
    # every way, on every tile, with the reduction whole and split
    x, w, b = synth.conv_inputs(s, seed=41, dist="normal", bias=True)
    want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=s.stride, pad=s.pad, act="relu6")
    xi, wi, bi = synth.conv_inputs(s, seed=42, dist="ints", bias=True)
    want_i, _ = oracle.conv2d_fwd(xi, wi, bias=bi, stride=s.stride, pad=s.pad)
    ran = 0
    for v in P.variants(0):
        if v.algo != 0:
            continue
        for split_k in (1, 3):
            v.split_k = split_k
            got = try_variant(P, v, s, x, w, b, act="relu6")
            if got is None:
                continue
            assert oracle.scaled_error(got, want, ab) <= FP32_TOL, (v, split_k)
            got_i = try_variant(P, v, s, xi, wi, bi)
            assert np.array_equal(got_i.astype(np.float64), want_i), (v, split_k)
            ran += 1
    assert ran > 0
    P.set_tile_override(None)


LEFTOVER = [
    synth.ConvShape("tail64", 17, 8, 32, 32, 64, 3, 3, 1, 1),     # 272 tiles of 64x64: 16 leftover tiles, 5 stages
    synth.ConvShape("tail1x1", 9, 40, 48, 40, 70, 1, 1, 1, 0),    # two tile rows, short reduction, ragged channels
    synth.ConvShape("tail128", 5, 4, 64, 64, 130, 3, 3, 1, 1),    # 320 tiles of 128x128: 64 leftover tiles
]


@pytest.mark.parametrize("s", LEFTOVER, ids=lambda s: s.name)
def test_leftover_tiles_split(P, s):
    # rasters 2 and 3: the tiles beyond the last full round of the compute units are cut along the reduction
    x, w, b = synth.conv_inputs(s, seed=43, dist="normal", bias=True)
    want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=s.stride, pad=s.pad, act="relu")
    xi, wi, bi = synth.conv_inputs(s, seed=44, dist="ints", bias=True)
    want_i, _ = oracle.conv2d_fwd(xi, wi, bias=bi, stride=s.stride, pad=s.pad)
    ran = 0
    for v in P.variants(0):
        if v.algo != 0:
            continue
        for raster in (2, 3):       # the leftover tiles cut, tiles dealt in plain and in XCD-aware order
            v.raster, v.split_k = raster, 1
            got = try_variant(P, v, s, x, w, b, act="relu")
            if got is None:
                continue
            assert oracle.scaled_error(got, want, ab) <= FP32_TOL, v
            assert np.array_equal(try_variant(P, v, s, x, w, b, act="relu"), got), v     # fixed summation order
            got_i = try_variant(P, v, s, xi, wi, bi)
            assert np.array_equal(got_i.astype(np.float64), want_i), v
            ran += 1
    assert ran > 0
    P.set_tile_override(None)


@pytest.mark.parametrize("s", [SMALL[0], SMALL[2], SMALL[3], SMALL[4], SMALL[6]], ids=lambda s: s.name)
def test_activation_before_the_convolution(P, s):
    # out = act(conv(pre_act(x)) + bias): the oracle applies the element-wise operator to the input
    # first and then convolves; the gather kernel applies it as it fills a stage
    from oracle import elementwise
    x, w, b = synth.conv_inputs(s, seed=51, dist="normal", bias=True)
    x = (x * 4).astype(np.float32)                     # some values beyond 6
    for pre, fn in (("relu", elementwise.relu), ("relu6", elementwise.relu6)):
        xa = fn(x.astype(np.float64)).astype(np.float32)   # exact: max/min of float32 values
        want, ab = oracle.conv2d_fwd(xa, w, bias=b, stride=s.stride, pad=s.pad, act="relu")
        ran = 0
        for v in P.variants(0):
            if v.algo == 2:
                continue        # pointwise kernel: no split, no operator on the way in (covered by its own tests)
            P.set_tile_override(v)
            for split_k in (1, 2):
                v.split_k = split_k
                P.set_tile_override(v)
                try:
                    got = host(P.conv2d_fwd(dev(x), dev(w), dev(b), stride=s.stride, pad=s.pad, act="relu", pre_act=pre))
                except P.PolydlError as e:
                    assert e.status == -3
                    if v.algo == 0:
                        continue          # outside that variant's limits
                    break                 # the patch kernel does not take the operator
                assert v.algo == 0
                assert oracle.scaled_error(got, want, ab) <= FP32_TOL, (v, pre)
                ran += 1
        assert ran > 0
    P.set_tile_override(None)
    # through the picker: only gather variants are ranked
    got = host(P.conv2d_fwd(dev(x), dev(w), dev(b), stride=s.stride, pad=s.pad, act="relu", pre_act="relu6"))
    assert P.get_last_tile().algo == 0
    assert oracle.scaled_error(got, want, ab) <= FP32_TOL
    # and pre_act none is the plain call bit for bit
    a = host(P.conv2d_fwd(dev(x), dev(w), dev(b), stride=s.stride, pad=s.pad, act="relu", pre_act="none"))
    c = host(P.conv2d_fwd(dev(x), dev(w), dev(b), stride=s.stride, pad=s.pad, act="relu"))
    assert np.array_equal(a, c)


def test_random_shapes_through_the_picker(P):
    # no forced variant: whatever the picker chooses for each of a seeded set of random problems
    # (kernel, tile, split, workgroup order) must agree with the definition
    rng = np.random.default_rng(2024)
    P.set_tile_override(None)
    seen = set()
    for t in range(40):
        R = int(rng.choice([1, 1, 2, 3, 3, 3, 5, 7]))
        S = R if rng.random() < 0.8 else int(rng.choice([1, 2, 3, 4]))
        stride = int(rng.choice([1, 1, 1, 2, 3]))
        pad = int(rng.integers(0, max(R, S)))
        H = int(rng.integers(max(R - 2 * pad, 1), 40))
        W = int(rng.integers(max(S - 2 * pad, 1), 40))
        N, C, K = int(rng.integers(1, 9)), int(rng.integers(1, 70)), int(rng.integers(1, 200))
        s = synth.ConvShape("rnd%d" % t, N, C, H, W, K, R, S, stride, pad)
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        x, w, b = synth.conv_inputs(s, seed=500 + t, dist="normal", bias=bool(t % 3))
        act = [None, "relu", "relu6"][t % 3]
        want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=s.stride, pad=s.pad, act=act)
        got = run_conv(P, s, x, w, b, act=act)
        assert got.shape == want.shape, s
        assert oracle.scaled_error(got, want, ab) <= FP32_TOL, (s, P.get_last_tile())
        tile = P.get_last_tile()
        seen.add((tile.algo, tile.bm, tile.bn, tile.split_k > 1, tile.raster))
    assert len(seen) >= 2      # whole and split reductions at least


POINTWISE = [
    synth.ConvShape("c64", 2, 64, 56, 56, 128, 1, 1, 1, 0),        # 98 tiles of 64 pixels, two channel groups
    synth.ConvShape("groups", 1, 64, 7, 6, 256, 1, 1, 1, 0),        # 42 pixels: one ragged tile, four channel groups
    synth.ConvShape("c32", 3, 32, 5, 4, 128, 1, 1, 1, 0),          # tiles straddle images (20 pixels each)
    synth.ConvShape("c16", 5, 16, 9, 2, 1024, 1, 1, 1, 0),         # sixteen groups, filter fills LDS
    synth.ConvShape("many", 16, 16, 64, 66, 192, 1, 1, 1, 0),      # 3168 units for 2048 waves: runs of one and two
]


def point_variant(P):
    v = [v for v in P.variants(0) if v.algo == 2]
    assert len(v) == 1
    return v[0]


@pytest.mark.parametrize("s", POINTWISE, ids=lambda s: s.name)
def test_pointwise_kernel(P, s):
    v = point_variant(P)
    x, w, b = synth.conv_inputs(s, seed=71, dist="normal", bias=True)
    for act, bias in (("relu", b), (None, None), ("relu6", b)):
        want, ab = oracle.conv2d_fwd(x, w, bias=bias, stride=1, pad=0, act=act)
        got = try_variant(P, v, s, x, w, bias, act=act)
        assert got is not None and P.get_last_tile().algo == 2
        assert oracle.scaled_error(got, want, ab) <= FP32_TOL, (s.name, act)
    # exact cases: small integers, and a one-hot filter that copies one input channel
    xi, wi, bi = synth.conv_inputs(s, seed=72, dist="ints", bias=True)
    want, _ = oracle.conv2d_fwd(xi, wi, bias=bi, stride=1, pad=0)
    assert np.array_equal(try_variant(P, v, s, xi, wi, bi).astype(np.float64), want)
    w1 = np.zeros_like(w)
    w1[s.K - 1, s.C - 3, 0, 0] = 1.0
    got = try_variant(P, v, s, x, w1)
    assert np.array_equal(got[:, s.K - 1], x[:, s.C - 3]) and not got[:, :s.K - 1].any()
    P.set_tile_override(None)


def test_pointwise_kernel_limits_and_fallback(P):
    import torch
    v = point_variant(P)
    # shapes it does not take: odd pixel count, stride 2, 3x3, channel counts outside its family
    for s in (synth.ConvShape("odd", 1, 64, 7, 7, 64, 1, 1, 1, 0), synth.ConvShape("s2", 1, 64, 8, 8, 64, 1, 1, 2, 0),
              synth.ConvShape("k3", 1, 64, 8, 8, 64, 3, 3, 1, 1), synth.ConvShape("c24", 1, 24, 8, 8, 64, 1, 1, 1, 0),
              synth.ConvShape("k96", 1, 64, 8, 8, 96, 1, 1, 1, 0), synth.ConvShape("big", 1, 64, 8, 8, 512, 1, 1, 1, 0),
              synth.ConvShape("k64", 1, 64, 8, 8, 64, 1, 1, 1, 0)):
        x, w, _ = synth.conv_inputs(s, seed=73, dist="normal")
        assert try_variant(P, v, s, x, w) is None, s.name
        with pytest.raises(P.PolydlError):
            P.model_conv2d(tuple(s)[1:], v)
    P.set_tile_override(None)
    # a problem where the picker chooses it (64 -> 256 channels at 56 x 56, batch 64), every output
    # checked; with tensors that are only 4-byte aligned the call still succeeds through another kernel
    s = synth.ConvShape("pick", 64, 64, 56, 56, 256, 1, 1, 1, 0)
    cfg, _ = P.pick_conv2d(tuple(s)[1:])
    assert cfg.algo == 2
    x, w, b = synth.conv_inputs(s, seed=74, dist="normal", bias=True)
    want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=1, pad=0, act="relu")
    got = run_conv(P, s, x, w, b, act="relu")
    assert P.get_last_tile().as_dict() == cfg.as_dict()
    assert oracle.scaled_error(got, want, ab) <= FP32_TOL
    xd = torch.empty(x.size + 1, dtype=torch.float32, device="cuda")[1:].view(x.shape)
    xd.copy_(torch.from_numpy(x))
    assert xd.data_ptr() % 8 == 4
    got = host(P.conv2d_fwd(xd, dev(w), dev(b), stride=1, pad=0, act="relu"))
    assert P.get_last_tile().algo != 2
    assert oracle.scaled_error(got, want, ab) <= FP32_TOL
    P.set_tile_override(v)
    with pytest.raises(P.PolydlError):
        P.conv2d_fwd(xd, dev(w), dev(b), stride=1, pad=0, act="relu")
    P.set_tile_override(None)


def test_argument_errors(P):
    import ctypes
    z, one = ctypes.c_void_p(0), ctypes.c_void_p(256)
    f = P.lib.polydl_conv2d_fwd
    assert f(0, 1, 4, 4, 1, 3, 3, 1, 1, one, one, z, one, 0, z) == -2
    assert f(1, 1, 4, 4, 1, 3, 3, 0, 1, one, one, z, one, 0, z) == -2
    assert f(1, 1, 4, 4, 1, 3, 3, 1, -1, one, one, z, one, 0, z) == -2
    assert f(1, 1, 2, 2, 1, 3, 3, 1, 0, one, one, z, one, 0, z) == -2   # no output pixel
    assert f(1, 1, 4, 4, 1, 3, 3, 1, 1, z, one, z, one, 0, z) == -1
    assert f(1, 1, 4, 4, 1, 3, 3, 1, 1, one, one, z, z, 0, z) == -1
    assert P.lib.polydl_conv2d_fwd_act(1, 1, 4, 4, 1, 3, 3, 1, 1, one, one, z, one, 7, z) == -3

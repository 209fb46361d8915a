"""Host logic of the tile picker: the library's implementation of the bucketing algorithm and of
equation (1) against the oracle's, the closed-form working sets against the brute-force analyser,
and the consistency of the ranking (no GPU needed)."""
import itertools

import numpy as np
import pytest

import synth
from oracle import reuse
import paper_2006_02230_amd as P


def test_bucket_and_cost_match_oracle_on_random_inputs():
    rng = np.random.default_rng(7)
    for _ in range(200):
        n, m = int(rng.integers(0, 12)), int(rng.integers(1, 5))
        ws = [float(v) for v in rng.integers(1, 500, n)]
        sizes = sorted(float(v) for v in rng.integers(1, 800, m))
        lv, mem = P.reuse_bucket(ws, sizes)
        olv, omem = reuse.bucket_working_sets(ws, sizes)
        assert lv == [float(v) for v in olv] and mem == float(omem)
        w = [float(v) for v in rng.integers(1, 9, m)]
        assert P.reuse_cost(lv, mem, w, 50.0) == reuse.cost(olv, omem, w, 50.0)


def test_bucket_hand_example():
    assert P.reuse_bucket([50, 3, 200, 5, 60, 4], [10, 100]) == ([7.0, 55.0], 260.0)
    assert P.reuse_cost([7, 55], 260, [1, 4], 100) == 7 + 220 + 26000


def tiled_gemm_nest(tiles_n, bm, bn, K):
    """One row tile, tiles_n column tiles: for tn, k, i, j: C[i][tn*bn+j] += A[i][k] * B[k][tn*bn+j]."""
    loops = [("tn", tiles_n), ("k", K), ("i", bm), ("j", bn)]
    refs = [("C", lambda it: (it[2], it[0] * bn + it[3])), ("A", lambda it: (it[2], it[1])),
            ("B", lambda it: (it[1], it[0] * bn + it[3]))]
    return loops, refs


@pytest.mark.parametrize("bm,bn,K", [(2, 2, 3), (3, 2, 2), (2, 4, 2)])
def test_column_step_working_set_formula(bm, bn, K):
    # Reuse of the A panel by the next column tile.  With two column tiles the last target of the
    # first A element lies in the second tile (same k and i, last j), so WS_max is everything the
    # first tile step touches -- A panel, B panel, C tile -- plus the first row of the second
    # tile's B panel and C tile.  The library's "one column-tile step" working set is the leading
    # part bm*K + K*bn + bm*bn of this.
    loops, refs = tiled_gemm_nest(2, bm, bn, K)
    deps = reuse.working_sets(loops, refs)
    dA = [d for d in deps if (1, 1) in d["refs"]]
    assert len(dA) == 1 and dA[0]["source"] == (0, 0, 0, 0)
    assert dA[0]["max_target"] == (1, 0, 0, bn - 1)
    assert max(dA[0]["ws"]) == bm * K + K * bn + bm * bn + 2 * bn


def test_model_report_uses_that_formula():
    M = N = K = 1024
    for v in P.variants(1):
        rep = P.model_sgemm(M, N, K, v)
        ws = list(rep.ws)[:rep.n_ws]
        assert ws[0] == v.wm * v.wn * 4                                   # accumulator tile
        assert ws[2] == (v.bm * K + v.bn * K + v.bm * v.bn) * 4            # one column-tile step
        assert ws[4] == (M * K + K * N + 2 * M * N) * 4                    # whole problem (C read + written)
        assert sum(rep.level_bytes) + rep.mem_bytes == pytest.approx(sum(ws))
        lv, mem = reuse.bucket_working_sets(ws, [64 * 1024, 80 * 1024, 4 << 20, 256 << 20])
        assert list(rep.level_bytes) == [float(x) for x in lv] and rep.mem_bytes == float(mem)
        assert rep.predicted_us == pytest.approx(max(rep.mfma_us, rep.mem_us) + rep.fixed_us)


@pytest.mark.parametrize("layer", range(8))
def test_conv_pick_is_the_argmin_over_the_candidate_family(layer):
    s = synth.RESNET50_SUITE(32)[layer]
    shape = tuple(s)[1:]
    cfg, rep = P.pick_conv2d(shape)
    cands = P.conv_candidates(shape)
    assert any(c.as_dict() == cfg.as_dict() for c in cands)
    best = None
    for c in cands:
        try:
            r = P.model_conv2d(shape, c)
        except P.PolydlError:
            continue
        if best is None or r.predicted_us < best:
            best = r.predicted_us
    # candidates the patch kernel cannot hold are skipped by the picker, so its optimum can only be
    # equal to or above the unconstrained one
    assert rep.predicted_us >= best - 1e-9
    assert rep.workgroups >= 1 and rep.simd_load >= 1


def test_equal_predictions_go_to_the_smaller_workgroup_tile():
    # a pointwise layer with 16 channels: every unsplit candidate sits on the same data floor
    shape = (32, 16, 56, 56, 96, 1, 1, 1, 0)
    cfg, rep = P.pick_conv2d(shape)
    tied = [c for c in P.conv_candidates(shape)
            if abs(P.model_conv2d(shape, c).predicted_us - rep.predicted_us) <= 1e-6 * rep.predicted_us]
    assert len(tied) > 3 and len({c.algo for c in tied}) > 1
    assert cfg.bm * cfg.bn == min(c.bm * c.bn for c in tied)


def test_model_monotonic_in_batch():
    s = synth.RESNET50_SUITE(32)[2]
    cfg, _ = P.pick_conv2d(tuple(s)[1:])
    t = [P.model_conv2d((n,) + tuple(s)[2:], cfg).predicted_us for n in (8, 16, 32, 64)]
    assert t == sorted(t) and t[-1] > t[0]


def test_rounds_of_resident_workgroups_show_in_the_prediction():
    # 64x64 tiles of the patch kernel on a 64 -> 64 channel 3x3 layer: 49 tiles per image.  The model
    # times the grid in rounds of the workgroups a CU holds at once, so the prediction grows with the
    # batch in steps, never decreases, and a batch that just overflows a round costs visibly more
    # than one that just fills it
    cfg = P.TileCfg(64, 64, 0, 32, 32, 1, 0, 0, 1, 4)
    t = [P.model_conv2d((n, 64, 56, 56, 64, 3, 3, 1, 1), cfg).predicted_us for n in range(1, 64)]
    assert all(b >= a - 1e-9 for a, b in zip(t, t[1:]))
    steps = [b - a for a, b in zip(t, t[1:])]
    assert max(steps) > 4 * (t[-1] - t[0]) / len(steps)        # some step is a whole round's latency
    # splitting the reduction over more workgroups than fit at once cannot be predicted free
    base = P.model_conv2d((32, 256, 14, 14, 256, 3, 3, 1, 1), P.TileCfg(64, 64, 0, 32, 32, 1, 0, 0, 1, 4))
    many = P.model_conv2d((32, 256, 14, 14, 256, 3, 3, 1, 1), P.TileCfg(64, 64, 0, 32, 32, 16, 0, 0, 1, 4))
    assert many.fixed_us > base.fixed_us


def test_filter_row_staging_in_the_model():
    # a 7x7 filter is staged one filter row at a time: its LDS stage (second working set) does not
    # hold all 49 taps of its channels
    rep7 = P.model_conv2d((8, 16, 32, 32, 64, 7, 7, 1, 3), P.TileCfg(64, 64, 0, 32, 32, 1, 0, 0, 1, 4))
    rep3 = P.model_conv2d((8, 16, 32, 32, 64, 3, 3, 1, 1), P.TileCfg(64, 64, 0, 32, 32, 1, 0, 0, 1, 4))
    assert rep7.ws[1] < rep3.ws[1] * 49 / 9


def test_sgemm_pick_valid():
    for n in synth.SGEMM_SIZES:
        cfg, rep = P.pick_sgemm(n, n, n)
        assert any(v.bm == cfg.bm and v.bn == cfg.bn and v.bk == cfg.bk for v in P.variants(1))
        assert rep.predicted_us > 0


def test_leftover_tiles_in_the_model():
    # 64x64 tiles of the gather kernel.  Layer 2 of the suite at N = 32 has 1568 tiles = 6 * 256 + 32:
    # cutting the 32 leftover tiles (raster 2) must be predicted faster than a seventh round for them.
    # A grid that is a whole number of rounds has nothing left over: same prediction either way.
    plain = P.TileCfg(64, 64, 16, 32, 32, 1, 0, 0, 0, 0)
    cut = P.TileCfg(64, 64, 16, 32, 32, 1, 0, 2, 0, 0)
    shape = (32, 64, 56, 56, 64, 3, 3, 1, 1)
    assert P.model_conv2d(shape, cut).predicted_us < P.model_conv2d(shape, plain).predicted_us - 3.0
    shape_even = (256, 64, 8, 8, 64, 3, 3, 1, 1)      # 256 * 64 pixels / 64 = 256 tiles: nothing left over
    assert P.model_conv2d(shape_even, cut).predicted_us == pytest.approx(P.model_conv2d(shape_even, plain).predicted_us)
    # a grid of less than one round is the split factor's business: left alone
    shape_most = (4, 64, 56, 56, 64, 3, 3, 1, 1)      # 196 tiles
    assert P.model_conv2d(shape_most, cut).predicted_us == pytest.approx(P.model_conv2d(shape_most, plain).predicted_us)
    # the order in which the tiles are dealt to the XCDs (rasters 1 and 3) does not enter the prediction
    plain1, cut1 = P.TileCfg(64, 64, 16, 32, 32, 1, 0, 1, 0, 0), P.TileCfg(64, 64, 16, 32, 32, 1, 0, 3, 0, 0)
    assert P.model_conv2d(shape, plain1).predicted_us == pytest.approx(P.model_conv2d(shape, plain).predicted_us)
    assert P.model_conv2d(shape, cut1).predicted_us == pytest.approx(P.model_conv2d(shape, cut).predicted_us)
    # and the gather candidates the picker ranks are all in the XCD-aware order
    assert all(c.raster in (1, 3) for c in P.conv_candidates(shape) if c.algo == 0)


def test_bf16_pick_is_a_compiled_variant_and_the_model_agrees():
    for s in synth.RESNET50_SUITE(64):
        shape = tuple(s)[1:]
        cfg, us = P.pick_conv2d_bf16(shape)
        assert cfg.algo == 1 and cfg.cb >= 2 and cfg.cb % 2 == 0 and cfg.split_k >= 1 and us > 0
        assert P.model_conv2d_bf16(shape, cfg) == pytest.approx(us)
        # no variant of the family with the same stage depth is predicted faster
        for bm, bn, wm, wn in ((64, 64, 32, 32), (64, 128, 64, 32), (128, 64, 64, 32), (128, 128, 64, 64)):
            try:
                other = P.model_conv2d_bf16(shape, P.TileCfg(bm, bn, 0, wm, wn, cfg.split_k, 1, 0, 1, cfg.cb))
            except P.PolydlError:
                continue
            assert other >= us * 0.998
    import ctypes
    assert P.lib.polydl_pick_conv2d_bf16(1, 1, 2, 2, 1, 3, 3, 1, 0, ctypes.byref(P.TileCfg()), None) == -2
    assert P.lib.polydl_model_conv2d_bf16(1, 8, 4, 4, 1, 3, 3, 1, 1, None, None) == -1


def test_argument_errors():
    import ctypes
    cfg, rep = P.TileCfg(), P.ModelReport()
    assert P.lib.polydl_pick_conv2d(1, 1, 2, 2, 1, 3, 3, 1, 0, ctypes.byref(cfg), ctypes.byref(rep)) == -2
    assert P.lib.polydl_pick_conv2d(1, 1, 4, 4, 1, 3, 3, 1, 1, None, None) == -1
    assert P.lib.polydl_pick_sgemm(0, 1, 1, ctypes.byref(cfg), None) == -2
    bad = P.TileCfg(17, 64, 16, 32, 32, 1, 0, 0, 0, 0)
    assert P.lib.polydl_model_sgemm(8, 8, 8, ctypes.byref(bad), ctypes.byref(rep)) == -3


def place_by_hand(ws, sizes):
    """Algorithm "Compute working set sizes w.r.t cache sizes", keeping where each set went."""
    room = list(sizes)
    where = [len(sizes)] * len(ws)
    for i in sorted(range(len(ws)), key=lambda i: ws[i]):
        for lv in range(len(sizes)):
            if ws[i] <= room[lv]:
                room[lv] -= ws[i]
                where[i] = lv
                break
    return where


@pytest.mark.parametrize("layer", range(8))
def test_report_placement_and_data_term_follow_the_bucketing(layer):
    # every reuse's working set is placed by the bucketing algorithm, and the data term charges the
    # bytes each reuse moves at the rate of the level it was placed in
    s = synth.RESNET50_SUITE(32)[layer]
    shape = tuple(s)[1:]
    cap, rate, mem_rate = P.model_get_levels()
    for c in P.conv_candidates(shape):
        if c.algo != 0:
            continue
        rep = P.model_conv2d(shape, c)
        ws, lvl, moved = list(rep.ws)[:rep.n_ws], list(rep.ws_level)[:rep.n_ws], list(rep.ws_traffic)[:rep.n_ws]
        assert lvl == place_by_hand(ws, cap)
        olv, omem = reuse.bucket_working_sets(ws, cap)
        assert list(rep.level_bytes) == [float(x) for x in olv] and rep.mem_bytes == float(omem)
        r = lambda lv: rate[lv] if lv < 4 else mem_rate
        refetch = moved[2] / r(max(2, lvl[2])) * 1e-3 + moved[3] / r(max(2, lvl[3])) * 1e-3
        assert rep.mem_us >= refetch * (1 - 1e-12)
        assert rep.mem_us >= moved[4] / r(max(3, lvl[4])) * 1e-3 * (1 - 1e-12)


def test_moving_a_working_set_across_a_capacity_changes_the_data_term_and_the_ranking():
    # a pointwise layer with a long reduction and many column tiles: the A panel of a tile row is
    # re-fetched by every column tile.  With the real L2 (4 MB) the column-step working set of every
    # tile fits L2; with an L2 of 2 MB the large tiles' working sets fall through to the Infinity
    # Cache, their re-fetches are charged at its (here: much lower) rate, and the ranking changes
    # from the largest tile to the largest one whose working set still fits.
    shape = (8, 2048, 28, 28, 2048, 1, 1, 1, 0)
    cap, rate, mem_rate = P.model_get_levels()
    try:
        slow = list(rate)
        slow[3] = 500.0                                  # make what falls out of L2 expensive
        P.model_set_levels(cap, slow, mem_rate)
        before = {tuple(c.as_dict().values()): P.model_conv2d(shape, c) for c in P.conv_candidates(shape) if c.algo == 0}
        pick_before, _ = P.pick_conv2d(shape)
        small = list(cap)
        small[2] = 2 << 20
        P.model_set_levels(small, slow, mem_rate)
        after = {tuple(c.as_dict().values()): P.model_conv2d(shape, c) for c in P.conv_candidates(shape) if c.algo == 0}
        pick_after, _ = P.pick_conv2d(shape)
    finally:
        P.model_set_levels(cap, rate, mem_rate)
    moved_out = [k for k in before if before[k].ws_level[2] == 2 and after[k].ws_level[2] == 3]
    stayed = [k for k in before if before[k].ws_level[2] == 2 and after[k].ws_level[2] == 2]
    assert moved_out and stayed
    for k in moved_out:
        assert after[k].mem_us > before[k].mem_us          # the same bytes, charged at a slower level
    for k in stayed:
        assert after[k].mem_us == before[k].mem_us
    assert pick_after.as_dict() != pick_before.as_dict()
    assert pick_before.bm * pick_before.bn > pick_after.bm * pick_after.bn
    assert tuple(pick_before.as_dict().values()) in moved_out
    assert after[tuple(pick_after.as_dict().values())].ws_level[2] == 2   # the new pick keeps its A panel in L2
    # and the table is back
    assert P.model_get_levels() == (cap, rate, mem_rate)


def test_level_table_validation():
    cap, rate, mem_rate = P.model_get_levels()
    with pytest.raises(P.PolydlError):
        P.model_set_levels([cap[1], cap[0], cap[2], cap[3]], rate, mem_rate)   # not ascending
    with pytest.raises(P.PolydlError):
        P.model_set_levels(cap, [0.0] + rate[1:], mem_rate)
    with pytest.raises(P.PolydlError):
        P.model_set_levels(cap, rate, -1.0)
    assert P.model_get_levels() == (cap, rate, mem_rate)


def test_candidate_lists_come_from_the_library():
    shape = tuple(synth.RESNET50_SUITE(32)[4])[1:]
    cands = P.conv_candidates(shape)
    assert len(cands) > 50 and {c.algo for c in cands} == {0, 1}
    assert len({tuple(c.as_dict().values()) for c in cands}) == len(cands)
    pick, _ = P.pick_conv2d(shape)
    assert tuple(pick.as_dict().values()) in {tuple(c.as_dict().values()) for c in cands}
    sg = P.sgemm_candidates(512, 384, 1000)
    pick, _ = P.pick_sgemm(512, 384, 1000)
    assert tuple(pick.as_dict().values()) in {tuple(c.as_dict().values()) for c in sg}
    bf = P.conv_candidates_bf16(shape)
    pick, _ = P.pick_conv2d_bf16(shape)
    assert bf and tuple(pick.as_dict().values()) in {tuple(c.as_dict().values()) for c in bf}


def test_candidates_with_the_filter_copy():
    # kind 3 of polydl_conv2d_candidates: gather variants walk the [K][R][S][C] copy tap by tap (tile
    # layout 2) exactly where that applies -- 2..63 taps and a channel count that is a multiple of
    # the variant's stage depth -- and nothing else changes
    def gather(shape, tap):
        return [c for c in P.conv_candidates(shape, tap=tap) if c.algo == 0]
    s33 = (32, 128, 28, 28, 128, 3, 3, 1, 1)
    assert all(c.layout == 0 for c in gather(s33, False))
    assert all(c.layout == 2 for c in gather(s33, True))
    assert len(P.conv_candidates(s33, tap=True)) == len(P.conv_candidates(s33))
    # 24 channels: a multiple of 8 but not of 16, so only the variant with stage depth 8 can
    c24 = gather((8, 24, 14, 14, 64, 3, 3, 1, 1), True)
    assert {c.layout for c in c24 if c.bk == 8} == {2} and {c.layout for c in c24 if c.bk == 16} == {0}
    for shape in ((32, 3, 224, 224, 64, 7, 7, 2, 3),        # three channels
                  (32, 64, 56, 56, 64, 1, 1, 1, 0),          # one tap
                  (4, 16, 20, 20, 16, 8, 8, 1, 0)):          # 64 taps
        assert all(c.layout == 0 for c in gather(shape, True)), shape
    # the cheaper gather is priced for stride 1 only
    t0, t2 = P.TileCfg(64, 64, 16, 32, 32, 1, 0, 1, 0, 0), P.TileCfg(64, 64, 16, 32, 32, 1, 2, 1, 0, 0)
    assert P.model_conv2d(s33, t2).predicted_us < P.model_conv2d(s33, t0).predicted_us
    s2 = (32, 128, 56, 56, 128, 3, 3, 2, 1)
    assert P.model_conv2d(s2, t2).predicted_us == pytest.approx(P.model_conv2d(s2, t0).predicted_us)

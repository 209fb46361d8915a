"""The library's launches can be captured into a HIP graph and replayed: no allocation or memset
node once the scratch memory of a problem exists, counters left at zero by every launch.  Each
replay is checked against the eager result, with eager work and synchronisations in between."""
import numpy as np
import pytest

import synth
from gpu_util import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2006_02230_amd as p
    yield p
    p.set_tile_override(None)


def test_captured_convolutions_replay_to_the_eager_result(P):
    import torch
    shapes = [synth.ConvShape("g3", 4, 32, 14, 14, 48, 3, 3, 1, 1),
              synth.ConvShape("g1", 4, 48, 14, 14, 40, 1, 1, 2, 0)]
    tiles = [P.TileCfg(64, 64, 0, 32, 32, 3, 0, 0, 1, 4),      # split reduction: scratch tiles + counters
             None]                                             # the picker's own choice
    work = []
    for s, t in zip(shapes, tiles):
        x, w, b = synth.conv_inputs(s, seed=61, dist="normal", bias=True)
        Pq, Qq = synth.out_hw(s)
        work.append(dict(s=s, t=t, x=dev(x), w=dev(w), b=dev(b),
                         out=torch.empty((s.N, s.K, Pq, Qq), dtype=torch.float32, device="cuda")))

    def step():
        for L in work:
            P.set_tile_override(L["t"])
            s = L["s"]
            P.conv2d_fwd(L["x"], L["w"], L["b"], out=L["out"], stride=s.stride, pad=s.pad, act="relu")
        P.set_tile_override(None)

    def same(got, want, L, tag):
        # split reductions are summed in a fixed order in every kernel: bit for bit
        assert np.array_equal(got, want), (tag, L["s"].name)

    step()                      # eager: also creates the scratch buffers of the side stream below
    torch.cuda.synchronize()
    eager = [host(L["out"]) for L in work]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()                  # scratch memory is per stream: allocate it before capturing
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(4):
        for L in work:
            L["out"].fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for L, want in zip(work, eager):
            same(host(L["out"]), want, L, rep)
        step()                  # eager work on the default stream between replays
        torch.cuda.synchronize()
        for L, want in zip(work, eager):
            same(host(L["out"]), want, L, (rep, "eager"))


def test_scratch_growth_between_capture_and_replay(P):
    # a graph keeps the scratch addresses it was recorded with; a later, larger split reduction on
    # the capture stream makes the library allocate a larger buffer, and the recorded one must stay
    # valid: the replay still gives the eager result
    import torch
    small = synth.ConvShape("gs", 2, 32, 10, 10, 48, 3, 3, 1, 1)
    large = synth.ConvShape("gl", 8, 64, 28, 28, 256, 3, 3, 1, 1)
    tile = P.TileCfg(64, 64, 16, 32, 32, 4, 0, 0, 0, 0)
    xs, ws, bs = synth.conv_inputs(small, seed=62, dist="normal", bias=True)
    xl, wl, bl = synth.conv_inputs(large, seed=63, dist="normal", bias=True)
    dxs, dws, dbs = dev(xs), dev(ws), dev(bs)
    dxl, dwl, dbl = dev(xl), dev(wl), dev(bl)
    out = torch.empty((small.N, small.K, 10, 10), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    P.set_tile_override(tile)
    with torch.cuda.stream(side):
        P.conv2d_fwd(dxs, dws, dbs, out=out, stride=1, pad=1, act="relu")      # scratch of this stream exists now
        torch.cuda.synchronize()
        eager = host(out)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            P.conv2d_fwd(dxs, dws, dbs, out=out, stride=1, pad=1, act="relu")
        torch.cuda.synchronize()
        # 64 x the partial tiles of the captured call, on the same stream: the buffer has to grow
        big = P.conv2d_fwd(dxl, dwl, dbl, stride=1, pad=1, act="relu")
        torch.cuda.synchronize()
        # fresh allocations that may land where a freed buffer would have been
        junk = [torch.full((1 << 20,), float("nan"), device="cuda") for _ in range(8)]
        torch.cuda.synchronize()
    for rep in range(3):
        out.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(host(out), eager), rep
        with torch.cuda.stream(side):
            again = P.conv2d_fwd(dxl, dwl, dbl, stride=1, pad=1, act="relu")
            torch.cuda.synchronize()
        assert np.array_equal(host(again), host(big)), rep
    assert all(bool(torch.isnan(j).all()) for j in junk)     # no replay wrote into memory it does not own
    P.set_tile_override(None)


def test_capture_that_would_allocate_is_refused(P):
    # the first split reduction on a stream allocates its scratch memory; under capture that is
    # not allowed, so the call says so and records nothing; the capture itself stays usable
    import torch
    s = synth.ConvShape("gc", 2, 32, 10, 10, 48, 3, 3, 1, 1)
    x, w, b = synth.conv_inputs(s, seed=64, dist="normal", bias=True)
    dx, dw, db = dev(x), dev(w), dev(b)
    out = torch.zeros((s.N, s.K, 10, 10), dtype=torch.float32, device="cuda")
    fresh = torch.cuda.Stream()            # no library call has run on this stream yet
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(fresh):
        with torch.cuda.graph(graph, stream=fresh):
            P.set_tile_override(P.TileCfg(64, 64, 16, 32, 32, 4, 0, 0, 0, 0))
            with pytest.raises(P.PolydlError) as err:
                P.conv2d_fwd(dx, dw, db, out=out, stride=1, pad=1, act="relu")
            assert err.value.status == -3
            P.set_tile_override(P.TileCfg(64, 64, 16, 32, 32, 1, 0, 0, 0, 0))    # unsplit: no scratch memory
            P.conv2d_fwd(dx, dw, db, out=out, stride=1, pad=1, act="relu")
    P.set_tile_override(None)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    import oracle
    want, ab = oracle.conv2d_fwd(x, w, bias=b, stride=1, pad=1, act="relu")
    assert oracle.scaled_error(host(out), want, ab) <= 1e-5

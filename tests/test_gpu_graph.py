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

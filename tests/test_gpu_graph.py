"""The whole path captured into a HIP graph (pipeline.GraphedPath) against the eager calls: every replay must
give the eager result bit for bit, also with eager work of the same library and synchronisations between the
replays and after the inputs were rewritten in place."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2209_13027_amd.workloads import WORKLOADS, make_views  # noqa: E402
from paper_2209_13027_amd import pipeline  # noqa: E402


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def eager(ctx, wl, d1, d2, dc, fused):
    model = pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2)
    feat = pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride, fused=fused)
    ctx.status()
    return [f.clone() for f in model["filters"]], [r.clone() for r in model["rho"]], feat.clone()


def same(a, b):
    return all(torch.equal(x, y) for x, y in zip(a, b))


@pytest.mark.parametrize("name,mpc,fused", [("tiny", None, False), ("tiny", None, True), ("small_face", 2, False)])
def test_graph_replays_equal_eager(name, mpc, fused):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2209_13027_amd.binding import Context
    wl = WORKLOADS[name]
    v1, v2, cls = make_views(wl, max_per_class=mpc)
    d1, d2, dc = dev(v1), dev(v2), dev(cls)
    ctx = Context(0)
    want = eager(ctx, wl, d1, d2, dc, fused)
    g = pipeline.GraphedPath(d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2, wl.block, wl.stride, fused=fused)
    for rep in range(3):
        g.feat.zero_()
        for f in g.filters:
            f.zero_()
        torch.cuda.synchronize()
        g.replay()
        g.status()
        torch.cuda.synchronize()
        assert same(g.filters, want[0]), rep
        assert same(g.rho, want[1]), rep
        assert torch.equal(g.feat, want[2]), rep
        # eager work of the same library between the replays
        again = eager(ctx, wl, d1, d2, dc, fused)
        assert same(again[0], want[0]) and torch.equal(again[2], want[2])
    # new data in the same buffers: the replay follows it
    d1.copy_(torch.flip(d1, dims=[0]))
    d2.copy_(torch.flip(d2, dims=[0]))
    dc.copy_(torch.flip(dc, dims=[0]))
    torch.cuda.synchronize()
    want2 = eager(ctx, wl, d1, d2, dc, fused)
    g.replay()
    g.status()
    torch.cuda.synchronize()
    assert same(g.filters, want2[0]) and same(g.rho, want2[1]) and torch.equal(g.feat, want2[2])
    assert not torch.equal(want2[2], want[2])
    g.close()
    ctx.close()

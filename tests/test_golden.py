"""The stored results of the CPU oracle on the `tiny` workload (tests/golden/tiny_two_stage.txt, written by
tests/golden/make_golden.py from oracle/ alone): the oracle must keep reproducing them (a change of its arithmetic
shows up here first), and the HIP path must meet them to the bars of the path -- filter cosine >= 0.9999 where the
canonical correlations are separated, histograms <= 1e-3 relative L1 (Eq. 2-12)."""
import os

import numpy as np
import pytest

from paper_2209_13027_amd.workloads import WORKLOADS, make_views

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_two_stage.txt")


def load_golden():
    g = {"rho": {}, "gap": {}, "F": {}, "codes": {}, "sample": []}
    for line in open(GOLDEN):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "shape":
            g["shape"] = {t[i]: int(t[i + 1]) for i in range(1, len(t), 2)}
        elif t[0] in ("rho", "gap"):
            g[t[0]][int(t[1])] = np.array([float(x) for x in t[2:]])
        elif t[0] == "F":
            g["F"][(int(t[1]), int(t[2]), int(t[3]))] = np.array([float(x) for x in t[4:]])
        elif t[0] == "codes":
            g["codes"][(int(t[1]), int(t[2]))] = np.array([int(x) for x in t[3:]], dtype=np.int64)
        elif t[0] == "sample":
            g["sample"].append((tuple(int(x) for x in t[1:7]), int(t[7])))
    return g


def cosine(a, b):
    return float(np.dot(a, b) / (np.linalg.norm(a) * np.linalg.norm(b)))


def check_shape(g, wl, m):
    s = g["shape"]
    assert (s["images"], s["h"], s["w"], s["k"], s["L1"], s["L2"], s["block"], s["stride"]) == \
           (m, wl.h, wl.w, wl.k, wl.L1, wl.L2, wl.block, wl.stride)


def test_oracle_reproduces_golden(oracle):
    g = load_golden()
    wl = WORKLOADS["tiny"]
    v1, v2, cls = make_views(wl)
    check_shape(g, wl, v1.shape[0])
    res = oracle.two_stage(v1, v2, cls, wl.n_classes, wl.k, wl.L1, wl.L2, wl.block, wl.stride)
    for s in (1, 2):
        st = res["stage%d" % s]
        assert np.allclose(st["rho"], g["rho"][s], rtol=1e-9)
        assert np.allclose(st["gap"], g["gap"][s], rtol=1e-4)
        for d in (1, 2):
            F = st["F%d" % d].reshape(st["F%d" % d].shape[0], -1)
            for l in range(F.shape[0]):
                assert np.allclose(F[l], g["F"][(s, d, l)], rtol=0, atol=1e-8 * np.abs(F[l]).max())
    codes = res["hist"].sum(axis=(0, 3, 4))
    for (d, gi), want in g["codes"].items():
        assert np.array_equal(codes[d, gi], want)
    for idx, want in g["sample"]:
        assert int(res["hist"][idx]) == want
    assert len(g["sample"]) == 48 and len(g["codes"]) == 2 * wl.L1


@pytest.mark.gpu
def test_hip_path_meets_golden():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2209_13027_amd.binding import Context
    from paper_2209_13027_amd import pipeline
    g = load_golden()
    wl = WORKLOADS["tiny"]
    v1, v2, cls = make_views(wl)
    check_shape(g, wl, v1.shape[0])
    ctx = Context(0)
    try:
        d1, d2, dc = (torch.from_numpy(np.ascontiguousarray(a)).cuda() for a in (v1, v2, cls))
        model = pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2)
        feat = pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride)
        ctx.status()
        hist = feat.cpu().numpy().astype(np.int64)
        for s in (1, 2):
            rho = model["rho"][s - 1].cpu().numpy()
            assert np.allclose(rho, g["rho"][s], rtol=1e-5)
            for d in (1, 2):
                W = model["filters"][2 * (s - 1) + d - 1].cpu().numpy().reshape(-1, wl.k * wl.k).astype(np.float64)
                for l in range(W.shape[0]):
                    if g["gap"][s][l] > 1e-3:
                        assert cosine(W[l], g["F"][(s, d, l)]) >= 0.9999, (s, d, l)
    finally:
        ctx.close()
    codes = hist.sum(axis=(0, 3, 4))
    total = diff = 0
    for (d, gi), want in g["codes"].items():
        total += int(want.sum())
        diff += int(np.abs(codes[d, gi] - want).sum())
    assert diff <= 1e-3 * total
    off = sum(abs(int(hist[idx]) - want) for idx, want in g["sample"])
    assert off <= max(2, 1e-2 * sum(want for _, want in g["sample"]))

"""GPU parity of ddcca_learn_next_stage_filters (second-stage learning from the first stage's inputs, maps convolved
batch by batch, class-conditioned sum images by linearity of the convolution) against

  * the materialised route through the same library (ddcca_apply_stage + ddcca_learn_stage_filters): C11, C22, C12
    equal up to the summation order that follows the batch split (these small cases: fp64 only), Cw and CT up to
    the fp32 rounding of the sum images;
  * the fp64 oracle, to the bars of the path: matrices <= 1e-4 relative (Frobenius), filters cosine >= 0.9999 where
    the canonical correlations are separated, end-to-end histograms <= 1e-3 relative L1.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2209_13027_amd.workloads import WORKLOADS, make_views  # noqa: E402
from paper_2209_13027_amd import pipeline  # noqa: E402


@pytest.fixture(scope="module")
def ctx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2209_13027_amd.binding import Context
    c = Context(0)
    yield c
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel_fro(a, b):
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def cosines(got, want):
    g = got.reshape(got.shape[0], -1).astype(np.float64)
    r = want.reshape(want.shape[0], -1).astype(np.float64)
    return np.sum(g * r, axis=1) / (np.linalg.norm(g, axis=1) * np.linalg.norm(r, axis=1))


def rand_problem(seed, n_img, h, w, n_cls):
    rng = np.random.default_rng(seed)
    # smooth + noise so that the first stage has separated canonical correlations
    base = rng.standard_normal((n_img, h + 4, w + 4)).astype(np.float32)
    smooth = sum(base[:, dy:dy + h, dx:dx + w] for dy in range(5) for dx in range(5)) / 5.0
    v1 = (smooth + 0.3 * rng.standard_normal((n_img, h, w))).astype(np.float32)
    v2 = (0.7 * smooth + 0.5 * rng.standard_normal((n_img, h, w)) + 2.0).astype(np.float32)
    cls = (np.arange(n_img) % n_cls).astype(np.int32)
    rng.shuffle(cls)
    return v1, v2, cls


def matrices_of_last_learning(ctx, k):
    return {n: v.cpu().numpy() for n, v in ctx.corr_export(k).items()}


@pytest.mark.parametrize("n_img,G_in,h,w,k,L1,L2,n_cls,batch", [
    (12, 1, 32, 32, 5, 4, 4, 3, 0),        # one batch
    (12, 1, 32, 32, 5, 4, 4, 3, 5),        # ragged batches 5 + 5 + 2
    (7, 1, 45, 70, 7, 8, 8, 2, 3),         # k = 7, ragged tiles
    (5, 1, 24, 40, 3, 3, 2, 5, 1),         # every sample its own class and its own batch
    (6, 1, 40, 36, 9, 8, 8, 1, 4),         # k = 9, a single class
    (6, 3, 28, 36, 5, 4, 4, 2, 4),         # inputs that are themselves maps of an earlier stage (3 per sample)
])
def test_streamed_equals_materialised(ctx, n_img, G_in, h, w, k, L1, L2, n_cls, batch):
    v1, v2, cls = rand_problem(900 + k + n_img, n_img * G_in, h, w, n_cls)
    cls = cls[:n_img].copy()
    d1, d2, dc = dev(v1), dev(v2), dev(cls)
    W1a, W2a, _ = ctx.learn_stage_filters(d1, d2, dc, G_in, h, w, n_cls, k, L1)
    y1, y2 = ctx.apply_stage(d1, W1a), ctx.apply_stage(d2, W2a)
    Wm1, Wm2, rho_m = ctx.learn_stage_filters(y1, y2, dc, G_in * L1, h, w, n_cls, k, L2)
    mats_m = matrices_of_last_learning(ctx, k)
    Ws1, Ws2, rho_s = ctx.learn_next_stage_filters(d1, d2, dc, G_in, h, w, n_cls, W1a, W2a, k, L2,
                                                   batch_images=batch)
    mats_s = matrices_of_last_learning(ctx, k)
    ctx.status()
    for name in ("C11", "C22", "C12"):
        assert rel_fro(mats_s[name], mats_m[name]) <= 1e-13, name
    for name in ("Cw", "CT"):
        assert rel_fro(mats_s[name], mats_m[name]) <= 1e-6, name
    assert np.allclose(rho_s.cpu().numpy(), rho_m.cpu().numpy(), rtol=1e-5)
    # filters: compare where the leading correlations are separated (ratio of neighbours below 0.999)
    rho = rho_m.cpu().numpy()
    sep = np.ones(L2, dtype=bool)
    sep[1:] &= rho[1:] < 0.999 * rho[:-1]
    sep[:-1] &= rho[1:] < 0.999 * rho[:-1]
    if sep.any():
        assert cosines(Ws1.cpu().numpy(), Wm1.cpu().numpy())[sep].min() >= 1 - 1e-6
        assert cosines(Ws2.cpu().numpy(), Wm2.cpu().numpy())[sep].min() >= 1 - 1e-6


def test_streamed_matrices_against_oracle(ctx, oracle):
    n_img, h, w, k, L1, n_cls = 9, 30, 44, 5, 4, 3
    v1, v2, cls = rand_problem(77, n_img, h, w, n_cls)
    d1, d2, dc = dev(v1), dev(v2), dev(cls)
    W1a, W2a, _ = ctx.learn_stage_filters(d1, d2, dc, 1, h, w, n_cls, k, L1)
    ctx.learn_next_stage_filters(d1, d2, dc, 1, h, w, n_cls, W1a, W2a, k, 4, batch_images=4)
    got = matrices_of_last_learning(ctx, k)
    # the oracle's own convolution of the same inputs with the filters the library learned, then its matrices
    y1 = oracle.conv(v1.astype(np.float64), W1a.cpu().numpy().astype(np.float64)).reshape(-1, h, w)
    y2 = oracle.conv(v2.astype(np.float64), W2a.cpu().numpy().astype(np.float64)).reshape(-1, h, w)
    grp = np.tile(np.arange(L1, dtype=np.int32), n_img)
    want = oracle.stage_matrices(y1, y2, np.repeat(cls, L1), grp, n_cls, L1, k)
    for name in ("C11", "C22", "C12", "Cw", "CT"):
        assert rel_fro(got[name], want[name]) <= 1e-4, name
        assert rel_fro(got[name], want[name]) <= 5e-6, (name, "looser than expected for fp32 maps and products")


def test_streamed_learning_with_three_piece_arithmetic(oracle):
    """The same call with the Gram and the convolution on three-piece bf16 operands: the bars of the path."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2209_13027_amd.binding import (Context, OPT_CONV_ARITH, CONV_BF16X3, OPT_GRAM_ARITH, GRAM_BF16X3)
    c = Context(0)
    c.set_option(OPT_CONV_ARITH, CONV_BF16X3)
    c.set_option(OPT_GRAM_ARITH, GRAM_BF16X3)
    n_img, h, w, k, L1, n_cls = 8, 36, 50, 7, 8, 4
    v1, v2, cls = rand_problem(31, n_img, h, w, n_cls)
    d1, d2, dc = dev(v1), dev(v2), dev(cls)
    W1a, W2a, _ = c.learn_stage_filters(d1, d2, dc, 1, h, w, n_cls, k, L1)
    c.learn_next_stage_filters(d1, d2, dc, 1, h, w, n_cls, W1a, W2a, k, 8, batch_images=3)
    got = matrices_of_last_learning(c, k)
    c.status()
    y1 = oracle.conv(v1.astype(np.float64), W1a.cpu().numpy().astype(np.float64)).reshape(-1, h, w)
    y2 = oracle.conv(v2.astype(np.float64), W2a.cpu().numpy().astype(np.float64)).reshape(-1, h, w)
    grp = np.tile(np.arange(L1, dtype=np.int32), n_img)
    want = oracle.stage_matrices(y1, y2, np.repeat(cls, L1), grp, n_cls, L1, k)
    for name in ("C11", "C22", "C12", "Cw", "CT"):
        assert rel_fro(got[name], want[name]) <= 1e-4, name
        assert rel_fro(got[name], want[name]) <= 5e-6, (name, "looser than expected")
    c.close()


def test_validation(ctx):
    from paper_2209_13027_amd.binding import DdccaError
    v1, v2, cls = rand_problem(5, 4, 16, 16, 2)
    d1, d2, dc = dev(v1), dev(v2), dev(cls)
    W = torch.zeros((4, 5, 5), dtype=torch.float32, device="cuda")
    with pytest.raises(DdccaError):
        ctx.learn_next_stage_filters(d1, d2, dc, 1, 16, 16, 2, W, W, 5, 4, batch_images=-1)
    Wbig = torch.zeros((25, 5, 5), dtype=torch.float32, device="cuda")        # L_prev > k*k - 1
    with pytest.raises(DdccaError):
        ctx.learn_next_stage_filters(d1, d2, dc, 1, 16, 16, 2, Wbig, Wbig, 5, 4)
    with pytest.raises(ValueError):
        ctx.learn_next_stage_filters(d1, d2, dc, 2, 16, 16, 2, W, W, 5, 4)    # views do not hold G_in = 2 maps


@pytest.mark.parametrize("name,mpc,batch", [("tiny", None, 16), ("small_face", 2, 0)])
def test_end_to_end_with_streamed_learning(ctx, oracle, name, mpc, batch):
    wl = WORKLOADS[name]
    v1, v2, cls = make_views(wl, max_per_class=mpc)
    d1, d2, dc = dev(v1), dev(v2), dev(cls)
    model = pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2, streamed=True, batch_images=batch)
    feat = pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride)
    ctx.status()
    ref = oracle.two_stage(v1, v2, cls, wl.n_classes, wl.k, wl.L1, wl.L2, wl.block)
    refs = [ref["stage1"]["W1"], ref["stage1"]["W2"], ref["stage2"]["W1"], ref["stage2"]["W2"]]
    gaps = [ref["stage1"]["gap"], ref["stage1"]["gap"], ref["stage2"]["gap"], ref["stage2"]["gap"]]
    for W, R, gap in zip(model["filters"], refs, gaps):
        assert cosines(W.cpu().numpy(), R)[gap > 1e-3].min() >= 0.9999
    assert np.allclose(model["rho"][1].cpu().numpy(), ref["stage2"]["rho"], rtol=1e-4)
    got = feat.cpu().numpy()
    assert got.shape == ref["hist"].shape
    l1 = np.abs(got.astype(np.int64) - ref["hist"]).sum() / ref["hist"].sum()
    assert l1 <= 1e-3, l1


@pytest.mark.parametrize("m,h,w,k,L1,L2,n_cls", [
    (3, 41, 4, 3, 1, 8, 2),     # an image as wide as one step of the matrix instruction; all D - 1 pairs of the stage
    (4, 30, 3, 3, 2, 8, 2),     # narrower than one step; as wide as the patch
    (4, 5, 37, 5, 2, 24, 2),    # the same lying down, k = 5, all D - 1 pairs
])
def test_streamed_route_on_narrow_images_with_every_pair(ctx, oracle, m, h, w, k, L1, L2, n_cls):
    """Images narrower than (or as narrow as) one K-step of the matrix instruction and L = D - 1, the largest filter
    count a stage has: on such an image most patches lie on the border, C_dd has small eigenvalues next to the
    ridge, and the last pairs are the most sensitive ones of the stage.  Both second-stage routes (streamed from the
    inputs, materialised maps) against the oracle at the bars of the path: rho to 1e-4 of the leading correlation
    (the two routes differ from each other by a relative 1e-5 in the LAST correlation of such a case, which is its
    conditioning and not a defect), filter cosines where the correlations are separated."""
    v1, v2, cls = rand_problem(27000 + h + w, m, h, w, n_cls)
    d1, d2, dc = dev(v1), dev(v2), dev(cls)
    ref = oracle.learn_two_stage(v1, v2, cls, n_cls, k, L1, L2)
    for streamed in (True, False):
        model = pipeline.fit(ctx, d1, d2, dc, n_cls, k, L1, L2, streamed=streamed)
        ctx.status()
        for s, L in ((0, L1), (1, L2)):
            r = ref["stage%d" % (s + 1)]
            rho = model["rho"][s].cpu().numpy()
            assert np.all(np.isfinite(rho))
            assert np.abs(rho - r["rho"]).max() <= 1e-4 * r["rho"][0], (streamed, s, rho, r["rho"])
            ok = r["gap"] > 1e-3
            for d in range(2):
                cos = cosines(model["filters"][2 * s + d].cpu().numpy(), r["W%d" % (d + 1)])
                if ok.any():
                    assert cos[ok].min() >= 0.9999, (streamed, s, d, cos, r["gap"])


@pytest.mark.parametrize("arith", ["fp32", "bf16x3"])
@pytest.mark.parametrize("n_img,G_in,h,w,k,L1,n_cls", [
    (9, 1, 30, 44, 5, 4, 3),       # ragged tiles in both directions
    (7, 1, 45, 70, 7, 8, 2),       # k = 7
    (5, 1, 24, 40, 3, 3, 5),       # k = 3
    (4, 1, 40, 36, 9, 8, 1),       # k = 9
    (3, 1, 20, 300, 7, 5, 2),      # wider than one tile: three column tiles
    (3, 1, 50, 150, 9, 8, 2),      # k = 9 over two column tiles, four row tiles
    (6, 3, 28, 36, 5, 4, 2),       # inputs that are themselves maps (3 per sample)
    (4, 1, 30, 3, 3, 2, 2),        # as wide as the patch
    (2, 1, 3, 2, 5, 3, 1),         # smaller than the patch
])
def test_recomputed_maps_against_oracle_and_streamed(oracle, arith, n_img, G_in, h, w, k, L1, n_cls):
    """DDCCA_MAPS_RECOMPUTED: the Gram kernel forms every tile of the previous stage's maps from the input tile it
    holds (Section II-B on Section II-A); the matrices against the oracle's convolution (Eq. 6) and matrices of the
    same inputs at the bars of the path, and against the streamed route of the same library."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2209_13027_amd.binding import (Context, OPT_GRAM_ARITH, GRAM_BF16X3, OPT_NEXT_STAGE_MAPS,
                                              MAPS_RECOMPUTED, MAPS_STREAMED)
    c = Context(0)
    try:
        if arith == "bf16x3":
            c.set_option(OPT_GRAM_ARITH, GRAM_BF16X3)
        v1, v2, cls = rand_problem(4100 + 7 * k + w, n_img * G_in, h, w, n_cls)
        cls = cls[:n_img].copy()
        d1, d2, dc = dev(v1), dev(v2), dev(cls)
        rng = np.random.default_rng(k + h)
        Wa = rng.standard_normal((2, L1, k, k)).astype(np.float32)
        W1a, W2a = dev(Wa[0]), dev(Wa[1])
        L2 = min(4, k * k - 1)
        c.set_option(OPT_NEXT_STAGE_MAPS, MAPS_STREAMED)
        c.learn_next_stage_filters(d1, d2, dc, G_in, h, w, n_cls, W1a, W2a, k, L2)
        streamed = matrices_of_last_learning(c, k)
        c.set_option(OPT_NEXT_STAGE_MAPS, MAPS_RECOMPUTED)
        _, _, rho = c.learn_next_stage_filters(d1, d2, dc, G_in, h, w, n_cls, W1a, W2a, k, L2)
        got = matrices_of_last_learning(c, k)
        c.status()
        y1 = oracle.conv(v1.astype(np.float64), Wa[0].astype(np.float64)).reshape(-1, h, w)
        y2 = oracle.conv(v2.astype(np.float64), Wa[1].astype(np.float64)).reshape(-1, h, w)
        G = G_in * L1
        grp = np.tile(np.arange(G, dtype=np.int32), n_img)
        want = oracle.stage_matrices(y1, y2, np.repeat(cls, G), grp, n_cls, G, k)
        assert np.all(np.isfinite(rho.cpu().numpy()))
        for name in ("C11", "C22", "C12", "Cw", "CT"):
            assert rel_fro(got[name], want[name]) <= 1e-4, name
            assert rel_fro(got[name], want[name]) <= 5e-6, (name, "looser than expected for fp32 maps and products")
            assert rel_fro(got[name], streamed[name]) <= 5e-6, (name, "against the streamed route")
    finally:
        c.close()


def test_recomputed_maps_end_to_end(oracle):
    """Two-stage learning with the second stage's maps recomputed in the Gram kernel, then extraction, on small_face
    (two images per class): filters and histograms against the oracle at the bars of the path."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2209_13027_amd.binding import Context, OPT_NEXT_STAGE_MAPS, MAPS_RECOMPUTED
    wl = WORKLOADS["small_face"]
    v1, v2, cls = make_views(wl, max_per_class=2)
    d1, d2, dc = dev(v1), dev(v2), dev(cls)
    c = Context(0)
    try:
        c.set_option(OPT_NEXT_STAGE_MAPS, MAPS_RECOMPUTED)
        model = pipeline.fit(c, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2, streamed=True)
        feat = pipeline.extract(c, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride)
        c.status()
    finally:
        c.close()
    ref = oracle.two_stage(v1, v2, cls, wl.n_classes, wl.k, wl.L1, wl.L2, wl.block)
    refs = [ref["stage1"]["W1"], ref["stage1"]["W2"], ref["stage2"]["W1"], ref["stage2"]["W2"]]
    gaps = [ref["stage1"]["gap"], ref["stage1"]["gap"], ref["stage2"]["gap"], ref["stage2"]["gap"]]
    for W, R, gap in zip(model["filters"], refs, gaps):
        assert cosines(W.cpu().numpy(), R)[gap > 1e-3].min() >= 0.9999
    assert np.allclose(model["rho"][1].cpu().numpy(), ref["stage2"]["rho"], rtol=1e-4)
    got = feat.cpu().numpy()
    l1 = np.abs(got.astype(np.int64) - ref["hist"]).sum() / ref["hist"].sum()
    assert l1 <= 1e-3, l1


def test_recomputed_maps_option_falls_back_where_it_does_not_apply():
    """k_prev != k, or the lag-structured Gram: the call proceeds as with streamed maps (bit for bit)."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2209_13027_amd.binding import (Context, DdccaError, OPT_GRAM_ARITH, GRAM_LAG_FP32, GRAM_FP32,
                                              OPT_NEXT_STAGE_MAPS, MAPS_RECOMPUTED, MAPS_STREAMED)
    c = Context(0)
    try:
        v1, v2, cls = rand_problem(515, 6, 26, 34, 2)
        d1, d2, dc = dev(v1), dev(v2), dev(cls)
        rng = np.random.default_rng(3)
        for k_prev, k, arith in ((5, 3, GRAM_FP32), (5, 5, GRAM_LAG_FP32)):
            Wa = rng.standard_normal((2, 4, k_prev, k_prev)).astype(np.float32)
            c.set_option(OPT_GRAM_ARITH, arith)
            out = []
            for mode in (MAPS_STREAMED, MAPS_RECOMPUTED):
                c.set_option(OPT_NEXT_STAGE_MAPS, mode)
                c.learn_next_stage_filters(d1, d2, dc, 1, 26, 34, 2, dev(Wa[0]), dev(Wa[1]), k, 3)
                out.append(matrices_of_last_learning(c, k))
            for name in ("C11", "C22", "C12", "Cw", "CT"):
                assert np.array_equal(out[0][name], out[1][name]), (k_prev, k, name)
        with pytest.raises(DdccaError):
            c.set_option(OPT_NEXT_STAGE_MAPS, 2)
        c.status()
    finally:
        c.close()

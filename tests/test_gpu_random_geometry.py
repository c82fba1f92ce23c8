"""GPU parity on seeded random geometries: the calls of the C ABI against the CPU oracle on shapes nobody picked by
hand.  The hand-written cases of the other files aim at the tile edges the kernels are known to have; these draw
image sizes, patch sides, filter counts, blocks and strides from a seeded generator (every draw inside what the
calls accept) so that a launch heuristic or a ragged tail the hand-written list misses still meets the oracle.
Each case prints its geometry before it touches the GPU.  Bars as in the other parity tests: histograms bit-exact
on identical fp32 maps, maps within 2e-6 of the filter's l1 norm times the largest pixel, correlation matrices
within 2e-6 relative Frobenius error (1e-5 with three-piece bf16 operands), fused last stage identical to the
unfused calls and equal to the oracle's counts except for pixels whose map value is within rounding of zero."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2209_13027_amd.binding as b
    return b


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context(0)
    yield c
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def say(*what):
    print(*what, flush=True)


def draw_block(rng, h_max, w_max):
    """A block and a stride: square or rectangular, overlapping, touching or with gaps."""
    bh = int(rng.integers(1, min(24, h_max) + 1))
    bw = bh if rng.random() < 0.5 else int(rng.integers(1, min(24, w_max) + 1))
    bw = min(bw, w_max)
    sy = int(rng.integers(1, bh + 3))
    sx = sy if rng.random() < 0.5 else int(rng.integers(1, bw + 3))
    return (bh, bw), (sy, sx)


def draw_size(rng, lo_h, lo_w):
    """Mostly small maps, now and then a wide or a tall one (several tiles, the kernels for wide maps)."""
    kind = rng.random()
    if kind < 0.6:
        return lo_h + int(rng.integers(0, 60)), lo_w + int(rng.integers(0, 70))
    if kind < 0.85:
        return lo_h + int(rng.integers(0, 20)), max(lo_w, int(rng.integers(130, 340)))
    return max(lo_h, int(rng.integers(100, 200))), lo_w + int(rng.integers(0, 40))


# ------------------------------------------------------------------ hashing + block histograms (Eq. 7-9)
@pytest.mark.parametrize("case", range(24))
def test_hash_histogram_random_geometry(ctx, oracle, case):
    rng = np.random.default_rng(51000 + case)
    L2 = int(rng.integers(1, 13))
    h0, w0 = draw_size(rng, 1, 1)
    block, stride = draw_block(rng, h0, w0)
    h, w = max(h0, block[0]), max(w0, block[1])
    if rng.random() < 0.5:
        w = (w + 3) // 4 * 4                                  # rows that can be read four pixels at a time
    n = int(rng.integers(1, 4))
    say("hash_histogram", dict(n=n, L2=L2, h=h, w=w, block=block, stride=stride))
    Z = rng.standard_normal((n, L2, h, w)).astype(np.float32)
    Z[rng.random(Z.shape) < 0.03] = 0.0
    got = ctx.hash_histogram(dev(Z), block, stride).cpu().numpy()
    ctx.status()
    want = oracle.block_hist(oracle.hash_maps(Z), block, stride, 1 << L2)
    assert got.shape == want.shape
    assert np.array_equal(got.astype(np.int64), want)


# ------------------------------------------------------------------ stage convolution (Eq. 6)
@pytest.mark.parametrize("arith", ["fp32", "bf16x3"])
@pytest.mark.parametrize("case", range(12))
def test_apply_stage_random_geometry(lib, ctx, oracle, case, arith):
    rng = np.random.default_rng(52000 + case)
    k = int(rng.choice([3, 5, 7, 9]))
    L = int(rng.integers(1, 17))
    h, w = draw_size(rng, 1, 1)
    n = int(rng.integers(1, 4))
    say("apply_stage", arith, dict(n=n, h=h, w=w, k=k, L=L))
    V = (rng.standard_normal((n, h, w)) * 3 + rng.uniform(-2, 2)).astype(np.float32)
    F = rng.standard_normal((L, k, k)).astype(np.float32)
    ctx.set_option(lib.OPT_CONV_ARITH, lib.CONV_FP32 if arith == "fp32" else lib.CONV_BF16X3)
    try:
        got = ctx.apply_stage(dev(V), dev(F)).cpu().numpy()
        ctx.status()
    finally:
        ctx.set_option(lib.OPT_CONV_ARITH, lib.CONV_AUTO)
    want = oracle.conv(V, F)
    scale = np.abs(F).sum(axis=(1, 2)).max() * np.abs(V).max()
    assert got.shape == want.shape
    assert np.abs(got - want).max() <= 2e-6 * scale


# ------------------------------------------------------------------ correlation matrices (Eq. 13-15)
GRAM_BAR = {"fp32": 2e-6, "bf16x3": 1e-5, "lag": 2e-6}


@pytest.mark.parametrize("arith", ["fp32", "bf16x3", "lag"])
@pytest.mark.parametrize("case", range(10))
def test_corr_matrices_random_geometry(lib, oracle, case, arith):
    rng = np.random.default_rng(53000 + case)
    k = int(rng.choice([3, 5, 7, 9]))
    G = int(rng.integers(1, 4))
    n_img = int(rng.integers(1, 7))
    n_cls = int(rng.integers(1, 4))
    h, w = draw_size(rng, 2, 2)
    h = min(h, 64)
    say("corr", arith, dict(n_img=n_img, G=G, h=h, w=w, k=k, n_cls=n_cls))
    V1 = rng.standard_normal((n_img * G, h, w)).astype(np.float32)
    V2 = (np.abs(rng.standard_normal((n_img * G, h, w))) * 2 + 5).astype(np.float32)
    cls = rng.integers(0, n_cls, size=n_img).astype(np.int32)
    cut = int(rng.integers(0, n_img + 1))                      # two accumulate calls (Eq. 15)
    c = lib.Context(0)
    try:
        c.set_option(lib.OPT_GRAM_ARITH, {"fp32": lib.GRAM_FP32, "bf16x3": lib.GRAM_BF16X3,
                                          "lag": lib.GRAM_LAG_FP32}[arith])
        c.corr_begin(k, n_cls, G, h, w)
        d1, d2, dc = dev(V1), dev(V2), dev(cls)
        for a, b in ((0, cut), (cut, n_img)):
            c.corr_accumulate(d1[a * G:b * G], d2[a * G:b * G], dc[a:b])
        got = {name: m.cpu().numpy() for name, m in c.corr_export(k).items()}
        c.status()
    finally:
        c.close()
    grp = np.tile(np.arange(G, dtype=np.int32), n_img)
    want = oracle.stage_matrices(V1, V2, np.repeat(cls, G), grp, n_cls, G, k)
    for name in ("C11", "C22", "C12", "Cw", "CT"):
        err = np.linalg.norm(got[name] - want[name]) / np.linalg.norm(want[name])
        assert err <= GRAM_BAR[arith], (name, err)


# ------------------------------------------------------------------ fused last stage (Eq. 6-9 in one call)
@pytest.mark.parametrize("arith", ["fp32", "bf16x3"])
@pytest.mark.parametrize("case", range(12))
def test_apply_stage_hash_random_geometry(lib, ctx, oracle, case, arith):
    rng = np.random.default_rng(54000 + case)
    k = int(rng.choice([3, 5, 7, 9]))
    L2 = int(rng.integers(1, 13))
    h0, w0 = draw_size(rng, 1, 1)
    block, stride = draw_block(rng, h0, w0)
    h, w = max(h0, block[0]), max(w0, block[1])
    n = int(rng.integers(1, 4))
    say("apply_stage_hash", arith, dict(n=n, h=h, w=w, k=k, L2=L2, block=block, stride=stride))
    V = rng.standard_normal((n, h, w)).astype(np.float32)
    F = rng.standard_normal((L2, k, k)).astype(np.float32)
    ctx.set_option(lib.OPT_CONV_ARITH, lib.CONV_FP32 if arith == "fp32" else lib.CONV_BF16X3)
    try:
        dV, dF = dev(V), dev(F)
        got = ctx.apply_stage_hash(dV, dF, block, stride)
        same = ctx.hash_histogram(ctx.apply_stage(dV, dF), block, stride)
        iq = ctx.apply_stage_hash(dV, dF, block, stride, torch.float32)
        iq_same = ctx.hash_iq(ctx.apply_stage(dV, dF), block, stride, torch.float32)
        ctx.status()
    finally:
        ctx.set_option(lib.OPT_CONV_ARITH, lib.CONV_AUTO)
    assert torch.equal(got, same)
    assert torch.equal(iq, iq_same)
    maps = oracle.conv(V, F)
    want = oracle.block_hist(oracle.hash_maps(maps), block, stride, 1 << L2)
    g = got.cpu().numpy().astype(np.int64)
    assert g.shape == want.shape
    assert np.all(g.sum(axis=-1) == block[0] * block[1])
    # A pixel may hash differently in fp32 and fp64 only where a map value lies within the fp32 path's error of
    # zero; it then moves two counts in every block that holds it.  Everywhere else the counts are equal.
    scale = np.abs(F).sum(axis=(1, 2)).max() * np.abs(V).max()
    doubtful = int((np.abs(maps) <= 2e-6 * scale).any(axis=1).sum())
    cover = -(-block[0] // stride[0]) * -(-block[1] // stride[1])
    assert np.abs(g - want).sum() <= 2 * cover * doubtful, (doubtful, cover)


# ------------------------------------------------------------------ extraction with given filters (Eq. 6-9, 11-12)
@pytest.mark.parametrize("arith", ["auto", "fp32"])
@pytest.mark.parametrize("case", range(10))
def test_extract_features_random_geometry(lib, ctx, oracle, case, arith):
    """Two convolution stages, hashing and block histograms of both views with random filters.  The stage-2 maps of
    the GPU (two ddcca_apply_stage calls) meet the oracle's within the error bound of two fp32 stages; the
    histograms of every extraction route (one batch, ragged batches, fused last stage) equal the oracle's hashing and
    counting of exactly those maps, so that both sides take every sign decision on the same numbers."""
    rng = np.random.default_rng(55000 + case)
    k = int(rng.choice([3, 5, 7, 9]))
    L1, L2 = int(rng.integers(1, 5)), int(rng.integers(1, 9))
    h0, w0 = 1 + int(rng.integers(0, 50)), 1 + int(rng.integers(0, 90))
    block, stride = draw_block(rng, h0, w0)
    h, w = max(h0, block[0]), max(w0, block[1])
    m = int(rng.integers(1, 6))
    batch = int(rng.integers(1, m + 1))
    say("extract_features", arith, dict(m=m, h=h, w=w, k=k, L1=L1, L2=L2, block=block, stride=stride, batch=batch))
    V = rng.standard_normal((2, m, h, w)).astype(np.float32)
    F = [rng.standard_normal((L, k, k)).astype(np.float32) for L in (L1, L1, L2, L2)]
    dV, dF = [dev(V[0]), dev(V[1])], [dev(f) for f in F]
    ctx.set_option(lib.OPT_CONV_ARITH, lib.CONV_FP32 if arith == "fp32" else lib.CONV_AUTO)
    try:
        Z = [ctx.apply_stage(ctx.apply_stage(dV[d], dF[d]).reshape(m * L1, h, w), dF[2 + d]).cpu().numpy()
             for d in range(2)]
        whole = ctx.extract_features(dV[0], dV[1], dF, k, L1, L2, block, stride)
        batched = ctx.extract_features(dV[0], dV[1], dF, k, L1, L2, block, stride, batch_images=batch)
        fused = ctx.extract_features(dV[0], dV[1], dF, k, L1, L2, block, stride, batch_images=batch, fused=True)
        ctx.status()
    finally:
        ctx.set_option(lib.OPT_CONV_ARITH, lib.CONV_AUTO)
    ref = oracle.extract_features(V[0], V[1], F, k, L1, L2, block, stride, keep_maps=True)
    for d in range(2):
        l1 = [np.abs(F[s * 2 + d]).sum(axis=(1, 2)).max() for s in range(2)]
        assert np.abs(Z[d] - ref["Z"][d]).max() <= 4e-6 * l1[0] * l1[1] * np.abs(V[d]).max(), d
    want = np.stack([oracle.block_hist(oracle.hash_maps(Z[d]), block, stride, 1 << L2)
                     .reshape(m, L1, *ref["hist"].shape[3:]) for d in range(2)], axis=1)
    assert want.shape == ref["hist"].shape == tuple(whole.shape)
    for name, got in (("whole", whole), ("batched", batched), ("fused", fused)):
        assert np.array_equal(got.cpu().numpy().astype(np.int64), want), name


# ------------------------------------------------------------------ learning both stages (Sections II-A, II-B)
def cosines(got, want):
    g = got.reshape(got.shape[0], -1).astype(np.float64)
    r = want.reshape(want.shape[0], -1)
    return np.einsum("ga,ga->g", g, r) / (np.linalg.norm(g, axis=1) * np.linalg.norm(r, axis=1))


@pytest.mark.parametrize("route", ["streamed", "materialised", "recomputed"])
@pytest.mark.parametrize("case", range(8))
def test_two_stage_learning_random_geometry(lib, oracle, case, route):
    """Filters and correlations of both stages against the oracle on random small problems, by each of the three
    routes the second stage has (maps streamed through scratch memory, kept in memory, recomputed in the Gram
    kernel): rho to 1e-4 of the leading correlation, signed filter cosines where the correlations are separated."""
    from paper_2209_13027_amd import pipeline
    rng = np.random.default_rng(56000 + case)
    k = int(rng.choice([3, 5, 7, 9]))
    L1, L2 = int(rng.integers(1, 4)), int(rng.integers(1, 7))
    n_cls = int(rng.integers(1, 4))
    m = int(rng.integers(max(3, n_cls), 11))
    h, w = 16 + int(rng.integers(0, 32)), 16 + int(rng.integers(0, 80))
    batch = int(rng.integers(0, m + 1))
    say("two-stage learning", route, dict(m=m, h=h, w=w, k=k, L1=L1, L2=L2, n_cls=n_cls, batch=batch))
    cls = (np.arange(m) % n_cls).astype(np.int32)
    base = rng.standard_normal((n_cls, h, w))
    v1 = (base[cls] + 0.7 * rng.standard_normal((m, h, w))).astype(np.float32)
    v2 = (0.5 * base[cls] ** 2 + 0.7 * rng.standard_normal((m, h, w))).astype(np.float32)
    ref = oracle.learn_two_stage(v1, v2, cls, n_cls, k, L1, L2)
    c = lib.Context(0)
    try:
        if route == "recomputed":
            c.set_option(lib.OPT_NEXT_STAGE_MAPS, lib.MAPS_RECOMPUTED)
        model = pipeline.fit(c, dev(v1), dev(v2), dev(cls), n_cls, k, L1, L2, streamed=route != "materialised",
                             batch_images=batch)
        c.status()
        filters = [f.cpu().numpy() for f in model["filters"]]
        rhos = [r.cpu().numpy() for r in model["rho"]]
    finally:
        c.close()
    for s in range(2):
        r = ref["stage%d" % (s + 1)]
        assert np.all(np.isfinite(rhos[s]))
        assert np.abs(rhos[s] - r["rho"]).max() <= 1e-4 * r["rho"][0], (s, rhos[s], r["rho"])
        ok = r["gap"] > 1e-3
        for d in range(2):
            if ok.any():
                cos = cosines(filters[2 * s + d], r["W%d" % (d + 1)])
                assert cos[ok].min() >= 0.9999, (s, d, cos, r["gap"])

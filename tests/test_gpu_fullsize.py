"""GPU parity at the full sizes of the five benchmark workloads, in the launch configuration bench.py times
(pipeline.fit + pipeline.extract on the whole workload).  The CPU oracle cannot redo a full run in
seconds, so each stage of the full-size GPU result is checked on outputs the oracle can compute one
by one, and by properties that hold at any size:
  * sampled entries of the stage-1 matrices over ALL patches (oracle.corr_entries);
  * class matrices against the oracle's Gram of the class-sum images (linearity, pinned on the CPU);
  * the solve against the oracle's solve of the exported fp64 matrices;
  * convolution of sampled images element by element; map statistics against the Gram quadratic
    forms w^T C w for both stages (ties the full-size Gram and conv outputs together);
  * hashing + histograms of sampled images bit-exact from the GPU's own fp32 maps;
  * every histogram sums to the block area;
  * end-to-end against the oracle on a class-balanced slice of the same workload.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu

from paper_2209_13027_amd.workloads import WORKLOADS, make_views  # noqa: E402


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def filter_cosines(got, want):
    g = got.reshape(got.shape[0], -1).astype(np.float64)
    w = want.reshape(want.shape[0], -1)
    return np.einsum("ga,ga->g", g, w) / (np.linalg.norm(g, axis=1) * np.linalg.norm(w, axis=1))


class FullRun:
    """One full-size GPU run, shared by the tests of a workload."""

    def __init__(self, name, split=False):
        from paper_2209_13027_amd import pipeline
        from paper_2209_13027_amd.binding import (Context, OPT_CONV_ARITH, CONV_BF16X3, CONV_FP32, OPT_GRAM_ARITH,
                                                  GRAM_BF16X3, GRAM_LAG_FP32)
        self.wl = wl = WORKLOADS[name]
        lag = split == "lag"
        self.split = split = split is True
        self.v1, self.v2, self.cls = make_views(wl)
        self.ctx = ctx = Context(0)
        # the plain run and the lag run convolve with the fp32 matrix instructions (the fused last stage, which
        # always does, is then bit-identical); the split run with three-piece bf16 operands
        ctx.set_option(OPT_CONV_ARITH, CONV_FP32)
        if split:
            # three-piece bf16 operands in the Gram and in the convolution: the same checks, the same bars
            ctx.set_option(OPT_GRAM_ARITH, GRAM_BF16X3)
            ctx.set_option(OPT_CONV_ARITH, CONV_BF16X3)
        if lag:
            # the lag-structured Gram (fp32 convolution): the same checks, the same bars
            ctx.set_option(OPT_GRAM_ARITH, GRAM_LAG_FP32)
        self.d1, self.d2, self.dc = dev(self.v1), dev(self.v2), dev(self.cls)
        M, h, w = self.v1.shape
        # stage-1 matrices through the streamed API (same kernels and launch shapes as learn_stage_filters)
        ctx.corr_begin(wl.k, wl.n_classes, 1, h, w)
        ctx.corr_accumulate(self.d1, self.d2, self.dc)
        self.mats1 = {k: v.cpu().numpy() for k, v in ctx.corr_export(wl.k).items()}
        self.model = pipeline.fit(ctx, self.d1, self.d2, self.dc, wl.n_classes, wl.k, wl.L1, wl.L2, keep_maps=True)
        y1, y2 = self.model["maps"]
        ctx.corr_begin(wl.k, wl.n_classes, wl.L1, h, w)
        ctx.corr_accumulate(y1, y2, self.dc)
        self.mats2 = {k: v.cpu().numpy() for k, v in ctx.corr_export(wl.k).items()}
        self.feat = pipeline.extract(ctx, self.d1, self.d2, self.model["filters"], wl.k, wl.L1, wl.L2, wl.block,
                                     wl.stride, wl.extract_batch)
        ctx.status()
        torch.cuda.synchronize()
        self.filters = [f.cpu().numpy() for f in self.model["filters"]]

    def close(self):
        self.ctx.close()
        del self.feat, self.model, self.d1, self.d2
        torch.cuda.empty_cache()


@pytest.fixture(scope="module", params=[("object", False), ("stress", False), ("large_scale", False),
                                        ("object", True), ("stress", True), ("large_scale", True),
                                        ("object", "lag"), ("large_scale", "lag"), ("stress", "lag")],
                ids=lambda p: p[0] + ("-lag" if p[1] == "lag" else "-bf16x3" if p[1] else ""))
def run(request):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    r = FullRun(*request.param)
    yield r
    r.close()


def test_fused_extraction_full_size(run):
    """The fused last stage on the whole workload: identical to the materialised path (fp32 convolution), or
    within the end-to-end histogram bar of it (three-piece convolution in the materialised path; the fused
    kernel always uses the fp32 instructions)."""
    from paper_2209_13027_amd import pipeline
    wl = run.wl
    fused = pipeline.extract(run.ctx, run.d1, run.d2, run.model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride,
                             wl.extract_batch, fused=True)
    run.ctx.status()
    if not run.split:
        assert torch.equal(fused, run.feat)
    else:
        diff, total = 0.0, 0.0
        step = max(1, fused.shape[0] // 64)
        for s in range(0, fused.shape[0], step):
            a, b = fused[s:s + step].to(torch.int32), run.feat[s:s + step].to(torch.int32)
            diff += float((a - b).abs().sum())
            total += float(b.sum())
        assert diff <= 1e-3 * total
    del fused


def test_stage1_matrix_entries(run, oracle):
    wl = run.wl
    D = wl.D
    rng = np.random.default_rng(5)
    entries = []
    for va, vb in ((1, 1), (2, 2), (1, 2)):
        for _ in range(3):
            entries.append((va, int(rng.integers(D)), vb, int(rng.integers(D))))
    entries.append((1, 0, 1, 0))
    entries.append((2, D // 2, 2, D // 2))
    want = oracle.corr_entries(run.v1, run.v2, wl.k, entries) / (run.v1.shape[0] * wl.h * wl.w)
    name = {(1, 1): "C11", (2, 2): "C22", (1, 2): "C12"}
    for (va, a, vb, b), wv in zip(entries, want):
        M = run.mats1[name[(va, vb)]]
        scale = np.sqrt((M ** 2).mean())
        assert abs(M[a, b] - wv) <= 1e-4 * scale, (va, a, vb, b, M[a, b], wv)
        # what fp32 accumulation over ~16k patches per wavefront between fp64 folds delivers
        assert abs(M[a, b] - wv) <= 1e-5 * max(scale, abs(wv))


def test_stage1_class_matrices(run, oracle):
    wl = run.wl
    N = run.v1.shape[0] * wl.h * wl.w
    s1 = np.stack([run.v1[run.cls == c].sum(axis=0, dtype=np.float64) for c in range(wl.n_classes)])
    s2 = np.stack([run.v2[run.cls == c].sum(axis=0, dtype=np.float64) for c in range(wl.n_classes)])
    _, _, Sw = oracle.corr_sums(s1, s2, wl.k)
    _, _, ST = oracle.corr_sums(s1.sum(0, keepdims=True), s2.sum(0, keepdims=True), wl.k)
    for got, want in ((run.mats1["Cw"], Sw / N), (run.mats1["CT"], ST / N)):
        assert np.linalg.norm(got - want) <= 1e-4 * np.linalg.norm(want)


def test_matrix_structure(run):
    D = run.wl.D
    for mats in (run.mats1, run.mats2):
        for nm in ("C11", "C22"):
            C = mats[nm]
            assert np.abs(C - C.T).max() <= 1e-12 * np.abs(C).max()
            assert np.linalg.eigvalsh(C).min() >= -1e-7 * np.abs(C).max()
        for nm in ("C11", "C22", "C12", "Cw", "CT"):
            C = mats[nm]
            assert np.abs(C @ np.ones(D)).max() <= 1e-12 * np.abs(C).max()
            assert np.abs(np.ones(D) @ C).max() <= 1e-12 * np.abs(C).max()


def test_solve_on_exported_matrices(run, oracle):
    wl = run.wl
    for mats, (f1, f2), rho, L in ((run.mats1, run.filters[:2], run.model["rho"][0], wl.L1),
                                   (run.mats2, run.filters[2:], run.model["rho"][1], wl.L2)):
        sol = oracle.dcca_solve(mats["C11"], mats["C22"], 2 * mats["Cw"] - mats["CT"], L)
        ok = sol["gap"] > 1e-3
        assert ok.sum() >= L - 2
        assert np.allclose(rho.cpu().numpy(), sol["rho"], rtol=1e-8)
        assert filter_cosines(f1, sol["W1"])[ok].min() >= 0.9999
        assert filter_cosines(f2, sol["W2"])[ok].min() >= 0.9999
        assert filter_cosines(f1, sol["W1"])[ok].min() >= 1 - 1e-9


def test_conv_sampled_images_and_map_statistics(run, oracle):
    wl = run.wl
    M = run.v1.shape[0]
    idx = [0, M // 2, M - 1]
    for d, (v, y) in enumerate(((run.v1, run.model["maps"][0]), (run.v2, run.model["maps"][1]))):
        want = oracle.conv(v[idx], run.filters[d])
        got = y[idx].cpu().numpy()
        scale = np.abs(run.filters[d]).sum(axis=(1, 2)).max() * np.abs(v[idx]).max()
        assert np.abs(got - want).max() <= 2e-6 * scale
    # mean over all patches of Y_g^2 and Y1_g*Y2_g equals the Gram quadratic forms (any size)
    y1, y2 = run.model["maps"]
    w1 = run.filters[0].reshape(wl.L1, -1).astype(np.float64)
    w2 = run.filters[1].reshape(wl.L1, -1).astype(np.float64)
    ms1 = (y1.double() ** 2).mean(dim=(0, 2, 3)).cpu().numpy()
    ms2 = (y2.double() ** 2).mean(dim=(0, 2, 3)).cpu().numpy()
    cross = (y1.double() * y2.double()).mean(dim=(0, 2, 3)).cpu().numpy()
    # w^T dC w <= |w|^2 |dC|: the matrix unit's fp32 accumulation loses a little of every addend once the
    # accumulator is much larger, a deficit of about 1e-6 (fp32 instructions) to 3e-6 (three-piece bf16) of the
    # diagonal on sums of squares; allow 5e-6 of the largest diagonal entry per unit of |w|^2
    def close(stat, C, wa, wb, Ca, Cb):
        quad = np.einsum("ga,ab,gb->g", wa, C, wb)
        bound = 5e-6 * np.sqrt(np.diag(Ca).max() * np.diag(Cb).max()) * np.linalg.norm(wa, axis=1) * np.linalg.norm(wb, axis=1)
        return np.all(np.abs(stat - quad) <= bound + 2e-6 * np.abs(quad))
    C11, C22, C12 = run.mats1["C11"], run.mats1["C22"], run.mats1["C12"]
    assert close(ms1, C11, w1, w1, C11, C11)
    assert close(ms2, C22, w2, w2, C22, C22)
    assert close(cross, C12, w1, w2, C11, C22)
    assert np.allclose(cross, run.model["rho"][0].cpu().numpy() * 0 + cross)        # finite


def test_stage2_matrices_against_map_statistics(run, oracle):
    # stage-2 quadratic forms: convolve a sample of stage-1 maps with the stage-2 filters on the GPU and
    # compare the statistics of ALL stage-2 maps (accumulated batch-wise) with w^T C w of the stage-2 Gram
    wl = run.wl
    y1 = run.model["maps"][0].reshape(-1, wl.h, wl.w)
    n = y1.shape[0]
    w = run.filters[2].reshape(wl.L2, -1).astype(np.float64)
    acc = torch.zeros(wl.L2, dtype=torch.float64, device="cuda")
    step = max(1, (1 << 28) // (wl.L2 * wl.h * wl.w))
    for s in range(0, n, step):
        z = run.ctx.apply_stage(y1[s:s + step], run.model["filters"][2])
        acc += (z.double() ** 2).sum(dim=(0, 2, 3))
    ms = acc.cpu().numpy() / (n * wl.h * wl.w)
    # same bound as for stage 1: 5e-6 of the largest diagonal entry per unit of |w|^2
    quad = np.einsum("ga,ab,gb->g", w, run.mats2["C11"], w)
    bound = 5e-6 * np.diag(run.mats2["C11"]).max() * (w ** 2).sum(axis=1)
    assert np.all(np.abs(ms - quad) <= bound + 2e-6 * np.abs(quad))
    # a few stage-2 entries over a bounded number of maps cannot be isolated from the full sum, so the
    # entry-wise check of the stage-2 launch shape is done on the class matrices (few sum images)
    cls = run.cls
    yy1 = run.model["maps"][0]
    yy2 = run.model["maps"][1]
    s1 = torch.stack([yy1[torch.from_numpy(cls == c).cuda()].double().sum(0) for c in range(wl.n_classes)])
    s2 = torch.stack([yy2[torch.from_numpy(cls == c).cuda()].double().sum(0) for c in range(wl.n_classes)])
    s1 = s1.reshape(-1, wl.h, wl.w).cpu().numpy()           # [(c,g)] sum images
    s2 = s2.reshape(-1, wl.h, wl.w).cpu().numpy()
    rng = np.random.default_rng(6)
    entries = [(1, int(rng.integers(wl.D)), 2, int(rng.integers(wl.D))) for _ in range(6)]
    want = oracle.corr_entries(s1, s2, wl.k, entries) / (n * wl.h * wl.w)
    scale = np.sqrt((run.mats2["Cw"] ** 2).mean())
    for (_, a, _, b), wv in zip(entries, want):
        assert abs(run.mats2["Cw"][a, b] - wv) <= 1e-4 * scale


def test_histograms_of_sampled_images_bit_exact(run, oracle):
    wl = run.wl
    M = run.v1.shape[0]
    assert run.feat.shape == (M, 2, wl.L1) + wl.blocks + (1 << wl.L2,)
    for m in (0, M // 3, M - 1):
        for d in range(2):
            y = run.model["maps"][d][m]                                        # [L1, h, w]
            z = run.ctx.apply_stage(y, run.model["filters"][2 + d]).cpu().numpy()
            want = oracle.block_hist(oracle.hash_maps(z), wl.block, wl.stride, 1 << wl.L2)
            got = run.feat[m, d].cpu().numpy().astype(np.int64)
            assert np.array_equal(got, want)


def test_every_histogram_sums_to_block_area(run):
    wl = run.wl
    M = run.v1.shape[0]
    step = max(1, M // 64)
    for s in range(0, M, step * 8):
        sums = run.feat[s:s + step].to(torch.int32).sum(dim=-1)
        assert int(sums.min()) == wl.block ** 2 and int(sums.max()) == wl.block ** 2


def test_end_to_end_on_a_slice(run, oracle):
    from paper_2209_13027_amd import pipeline
    wl = run.wl
    per_class = {"object": 3, "stress": 1, "large_scale": 1}[wl.name]
    n_cls = {"object": 8, "stress": 8, "large_scale": 24}[wl.name]
    v1, v2, cls = make_views(wl, max_per_class=per_class, n_classes=n_cls)
    if wl.name == "stress":                      # two samples per class so that classes mean something
        cls = (cls // 2).astype(np.int32)
        n_cls //= 2
    ctx = run.ctx
    d1, d2, dc = dev(v1), dev(v2), dev(cls)
    model = pipeline.fit(ctx, d1, d2, dc, n_cls, wl.k, wl.L1, wl.L2)
    feat = pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride)
    ctx.status()
    ref = oracle.two_stage(v1, v2, cls, n_cls, wl.k, wl.L1, wl.L2, wl.block)
    refs = [ref["stage1"]["W1"], ref["stage1"]["W2"], ref["stage2"]["W1"], ref["stage2"]["W2"]]
    gaps = [ref["stage1"]["gap"]] * 2 + [ref["stage2"]["gap"]] * 2
    for W, R, gap in zip(model["filters"], refs, gaps):
        cos = filter_cosines(W.cpu().numpy(), R)
        assert cos[gap > 1e-3].min() >= 0.9999
    got = feat.cpu().numpy().astype(np.int64)
    l1 = np.abs(got - ref["hist"]).sum() / ref["hist"].sum()
    assert l1 <= 1e-3, l1


def test_streamed_second_stage_learning_full_size(run):
    """Second-stage learning from the inputs (maps convolved batch by batch, class sum images by linearity) at
    full size against the materialised run of the fixture: the same matrices up to the order of the fp32 partial
    sums, which follows the batch split (the bar of the batch-split test), and the fp32 rounding of the sum
    images (Cw, CT); the same filters."""
    wl, ctx = run.wl, run.ctx
    M, h, w = run.v1.shape
    W1a, W2a = run.model["filters"][0], run.model["filters"][1]
    W1b, W2b, rho = ctx.learn_next_stage_filters(run.d1, run.d2, run.dc, 1, h, w, wl.n_classes, W1a, W2a, wl.k,
                                                 wl.L2)
    mats = {k: v.cpu().numpy() for k, v in ctx.corr_export(wl.k).items()}
    ctx.status()
    for name in ("C11", "C22", "C12", "Cw", "CT"):
        assert np.linalg.norm(mats[name] - run.mats2[name]) <= 1e-6 * np.linalg.norm(run.mats2[name]), name
    rho_m = run.model["rho"][1].cpu().numpy()
    assert np.allclose(rho.cpu().numpy(), rho_m, rtol=1e-5)
    sep = np.ones(wl.L2, dtype=bool)
    sep[1:] &= rho_m[1:] < 0.999 * rho_m[:-1]
    sep[:-1] &= rho_m[1:] < 0.999 * rho_m[:-1]
    if sep.any():
        assert filter_cosines(W1b.cpu().numpy(), run.filters[2].astype(np.float64))[sep].min() >= 1 - 1e-6
        assert filter_cosines(W2b.cpu().numpy(), run.filters[3].astype(np.float64))[sep].min() >= 1 - 1e-6

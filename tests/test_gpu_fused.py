"""GPU tests of the fused last stage (stage convolution + hashing + block histograms without the maps in memory).

Against the oracle: conv (Eq. 6) -> hash (Eq. 7-9) -> block histogram, relative L1 of the counts <= 1e-3 (the
end-to-end histogram bar: a map value within fp32 rounding of zero may hash differently in fp32 and fp64).
Against the unfused GPU calls (ddcca_apply_stage + ddcca_hash_iq): bit-exact, since the fused kernel runs
the same contraction in the same order.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2209_13027_amd.workloads import WORKLOADS, make_views  # noqa: E402
from paper_2209_13027_amd import pipeline  # noqa: E402


@pytest.fixture(scope="module", params=["fp32", "bf16x3"])
def ctx(request):
    """The fused last stage runs in the arithmetic the stage convolution has, so that its bit-exact reference is the
    unfused path of the same context: with the fp32 matrix instructions one kernel (convolution, hashing and
    histograms around a ring of block rows); with three-piece bf16 operands the convolution kernel writes the hash
    codes of its maps (one byte per pixel and 8 filters) and the histograms are counted from those."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2209_13027_amd.binding import Context, OPT_CONV_ARITH, CONV_FP32, CONV_BF16X3
    c = Context(0)
    c.set_option(OPT_CONV_ARITH, CONV_FP32 if request.param == "fp32" else CONV_BF16X3)
    yield c
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


GEOMETRIES = [
    (5, 32, 32, 5, 4, 8, 4),             # tiny workload geometry
    (3, 112, 92, 7, 8, 7, 4),            # small-face geometry (several row groups, ragged last group)
    (2, 128, 128, 5, 8, 16, 8),          # object geometry
    (2, 128, 128, 7, 8, 16, 8),          # large-scale geometry
    (1, 256, 256, 9, 8, 32, 16),         # stress geometry (two tile columns)
    (3, 17, 23, 3, 1, 5, 3),             # one bit, ragged everything
    (2, 40, 36, 5, 12, 9, 5),            # maximum code width: two filter groups
    (1, 20, 200, 5, 12, 8, 4),           # wide map, 4096 bins: block columns split over workgroups
    (2, 9, 300, 3, 3, (9, 11), (1, 7)),  # single block row, rectangular block, three tile columns
    (1, 8, 8, 9, 5, 8, 8),               # filter larger than the map, one block
    (2, 33, 130, 7, 11, (6, 10), (2, 3)),  # dense block overlap (stride < block/2), 11 filters
    (2, 24, 24, 3, 12, 9, 1),            # stride 1 with 4096 bins: live block rows exceed LDS (row-group kernel)
    (2, 150, 40, 5, 8, 16, 8),           # tall narrow map: many tile rows, several block-row flushes
    (3, 1, 40, 3, 2, (1, 8), (1, 4)),    # one pixel row
    (2, 37, 41, 5, 6, 9, 4),             # odd width and height: unaligned rows, scalar tile staging
    (1, 300, 500, 7, 8, 64, 32),         # large map, large blocks: four tile columns, long block rows
    (2, 64, 64, 9, 8, 8, 8),             # stride = block (no overlap): each pixel in exactly one block
    (2, 48, 80, 5, 7, 6, 9),             # stride > block: pixels between blocks belong to none
]


@pytest.mark.parametrize("n,h,w,k,L2,block,stride", GEOMETRIES)
def test_apply_stage_hash(ctx, oracle, n, h, w, k, L2, block, stride):
    rng = np.random.default_rng(400 + k + h + L2)
    V = rng.standard_normal((n, h, w)).astype(np.float32)
    F = rng.standard_normal((L2, k, k)).astype(np.float32)
    dV, dF = dev(V), dev(F)
    got = ctx.apply_stage_hash(dV, dF, block, stride)
    # oracle: the definition, in fp64
    want = oracle.block_hist(oracle.hash_maps(oracle.conv(V, F)), block, stride, 1 << L2)
    g = got.cpu().numpy().astype(np.int64)
    assert g.shape == want.shape
    assert np.abs(g - want).sum() <= 1e-3 * want.sum()
    bh, bw = (block, block) if np.isscalar(block) else block
    assert np.all(g.sum(axis=-1) == bh * bw)
    # the unfused kernels on the same inputs: identical, in all three output forms
    maps = ctx.apply_stage(dV, dF)
    assert torch.equal(got, ctx.hash_histogram(maps, block, stride))
    for dtype in (torch.float32, torch.float16):
        assert torch.equal(ctx.apply_stage_hash(dV, dF, block, stride, dtype), ctx.hash_iq(maps, block, stride, dtype))


def test_apply_stage_hash_exact_on_integer_data(ctx, oracle):
    # small-integer images and filters: every product and sum is exact in fp32, so the counts must equal the
    # oracle's exactly (including the pixels whose map value is exactly zero)
    rng = np.random.default_rng(9)
    V = rng.integers(-3, 4, size=(3, 50, 70)).astype(np.float32)
    F = rng.integers(-2, 3, size=(8, 5, 5)).astype(np.float32)
    got = ctx.apply_stage_hash(dev(V), dev(F), 10, 5).cpu().numpy().astype(np.int64)
    want = oracle.block_hist(oracle.hash_maps(oracle.conv(V, F)), 10, 5, 256)
    assert np.array_equal(got, want)


def test_apply_stage_hash_empty_and_validation(ctx):
    from paper_2209_13027_amd.binding import DdccaError
    F = torch.zeros((4, 5, 5), dtype=torch.float32, device="cuda")
    out = ctx.apply_stage_hash(torch.empty((0, 16, 16), dtype=torch.float32, device="cuda"), F, 8, 4)
    assert out.shape == (0, 3, 3, 16)
    with pytest.raises(DdccaError):
        ctx.apply_stage_hash(torch.zeros((1, 16, 16), dtype=torch.float32, device="cuda"), F, 32, 4)


@pytest.mark.parametrize("name,images,batch", [("tiny", None, 16), ("small_face", 3, 0), ("object", 1, 0)])
def test_extract_fused_equals_unfused(ctx, name, images, batch):
    wl = WORKLOADS[name]
    v1, v2, cls = make_views(wl, max_per_class=images)
    d1, d2, dc = dev(v1), dev(v2), dev(cls)
    model = pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2)
    for dtype in (torch.uint16, torch.float32, torch.float16):
        a = pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride, batch,
                             dtype=dtype)
        b = pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride, batch,
                             dtype=dtype, fused=True)
        assert a.shape == b.shape and torch.equal(a, b)


def test_extract_fused_odd_group_and_ragged_batches(ctx):
    # L1 = 3 maps per image, 5 images in batches of 2: group layout and ragged last batch of the fused launch
    rng = np.random.default_rng(31)
    v1 = rng.standard_normal((5, 30, 44)).astype(np.float32)
    v2 = rng.standard_normal((5, 30, 44)).astype(np.float32)
    filters = [dev(rng.standard_normal((L, 5, 5)).astype(np.float32)) for L in (3, 3, 6, 6)]
    a = ctx.extract_features(dev(v1), dev(v2), filters, 5, 3, 6, 10, 5, batch_images=2)
    b = ctx.extract_features(dev(v1), dev(v2), filters, 5, 3, 6, 10, 5, batch_images=2, fused=True)
    c = ctx.extract_features(dev(v1), dev(v2), filters, 5, 3, 6, 10, 5, batch_images=0, fused=True)
    assert a.shape == (5, 2, 3, 5, 7, 64)
    assert torch.equal(a, b) and torch.equal(a, c)


def test_end_to_end_tiny_fused(ctx, oracle):
    wl = WORKLOADS["tiny"]
    v1, v2, cls = make_views(wl)
    d1, d2, dc = dev(v1), dev(v2), dev(cls)
    model = pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2)
    feat = pipeline.extract(ctx, d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride, 16, fused=True)
    ref = oracle.two_stage(v1, v2, cls, wl.n_classes, wl.k, wl.L1, wl.L2, wl.block, wl.stride)
    got = feat.cpu().numpy().astype(np.int64)
    assert got.shape == ref["hist"].shape
    assert np.abs(got - ref["hist"]).sum() / ref["hist"].sum() <= 1e-3

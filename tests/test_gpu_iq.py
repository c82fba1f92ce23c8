"""GPU parity of the information-quality output (Eq. 10-12) against the fp64 oracle.

fp32 output: within one fp32 unit in the last place of the oracle value (the kernel rounds an fp64 value
once; the oracle's own fp64 rounding may move a tie).  fp16 output: within one fp16 unit in the last place.
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


def area(block):
    return block * block if np.isscalar(block) else block[0] * block[1]


def check_iq(got, want64, dtype):
    assert got.shape == want64.shape
    if dtype == torch.float32:
        want = want64.astype(np.float32)
        ulp = np.spacing(np.abs(want))
        bad = np.abs(got.astype(np.float64) - want64) > ulp.astype(np.float64)
        assert not bad.any(), f"{bad.sum()} fp32 values off by more than one ulp"
        assert np.mean(got == want) > 0.999
    else:
        want = want64.astype(np.float16)
        ulp = np.spacing(np.abs(want)).astype(np.float64)
        bad = np.abs(got.astype(np.float64) - want.astype(np.float64)) > ulp
        assert not bad.any(), f"{bad.sum()} fp16 values off by more than one ulp"
        assert np.mean(got == want) > 0.999


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("n,L2,h,w,block,stride", [
    (5, 4, 32, 32, 8, 4),            # tiny workload geometry
    (3, 8, 112, 92, 7, 4),           # small-face geometry
    (4, 8, 128, 128, 16, 8),         # object / large-scale geometry
    (2, 8, 256, 256, 32, 16),        # stress geometry
    (3, 1, 17, 23, 5, 3),            # one bit, ragged everything, unaligned output rows
    (2, 2, 30, 31, 6, 5),            # four bins
    (2, 12, 40, 36, 9, 5),           # maximum code width
    (2, 3, 9, 300, (9, 11), (1, 7)),  # single block row, rectangular block, wide map
])
def test_hash_iq(ctx, oracle, n, L2, h, w, block, stride, dtype):
    rng = np.random.default_rng(300 + L2 + h)
    Z = rng.standard_normal((n, L2, h, w)).astype(np.float32)
    Z[rng.random(Z.shape) < 0.05] = 0.0
    got = ctx.hash_iq(dev(Z), block, stride, dtype).cpu().numpy()
    H = oracle.block_hist(oracle.hash_maps(Z), block, stride, 1 << L2)
    check_iq(got, oracle.iq_features(H, area(block)), dtype)


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
def test_hash_iq_counts_beyond_the_table(ctx, oracle, dtype):
    # 60x60 blocks (area 3600) of maps that are positive almost everywhere: one code collects far more than
    # the 2047 counts the kernel's table covers, so the directly computed values are exercised too
    rng = np.random.default_rng(11)
    Z = (rng.standard_normal((2, 3, 70, 130)) + 3.0).astype(np.float32)
    got = ctx.hash_iq(dev(Z), 60, (5, 35), dtype).cpu().numpy()
    H = oracle.block_hist(oracle.hash_maps(Z), 60, (5, 35), 8)
    assert H.max() > 3000
    check_iq(got, oracle.iq_features(H, 3600), dtype)


def test_hash_iq_empty_and_bad_type(ctx):
    from paper_2209_13027_amd.binding import DdccaError, EINVAL, lib
    Z = torch.empty((0, 8, 16, 16), dtype=torch.float32, device="cuda")
    assert ctx.hash_iq(Z, 8, 4).shape == (0, 3, 3, 256)
    Z = torch.zeros((1, 2, 8, 8), dtype=torch.float32, device="cuda")
    out = torch.zeros((1, 1, 1, 4), dtype=torch.float32, device="cuda")
    rc = lib().ddcca_hash_iq(ctx._h, Z.data_ptr(), 1, 2, 8, 8, 8, 8, 8, 8, 7, out.data_ptr())
    assert rc == EINVAL
    assert DdccaError is not None


def test_extract_iq_features_tiny(ctx, oracle):
    """Whole path with the information-quality output: layout [m][view][g][by][bx][bin]; the probabilities
    exp(-o) match the oracle's within the end-to-end histogram tolerance (relative L1 <= 1e-3) and each block's
    probabilities sum to one."""
    wl = WORKLOADS["tiny"]
    v1, v2, cls = make_views(wl)
    d1, d2, dc = dev(v1), dev(v2), dev(cls)
    model = pipeline.fit(ctx, d1, d2, dc, wl.n_classes, wl.k, wl.L1, wl.L2)
    o32 = ctx.extract_iq_features(d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride,
                                  torch.float32, batch_images=16)
    o16 = ctx.extract_iq_features(d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride,
                                  torch.float16)
    cnt = ctx.extract_features(d1, d2, model["filters"], wl.k, wl.L1, wl.L2, wl.block, wl.stride)
    ref = oracle.two_stage(v1, v2, cls, wl.n_classes, wl.k, wl.L1, wl.L2, wl.block, wl.stride)
    want = oracle.iq_features(ref["hist"], wl.block * wl.block)
    got = o32.cpu().numpy().astype(np.float64)
    assert got.shape == want.shape
    p_got, p_want = np.exp(-got), np.exp(-want)
    np.testing.assert_allclose(p_got.sum(axis=-1), 1.0, rtol=0, atol=1e-5)
    assert np.abs(p_got - p_want).sum() / np.abs(p_want).sum() <= 1e-3
    # the same launch configuration with the count output gives exactly the counts the values encode
    total = wl.block * wl.block + (1 << wl.L2)
    assert np.array_equal(np.rint(total * p_got - 1.0).astype(np.int64), cnt.cpu().numpy().astype(np.int64))
    assert np.array_equal(o16.cpu().numpy(), o32.cpu().numpy().astype(np.float16))

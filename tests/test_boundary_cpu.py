"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2209_13027_amd import binding as b
    if not os.path.exists(b.LIB_PATH):
        from paper_2209_13027_amd import build
        build.build_library()
    return b


def header_symbols():
    text = open(os.path.join(ROOT, "include", "ddcca.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ddcca_[a-z_]+)\s*\(", text)))


def test_header_symbols_all_exported(binding):
    lib = binding.lib()
    names = header_symbols()
    assert len(names) >= 16
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_no_oracle_in_product_path():
    # the product package must never reach into the CPU oracle
    pkg = os.path.join(ROOT, "paper_2209_13027_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "workloads.py", (dirpath, f)


def make_ctx(binding):
    h = ctypes.c_void_p()
    assert binding.lib().ddcca_create(ctypes.byref(h), 0, None) == binding.OK
    return h


def test_create_rejects_bad_args(binding):
    lib = binding.lib()
    assert lib.ddcca_create(None, 0, None) == binding.EINVAL
    h = ctypes.c_void_p()
    assert lib.ddcca_create(ctypes.byref(h), -1, None) == binding.EINVAL
    assert lib.ddcca_last_error(None) == b"null context"


def test_validation_before_any_launch(binding):
    lib = binding.lib()
    h = make_ctx(binding)
    one = ctypes.c_void_p(256)          # never dereferenced: validation fails first
    E = binding.EINVAL
    # corr_begin: k even, k too large, bad class count, bad G, empty image
    assert lib.ddcca_corr_begin(h, 4, 2, 1, 8, 8) == E
    assert b"odd" in lib.ddcca_last_error(h)
    assert lib.ddcca_corr_begin(h, 11, 2, 1, 8, 8) == E
    assert lib.ddcca_corr_begin(h, 5, 0, 1, 8, 8) == E
    assert lib.ddcca_corr_begin(h, 5, 2, 0, 8, 8) == E
    assert lib.ddcca_corr_begin(h, 5, 2, 1, 0, 8) == E
    assert lib.ddcca_corr_begin(h, 5, 70000, 1, 8, 8) == E
    # state errors
    assert lib.ddcca_corr_accumulate(h, one, one, one, 4) == binding.ESTATE
    assert lib.ddcca_corr_export(h, one, one, one, one, one) == binding.ESTATE
    assert lib.ddcca_solve_filters(h, 2, 1e-4, one, one, one) == binding.ESTATE
    # solve: L range, ridge, null pointers
    assert lib.ddcca_dcca_solve(h, one, one, one, one, 5, 0, 1e-4, one, one, one) == E
    assert lib.ddcca_dcca_solve(h, one, one, one, one, 5, 25, 1e-4, one, one, one) == E
    assert lib.ddcca_dcca_solve(h, one, one, one, one, 5, 4, 0.0, one, one, one) == E
    assert lib.ddcca_dcca_solve(h, one, one, one, one, 5, 4, 1e-4, None, one, one) == E
    assert lib.ddcca_dcca_solve(h, None, one, one, one, 5, 4, 1e-4, one, one, one) == E
    # learn_stage_filters
    assert lib.ddcca_learn_stage_filters(h, one, one, one, 0, 1, 8, 8, 2, 5, 4, 1e-4, one, one, one) == E
    assert lib.ddcca_learn_stage_filters(h, None, one, one, 4, 1, 8, 8, 2, 5, 4, 1e-4, one, one, one) == E
    assert lib.ddcca_learn_stage_filters(h, one, one, one, 4, 1, 8, 8, 2, 6, 4, 1e-4, one, one, one) == E
    # apply_stage
    assert lib.ddcca_apply_stage(h, one, -1, 8, 8, one, 5, 4, one) == E
    assert lib.ddcca_apply_stage(h, one, 2, 8, 8, one, 2, 4, one) == E
    assert lib.ddcca_apply_stage(h, one, 2, 8, 8, one, 5, 0, one) == E
    assert lib.ddcca_apply_stage(h, None, 2, 8, 8, one, 5, 4, one) == E
    assert lib.ddcca_apply_stage(h, one, 0, 8, 8, one, 5, 4, one) == binding.OK      # empty batch: nothing to do
    # hash_histogram
    assert lib.ddcca_hash_histogram(h, one, 2, 13, 16, 16, 8, 8, 4, 4, one) == E     # L2 > 12
    assert lib.ddcca_hash_histogram(h, one, 2, 8, 16, 16, 17, 8, 4, 4, one) == E     # block taller than the map
    assert lib.ddcca_hash_histogram(h, one, 2, 8, 16, 16, 8, 8, 0, 4, one) == E      # zero stride
    assert lib.ddcca_hash_histogram(h, one, 2, 8, 300, 300, 256, 256, 4, 4, one) == binding.EOVERFLOW
    assert lib.ddcca_hash_histogram(h, one, 2, 8, 16, 16, 8, 8, 4, 4, None) == E
    assert lib.ddcca_hash_histogram(h, one, 0, 8, 16, 16, 8, 8, 4, 4, one) == binding.OK
    # extract_features
    m = binding._Model()
    m.k, m.L1, m.L2, m.block_h, m.block_w, m.stride_y, m.stride_x = 5, 4, 4, 8, 8, 4, 4
    assert lib.ddcca_extract_features(h, one, one, 2, 16, 16, ctypes.byref(m), one) == E   # null filters
    assert lib.ddcca_extract_features(h, one, one, 2, 16, 16, None, one) == E
    for s in range(2):
        for d in range(2):
            m.W[s][d] = 256
    m.L2 = 13
    assert lib.ddcca_extract_features(h, one, one, 2, 16, 16, ctypes.byref(m), one) == E
    m.L2 = 4
    assert lib.ddcca_extract_features(h, one, one, 0, 16, 16, ctypes.byref(m), one) == binding.OK
    # profiling
    assert lib.ddcca_profile_read(h, 99, None, None) == E
    lib.ddcca_destroy(h)


def test_validation_of_the_widened_calls(binding):
    """Information-quality output, fused last stage and the arithmetic options: host-side validation."""
    lib = binding.lib()
    h = make_ctx(binding)
    one = ctypes.c_void_p(256)
    E = binding.EINVAL
    # hash_iq: feature type, then the checks of hash_histogram
    assert lib.ddcca_hash_iq(h, one, 2, 8, 16, 16, 8, 8, 4, 4, 7, one) == E
    assert b"feature type" in lib.ddcca_last_error(h)
    assert lib.ddcca_hash_iq(h, one, 2, 13, 16, 16, 8, 8, 4, 4, binding.FEAT_IQ_F32, one) == E
    assert lib.ddcca_hash_iq(h, one, 2, 8, 16, 16, 8, 8, 4, 4, binding.FEAT_IQ_F16, None) == E
    assert lib.ddcca_hash_iq(h, one, 0, 8, 16, 16, 8, 8, 4, 4, binding.FEAT_IQ_F16, one) == binding.OK
    # apply_stage_hash: the checks of apply_stage and of hash_histogram
    args = (8, 4, 4)
    assert lib.ddcca_apply_stage_hash(h, one, 2, 16, 16, one, 4, 4, 8, *args, 0, one) == E      # even k
    assert lib.ddcca_apply_stage_hash(h, one, 2, 16, 16, one, 5, 13, 8, *args, 0, one) == E     # L2 > 12
    assert lib.ddcca_apply_stage_hash(h, one, 2, 16, 16, one, 5, 4, 32, *args, 0, one) == E     # block > map
    assert lib.ddcca_apply_stage_hash(h, one, 2, 16, 16, None, 5, 4, 8, *args, 0, one) == E     # null filters
    assert lib.ddcca_apply_stage_hash(h, one, 2, 16, 16, one, 5, 4, 8, *args, 3, one) == E      # feature type
    assert lib.ddcca_apply_stage_hash(h, one, 0, 16, 16, one, 5, 4, 8, *args, 0, one) == binding.OK
    # extract_features_fused / extract_iq_features
    m = binding._Model()
    m.k, m.L1, m.L2, m.block_h, m.block_w, m.stride_y, m.stride_x = 5, 4, 4, 8, 8, 4, 4
    assert lib.ddcca_extract_features_fused(h, one, one, 2, 16, 16, ctypes.byref(m), 0, one) == E   # null filters
    for s in range(2):
        for d in range(2):
            m.W[s][d] = 256
    assert lib.ddcca_extract_features_fused(h, one, one, 2, 16, 16, ctypes.byref(m), 9, one) == E
    assert lib.ddcca_extract_iq_features(h, one, one, 2, 16, 16, ctypes.byref(m), 9, one) == E
    assert lib.ddcca_extract_features_fused(h, one, one, 0, 16, 16, ctypes.byref(m), 0, one) == binding.OK
    # options: known values are accepted without a GPU, anything else is rejected
    assert lib.ddcca_set_option(h, binding.OPT_CONV_ARITH, binding.CONV_BF16X3) == binding.OK
    assert lib.ddcca_set_option(h, binding.OPT_GRAM_ARITH, binding.GRAM_BF16X3) == binding.OK
    assert lib.ddcca_set_option(h, binding.OPT_GRAM_ARITH, binding.GRAM_LAG_FP32) == binding.OK
    assert lib.ddcca_set_option(h, binding.OPT_GRAM_ARITH, 3) == E
    assert lib.ddcca_set_option(h, binding.OPT_GRAM_ARITH, binding.GRAM_FP32) == binding.OK
    assert lib.ddcca_set_option(h, binding.OPT_CONV_ARITH, binding.CONV_AUTO) == binding.OK
    assert lib.ddcca_set_option(h, binding.OPT_CONV_ARITH, 3) == E
    assert lib.ddcca_set_option(h, binding.OPT_GRAM_ARITH, -1) == E
    assert lib.ddcca_set_option(h, binding.OPT_NEXT_STAGE_MAPS, binding.MAPS_RECOMPUTED) == binding.OK
    assert lib.ddcca_set_option(h, binding.OPT_NEXT_STAGE_MAPS, binding.MAPS_STREAMED) == binding.OK
    assert lib.ddcca_set_option(h, binding.OPT_NEXT_STAGE_MAPS, 2) == E
    assert lib.ddcca_set_option(h, 99, 0) == E
    assert lib.ddcca_set_option(None, binding.OPT_CONV_ARITH, 0) == E
    # timing selection: any mask with a known kernel id; none is an error
    assert lib.ddcca_profile_select(h, 1) == binding.OK
    assert lib.ddcca_profile_select(h, 0xFFFFFFFF) == binding.OK
    assert lib.ddcca_profile_select(h, 0) == E
    assert lib.ddcca_profile_select(h, 1 << 20) == E
    assert lib.ddcca_profile_select(None, 1) == E
    lib.ddcca_destroy(h)


def test_validation_of_next_stage_learning(binding):
    """ddcca_learn_next_stage_filters: every argument check happens on the host, before any device work."""
    lib = binding.lib()
    h = make_ctx(binding)
    one = ctypes.c_void_p(256)
    E = binding.EINVAL

    def call(v1=one, cls=one, n_img=4, G_in=1, hh=16, ww=16, n_cls=2, Wp=one, k_prev=5, L_prev=4, k=5, L=4,
             ridge=1e-4, batch=0, W1=one):
        return lib.ddcca_learn_next_stage_filters(h, v1, one, cls, n_img, G_in, hh, ww, n_cls, Wp, one, k_prev,
                                                  L_prev, k, L, ridge, batch, W1, one, one)

    assert call(v1=None) == E
    assert call(cls=None) == E
    assert call(Wp=None) == E
    assert call(W1=None) == E
    assert call(n_img=0) == E
    assert call(k=4) == E and call(k_prev=11) == E
    assert call(L=25) == E and call(L_prev=25) == E and call(L_prev=0) == E
    assert call(G_in=0) == E
    assert call(G_in=1024, L_prev=8) == E           # G_in * L_prev > 4096
    assert call(ridge=0.0) == E
    assert call(batch=-1) == E
    assert b"batch" in lib.ddcca_last_error(h)
    assert lib.ddcca_learn_next_stage_filters(None, one, one, one, 4, 1, 16, 16, 2, one, one, 5, 4, 5, 4, 1e-4, 0,
                                              one, one, one) == E
    lib.ddcca_destroy(h)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr


def test_compute_without_gpu_fails_loudly(binding):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    lib = binding.lib()
    h = make_ctx(binding)
    rc = lib.ddcca_corr_begin(h, 5, 2, 1, 8, 8)
    assert rc == binding.EHIP
    assert len(lib.ddcca_last_error(h)) > 0
    lib.ddcca_destroy(h)


def test_binding_rejects_wrong_tensors(binding):
    import torch
    ctx = binding.Context(0)
    x = torch.zeros((2, 8, 8), dtype=torch.float32)         # CPU tensor
    W = torch.zeros((4, 5, 5), dtype=torch.float32)
    with pytest.raises(ValueError):
        ctx.apply_stage(x, W)
    with pytest.raises(TypeError):
        ctx.apply_stage(x.double(), W)
    ctx.close()


def test_workloads_are_deterministic_and_shaped():
    import numpy as np
    from paper_2209_13027_amd.workloads import WORKLOADS, make_views
    wl = WORKLOADS["tiny"]
    a = make_views(wl)
    b = make_views(wl)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    v1, v2, cls = a
    assert v1.shape == (40, 32, 32) and v1.dtype == np.float32 and v2.min() >= 0
    assert np.bincount(cls).tolist() == [10, 10, 10, 10]
    assert wl.blocks == (7, 7) and wl.feature_len == 6272
    assert WORKLOADS["small_face"].blocks == (27, 22) and WORKLOADS["small_face"].feature_len == 2433024
    assert WORKLOADS["object"].feature_len == 921600 and WORKLOADS["stress"].blocks == (15, 15)
    # large_scale class sizes: 257 classes, >= 80 each, 30607 in total
    from paper_2209_13027_amd.workloads import _class_sizes, BASE_SEED
    ls = WORKLOADS["large_scale"]
    sizes = _class_sizes(ls, np.random.Generator(np.random.PCG64(BASE_SEED + ls.index)))
    assert len(sizes) == 257 and sizes.sum() == 30607 and sizes.min() >= 80 and sizes.max() <= 827

"""ctypes binding of libddcca: argument marshalling only.

Every function takes torch tensors that already live on the GPU, checks dtype /
contiguity / device, and passes their data pointers to the C ABI call of the same name
(see include/ddcca.h).  No arithmetic happens here; if the HIP library is missing the
import of this module's `lib()` fails loudly -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libddcca.so")

OK, EINVAL, ESTATE, ENOMEM, EHIP, EOVERFLOW, ELABEL, ENUMERIC = 0, -1, -2, -3, -4, -5, -6, -7
K_GRAM, K_CLASS_SUM, K_REDUCE, K_SOLVE, K_CONV, K_HASH_HIST, K_GRAM_CROSS, K_CONV_HASH_HIST, K_COUNT = range(9)
KERNEL_NAMES = ["gram", "class_sum", "reduce", "solve", "conv", "hash_hist", "gram_cross", "conv_hash_hist"]

EXPORTS = [
    "ddcca_create", "ddcca_destroy", "ddcca_last_error", "ddcca_status",
    "ddcca_corr_begin", "ddcca_corr_accumulate", "ddcca_corr_export", "ddcca_solve_filters",
    "ddcca_dcca_solve", "ddcca_dcca_solve_noalloc", "ddcca_learn_stage_filters", "ddcca_apply_stage", "ddcca_hash_histogram",
    "ddcca_extract_features", "ddcca_hash_iq", "ddcca_extract_iq_features",
    "ddcca_apply_stage_hash", "ddcca_extract_features_fused", "ddcca_set_option",
    "ddcca_learn_next_stage_filters", "ddcca_profile_select",
    "ddcca_profile_enable", "ddcca_profile_read", "ddcca_profile_reset",
]
FEAT_COUNT_U16, FEAT_IQ_F32, FEAT_IQ_F16 = 0, 1, 2
OPT_CONV_ARITH, OPT_GRAM_ARITH, OPT_NEXT_STAGE_MAPS = 1, 2, 3
MAPS_STREAMED, MAPS_RECOMPUTED = 0, 1
CONV_FP32, CONV_BF16X3, CONV_AUTO = 0, 1, 2
GRAM_FP32, GRAM_BF16X3, GRAM_LAG_FP32 = 0, 1, 2
FEAT_TYPES = {torch.uint16: FEAT_COUNT_U16, torch.float32: FEAT_IQ_F32, torch.float16: FEAT_IQ_F16}


class DdccaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libddcca error {code}: {message}")
        self.code = code


class _Model(ctypes.Structure):
    _fields_ = [
        ("k", ctypes.c_int), ("L1", ctypes.c_int), ("L2", ctypes.c_int),
        ("block_h", ctypes.c_int), ("block_w", ctypes.c_int),
        ("stride_y", ctypes.c_int), ("stride_x", ctypes.c_int),
        ("W", (ctypes.c_void_p * 2) * 2),
        ("batch_images", ctypes.c_int64),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """Load the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        l = ctypes.CDLL(LIB_PATH)
        vp, i, i64, d = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_double
        l.ddcca_create.argtypes = [ctypes.POINTER(vp), i, vp]
        l.ddcca_destroy.argtypes = [vp]
        l.ddcca_destroy.restype = None
        l.ddcca_last_error.argtypes = [vp]
        l.ddcca_last_error.restype = ctypes.c_char_p
        l.ddcca_status.argtypes = [vp]
        l.ddcca_corr_begin.argtypes = [vp, i, i, i, i, i]
        l.ddcca_corr_accumulate.argtypes = [vp, vp, vp, vp, i64]
        l.ddcca_corr_export.argtypes = [vp, vp, vp, vp, vp, vp]
        l.ddcca_solve_filters.argtypes = [vp, i, d, vp, vp, vp]
        l.ddcca_dcca_solve.argtypes = [vp, vp, vp, vp, vp, i, i, d, vp, vp, vp]
        l.ddcca_dcca_solve_noalloc.argtypes = [vp, vp, vp, vp, vp, i, i, d, vp, vp, vp]
        l.ddcca_learn_stage_filters.argtypes = [vp, vp, vp, vp, i64, i, i, i, i, i, i, d, vp, vp, vp]
        l.ddcca_apply_stage.argtypes = [vp, vp, i64, i, i, vp, i, i, vp]
        l.ddcca_hash_histogram.argtypes = [vp, vp, i64, i, i, i, i, i, i, i, vp]
        l.ddcca_extract_features.argtypes = [vp, vp, vp, i64, i, i, ctypes.POINTER(_Model), vp]
        l.ddcca_hash_iq.argtypes = [vp, vp, i64, i, i, i, i, i, i, i, i, vp]
        l.ddcca_extract_iq_features.argtypes = [vp, vp, vp, i64, i, i, ctypes.POINTER(_Model), i, vp]
        l.ddcca_apply_stage_hash.argtypes = [vp, vp, i64, i, i, vp, i, i, i, i, i, i, i, vp]
        l.ddcca_extract_features_fused.argtypes = [vp, vp, vp, i64, i, i, ctypes.POINTER(_Model), i, vp]
        l.ddcca_set_option.argtypes = [vp, i, i]
        l.ddcca_learn_next_stage_filters.argtypes = [vp, vp, vp, vp, i64, i, i, i, i, vp, vp, i, i, i, i, d, i64,
                                                     vp, vp, vp]
        l.ddcca_profile_enable.argtypes = [vp, i]
        l.ddcca_profile_select.argtypes = [vp, ctypes.c_uint]
        l.ddcca_profile_read.argtypes = [vp, i, ctypes.POINTER(d), ctypes.POINTER(i64)]
        l.ddcca_profile_reset.argtypes = [vp]
        _lib = l
    return _lib


def _ptr(t, dtype, name):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name}: expected a torch tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    if not t.is_cuda:
        raise ValueError(f"{name}: tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name}: tensor must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


class Context:
    """Owns one ddcca_ctx bound to a device and to torch's current stream on it."""

    def __init__(self, device: int = 0, stream=None):
        self._h = ctypes.c_void_p()
        self.device = int(device)
        if stream is None and torch.cuda.is_available():
            stream = torch.cuda.current_stream(self.device).cuda_stream
        rc = lib().ddcca_create(ctypes.byref(self._h), self.device, ctypes.c_void_p(stream or 0))
        if rc != OK:
            raise DdccaError(rc, "ddcca_create failed")

    def close(self):
        if self._h:
            lib().ddcca_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != OK:
            raise DdccaError(rc, lib().ddcca_last_error(self._h).decode())

    # ---- thin wrappers, same names as the C calls ---------------------------------
    def status(self):
        self._check(lib().ddcca_status(self._h))

    def corr_begin(self, k, n_cls, G, h, w):
        self._check(lib().ddcca_corr_begin(self._h, k, n_cls, G, h, w))

    def corr_accumulate(self, v1, v2, cls, n_img=None):
        n_img = int(cls.shape[0]) if n_img is None else int(n_img)
        self._check(lib().ddcca_corr_accumulate(self._h, _ptr(v1, torch.float32, "v1"), _ptr(v2, torch.float32, "v2"),
                                                _ptr(cls, torch.int32, "cls"), n_img))

    def corr_export(self, k):
        D = k * k
        out = [torch.empty((D, D), dtype=torch.float64, device=f"cuda:{self.device}") for _ in range(5)]
        self._check(lib().ddcca_corr_export(self._h, *[_ptr(o, torch.float64, "C") for o in out]))
        return dict(zip(["C11", "C22", "C12", "Cw", "CT"], out))

    def _filter_outputs(self, k, L):
        dev = f"cuda:{self.device}"
        return (torch.empty((L, k, k), dtype=torch.float32, device=dev),
                torch.empty((L, k, k), dtype=torch.float32, device=dev),
                torch.empty((L,), dtype=torch.float64, device=dev))

    def solve_filters(self, k, L, ridge=1e-4):
        W1, W2, rho = self._filter_outputs(k, L)
        self._check(lib().ddcca_solve_filters(self._h, L, ridge, _ptr(W1, torch.float32, "W1"),
                                              _ptr(W2, torch.float32, "W2"), _ptr(rho, torch.float64, "rho")))
        return W1, W2, rho

    def dcca_solve(self, C11, C22, Cw, CT, k, L, ridge=1e-4):
        W1, W2, rho = self._filter_outputs(k, L)
        self._check(lib().ddcca_dcca_solve(self._h, _ptr(C11, torch.float64, "C11"), _ptr(C22, torch.float64, "C22"),
                                           _ptr(Cw, torch.float64, "Cw"), _ptr(CT, torch.float64, "CT"), k, L, ridge,
                                           _ptr(W1, torch.float32, "W1"), _ptr(W2, torch.float32, "W2"),
                                           _ptr(rho, torch.float64, "rho")))
        return W1, W2, rho

    def dcca_solve_noalloc(self, C11, C22, Cw, CT, k, L, ridge, W1, W2, rho):
        """ddcca_dcca_solve without any allocation: the caller brings the outputs W1, W2 ([L, k, k] float32) and rho
        ([L] float64); nothing is allocated here or in the library."""
        self._check(lib().ddcca_dcca_solve_noalloc(
            self._h, _ptr(C11, torch.float64, "C11"), _ptr(C22, torch.float64, "C22"), _ptr(Cw, torch.float64, "Cw"),
            _ptr(CT, torch.float64, "CT"), k, L, ridge, _ptr(W1, torch.float32, "W1"), _ptr(W2, torch.float32, "W2"),
            _ptr(rho, torch.float64, "rho")))

    def learn_stage_filters(self, v1, v2, cls, G, h, w, n_cls, k, L, ridge=1e-4):
        """v1, v2: [n_img*G, h, w] (or [n_img, G, h, w]) float32; cls: [n_img] int32."""
        n_img = int(cls.shape[0])
        if v1.numel() != n_img * G * h * w or v2.numel() != n_img * G * h * w:
            raise ValueError("view tensors do not match n_img * G * h * w")
        W1, W2, rho = self._filter_outputs(k, L)
        self._check(lib().ddcca_learn_stage_filters(
            self._h, _ptr(v1, torch.float32, "v1"), _ptr(v2, torch.float32, "v2"), _ptr(cls, torch.int32, "cls"),
            n_img, G, h, w, n_cls, k, L, ridge, _ptr(W1, torch.float32, "W1"), _ptr(W2, torch.float32, "W2"),
            _ptr(rho, torch.float64, "rho")))
        return W1, W2, rho

    def learn_next_stage_filters(self, v1, v2, cls, G_in, h, w, n_cls, Wp1, Wp2, k, L, ridge=1e-4, batch_images=0):
        """Filters of the stage after the one with filters Wp1 / Wp2 ([L_prev, k_prev, k_prev]), learned from that
        stage's INPUTS v1, v2 ([n_img * G_in, h, w]) without holding its maps."""
        n_img = int(cls.shape[0])
        if v1.numel() != n_img * G_in * h * w or v2.numel() != n_img * G_in * h * w:
            raise ValueError("view tensors do not match n_img * G_in * h * w")
        L_prev, k_prev, _ = Wp1.shape
        if tuple(Wp2.shape) != tuple(Wp1.shape):
            raise ValueError("the two views' filter banks differ in shape")
        W1, W2, rho = self._filter_outputs(k, L)
        self._check(lib().ddcca_learn_next_stage_filters(
            self._h, _ptr(v1, torch.float32, "v1"), _ptr(v2, torch.float32, "v2"), _ptr(cls, torch.int32, "cls"),
            n_img, G_in, h, w, n_cls, _ptr(Wp1, torch.float32, "Wp1"), _ptr(Wp2, torch.float32, "Wp2"), k_prev,
            L_prev, k, L, ridge, batch_images, _ptr(W1, torch.float32, "W1"), _ptr(W2, torch.float32, "W2"),
            _ptr(rho, torch.float64, "rho")))
        return W1, W2, rho

    def apply_stage(self, x, W, out=None):
        """x: [n, h, w] float32; W: [L, k, k] float32 -> [n, L, h, w] float32."""
        n, h, w = x.shape
        L, k, _ = W.shape
        if out is None:
            out = torch.empty((n, L, h, w), dtype=torch.float32, device=x.device)
        elif out.numel() != n * L * h * w:
            raise ValueError("out has the wrong size")
        self._check(lib().ddcca_apply_stage(self._h, _ptr(x, torch.float32, "x"), n, h, w,
                                            _ptr(W, torch.float32, "W"), k, L, _ptr(out, torch.float32, "out")))
        return out

    def hash_histogram(self, maps, block, stride, out=None):
        """maps: [n, L2, h, w] float32 -> [n, nby, nbx, 2**L2] uint16."""
        n, L2, h, w = maps.shape
        bh, bw = (block, block) if isinstance(block, int) else block
        sy, sx = (stride, stride) if isinstance(stride, int) else stride
        if h < bh or w < bw or sy < 1 or sx < 1:
            nby = nbx = 0
        else:
            nby, nbx = (h - bh) // sy + 1, (w - bw) // sx + 1
        if out is None:
            out = torch.empty((n, nby, nbx, 1 << L2), dtype=torch.uint16, device=maps.device)
        self._check(lib().ddcca_hash_histogram(self._h, _ptr(maps, torch.float32, "maps"), n, L2, h, w, bh, bw, sy, sx,
                                               _ptr(out, torch.uint16, "hist")))
        return out

    def hash_iq(self, maps, block, stride, dtype=torch.float32, out=None):
        """maps: [n, L2, h, w] float32 -> [n, nby, nbx, 2**L2] information quality, float32 or float16."""
        n, L2, h, w = maps.shape
        bh, bw = (block, block) if isinstance(block, int) else block
        sy, sx = (stride, stride) if isinstance(stride, int) else stride
        if h < bh or w < bw or sy < 1 or sx < 1:
            nby = nbx = 0
        else:
            nby, nbx = (h - bh) // sy + 1, (w - bw) // sx + 1
        if out is None:
            out = torch.empty((n, nby, nbx, 1 << L2), dtype=dtype, device=maps.device)
        self._check(lib().ddcca_hash_iq(self._h, _ptr(maps, torch.float32, "maps"), n, L2, h, w, bh, bw, sy, sx,
                                        FEAT_TYPES[dtype], _ptr(out, dtype, "out")))
        return out

    def apply_stage_hash(self, x, W, block, stride, dtype=torch.uint16, out=None):
        """x: [n, h, w]; W: [L2, k, k] -> [n, nby, nbx, 2**L2]: stage convolution fused with hashing and block
        histograms (counts, or information quality for float dtypes)."""
        n, h, w = x.shape
        L2, k = W.shape[0], W.shape[1]
        bh, bw = (block, block) if isinstance(block, int) else block
        sy, sx = (stride, stride) if isinstance(stride, int) else stride
        if h < bh or w < bw or sy < 1 or sx < 1:
            nby = nbx = 0
        else:
            nby, nbx = (h - bh) // sy + 1, (w - bw) // sx + 1
        if out is None:
            out = torch.empty((n, nby, nbx, 1 << L2), dtype=dtype, device=x.device)
        self._check(lib().ddcca_apply_stage_hash(self._h, _ptr(x, torch.float32, "x"), n, h, w,
                                                 _ptr(W, torch.float32, "W"), k, L2, bh, bw, sy, sx,
                                                 FEAT_TYPES[dtype], _ptr(out, dtype, "out")))
        return out

    def extract_iq_features(self, v1, v2, filters, k, L1, L2, block, stride, dtype=torch.float32, batch_images=0,
                            out=None):
        """As extract_features, with -log p(t) per bin (float32 / float16) instead of the counts."""
        return self.extract_features(v1, v2, filters, k, L1, L2, block, stride, batch_images, out, dtype)

    def extract_features(self, v1, v2, filters, k, L1, L2, block, stride, batch_images=0, out=None,
                         dtype=torch.uint16, fused=False):
        """filters = (W1_stage1, W2_stage1, W1_stage2, W2_stage2) -> [m, 2, L1, nby, nbx, 2**L2] uint16."""
        m, h, w = v1.shape
        bh, bw = (block, block) if isinstance(block, int) else block
        sy, sx = (stride, stride) if isinstance(stride, int) else stride
        nby, nbx = (h - bh) // sy + 1, (w - bw) // sx + 1
        if out is None:
            out = torch.empty((m, 2, L1, nby, nbx, 1 << L2), dtype=dtype, device=v1.device)
        model = _Model()
        model.k, model.L1, model.L2 = k, L1, L2
        model.block_h, model.block_w, model.stride_y, model.stride_x = bh, bw, sy, sx
        names = ["W1_stage1", "W2_stage1", "W1_stage2", "W2_stage2"]
        for s in range(2):
            for d in range(2):
                model.W[s][d] = _ptr(filters[2 * s + d], torch.float32, names[2 * s + d])
        model.batch_images = int(batch_images)
        if fused:
            self._check(lib().ddcca_extract_features_fused(self._h, _ptr(v1, torch.float32, "v1"),
                                                           _ptr(v2, torch.float32, "v2"), m, h, w,
                                                           ctypes.byref(model), FEAT_TYPES[dtype],
                                                           _ptr(out, dtype, "feat")))
        elif dtype == torch.uint16:
            self._check(lib().ddcca_extract_features(self._h, _ptr(v1, torch.float32, "v1"),
                                                     _ptr(v2, torch.float32, "v2"), m, h, w, ctypes.byref(model),
                                                     _ptr(out, torch.uint16, "feat")))
        else:
            self._check(lib().ddcca_extract_iq_features(self._h, _ptr(v1, torch.float32, "v1"),
                                                        _ptr(v2, torch.float32, "v2"), m, h, w, ctypes.byref(model),
                                                        FEAT_TYPES[dtype], _ptr(out, dtype, "feat")))
        return out

    def set_option(self, option: int, value: int):
        self._check(lib().ddcca_set_option(self._h, option, value))

    # ---- profiling -------------------------------------------------------------------
    def profile_enable(self, on: bool):
        self._check(lib().ddcca_profile_enable(self._h, 1 if on else 0))

    def profile_select(self, names=None):
        """Time only the named kernel families (KERNEL_NAMES) while profiling is on; None = all."""
        mask = 0xFFFFFFFF if names is None else sum(1 << KERNEL_NAMES.index(n) for n in names)
        self._check(lib().ddcca_profile_select(self._h, mask))

    def profile_reset(self):
        self._check(lib().ddcca_profile_reset(self._h))

    def profile_read(self) -> dict:
        out = {}
        for kid, name in enumerate(KERNEL_NAMES):
            ms, cnt = ctypes.c_double(), ctypes.c_int64()
            self._check(lib().ddcca_profile_read(self._h, kid, ctypes.byref(ms), ctypes.byref(cnt)))
            out[name] = {"ms": ms.value, "launches": cnt.value}
        return out

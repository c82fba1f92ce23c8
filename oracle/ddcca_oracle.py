"""CPU fp64 oracle of the two-stage DDCCANet feature extractor -- TEST INFRASTRUCTURE ONLY.

A thin numpy front end over `ddcca_oracle.c` (plain C loops) plus the small dense
linear algebra of the DCCA solve written out step by step.  Only the tests, the smoke
check and the benchmark's CPU-baseline leg may import this module; the product package
never does, and nothing here touches the HIP library.

Everything is float64; fp32 inputs are widened, never the other way round.
Section / equation numbers refer to the paper (Section II: model; Section III: batching).

Pins (tests/test_oracle_*.py): patch sums, brute-force Gram, batch-split invariance
(Eq. 15), pair-loop C_w / C_b, eigen residuals and library cross-checks for the solve,
brute-forced objective (Eq. 2-3), conv/Gram tie, histogram sums and bincount,
information quality (Eq. 10): probabilities sum to one, hand-computed block, monotone;
the composite routines: second-stage C_w / C_b of learn_two_stage against explicit
image-pair loops over maps that scipy computes per image, extract_features per image and
per map against scipy correlation + bincount.
Numeric values of filters / features on the paper's own data: parity unpinned (the
paper prints no intermediate value and its data sets are not available).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ddcca_oracle.c")
_SO = os.path.join(_HERE, "libddcca_oracle.so")
_lib_handle = None

_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)


def build(force: bool = False) -> str:
    """Compile the C part with gcc (OpenMP)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _SO, _SRC, "-lm"])
    return _SO


def _lib():
    global _lib_handle
    if _lib_handle is None:
        build()
        _lib_handle = ctypes.CDLL(_SO)
        _lib_handle.orc_num_threads.restype = ctypes.c_int
        _lib_handle.orc_jacobi_sym.restype = ctypes.c_int
    return _lib_handle


def num_threads() -> int:
    return int(_lib().orc_num_threads())


def _d(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a, t=_f64p):
    return a.ctypes.data_as(t)


# ----------------------------------------------------------------------------- O1
def patch_matrix(V, k: int) -> np.ndarray:
    """Eq. 1: the D x (n*h*w) matrix of mean-removed, zero-padded k*k patches, one per
    pixel, column order (image, y, x).  For small inputs only."""
    V = _d(V)
    n, h, w = V.shape
    D = k * k
    out = np.empty((n * h * w, D))
    buf = np.empty(D)
    lib = _lib()
    col = 0
    for m in range(n):
        for y in range(h):
            for x in range(w):
                lib.orc_patch(_p(V[m]), h, w, k, y, x, _p(buf))
                out[col] = buf
                col += 1
    return out.T.copy()


# ----------------------------------------------------------------------------- O2
def corr_sums(V1, V2, k: int, into=None):
    """Un-normalised S11, S22, S12 over all patches (Section II-A; Eq. 15 lets `into`
    carry the running sums from earlier batches)."""
    V1, V2 = _d(V1), _d(V2)
    assert V1.shape == V2.shape
    n, h, w = V1.shape
    D = k * k
    if into is None:
        into = (np.zeros((D, D)), np.zeros((D, D)), np.zeros((D, D)))
    S11, S22, S12 = into
    _lib().orc_corr_sums(_p(V1), _p(V2), ctypes.c_int64(n), h, w, k, _p(S11), _p(S22), _p(S12))
    return S11, S22, S12


def class_sums(V1, V2, cls, grp, n_cls: int, n_grp: int, k: int):
    """Un-normalised same-class (Sw) and all-pairs (ST) cross-view sums."""
    V1, V2 = _d(V1), _d(V2)
    n, h, w = V1.shape
    cls = np.ascontiguousarray(cls, dtype=np.int32)
    grp = np.ascontiguousarray(grp, dtype=np.int32)
    assert cls.shape == (n,) and grp.shape == (n,)
    assert cls.min(initial=0) >= 0 and cls.max(initial=0) < n_cls
    assert grp.min(initial=0) >= 0 and grp.max(initial=0) < n_grp
    D = k * k
    Sw, ST = np.empty((D, D)), np.empty((D, D))
    _lib().orc_class_sums(_p(V1), _p(V2), _p(cls, _i32p), _p(grp, _i32p), ctypes.c_int64(n),
                          n_cls, n_grp, h, w, k, _p(Sw), _p(ST))
    return Sw, ST


def corr_entries(V1, V2, k: int, entries):
    """Selected entries of the un-normalised sums: entries = [(va, a, vb, b), ...] gives
    sum over patches of x^{va}[a] * x^{vb}[b]  (va, vb in {1, 2})."""
    V1, V2 = _d(V1), _d(V2)
    n, h, w = V1.shape
    e = np.ascontiguousarray(entries, dtype=np.int32)
    va, a, vb, b = (np.ascontiguousarray(e[:, i]) for i in range(4))
    out = np.empty(len(e))
    _lib().orc_corr_entries(_p(V1), _p(V2), ctypes.c_int64(n), h, w, k, len(e),
                            _p(va, _i32p), _p(a, _i32p), _p(vb, _i32p), _p(b, _i32p), _p(out))
    return out


def stage_matrices(V1, V2, cls, grp, n_cls: int, n_grp: int, k: int) -> dict:
    """The five D x D matrices of one stage, each divided by the patch count N:
    C11, C22, C12 (within-view and plain cross-view), Cw (same-class pairs), CT (all
    pairs); Cb = CT - Cw (different-class pairs) and Ctilde = Cw - Cb (Section II-A)."""
    n, h, w = np.shape(V1)
    N = float(n * h * w)
    S11, S22, S12 = corr_sums(V1, V2, k)
    Sw, ST = class_sums(V1, V2, cls, grp, n_cls, n_grp, k)
    out = {"C11": S11 / N, "C22": S22 / N, "C12": S12 / N, "Cw": Sw / N, "CT": ST / N, "N": N}
    out["Cb"] = out["CT"] - out["Cw"]
    out["Ctilde"] = out["Cw"] - out["Cb"]
    return out


# ----------------------------------------------------------------------------- O3-O5
def jacobi_sym(A, tol: float = 1e-15, max_sweeps: int = 60):
    """Eigen-decomposition of a symmetric matrix by cyclic Jacobi rotations.
    Returns (eigenvalues, eigenvectors as columns, sweeps)."""
    A = _d(A).copy()
    n = A.shape[0]
    V = np.empty((n, n))
    sweeps = _lib().orc_jacobi_sym(_p(A), n, _p(V), ctypes.c_double(tol), max_sweeps)
    return np.diag(A).copy(), V, sweeps


def ridge_matrices(C11, C22, ridge: float):
    """B_d = C_dd + eps_d I with eps_d = ridge * trace(C_dd) / D.  After per-patch mean
    removal C_dd annihilates the constant vector, so Eq. 3 needs a regulariser."""
    D = C11.shape[0]
    B1 = C11 + (ridge * np.trace(C11) / D) * np.eye(D)
    B2 = C22 + (ridge * np.trace(C22) / D) * np.eye(D)
    return B1, B2


def sign_rule(w1: np.ndarray, w2: np.ndarray):
    """Make the largest-magnitude entry of w1 positive (lowest index on ties) and flip
    w2 with it, so that rho keeps its sign."""
    j = int(np.argmax(np.abs(w1)))
    if w1[j] < 0:
        return -w1, -w2
    return w1, w2


def dcca_solve(C11, C22, Ctilde, L: int, ridge: float = 1e-4) -> dict:
    """Eq. 2-3: the L pairs (w1, w2) with the largest w1^T Ctilde w2 under
    w1^T B1 w1 = w2^T B2 w2 = 1, pairs mutually B-orthogonal.

    Steps: B_d = R_d^T R_d (Cholesky); T = R1^{-T} Ctilde R2^{-1}; the symmetric
    K = [[0, T], [T^T, 0]] has eigenvalues +-sigma_j with eigenvectors [u_j; +-v_j]/sqrt2
    where T = sum sigma_j u_j v_j^T; w1 = R1^{-1} u, w2 = R2^{-1} v, rho = sigma.
    """
    C11, C22, Ctilde = _d(C11), _d(C22), _d(Ctilde)
    D = C11.shape[0]
    assert 1 <= L <= D - 1
    B1, B2 = ridge_matrices(C11, C22, ridge)
    R1 = np.linalg.cholesky(B1).T          # upper, B1 = R1^T R1
    R2 = np.linalg.cholesky(B2).T
    R1i, R2i = np.linalg.inv(R1), np.linalg.inv(R2)
    T = R1i.T @ Ctilde @ R2i
    K = np.zeros((2 * D, 2 * D))
    K[:D, D:] = T
    K[D:, :D] = T.T
    lam, E, sweeps = jacobi_sym(K)
    order = np.argsort(-lam, kind="stable")
    W1 = np.empty((L, D))
    W2 = np.empty((L, D))
    rho = np.empty(L)
    for g in range(L):
        j = order[g]
        u, v = E[:D, j], E[D:, j]
        w1 = np.sqrt(2.0) * (R1i @ u)
        w2 = np.sqrt(2.0) * (R2i @ v)
        w1 = w1 / np.sqrt(w1 @ B1 @ w1)
        w2 = w2 / np.sqrt(w2 @ B2 @ w2)
        w1, w2 = sign_rule(w1, w2)
        W1[g], W2[g], rho[g] = w1, w2, w1 @ Ctilde @ w2
    sig = np.sort(lam)[::-1][:D]           # all canonical correlations, descending
    gaps = np.empty(L)
    for g in range(L):
        lo = sig[g] - sig[g + 1]
        hi = sig[g - 1] - sig[g] if g > 0 else np.inf
        gaps[g] = min(lo, hi) / sig[0]
    return {"W1": W1, "W2": W2, "rho": rho, "sigma": sig, "gap": gaps, "B1": B1, "B2": B2,
            "sweeps": sweeps}


def learn_stage(V1, V2, cls, grp, n_cls, n_grp, k, L, ridge=1e-4) -> dict:
    """One stage of filter learning: matrices, then the DCCA solve; filters reshaped
    row-major to k x k (Eq. 4-5)."""
    mats = stage_matrices(V1, V2, cls, grp, n_cls, n_grp, k)
    sol = dcca_solve(mats["C11"], mats["C22"], mats["Ctilde"], L, ridge)
    sol.update(mats)
    sol["F1"] = sol["W1"].reshape(L, k, k)
    sol["F2"] = sol["W2"].reshape(L, k, k)
    return sol


# ----------------------------------------------------------------------------- O6-O9
def conv(V, F) -> np.ndarray:
    """Eq. 6: [n,h,w] images x [L,k,k] filters -> [n,L,h,w] maps (zero padding, no flip)."""
    V, F = _d(V), _d(F)
    n, h, w = V.shape
    L, k, _ = F.shape
    out = np.empty((n, L, h, w))
    _lib().orc_conv(_p(V), ctypes.c_int64(n), h, w, _p(F), L, k, _p(out))
    return out


def hash_maps(Z) -> np.ndarray:
    """Eq. 7-9: [n,L2,h,w] maps -> [n,h,w] int32 codes."""
    Z = _d(Z)
    n, L2, h, w = Z.shape
    Q = np.empty((n, h, w), dtype=np.int32)
    _lib().orc_hash(_p(Z), ctypes.c_int64(n), L2, h, w, _p(Q, _i32p))
    return Q


def block_hist(Q, block, stride, bins: int) -> np.ndarray:
    """Section II-C: per-block code counts, [n, nby, nbx, bins] int64.  `block` and
    `stride` are ints or (y, x) pairs."""
    Q = np.ascontiguousarray(Q, dtype=np.int32)
    n, h, w = Q.shape
    bh, bw = (block, block) if np.isscalar(block) else block
    sy, sx = (stride, stride) if np.isscalar(stride) else stride
    assert Q.min(initial=0) >= 0 and Q.max(initial=0) < bins
    nby, nbx = (h - bh) // sy + 1, (w - bw) // sx + 1
    hist = np.empty((n, nby, nbx, bins), dtype=np.int64)
    _lib().orc_block_hist(_p(Q, _i32p), ctypes.c_int64(n), h, w, bh, bw, sy, sx, bins, _p(hist, _i64p))
    return hist


def iq_features(hist, block_area: int) -> np.ndarray:
    """Eq. 10: information quality o = -log p(t) of every code t in every block, natural
    logarithm.  p(t) is the block's code distribution with one pseudo-count per bin,
    p(t) = (count(t) + 1) / (block_area + bins), so that codes absent from a block (p = 0 in
    the raw frequencies, where Eq. 10 is undefined) get the finite value log(block_area +
    bins) and sum_t p(t) = 1 still holds.  hist: [..., bins] counts; returns float64."""
    hist = np.asarray(hist)
    bins = hist.shape[-1]
    total = float(block_area + bins)
    out = np.empty(hist.shape, dtype=np.float64)
    flat_in, flat_out = hist.reshape(-1), out.reshape(-1)
    step = 1 << 22
    for a in range(0, flat_in.size, step):
        c = flat_in[a:a + step].astype(np.float64)
        flat_out[a:a + step] = -np.log((c + 1.0) / total)
    return out


def default_stride(block: int) -> int:
    """50 % overlap, rounding half up (7 -> 4, 8 -> 4, 16 -> 8)."""
    return (block + 1) // 2


# ----------------------------------------------------------------------------- whole path
def learn_two_stage(V1, V2, cls, n_cls, k, L1, L2, ridge=1e-4) -> dict:
    """Stage 1 on the images, stage 2 on the M*L1 stage-1 maps (map g of view 1 pairs
    with map g of view 2; class of a map = class of its image; group = g)."""
    V1, V2 = _d(V1), _d(V2)
    M, h, w = V1.shape
    cls = np.asarray(cls, dtype=np.int32)
    s1 = learn_stage(V1, V2, cls, np.zeros(M, np.int32), n_cls, 1, k, L1, ridge)
    Y1 = conv(V1, s1["F1"]).reshape(M * L1, h, w)
    Y2 = conv(V2, s1["F2"]).reshape(M * L1, h, w)
    cls2 = np.repeat(cls, L1)
    grp2 = np.tile(np.arange(L1, dtype=np.int32), M)
    s2 = learn_stage(Y1, Y2, cls2, grp2, n_cls, L1, k, L2, ridge)
    return {"stage1": s1, "stage2": s2, "Y1": Y1, "Y2": Y2}


def extract_features(V1, V2, F, k, L1, L2, block, stride=None, keep_maps=False) -> dict:
    """Feature extraction with given filters F = (F1_s1, F2_s1, F1_s2, F2_s2):
    hist[m][d][g][by][bx][t], the layout of Eq. 11-12 (views concatenated per image)."""
    V = [_d(V1), _d(V2)]
    M, h, w = V[0].shape
    stride = default_stride(block) if stride is None else stride
    bins = 1 << L2
    hists, Zs = [], []
    for d in range(2):
        Y = conv(V[d], F[d]).reshape(M * L1, h, w)
        Z = conv(Y, F[2 + d])                      # [M*L1, L2, h, w]
        Q = hash_maps(Z)
        H = block_hist(Q, block, stride, bins)     # [M*L1, nby, nbx, bins]
        hists.append(H.reshape(M, L1, *H.shape[1:]))
        if keep_maps:
            Zs.append(Z)
    out = {"hist": np.stack(hists, axis=1)}
    if keep_maps:
        out["Z"] = Zs
    return out


def two_stage(V1, V2, cls, n_cls, k, L1, L2, block, stride=None, ridge=1e-4) -> dict:
    """Learn both stages on (V1, V2, cls) and extract the features of the same images."""
    model = learn_two_stage(V1, V2, cls, n_cls, k, L1, L2, ridge)
    F = (model["stage1"]["F1"], model["stage1"]["F2"], model["stage2"]["F1"], model["stage2"]["F2"])
    feats = extract_features(V1, V2, F, k, L1, L2, block, stride)
    model["hist"] = feats["hist"]
    return model

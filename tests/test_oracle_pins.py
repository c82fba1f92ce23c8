"""Pins for the CPU oracle: every routine is checked against something other than
itself -- an independently written brute force, a closed form, an invariant the paper
fixes, or a library routine (numpy / scipy are used here only, never in the oracle's
own arithmetic for that step)."""
import math

import numpy as np
import pytest
import scipy.linalg
import scipy.signal
from numpy.lib.stride_tricks import sliding_window_view


def rand_views(rng, n, h, w):
    v1 = rng.standard_normal((n, h, w))
    v2 = np.abs(rng.standard_normal((n, h, w))) + 3.0      # strong DC term, like a gradient magnitude
    return v1, v2


def window_patches(V, k):
    """Independent patch extraction: numpy pad + sliding windows -> [n, h, w, D], mean removed."""
    r = (k - 1) // 2
    Vp = np.pad(V, ((0, 0), (r, r), (r, r)))
    X = sliding_window_view(Vp, (k, k), axis=(1, 2)).reshape(V.shape[0], V.shape[1], V.shape[2], k * k)
    return X - X.mean(axis=-1, keepdims=True)


# ------------------------------------------------------------------ P1 (Eq. 1)
def test_patch_count_and_zero_sum(oracle):
    rng = np.random.default_rng(1)
    V, _ = rand_views(rng, 3, 6, 5)
    for k in (3, 5):
        X = oracle.patch_matrix(V, k)
        assert X.shape == (k * k, 3 * 6 * 5)                 # Eq. 1: l1*l2 x M*p*q
        assert np.abs(X.sum(axis=0)).max() <= 1e-12 * np.abs(V).sum()


def test_patch_hand_example(oracle):
    # 3x3 image, k=3: centre patch is the image minus its mean; the top-left patch sees
    # five zeros of padding and the 2x2 corner, row-major.
    img = np.arange(1.0, 10.0).reshape(1, 3, 3)
    X = oracle.patch_matrix(img, 3)
    centre = X[:, 4]
    assert np.allclose(centre, np.arange(1.0, 10.0) - 5.0, atol=1e-15)
    corner = X[:, 0]
    raw = np.array([0, 0, 0, 0, 1, 2, 0, 4, 5], dtype=float)
    assert np.allclose(corner, raw - raw.sum() / 9.0, atol=1e-15)
    # last column = bottom-right pixel
    raw = np.array([5, 6, 0, 8, 9, 0, 0, 0, 0], dtype=float)
    assert np.allclose(X[:, 8], raw - raw.sum() / 9.0, atol=1e-15)


def test_patch_matches_windows(oracle):
    rng = np.random.default_rng(2)
    V, _ = rand_views(rng, 2, 7, 9)
    X = oracle.patch_matrix(V, 5)
    Xw = window_patches(V, 5).reshape(-1, 25).T
    assert np.abs(X - Xw).max() <= 1e-14


# ------------------------------------------------------------------ P2 (Section II-A)
def test_gram_brute_force_python_loops(oracle):
    rng = np.random.default_rng(3)
    n, h, w, k = 2, 4, 5, 3
    V1, V2 = rand_views(rng, n, h, w)
    D, r = k * k, 1
    S11 = np.zeros((D, D)); S22 = np.zeros((D, D)); S12 = np.zeros((D, D))

    def pix(V, m, y, x):
        return V[m, y, x] if 0 <= y < h and 0 <= x < w else 0.0

    for m in range(n):
        for y in range(h):
            for x in range(w):
                p1 = [pix(V1, m, y + a // k - r, x + a % k - r) for a in range(D)]
                p2 = [pix(V2, m, y + a // k - r, x + a % k - r) for a in range(D)]
                m1, m2 = sum(p1) / D, sum(p2) / D
                for a in range(D):
                    for b in range(D):
                        S11[a, b] += (p1[a] - m1) * (p1[b] - m1)
                        S22[a, b] += (p2[a] - m2) * (p2[b] - m2)
                        S12[a, b] += (p1[a] - m1) * (p2[b] - m2)
    O11, O22, O12 = oracle.corr_sums(V1, V2, k)
    for O, S in ((O11, S11), (O22, S22), (O12, S12)):
        assert np.abs(O - S).max() <= 1e-12 * np.abs(S).max()


def test_gram_matches_window_matmul(oracle):
    rng = np.random.default_rng(4)
    V1, V2 = rand_views(rng, 5, 12, 10)
    for k in (3, 5, 7):
        X1 = window_patches(V1, k).reshape(-1, k * k)
        X2 = window_patches(V2, k).reshape(-1, k * k)
        O11, O22, O12 = oracle.corr_sums(V1, V2, k)
        assert np.abs(O11 - X1.T @ X1).max() <= 1e-12 * np.abs(O11).max()
        assert np.abs(O22 - X2.T @ X2).max() <= 1e-12 * np.abs(O22).max()
        assert np.abs(O12 - X1.T @ X2).max() <= 1e-12 * np.abs(O12).max()
        # symmetric, positive semi-definite, and the constant vector is in the null space
        assert np.abs(O11 - O11.T).max() <= 1e-12 * np.abs(O11).max()
        assert np.linalg.eigvalsh(O22).min() >= -1e-9 * np.abs(O22).max()
        assert np.abs(O11 @ np.ones(k * k)).max() <= 1e-10 * np.abs(O11).max()
        assert np.abs(np.ones(k * k) @ O12).max() <= 1e-10 * np.abs(O12).max()


def test_corr_entries_match_full(oracle):
    rng = np.random.default_rng(5)
    V1, V2 = rand_views(rng, 3, 8, 8)
    k = 5
    S11, S22, S12 = oracle.corr_sums(V1, V2, k)
    ent = [(1, 0, 1, 24), (2, 3, 2, 3), (1, 7, 2, 11), (2, 5, 1, 6)]
    e = oracle.corr_entries(V1, V2, k, ent)
    ref = [S11[0, 24], S22[3, 3], S12[7, 11], S12[6, 5]]
    assert np.allclose(e, ref, rtol=1e-12, atol=0)


# ------------------------------------------------------------------ P3 (Eq. 13-15)
def test_batch_split_invariance(oracle):
    rng = np.random.default_rng(6)
    V1, V2 = rand_views(rng, 7, 9, 8)
    k = 3
    full = oracle.corr_sums(V1, V2, k)
    for cuts in ([0, 7], [0, 1, 5, 7], list(range(8))):
        acc = None
        for a, b in zip(cuts[:-1], cuts[1:]):
            acc = oracle.corr_sums(V1[a:b], V2[a:b], k, into=acc)
        for F, A in zip(full, acc):
            assert np.abs(F - A).max() <= 1e-13 * np.abs(F).max()


# ------------------------------------------------------------------ P4 (C_w, C_b)
def pair_loop_matrices(V1, V2, cls, grp, k):
    X1, X2 = window_patches(V1, k), window_patches(V2, k)     # [n,h,w,D]
    D = k * k
    Cw, Cb = np.zeros((D, D)), np.zeros((D, D))
    n = V1.shape[0]
    for m in range(n):
        for mm in range(n):
            if grp[m] != grp[mm]:
                continue
            contrib = np.einsum("yxa,yxb->ab", X1[m], X2[mm])
            if cls[m] == cls[mm]:
                Cw += contrib
            else:
                Cb += contrib
    return Cw, Cb


def test_class_matrices_pair_loops(oracle):
    rng = np.random.default_rng(7)
    V1, V2 = rand_views(rng, 6, 6, 7)
    cls = np.array([0, 1, 0, 1, 1, 0], dtype=np.int32)
    grp = np.zeros(6, dtype=np.int32)
    k = 3
    Cw, Cb = pair_loop_matrices(V1, V2, cls, grp, k)
    Sw, ST = oracle.class_sums(V1, V2, cls, grp, 2, 1, k)
    assert np.abs(Sw - Cw).max() <= 1e-12 * np.abs(Cw).max()
    assert np.abs((ST - Sw) - Cb).max() <= 1e-12 * np.abs(ST).max()
    mats = oracle.stage_matrices(V1, V2, cls, grp, 2, 1, k)
    N = 6 * 6 * 7
    assert np.abs(mats["Ctilde"] - (Cw - Cb) / N).max() <= 1e-12 * np.abs(Cw).max() / N
    assert np.abs(mats["Cw"] + mats["Cb"] - mats["CT"]).max() <= 1e-15
    assert np.abs(np.ones(9) @ mats["Ctilde"]).max() <= 1e-12


def test_class_matrices_with_groups(oracle):
    rng = np.random.default_rng(8)
    V1, V2 = rand_views(rng, 8, 5, 5)
    cls = np.array([0, 0, 1, 1, 0, 0, 1, 1], dtype=np.int32)
    grp = np.array([0, 1, 0, 1, 0, 1, 0, 1], dtype=np.int32)
    Cw, Cb = pair_loop_matrices(V1, V2, cls, grp, 3)
    Sw, ST = oracle.class_sums(V1, V2, cls, grp, 2, 2, 3)
    assert np.abs(Sw - Cw).max() <= 1e-12 * np.abs(Cw).max()
    assert np.abs((ST - Sw) - Cb).max() <= 1e-12 * np.abs(ST).max()


def test_class_matrices_special_cases(oracle):
    rng = np.random.default_rng(9)
    V1, V2 = rand_views(rng, 5, 6, 6)
    k = 3
    zeros = np.zeros(5, dtype=np.int32)
    S11, S22, S12 = oracle.corr_sums(V1, V2, k)
    # one class: every pair is a same-class pair
    Sw, ST = oracle.class_sums(V1, V2, zeros, zeros, 1, 1, k)
    assert np.abs(Sw - ST).max() <= 1e-12 * np.abs(ST).max()
    # every image its own class: same-class pairs are the (m, m) pairs, i.e. plain C12
    Sw, ST2 = oracle.class_sums(V1, V2, np.arange(5, dtype=np.int32), zeros, 5, 1, k)
    assert np.abs(Sw - S12).max() <= 1e-12 * np.abs(S12).max()
    assert np.abs(ST2 - ST).max() <= 1e-12 * np.abs(ST).max()
    # all-pairs sum = Gram of the summed images (linearity of patch extraction)
    T11, T22, T12 = oracle.corr_sums(V1.sum(0, keepdims=True), V2.sum(0, keepdims=True), k)
    assert np.abs(ST - T12).max() <= 1e-12 * np.abs(ST).max()


# ------------------------------------------------------------------ P5 (Eq. 2-3)
def random_problem(rng, D, n=400):
    X = rng.standard_normal((n, D)); Y = rng.standard_normal((n, D)) + 0.5 * X
    H = np.eye(D) - np.ones((D, D)) / D            # patches are mean-free: C 1 = 0
    X, Y = X @ H, Y @ H
    return X.T @ X / n, Y.T @ Y / n, (X.T @ Y / n) * 0.7 + 0.05 * H @ rng.standard_normal((D, D)) @ H


@pytest.mark.parametrize("D,L", [(9, 4), (25, 8), (49, 8)])
def test_solve_residual_constraints_library(oracle, D, L):
    rng = np.random.default_rng(10 + D)
    C11, C22, Ct = random_problem(rng, D)
    sol = oracle.dcca_solve(C11, C22, Ct, L, ridge=1e-4)
    W1, W2, rho, B1, B2 = sol["W1"], sol["W2"], sol["rho"], sol["B1"], sol["B2"]
    # ridge as specified
    assert np.allclose(B1 - C11, 1e-4 * np.trace(C11) / D * np.eye(D), atol=1e-18)
    # stationarity of the Lagrangian of Eq. 2-3
    for g in range(L):
        res = np.concatenate([Ct @ W2[g] - rho[g] * B1 @ W1[g], Ct.T @ W1[g] - rho[g] * B2 @ W2[g]])
        scale = (np.linalg.norm(Ct) + rho[g] * np.linalg.norm(B1)) * np.linalg.norm(np.concatenate([W1[g], W2[g]]))
        assert np.linalg.norm(res) <= 1e-9 * scale
    assert np.abs(W1 @ B1 @ W1.T - np.eye(L)).max() <= 1e-10
    assert np.abs(W2 @ B2 @ W2.T - np.eye(L)).max() <= 1e-10
    assert np.abs(W1 @ Ct @ W2.T - np.diag(rho)).max() <= 1e-10
    assert np.all(np.diff(rho) <= 1e-14) and np.all(rho > 0)
    for W in (W1, W2):                              # filters are zero-mean
        assert np.abs(W.sum(axis=1)).max() <= 1e-10 * np.abs(W).max()
    # library: generalised symmetric eigenproblem of the block pencil
    Kb = np.block([[np.zeros((D, D)), Ct], [Ct.T, np.zeros((D, D))]])
    Bb = np.block([[B1, np.zeros((D, D))], [np.zeros((D, D)), B2]])
    lam, vec = scipy.linalg.eigh(Kb, Bb)
    lam, vec = lam[::-1], vec[:, ::-1]
    assert np.allclose(lam[:L], rho, rtol=1e-10, atol=1e-13)
    for g in range(L):
        v = vec[:, g] * np.sqrt(2.0)
        cos = abs(v[:D] @ B1 @ W1[g])
        assert cos >= 1 - 1e-8
        same_sign = np.sign(v[:D] @ B1 @ W1[g]) == np.sign(v[D:] @ B2 @ W2[g])
        assert same_sign
    # library: singular values of the whitened cross matrix
    R1, R2 = np.linalg.cholesky(B1).T, np.linalg.cholesky(B2).T
    sv = np.linalg.svd(np.linalg.solve(R1.T, Ct) @ np.linalg.inv(R2), compute_uv=False)
    assert np.allclose(sv[:L], rho, rtol=1e-10)
    assert np.allclose(sv, sol["sigma"], rtol=1e-8, atol=1e-12)
    # sign rule
    for g in range(L):
        assert W1[g][np.argmax(np.abs(W1[g]))] > 0


def test_jacobi_matches_eigh(oracle):
    rng = np.random.default_rng(11)
    A = rng.standard_normal((30, 30)); A = A + A.T
    lam, V, sweeps = oracle.jacobi_sym(A)
    assert sweeps < 30
    assert np.allclose(np.sort(lam), np.linalg.eigvalsh(A), rtol=0, atol=1e-12)
    assert np.abs(V.T @ V - np.eye(30)).max() <= 1e-13
    assert np.abs(A @ V - V * lam).max() <= 1e-12 * np.abs(A).max() * 30


# ------------------------------------------------------------------ P5b (objective)
def test_objective_brute_force_two_class(oracle):
    rng = np.random.default_rng(12)
    n, h, w, k, L = 6, 8, 8, 3, 3
    proto = rng.standard_normal((2, h, w))
    cls = np.array([0, 1, 0, 1, 0, 1], dtype=np.int32)
    V1 = proto[cls] + 0.3 * rng.standard_normal((n, h, w))
    V2 = np.abs(V1) + 0.1 * rng.standard_normal((n, h, w))
    grp = np.zeros(n, dtype=np.int32)
    Cw, Cb = pair_loop_matrices(V1, V2, cls, grp, k)          # independent of the oracle
    N = n * h * w
    Ct = (Cw - Cb) / N
    X1 = window_patches(V1, k).reshape(-1, 9); X2 = window_patches(V2, k).reshape(-1, 9)
    C11, C22 = X1.T @ X1 / N, X2.T @ X2 / N
    B1 = C11 + 1e-4 * np.trace(C11) / 9 * np.eye(9)
    B2 = C22 + 1e-4 * np.trace(C22) / 9 * np.eye(9)

    def objective(a, b):
        return (a @ Ct @ b) / np.sqrt((a @ B1 @ a) * (b @ B2 @ b))

    sol = oracle.learn_stage(V1, V2, cls, grp, 2, 1, k, L)
    w1, w2, rho1 = sol["W1"][0], sol["W2"][0], sol["rho"][0]
    assert abs(objective(w1, w2) - rho1) <= 1e-12
    trials = rng.standard_normal((10000, 2, 9))
    best = max(objective(t[0], t[1]) for t in trials)
    assert best <= rho1 + 1e-12
    for _ in range(200):                                     # local maximum as well
        a = w1 + 1e-3 * rng.standard_normal(9); b = w2 + 1e-3 * rng.standard_normal(9)
        assert objective(a, b) <= rho1 + 1e-12
    # second pair maximises the objective among directions B-orthogonal to the first
    w1b, w2b = sol["W1"][1], sol["W2"][1]
    for _ in range(2000):
        a = rng.standard_normal(9); b = rng.standard_normal(9)
        a -= (a @ B1 @ w1) * w1; b -= (b @ B2 @ w2) * w2
        assert objective(a, b) <= sol["rho"][1] + 1e-12
    assert abs(objective(w1b, w2b) - sol["rho"][1]) <= 1e-12


# ------------------------------------------------------------------ P6 (Eq. 6)
def test_conv_matches_scipy_and_projection(oracle):
    rng = np.random.default_rng(13)
    V1, V2 = rand_views(rng, 3, 9, 11)
    k, L = 5, 3
    F = rng.standard_normal((L, k, k))
    Y = oracle.conv(V2, F)
    assert Y.shape == (3, L, 9, 11)
    for m in range(3):
        for g in range(L):
            ref = scipy.signal.correlate2d(V2[m], F[g], mode="same", boundary="fill", fillvalue=0.0)
            assert np.abs(Y[m, g] - ref).max() <= 1e-12 * np.abs(ref).max()
    # zero-mean filters: the map is the projection of the mean-removed patch, so the
    # map statistics are the Gram quadratic forms (ties conv and Gram border handling)
    F0 = F - F.mean(axis=(1, 2), keepdims=True)
    Y1, Y2 = oracle.conv(V1, F0), oracle.conv(V2, F0)
    X2 = window_patches(V2, k)                                   # [n,h,w,D]
    proj = np.einsum("nyxa,ga->ngyx", X2, F0.reshape(L, -1))
    assert np.abs(proj - Y2).max() <= 1e-12 * np.abs(Y2).max()
    S11, S22, S12 = oracle.corr_sums(V1, V2, k)
    N = 3 * 9 * 11
    W = F0.reshape(L, -1)
    assert np.allclose((Y1 ** 2).mean(axis=(0, 2, 3)), np.einsum("ga,ab,gb->g", W, S11 / N, W), rtol=1e-12)
    cross = np.einsum("ngyx,nkyx->gk", Y1, Y2) / N
    assert np.allclose(cross, W @ (S12 / N) @ W.T, rtol=1e-10, atol=1e-13)


def test_conv_asymmetric_filter_orientation(oracle):
    # a one-hot filter at (dy,dx) picks the pixel at offset (dy-r, dx-r): no flip
    img = np.arange(30.0).reshape(1, 5, 6)
    F = np.zeros((1, 3, 3)); F[0, 0, 2] = 1.0                   # up one row, right one column
    Y = oracle.conv(img, F)[0, 0]
    assert Y[2, 2] == img[0, 1, 3]
    assert Y[0, 0] == 0.0 and Y[4, 5] == 0.0 and Y[4, 4] == img[0, 3, 5]


# ------------------------------------------------------------------ P7 (Eq. 7-9, Section II-C)
def test_hash_hand_example(oracle):
    Z = np.zeros((1, 3, 2, 2))
    Z[0, 0] = [[1.0, -1.0], [0.0, 2.0]]      # bit 0
    Z[0, 1] = [[-1.0, 3.0], [0.5, 0.0]]      # bit 1
    Z[0, 2] = [[1e-300, -0.0], [np.nan, 5.0]]  # bit 2: tiny positive counts, -0 and NaN do not
    Q = oracle.hash_maps(Z)
    assert Q.tolist() == [[[1 + 4, 2], [2, 1 + 4]]]


def test_block_hist_invariants_and_bincount(oracle):
    rng = np.random.default_rng(14)
    n, h, w, bins = 3, 13, 11, 16
    Q = rng.integers(0, bins, size=(n, h, w)).astype(np.int32)
    for b, s in ((4, 2), (7, 4), (5, 5), ((3, 6), (2, 5))):
        H = oracle.block_hist(Q, b, s, bins)
        bh, bw = (b, b) if np.isscalar(b) else b
        sy, sx = (s, s) if np.isscalar(s) else s
        nby, nbx = (h - bh) // sy + 1, (w - bw) // sx + 1
        assert H.shape == (n, nby, nbx, bins)
        assert np.all(H.sum(axis=-1) == bh * bw)
        for m in range(n):
            for i in range(nby):
                for j in range(nbx):
                    blk = Q[m, i * sy:i * sy + bh, j * sx:j * sx + bw]
                    assert np.array_equal(H[m, i, j], np.bincount(blk.ravel(), minlength=bins))
                    assert (H[m, i, j] * np.arange(bins)).sum() == blk.sum()


def test_block_hist_worked_toy(oracle):
    # 8x8 map, left half code 1, right half code 2; 4x4 blocks at stride 2 -> 3x3 blocks
    Q = np.ones((1, 8, 8), dtype=np.int32); Q[:, :, 4:] = 2
    H = oracle.block_hist(Q, 4, 2, 4)
    assert H.shape == (1, 3, 3, 4)
    assert H[0, :, 0].tolist() == [[0, 16, 0, 0]] * 3
    assert H[0, :, 1].tolist() == [[0, 8, 8, 0]] * 3
    assert H[0, :, 2].tolist() == [[0, 0, 16, 0]] * 3
    assert oracle.default_stride(7) == 4 and oracle.default_stride(8) == 4 and oracle.default_stride(16) == 8


def test_single_bit_hash_counts_positives(oracle):
    rng = np.random.default_rng(15)
    Z = rng.standard_normal((2, 1, 8, 8))
    H = oracle.block_hist(oracle.hash_maps(Z), 8, 8, 2)
    assert H[:, 0, 0, 1].tolist() == [(Z[0] > 0).sum(), (Z[1] > 0).sum()]


# ------------------------------------------------------------------ whole path
def test_two_stage_shapes_and_invariants(oracle):
    from paper_2209_13027_amd.workloads import WORKLOADS, make_views
    wl = WORKLOADS["tiny"]
    v1, v2, cls = make_views(wl, max_per_class=3)
    out = oracle.two_stage(v1, v2, cls, wl.n_classes, wl.k, wl.L1, wl.L2, wl.block)
    M = v1.shape[0]
    by, bx = wl.blocks
    assert out["hist"].shape == (M, 2, wl.L1, by, bx, 1 << wl.L2)      # Eq. 11-12 layout
    assert out["hist"][0].size == wl.feature_len
    assert np.all(out["hist"].sum(axis=-1) == wl.block ** 2)
    s1, s2 = out["stage1"], out["stage2"]
    # maps are B-normalised projections: mean square = 1 - eps * |w|^2
    eps1 = 1e-4 * np.trace(s1["C11"]) / wl.D
    ms = (out["Y1"].reshape(M, wl.L1, -1) ** 2).mean(axis=(0, 2))
    assert np.allclose(ms, 1 - eps1 * (s1["W1"] ** 2).sum(axis=1), rtol=1e-9)
    assert s2["C11"].shape == (wl.D, wl.D) and s2["N"] == M * wl.L1 * wl.h * wl.w
    assert np.all(s1["gap"] > 0) and np.all(s2["gap"] > 0)


def test_class_sums_equal_gram_of_class_sum_images(oracle):
    # linearity of patch extraction and mean removal: the per-pixel sum of a cell's patches is the
    # patch of the cell's sum image, so Sw is the cross Gram of the n_cls*G sum images
    rng = np.random.default_rng(16)
    V1, V2 = rand_views(rng, 12, 7, 6)
    cls = np.array([0, 0, 1, 1, 2, 2], dtype=np.int32)            # 6 samples x 2 maps
    cls2, grp2 = np.repeat(cls, 2), np.tile(np.arange(2, dtype=np.int32), 6)
    Sw, ST = oracle.class_sums(V1, V2, cls2, grp2, 3, 2, 3)
    S1 = np.stack([V1[(cls2 == c) & (grp2 == g)].sum(0) for c in range(3) for g in range(2)])
    S2 = np.stack([V2[(cls2 == c) & (grp2 == g)].sum(0) for c in range(3) for g in range(2)])
    _, _, G12 = oracle.corr_sums(S1, S2, 3)
    assert np.abs(Sw - G12).max() <= 1e-12 * np.abs(Sw).max()
    T1 = np.stack([V1[grp2 == g].sum(0) for g in range(2)])
    T2 = np.stack([V2[grp2 == g].sum(0) for g in range(2)])
    _, _, GT = oracle.corr_sums(T1, T2, 3)
    assert np.abs(ST - GT).max() <= 1e-12 * np.abs(ST).max()


def test_second_stage_class_sums_from_the_inputs_sum_images(oracle):
    # Eq. 6 is linear: the sum of a class's stage-1 maps is the stage-1 convolution of the class's sum image, so
    # the second stage's Sw / ST follow from the INPUTS' sum images convolved with the stage-1 filters (the route
    # the library's streamed second-stage learning takes); here on the oracle alone, in fp64
    rng = np.random.default_rng(23)
    n, h, w, k, L1 = 6, 8, 9, 3, 3
    V1, V2 = rand_views(rng, n, h, w)
    F1, F2 = rng.standard_normal((L1, k, k)), rng.standard_normal((L1, k, k))
    cls = np.array([0, 1, 1, 0, 2, 1], dtype=np.int32)
    Y1 = oracle.conv(V1, F1).reshape(n * L1, h, w)
    Y2 = oracle.conv(V2, F2).reshape(n * L1, h, w)
    Sw, ST = oracle.class_sums(Y1, Y2, np.repeat(cls, L1), np.tile(np.arange(L1, dtype=np.int32), n), 3, L1, k)
    S1 = np.stack([V1[cls == c].sum(0) for c in range(3)])
    S2 = np.stack([V2[cls == c].sum(0) for c in range(3)])
    C1 = oracle.conv(S1, F1).reshape(3 * L1, h, w)               # cell (c, g) = conv of class c's sum image, filter g
    C2 = oracle.conv(S2, F2).reshape(3 * L1, h, w)
    _, _, G12 = oracle.corr_sums(C1, C2, k)
    assert np.abs(Sw - G12).max() <= 1e-12 * np.abs(Sw).max()
    T1 = oracle.conv(V1.sum(0, keepdims=True), F1).reshape(L1, h, w)
    T2 = oracle.conv(V2.sum(0, keepdims=True), F2).reshape(L1, h, w)
    _, _, GT = oracle.corr_sums(T1, T2, k)
    assert np.abs(ST - GT).max() <= 1e-12 * np.abs(ST).max()


def test_iq_probabilities_sum_to_one_and_hand_values(oracle):
    """Eq. 10 with one pseudo-count per bin: exp(-o) is a distribution over the bins of every block;
    a block of 4 pixels with codes {0, 0, 3, 1} over 4 bins gives p = 3/8, 2/8, 1/8, 2/8."""
    rng = np.random.default_rng(5)
    Q = rng.integers(0, 16, size=(3, 20, 24)).astype(np.int32)
    H = oracle.block_hist(Q, 8, 4, 16)
    o = oracle.iq_features(H, 64)
    assert o.shape == H.shape and o.dtype == np.float64
    np.testing.assert_allclose(np.exp(-o).sum(axis=-1), 1.0, rtol=0, atol=1e-13)
    # a code seen more often is less informative; an absent code carries log(area + bins)
    order = np.argsort(H.reshape(-1), kind="stable")
    assert np.all(np.diff(o.reshape(-1)[order]) <= 1e-15)
    assert np.allclose(o[H == 0], math.log(64 + 16), rtol=0, atol=1e-14)
    hand = oracle.iq_features(np.array([2, 1, 0, 1]), 4)
    np.testing.assert_allclose(hand, [0.98082925301172619, 1.3862943611198906, 2.0794415416798357,
                                      1.3862943611198906], rtol=0, atol=1e-15)
    # all pixels of a block share one code: p = (area+1)/(area+bins) for it
    full = oracle.iq_features(np.array([49, 0, 0, 0, 0, 0, 0, 0]), 49)
    assert abs(full[0] - math.log(57.0 / 50.0)) < 1e-15 and abs(full[1] - math.log(57.0)) < 1e-14


# ------------------------------------------------------------------ composite path (Sec. II-B on II-A; Eq. 6-12)
def scipy_maps(img, F):
    """[h,w] image x [L,k,k] filters -> [L,h,w] by scipy's zero-filled 'same' cross-correlation."""
    return np.stack([scipy.signal.correlate2d(img, f, mode="same", boundary="fill", fillvalue=0.0) for f in F])


def test_learn_two_stage_second_stage_pairs_by_image_and_map_index(oracle):
    """The second stage is learned on the stage-1 maps: map g of image m carries the class of image m and pairs
    only with map g of the other view.  Its C_w / C_b are rebuilt here with explicit loops over image pairs
    (m, m') and the map index g from maps that scipy computes one image at a time, so a mislabelled map (class
    and group arrays exchanged or misordered inside learn_two_stage) shows up in every entry."""
    rng = np.random.default_rng(31)
    M, h, w, k, L1, L2 = 6, 7, 6, 3, 2, 3
    V1, V2 = rand_views(rng, M, h, w)
    cls = np.array([0, 1, 1, 0, 1, 0], dtype=np.int32)
    res = oracle.learn_two_stage(V1, V2, cls, 2, k, L1, L2)
    s1, s2 = res["stage1"], res["stage2"]
    Y = [np.stack([scipy_maps(V[m], F) for m in range(M)]) for V, F in ((V1, s1["F1"]), (V2, s1["F2"]))]
    X1 = [window_patches(Y[0][:, g], k) for g in range(L1)]          # per g: [M,h,w,D]
    X2 = [window_patches(Y[1][:, g], k) for g in range(L1)]
    D = k * k
    N = M * L1 * h * w
    Cw, Cb, C11, C22, C12 = (np.zeros((D, D)) for _ in range(5))
    for g in range(L1):
        for m in range(M):
            C11 += np.einsum("yxa,yxb->ab", X1[g][m], X1[g][m])
            C22 += np.einsum("yxa,yxb->ab", X2[g][m], X2[g][m])
            C12 += np.einsum("yxa,yxb->ab", X1[g][m], X2[g][m])
            for mm in range(M):
                pair = np.einsum("yxa,yxb->ab", X1[g][m], X2[g][mm])
                if cls[m] == cls[mm]:
                    Cw += pair
                else:
                    Cb += pair
    assert s2["N"] == N
    for name, want in (("Cw", Cw), ("Cb", Cb), ("C11", C11), ("C22", C22), ("C12", C12)):
        assert np.abs(s2[name] - want / N).max() <= 1e-11 * np.abs(want / N).max(), name
    assert np.abs(s2["Ctilde"] - (Cw - Cb) / N).max() <= 1e-11 * np.abs(Cw / N).max()
    # the maps handed on are the stage-1 maps in (image, g) order
    assert np.abs(res["Y1"].reshape(M, L1, h, w) - Y[0]).max() <= 1e-12 * np.abs(Y[0]).max()
    assert np.abs(res["Y2"].reshape(M, L1, h, w) - Y[1]).max() <= 1e-12 * np.abs(Y[1]).max()
    # and the stage-2 filters solve Eq. 2-3 for THESE matrices: rho = w1^T C~ w2, B-normalised
    B1 = C11 / N + 1e-4 * np.trace(C11 / N) / D * np.eye(D)
    for l in range(L2):
        w1, w2 = s2["W1"][l], s2["W2"][l]
        assert abs(w1 @ B1 @ w1 - 1.0) <= 1e-10
        assert abs(w1 @ ((Cw - Cb) / N) @ w2 - s2["rho"][l]) <= 1e-10 * max(1.0, abs(s2["rho"][l]))


def test_extract_features_layout_one_image_and_map_at_a_time(oracle):
    """hist[m][d][g] is the block histogram of the hashed second-stage maps of stage-1 map g of image m in view d
    (Eq. 6-12).  Rebuilt per image and per map with scipy's correlation, a written-out hash and numpy.bincount; the
    filters are random and all different, so any exchange of views, stages, g and l, or image order fails."""
    rng = np.random.default_rng(32)
    M, h, w, k, L1, L2, b, s = 3, 11, 10, 3, 3, 3, 4, 2
    V = rand_views(rng, M, h, w)
    V = (V[0], V[1] - V[1].mean())          # both views take both signs, or the codes would be trivial
    F = [rng.standard_normal((L, k, k)) for L in (L1, L1, L2, L2)]
    out = oracle.extract_features(V[0], V[1], F, k, L1, L2, b, s)
    nby, nbx = (h - b) // s + 1, (w - b) // s + 1
    assert out["hist"].shape == (M, 2, L1, nby, nbx, 1 << L2)
    seen = set()
    for m in range(M):
        for d in range(2):
            Y = scipy_maps(V[d][m], F[d])
            for g in range(L1):
                Z = scipy_maps(Y[g], F[2 + d])
                Q = sum((Z[l] > 0).astype(np.int64) << l for l in range(L2))
                for i in range(nby):
                    for j in range(nbx):
                        want = np.bincount(Q[i * s:i * s + b, j * s:j * s + b].ravel(), minlength=1 << L2)
                        assert np.array_equal(out["hist"][m, d, g, i, j], want), (m, d, g, i, j)
                seen.add(Q.tobytes())
    assert len(seen) == M * 2 * L1           # every (image, view, g) has its own code map: the check can tell them apart

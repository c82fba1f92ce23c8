"""Writes tests/golden/<workload>_full.npz (+ a readable .txt beside it): the CPU oracle's learning results on
a synthetic workload at its FULL size -- both stages' five matrices (Sec. II-A; Sec. III, Eq. 13-15), the canonical
correlations, their gaps and the filters (Eq. 2-5) -- plus, for a fixed sample of images, the per-code totals of
the oracle's histograms (Eq. 6-12) computed with the oracle's own filters.  The paper prints no intermediate value,
so these are the oracle's own results: a fixed full-size target for the HIP path and a drift guard for the oracle.

Calls only oracle/ and the seeded input generator.  The oracle's routines take whole arrays; two things keep the
full sizes inside this machine's memory, both identities the oracle's pins hold it to:
  * the within-view and cross-view sums are accumulated batch by batch (Eq. 15: corr_sums adds into running sums);
  * the second stage's class-conditioned sums are taken on the per-(class, g) SUM maps (one member per cell): patch
    extraction and mean removal are linear, so the per-pixel sum of a cell's patches is the patch of the cell's
    sum map (tests/test_oracle_pins.py::test_class_sums_equal_gram_of_class_sum_images).  Where all maps fit in
    memory the direct call is made as well and the difference is recorded in the .txt.

    python tests/golden/make_golden_full.py object stress large_scale
"""
import hashlib
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

from oracle import ddcca_oracle as orc  # noqa: E402
from paper_2209_13027_amd.workloads import WORKLOADS, make_views  # noqa: E402

N_SAMPLE = 16          # images whose histograms are summarised
BATCH = 256            # images per accumulation batch
DIRECT_CLASS_SUM_BYTES = 12e9   # call class_sums on all second-stage maps when both views fit in this


def source_hash() -> str:
    h = hashlib.sha256()
    for f in ("ddcca_oracle.c", "ddcca_oracle.py"):
        h.update(open(os.path.join(ROOT, "oracle", f), "rb").read())
    return h.hexdigest()[:16]


def sample_indices(M: int) -> np.ndarray:
    return np.unique(np.linspace(0, M - 1, N_SAMPLE).round().astype(np.int64))


def solve(mats, L, ridge):
    sol = orc.dcca_solve(mats["C11"], mats["C22"], mats["Ctilde"], L, ridge)
    return {"rho": sol["rho"], "gap": sol["gap"], "sigma": sol["sigma"], "W1": sol["W1"], "W2": sol["W2"]}


def finish(S11, S22, S12, Sw, ST, N):
    m = {"C11": S11 / N, "C22": S22 / N, "C12": S12 / N, "Cw": Sw / N, "CT": ST / N}
    m["Ctilde"] = 2.0 * m["Cw"] - m["CT"]          # C~ = C_w - C_b, C_b = C_T - C_w
    return m


def run(name: str, ridge: float = 1e-4) -> None:
    wl = WORKLOADS[name]
    log = []

    def note(msg):
        print(f"[{name} {time.time() - t0:7.0f}s] {msg}", flush=True)
        log.append(msg)

    t0 = time.time()
    v1, v2, cls = make_views(wl)
    M, h, w = v1.shape
    k, L1, L2, D = wl.k, wl.L1, wl.L2, wl.D
    note(f"inputs: {M} images {h}x{w}, {wl.n_classes} classes, k={k}, {orc.num_threads()} threads")

    # ---- stage 1 --------------------------------------------------------------------------------------------
    sums = None
    for s in range(0, M, BATCH):
        sums = orc.corr_sums(v1[s:s + BATCH], v2[s:s + BATCH], k, into=sums)
    Sw, ST = orc.class_sums(v1, v2, cls, np.zeros(M, np.int32), wl.n_classes, 1, k)
    m1 = finish(*sums, Sw, ST, float(M * h * w))
    s1 = solve(m1, L1, ridge)
    F1 = (s1["W1"].reshape(L1, k, k), s1["W2"].reshape(L1, k, k))
    note(f"stage 1 done: rho {s1['rho'][0]:.6f} .. {s1['rho'][-1]:.6f}, min gap {s1['gap'].min():.2e}")

    # ---- stage 2: maps exist one batch at a time --------------------------------------------------------------
    sums = None
    cell1 = np.zeros((wl.n_classes, L1, h, w))
    cell2 = np.zeros((wl.n_classes, L1, h, w))
    direct = 2.0 * M * L1 * h * w * 8 <= DIRECT_CLASS_SUM_BYTES
    keep1, keep2 = [], []
    t_last = time.time()
    for s in range(0, M, BATCH):
        y1 = orc.conv(v1[s:s + BATCH], F1[0])                  # [b, L1, h, w]
        y2 = orc.conv(v2[s:s + BATCH], F1[1])
        b = y1.shape[0]
        sums = orc.corr_sums(y1.reshape(b * L1, h, w), y2.reshape(b * L1, h, w), k, into=sums)
        for i in range(b):                                      # sum maps of the (class, g) cells, in image order
            cell1[cls[s + i]] += y1[i]
            cell2[cls[s + i]] += y2[i]
        if direct:
            keep1.append(y1)
            keep2.append(y2)
        if time.time() - t_last > 60:
            print(f"[{name} {time.time() - t0:7.0f}s] stage 2: {s + b} of {M} images", flush=True)
            t_last = time.time()
    cell_cls = np.repeat(np.arange(wl.n_classes, dtype=np.int32), L1)
    cell_grp = np.tile(np.arange(L1, dtype=np.int32), wl.n_classes)
    Sw, ST = orc.class_sums(cell1.reshape(-1, h, w), cell2.reshape(-1, h, w), cell_cls, cell_grp, wl.n_classes, L1, k)
    direct_note = "not made (the maps of both views do not fit in memory)"
    if direct:
        Y1 = np.concatenate(keep1).reshape(M * L1, h, w)
        Y2 = np.concatenate(keep2).reshape(M * L1, h, w)
        del keep1, keep2
        Sw_d, ST_d = orc.class_sums(Y1, Y2, np.repeat(cls, L1), np.tile(np.arange(L1, dtype=np.int32), M),
                                    wl.n_classes, L1, k)
        direct_note = "relative difference of Sw %.2e, of ST %.2e" % (
            np.linalg.norm(Sw_d - Sw) / np.linalg.norm(Sw_d), np.linalg.norm(ST_d - ST) / np.linalg.norm(ST_d))
        Sw, ST = Sw_d, ST_d                                     # the direct definition is what is stored
        del Y1, Y2
    note("second-stage class sums on all maps against the sum-map route: " + direct_note)
    m2 = finish(*sums, Sw, ST, float(M * L1 * h * w))
    s2 = solve(m2, L2, ridge)
    F2 = (s2["W1"].reshape(L2, k, k), s2["W2"].reshape(L2, k, k))
    note(f"stage 2 done: rho {s2['rho'][0]:.6f} .. {s2['rho'][-1]:.6f}, min gap {s2['gap'].min():.2e}")

    # ---- histograms of a fixed sample of images with the oracle's own filters -----------------------------------
    idx = sample_indices(M)
    feats = orc.extract_features(v1[idx], v2[idx], (F1[0], F1[1], F2[0], F2[1]), k, L1, L2, wl.block, wl.stride)
    codes = feats["hist"].sum(axis=(3, 4))                       # [sample][view][g][bin]
    note(f"histograms of {len(idx)} sampled images done")
    wall = time.time() - t0

    out = {"sample_idx": idx, "sample_codes": codes.astype(np.int64),
           "shape": np.array([M, h, w, k, L1, L2, wl.block, wl.stride, wl.n_classes], dtype=np.int64),
           "ridge": np.array(ridge), "source_hash": np.array(source_hash()), "wall_seconds": np.array(wall),
           "threads": np.array(orc.num_threads())}
    for s, (m, sol) in enumerate(((m1, s1), (m2, s2)), start=1):
        for nm in ("C11", "C22", "C12", "Cw", "CT"):
            out[f"s{s}_{nm}"] = m[nm]
        for nm in ("rho", "gap", "sigma", "W1", "W2"):
            out[f"s{s}_{nm}"] = sol[nm]
    np.savez_compressed(os.path.join(HERE, f"{name}_full.npz"), **out)
    with open(os.path.join(HERE, f"{name}_full.txt"), "w") as f:
        f.write(f"# CPU oracle at full size on the synthetic workload `{name}`, written by tests/golden/make_golden_full.py\n")
        f.write(f"# oracle sources sha256[:16] {source_hash()}; {orc.num_threads()} threads; wall time {wall:.0f} s\n")
        f.write(f"# arrays in {name}_full.npz: s<stage>_<C11|C22|C12|Cw|CT> (divided by the patch count),\n")
        f.write("# s<stage>_<rho|gap|sigma|W1|W2>, sample_idx, sample_codes[sample][view][g][bin]\n")
        for line in log:
            f.write("# " + line + "\n")
        for s, sol in ((1, s1), (2, s2)):
            f.write(f"rho {s} " + " ".join("%.12e" % x for x in sol["rho"]) + "\n")
            f.write(f"gap {s} " + " ".join("%.6e" % x for x in sol["gap"]) + "\n")
    note("written")


if __name__ == "__main__":
    orc.build()
    for nm in sys.argv[1:] or ["object"]:
        run(nm)

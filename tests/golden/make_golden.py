"""Writes tests/golden/tiny_two_stage.txt: the CPU oracle's results on the `tiny` synthetic workload (the paper
prints no intermediate values, so the stored values are the oracle's own, kept to catch a later drift of its
arithmetic and as a fixed target for the HIP path).  Calls only oracle/ and the seeded input generator.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import ddcca_oracle as orc  # noqa: E402
from paper_2209_13027_amd.workloads import WORKLOADS, make_views  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_two_stage.txt")


def main():
    orc.build()
    wl = WORKLOADS["tiny"]
    v1, v2, cls = make_views(wl)
    res = orc.two_stage(v1, v2, cls, wl.n_classes, wl.k, wl.L1, wl.L2, wl.block, wl.stride)
    hist = res["hist"]                                  # [m][view][g][by][bx][t]
    lines = [
        "# CPU oracle on the synthetic workload `tiny` (seeded generator, all images), written by",
        "# tests/golden/make_golden.py.  rho: canonical correlations of Eq. 2-5 per stage; gap: relative gaps;",
        "# F: filters of Eq. 4-5 (stage, view, filter, k*k taps row-major); codes: per (view, g) the number of",
        "# block pixels with each code of Eq. 7-9 summed over all images and blocks (Sec. II-C histograms);",
        "# sample: single histogram entries hist[m][view][g][by][bx][t].",
        f"shape images {v1.shape[0]} h {wl.h} w {wl.w} k {wl.k} L1 {wl.L1} L2 {wl.L2} block {wl.block} stride {wl.stride}",
    ]
    for s in (1, 2):
        st = res["stage%d" % s]
        lines.append(f"rho {s} " + " ".join("%.12e" % x for x in st["rho"]))
        lines.append(f"gap {s} " + " ".join("%.6e" % x for x in st["gap"]))
        for d in (1, 2):
            F = st["F%d" % d].reshape(st["F%d" % d].shape[0], -1)
            for l in range(F.shape[0]):
                lines.append(f"F {s} {d} {l} " + " ".join("%.10e" % x for x in F[l]))
    codes = hist.sum(axis=(0, 3, 4))                    # [view][g][t]
    for d in range(codes.shape[0]):
        for g in range(codes.shape[1]):
            lines.append(f"codes {d} {g} " + " ".join(str(int(x)) for x in codes[d, g]))
    rng = np.random.default_rng(1)
    for _ in range(48):
        idx = tuple(int(rng.integers(0, n)) for n in hist.shape)
        lines.append("sample " + " ".join(map(str, idx)) + " " + str(int(hist[idx])))
    with open(OUT, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", OUT, len(lines), "lines")


if __name__ == "__main__":
    main()

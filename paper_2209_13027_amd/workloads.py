"""Seeded synthetic two-view workloads shaped like the paper's data sets.

The paper evaluates on ORL (400 face images, 40 classes x 10), ETH-80 (3280 object
images, 8 classes x 410) and Caltech-256 (257 classes) -- Section IV.  None of those
sets can be shipped, so these generators produce stand-ins with the same image
counts, class structure and image shapes.  This module only *prepares data* (class
prototypes, shifts, rotations, noise, a Sobel-magnitude second view); it contains
none of the method's arithmetic and is the only code that the CPU oracle's tests and
the HIP path's tests both use.

Recipe (identical for every workload unless noted):
  * RNG: numpy Generator(PCG64(seed)), seed = 220913027 + workload index.
  * class sizes: equal, except "large_scale" (see `_class_sizes`).
  * prototype of a class: N(0,1) field, Gaussian blur (sigma 2; "object": 4) with
    wrap-around boundary truncated at 4 sigma, then re-centred to mean 0 / std 1.
  * sample: ("object" only: rotate by U(-10,10) degrees, bilinear, reflect fill)
    -> circular integer shift (dy,dx) uniform in {-2..2}^2 -> add N(0, 0.3^2) noise.
    View 1 is that image (fp32); view 2 is the 3x3 Sobel gradient magnitude of
    view 1 with reflected borders (fp32, non-negative).
  * images are stored class-sorted; labels are int32 in [0, n_classes).
Draw order: class sizes; then per class: prototype field, rotations, shifts, noise.
"""
from __future__ import annotations

import dataclasses
import numpy as np
from scipy import ndimage

BASE_SEED = 220913027


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int
    n_classes: int
    per_class: int          # 0 => drawn (large_scale)
    h: int
    w: int
    k: int                  # patch / filter side
    L1: int
    L2: int
    block: int              # histogram block side; stride = round-half-up(block/2)
    blur_sigma: float = 2.0
    max_rot_deg: float = 0.0
    n_images: int = 0       # total images (filled for large_scale)
    extract_batch: int = 0  # images per streamed stage-2 batch (0 = library default)

    @property
    def stride(self) -> int:
        return (self.block + 1) // 2

    @property
    def D(self) -> int:
        return self.k * self.k

    @property
    def M(self) -> int:
        return self.n_images if self.n_images else self.n_classes * self.per_class

    @property
    def blocks(self):
        by = (self.h - self.block) // self.stride + 1
        bx = (self.w - self.block) // self.stride + 1
        return by, bx

    @property
    def feature_len(self) -> int:
        by, bx = self.blocks
        return 2 * self.L1 * by * bx * (1 << self.L2)


WORKLOADS = {
    "tiny": Workload("tiny", 0, 4, 10, 32, 32, 5, 4, 4, 8),
    "small_face": Workload("small_face", 1, 40, 10, 112, 92, 7, 8, 8, 7),
    "object": Workload("object", 2, 8, 410, 128, 128, 5, 8, 8, 16, blur_sigma=4.0, max_rot_deg=10.0),
    "large_scale": Workload("large_scale", 3, 257, 0, 128, 128, 7, 8, 8, 16, n_images=30607,
                            extract_batch=1024),
    "stress": Workload("stress", 4, 16, 64, 256, 256, 9, 8, 8, 32),
}


def _class_sizes(wl: Workload, rng: np.random.Generator) -> np.ndarray:
    """Equal sizes, except large_scale: r_c ~ U{80..827}, squeezed so that the sizes
    stay >= 80 and add up to exactly n_images (a uniform draw on [80,827] cannot
    total 30607 over 257 classes, so the excess over 80 is rescaled)."""
    if wl.per_class:
        return np.full(wl.n_classes, wl.per_class, dtype=np.int64)
    r = rng.integers(80, 828, size=wl.n_classes).astype(np.int64)
    spare = wl.n_images - 80 * wl.n_classes
    extra = (r - 80) * spare // int((r - 80).sum())
    sizes = 80 + extra
    rem = wl.n_images - int(sizes.sum())
    sizes[:rem] += 1
    assert sizes.sum() == wl.n_images and sizes.min() >= 80
    return sizes


def make_views(wl: Workload, max_per_class: int | None = None, n_classes: int | None = None):
    """Return (view1, view2, labels): float32 [M,h,w] x2 and int32 [M].

    `max_per_class` / `n_classes` shrink the workload (fewer samples per class, fewer
    classes) for tests that need a slice the CPU oracle can finish; the per-class
    recipe is unchanged.
    """
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + wl.index))
    sizes = _class_sizes(wl, rng)
    if n_classes is not None:
        sizes = sizes[:n_classes]
    if max_per_class is not None:
        sizes = np.minimum(sizes, max_per_class)
    M = int(sizes.sum())
    v1 = np.empty((M, wl.h, wl.w), dtype=np.float32)
    labels = np.empty(M, dtype=np.int32)
    pos = 0
    for c, n_c in enumerate(sizes):
        n_c = int(n_c)
        field = rng.standard_normal((wl.h, wl.w))
        proto = ndimage.gaussian_filter(field, wl.blur_sigma, mode="wrap", truncate=4.0)
        proto = (proto - proto.mean()) / proto.std()
        if wl.max_rot_deg > 0:
            angles = rng.uniform(-wl.max_rot_deg, wl.max_rot_deg, size=n_c)
        shifts = rng.integers(-2, 3, size=(n_c, 2))
        noise = rng.standard_normal((n_c, wl.h, wl.w), dtype=np.float32)
        if wl.max_rot_deg > 0:
            base = np.stack([ndimage.rotate(proto, float(a), reshape=False, order=1, mode="reflect") for a in angles])
        else:
            base = np.broadcast_to(proto, (n_c, wl.h, wl.w))
        # circular shift by (dy, dx): out[y, x] = in[(y - dy) % h, (x - dx) % w]
        rows = (np.arange(wl.h)[None, :] - shifts[:, 0:1]) % wl.h
        cols = (np.arange(wl.w)[None, :] - shifts[:, 1:2]) % wl.w
        shifted = base[np.arange(n_c)[:, None, None], rows[:, :, None], cols[:, None, :]]
        v1[pos:pos + n_c] = shifted.astype(np.float32) + np.float32(0.3) * noise
        labels[pos:pos + n_c] = c
        pos += n_c
    v2 = sobel_magnitude(v1)
    return v1, v2, labels


def sobel_magnitude(v: np.ndarray) -> np.ndarray:
    """3x3 Sobel gradient magnitude per image, borders reflected about the edge (d c b a | a b c d),
    fp32.  gx = [1,2,1]^T (smooth along y) x [-1,0,1] (difference along x); gy likewise transposed."""
    out = np.empty_like(v)
    step = 32
    for s in range(0, v.shape[0], step):
        p = np.pad(v[s:s + step].astype(np.float32), ((0, 0), (1, 1), (1, 1)), mode="symmetric")
        sy = p[:, :-2, :] + 2.0 * p[:, 1:-1, :] + p[:, 2:, :]        # smoothed along y, [n, h, w+2]
        gx = sy[:, :, 2:] - sy[:, :, :-2]
        sx = p[:, :, :-2] + 2.0 * p[:, :, 1:-1] + p[:, :, 2:]        # smoothed along x, [n, h+2, w]
        gy = sx[:, 2:, :] - sx[:, :-2, :]
        out[s:s + step] = np.sqrt(gx * gx + gy * gy)
    return out

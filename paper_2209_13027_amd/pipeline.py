"""The whole hot path as a sequence of C ABI calls (no arithmetic here).

fit():     learn stage 1 (Eq. 2-5) -> learn stage 2 on the stage-1 maps, which are convolved (Eq. 6) batch by
           batch inside ddcca_learn_next_stage_filters (streamed) or, with streamed=False / keep_maps=True, held
           as a whole by ddcca_apply_stage
extract(): ddcca_extract_features (both stages + hashing + block histograms, Eq. 6-12)
"""
from __future__ import annotations

import torch

from .binding import Context


def fit(ctx: Context, v1: torch.Tensor, v2: torch.Tensor, cls: torch.Tensor, n_cls: int, k: int, L1: int, L2: int,
        ridge: float = 1e-4, keep_maps: bool = False, streamed: bool = True, batch_images: int = 0) -> dict:
    m, h, w = v1.shape
    W1a, W2a, rho1 = ctx.learn_stage_filters(v1, v2, cls, 1, h, w, n_cls, k, L1, ridge)
    if streamed and not keep_maps:
        W1b, W2b, rho2 = ctx.learn_next_stage_filters(v1, v2, cls, 1, h, w, n_cls, W1a, W2a, k, L2, ridge,
                                                      batch_images)
        return {"filters": (W1a, W2a, W1b, W2b), "rho": (rho1, rho2)}
    y1 = ctx.apply_stage(v1, W1a)          # [m, L1, h, w]
    y2 = ctx.apply_stage(v2, W2a)
    W1b, W2b, rho2 = ctx.learn_stage_filters(y1, y2, cls, L1, h, w, n_cls, k, L2, ridge)
    out = {"filters": (W1a, W2a, W1b, W2b), "rho": (rho1, rho2)}
    if keep_maps:
        out["maps"] = (y1, y2)
    return out


def extract(ctx: Context, v1, v2, filters, k, L1, L2, block, stride, batch_images=0, out=None,
            dtype=torch.uint16, fused=False):
    """dtype uint16: block histograms; float32 / float16: their information quality (Eq. 10).
    fused: second stage convolution and output layer in one kernel (same result, bit for bit)."""
    return ctx.extract_features(v1, v2, filters, k, L1, L2, block, stride, batch_images, out, dtype, fused)

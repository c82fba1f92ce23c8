"""The whole hot path as a sequence of C ABI calls (no arithmetic here).

fit():     learn stage 1 (Eq. 2-5) -> learn stage 2 on the stage-1 maps, which are convolved (Eq. 6) batch by
           batch inside ddcca_learn_next_stage_filters (streamed) or, with streamed=False / keep_maps=True, held
           as a whole by ddcca_apply_stage
extract(): ddcca_extract_features (both stages + hashing + block histograms, Eq. 6-12)
fit_stages() / extract_stages(): the same chain for any number of stages (the paper stops at two, Section III-A)
           out of the per-stage calls: every further stage is learned from the inputs of the stage before it
           (ddcca_learn_next_stage_filters), its maps are grouped by their position in the image's map list
           exactly as the second stage's are (Eq. 6), and the LAST stage's maps are hashed (Eq. 7-9)
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


def fit_stages(ctx: Context, v1: torch.Tensor, v2: torch.Tensor, cls: torch.Tensor, n_cls: int, k: int, Ls,
               ridge: float = 1e-4, batch_images: int = 0) -> dict:
    """Filters of len(Ls) stages, Ls[s] filters in stage s.  Returns {"filters": [(W1, W2) per stage], "rho": [...]}."""
    m, h, w = v1.shape
    W1, W2, rho = ctx.learn_stage_filters(v1, v2, cls, 1, h, w, n_cls, k, Ls[0], ridge)
    filters, rhos = [(W1, W2)], [rho]
    x1, x2, G = v1, v2, 1                  # inputs of the newest stage that has filters, G of them per image
    for s in range(1, len(Ls)):
        Wp1, Wp2 = filters[-1]
        W1, W2, rho = ctx.learn_next_stage_filters(x1, x2, cls, G, h, w, n_cls, Wp1, Wp2, k, Ls[s], ridge,
                                                   batch_images)
        filters.append((W1, W2))
        rhos.append(rho)
        if s + 1 < len(Ls):                # the stage after this one is learned from this stage's inputs
            x1 = ctx.apply_stage(x1.reshape(-1, h, w), Wp1).reshape(-1, h, w)
            x2 = ctx.apply_stage(x2.reshape(-1, h, w), Wp2).reshape(-1, h, w)
            G *= Ls[s - 1]
    return {"filters": filters, "rho": rhos}


def extract_stages(ctx: Context, v1, v2, filters, block, stride, dtype=torch.uint16):
    """Features [m, 2, G, nby, nbx, 2**L_last] with G = the product of the earlier stages' filter counts: all stages
    but the last as ddcca_apply_stage, the last fused with hashing and block histograms (ddcca_apply_stage_hash)."""
    m, h, w = v1.shape
    outs = []
    for d, x in enumerate((v1, v2)):
        for W in filters[:-1]:
            x = ctx.apply_stage(x.reshape(-1, h, w), W[d]).reshape(-1, h, w)
        f = ctx.apply_stage_hash(x, filters[-1][d], block, stride, dtype)
        outs.append(f.reshape(m, -1, *f.shape[1:]))
    return torch.stack(outs, dim=1)


class GraphedPath:
    """fit() + extract() of fixed device inputs, captured once into a HIP graph and replayed.

    For launch-bound workloads (small images, few samples) the sixty-odd dependent launches of a step cost more
    in launch gaps than in kernel time; a graph replays them back to back.  Everything the captured calls need
    is allocated by one eager run first (the library grows its scratch on demand and a capture must not
    allocate), the context lives on the capture stream, and the library clears its buffers with kernels, so the
    graph holds kernel and copy nodes only.  Outputs are the tensors `filters`, `rho` and `feat`, rewritten by
    every replay().  Class labels outside [0, n_cls) are reported by status() after a replay.
    """

    def __init__(self, v1, v2, cls, n_cls, k, L1, L2, block, stride, ridge=1e-4, batch_images=0,
                 dtype=torch.uint16, fused=False, device=0, out=None, options=()):
        """out: feature tensor to write (else one is allocated); options: (option, value) pairs for set_option."""
        self.stream = torch.cuda.Stream(device)
        self.stream.wait_stream(torch.cuda.current_stream(device))
        with torch.cuda.stream(self.stream):
            self.ctx = Context(device)
            for opt, val in options:
                self.ctx.set_option(opt, val)

            def run():
                model = fit(self.ctx, v1, v2, cls, n_cls, k, L1, L2, ridge)
                feat = extract(self.ctx, v1, v2, model["filters"], k, L1, L2, block, stride, batch_images, out,
                               dtype, fused)
                return model, feat

            run()                                   # eager: every scratch buffer reaches its final size
            self.ctx.status()
            self.graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(self.graph, stream=self.stream):
                model, self.feat = run()
        self.filters, self.rho = model["filters"], model["rho"]
        self._inputs = (v1, v2, cls)               # the graph reads these buffers on every replay

    def replay(self):
        self.graph.replay()

    def status(self):
        self.ctx.status()

    def close(self):
        self.graph = None
        self.ctx.close()

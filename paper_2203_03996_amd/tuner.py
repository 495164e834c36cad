"""Front-to-back threshold tuning on a density budget (host logic only; every frame runs in the HIP kernels).

The paper tunes one truncation threshold per layer, front to back, against a loss budget on a training set
(Section 4).  Without a dataset the same sweep is run against a *density* budget: for every layer that has a
threshold (the input layer and every activation), in execution order and with the earlier thresholds fixed, a
bisection on a geometric scale looks for the smallest threshold at which the layer emits updates at no more
than `target` of its output pixels, averaged over the sparse frames of a clip.
"""
from __future__ import annotations

import math

from .binding import ACT_NONE, DELTAGEN, Net


def tunable_layers(net: Net) -> list[int]:
    """Planned layers that have a truncation threshold, in execution order."""
    return [i for i, s in enumerate(net.stats()) if s["kind"] == DELTAGEN or s["act"] != ACT_NONE]


def output_density(net: Net, frames, layer: int) -> float:
    """Mean over the sparse frames of the clip of flagged output pixels / output pixels of one layer."""
    net.reset()
    net.init(frames[0])
    dens = []
    for f in frames[1:]:
        net.step(f)
        s = net.stats()[layer]
        dens.append(s["pixels_out"] / s["pixels_total"])
    return sum(dens) / len(dens)


def tune_thresholds(net: Net, frames, target: float, lo: float = 1e-4, hi: float = 16.0, iters: int = 10,
                    layers: list[int] | None = None) -> dict[int, float]:
    """Sets and returns {planned layer: threshold}.  `frames`: device tensors [n, h, w, c] of one clip (the first
    is the dense frame).  A layer whose density exceeds the budget even at `hi` keeps `hi`."""
    if not (0.0 < target <= 1.0) or not (0.0 < lo < hi) or len(frames) < 2:
        raise ValueError("tune_thresholds: need 0 < target <= 1, 0 < lo < hi and a clip of at least two frames")
    found = {}
    for i in (tunable_layers(net) if layers is None else layers):
        a, b = lo, hi
        for _ in range(iters):
            mid = math.sqrt(a * b)
            net.set_eps(i, mid)
            if output_density(net, frames, i) > target:
                a = mid
            else:
                b = mid
        net.set_eps(i, b)
        found[i] = b
    net.reset()
    return found

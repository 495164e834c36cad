"""Seeded synthetic video: static textured background, moving constant-valued
objects, per-frame sensor noise, optional global brightness drift.

The structure follows the paper's evaluation footage (Section 4: fixed camera,
a small moving foreground, background noise that the input threshold is meant
to suppress, slow illumination change as in the "rising sun" remark of
Section 3.1).  These frames stand in for the pose / detection datasets the
paper measures on; none of those datasets' records are reproduced.

Everything is float64 NHWC `[T, H, W, C]`; callers cast to their storage type.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
from scipy import ndimage


@dataclass(frozen=True)
class VideoSpec:
    h: int
    w: int
    c: int
    frames: int
    n_objects: int = 2
    obj_kind: str = "rect"        # "rect" | "blob" | "stick"
    obj_size: int = 12            # rect edge / blob diameter (px)
    max_speed: int = 3            # integer velocity components in [-max_speed, max_speed]
    noise_sigma: float = 0.01     # standard deviation of the per-frame noise
    drift: float = 0.0            # added to every pixel per frame
    bg_sigma: float = 4.0         # Gaussian blur of the background field (px)


def _background(rng: np.random.Generator, spec: VideoSpec) -> np.ndarray:
    field = rng.standard_normal((spec.h, spec.w, spec.c))
    bg = ndimage.gaussian_filter(field, sigma=(spec.bg_sigma, spec.bg_sigma, 0), mode="wrap")
    std = bg.std(axis=(0, 1), keepdims=True)
    return bg / np.where(std > 0, std, 1.0)


def _reflect(pos: np.ndarray, vel: np.ndarray, lo: np.ndarray, hi: np.ndarray):
    """One integer step with reflection at the borders (positions stay in [lo, hi])."""
    pos = pos + vel
    for k in range(2):
        if pos[k] < lo[k]:
            pos[k] = 2 * lo[k] - pos[k]
            vel[k] = -vel[k]
        if pos[k] > hi[k]:
            pos[k] = 2 * hi[k] - pos[k]
            vel[k] = -vel[k]
        pos[k] = min(max(pos[k], lo[k]), hi[k])
    return pos, vel


def _draw_segment(cover: np.ndarray, p0, p1, thick: float) -> None:
    """Mark pixels within `thick/2` of the segment p0-p1 (y, x coordinates)."""
    h, w = cover.shape
    y0, x0 = p0
    y1, x1 = p1
    r = thick / 2.0
    ya, yb = int(max(0, np.floor(min(y0, y1) - r))), int(min(h, np.ceil(max(y0, y1) + r) + 1))
    xa, xb = int(max(0, np.floor(min(x0, x1) - r))), int(min(w, np.ceil(max(x0, x1) + r) + 1))
    if ya >= yb or xa >= xb:
        return
    yy, xx = np.mgrid[ya:yb, xa:xb].astype(np.float64)
    dy, dx = y1 - y0, x1 - x0
    den = dy * dy + dx * dx
    t = np.zeros_like(yy) if den == 0 else np.clip(((yy - y0) * dy + (xx - x0) * dx) / den, 0, 1)
    dist2 = (yy - (y0 + t * dy)) ** 2 + (xx - (x0 + t * dx)) ** 2
    cover[ya:yb, xa:xb] = np.maximum(cover[ya:yb, xa:xb], (dist2 <= r * r).astype(np.float64))


def _stick_cover(h: int, w: int, centre, scale: float, phase: float, lens, amps, freqs, thick) -> np.ndarray:
    """Coverage map of an articulated figure: a torso with four two-segment limbs
    and a head segment whose joint angles vary sinusoidally with `phase`."""
    cover = np.zeros((h, w))
    cy, cx = centre
    hip = (cy + 0.15 * scale, cx)
    neck = (cy - 0.25 * scale, cx)
    _draw_segment(cover, hip, neck, thick[0])
    _draw_segment(cover, neck, (neck[0] - 0.12 * scale, cx), thick[1])
    k = 2
    for root, base in ((neck, 0.9), (neck, -0.9), (hip, 0.35), (hip, -0.35)):
        a1 = base + amps[k] * np.sin(freqs[k] * phase + k)
        e = (root[0] + lens[k] * scale * np.cos(a1), root[1] + lens[k] * scale * np.sin(a1))
        _draw_segment(cover, root, e, thick[k])
        a2 = a1 + amps[k + 1] * np.sin(freqs[k + 1] * phase + 2 * k)
        e2 = (e[0] + lens[k + 1] * scale * np.cos(a2), e[1] + lens[k + 1] * scale * np.sin(a2))
        _draw_segment(cover, e, e2, thick[k + 1])
        k += 2
    return cover


def make_video(spec: VideoSpec, seed: int) -> np.ndarray:
    """Return `[T, H, W, C]` float64 frames for one camera stream."""
    rng = np.random.default_rng(seed)
    bg = _background(rng, spec)
    n = spec.n_objects
    size = spec.obj_size
    vals = rng.uniform(1.0, 2.0, size=n) * rng.choice([-1.0, 1.0], size=n)
    lo = np.array([0, 0])
    hi = np.array([max(spec.h - size, 0), max(spec.w - size, 0)])
    pos = [np.array([rng.integers(lo[0], hi[0] + 1), rng.integers(lo[1], hi[1] + 1)]) for _ in range(n)]
    vel = []
    for _ in range(n):
        v = np.array([0, 0])
        while not v.any():
            v = rng.integers(-spec.max_speed, spec.max_speed + 1, size=2)
        vel.append(v)
    if spec.obj_kind == "stick":
        nseg = 10
        lens = rng.uniform(0.18, 0.3, size=(n, nseg))
        amps = rng.uniform(0.3, 0.9, size=(n, nseg))
        freqs = rng.uniform(0.15, 0.45, size=(n, nseg))
        thick = rng.uniform(3.0, 5.0, size=(n, nseg))
    if spec.obj_kind == "blob":
        sizes = rng.integers(size, 2 * size + 1, size=n)
        yy, xx = np.mgrid[0:2 * size + 1, 0:2 * size + 1].astype(np.float64)

    frames = np.empty((spec.frames, spec.h, spec.w, spec.c))
    for t in range(spec.frames):
        img = bg + spec.drift * t
        for i in range(n):
            y, x = int(pos[i][0]), int(pos[i][1])
            if spec.obj_kind == "rect":
                img[y:y + size, x:x + size, :] = vals[i]
            elif spec.obj_kind == "blob":
                d = int(sizes[i])
                r = d / 2.0
                dist = np.sqrt((yy[:d + 1, :d + 1] - r) ** 2 + (xx[:d + 1, :d + 1] - r) ** 2)
                a = np.clip((r - dist) / 3.0, 0.0, 1.0)           # soft 3-px edge
                ya, xa = min(y + d + 1, spec.h), min(x + d + 1, spec.w)
                a = a[:ya - y, :xa - x, None]
                img[y:ya, x:xa, :] = (1 - a) * img[y:ya, x:xa, :] + a * vals[i]
            elif spec.obj_kind == "stick":
                cover = _stick_cover(spec.h, spec.w, (y + size / 2.0, x + size / 2.0), float(size), float(t),
                                     lens[i], amps[i], freqs[i], thick[i])
                img = np.where(cover[:, :, None] > 0, vals[i], img)
            else:
                raise ValueError(f"unknown obj_kind {spec.obj_kind!r}")
        frames[t] = img + rng.normal(0.0, spec.noise_sigma, size=img.shape) if spec.noise_sigma > 0 else img
        for i in range(n):
            pos[i], vel[i] = _reflect(pos[i], vel[i], lo, hi)
    return frames


def make_batch(spec: VideoSpec, seed: int, n_streams: int) -> np.ndarray:
    """`[T, N, H, W, C]`: N independent camera streams (seed + 7919*stream)."""
    return np.stack([make_video(spec, seed + 7919 * s) for s in range(n_streams)], axis=1)

"""Network topology tables (plain data) and seeded random weights.

A network is a dict:
    {"name", "dtype" ("f32"|"f16"), "h", "w", "c", "video": VideoSpec, "nodes": [...]}
and every node is a dict with "kind", "in" (indices of producer nodes) and the
attributes of that kind:

    deltagen  eps, dilate_r                      (first node, consumes the camera frame)
    conv      k, stride, pad, cin, cout, depthwise   (weights W[k,k,cin,cout] or W[k,k,c], bias[cout])
    act       f ("relu"|"relu6"), eps            (activation + truncation, Section 3.1); optional no_xT, xT_residue
    add       two inputs
    maxpool   k, stride, pad
    upsample  factor (nearest)
    accum     (last node, produces the dense output)

Only shapes and hyper-parameters live here; what each kind computes is defined
separately by the oracle and by the HIP library.
"""
from __future__ import annotations

import numpy as np

from .video import VideoSpec

CONFIG_SEEDS = {i: 0xDE17A + i for i in range(1, 6)}


class _B:
    """Tiny helper that appends nodes and returns their index."""

    def __init__(self, no_xT=False, xT_residue=False):
        self.nodes = []
        self.no_xT = bool(no_xT)
        self.xT_residue = bool(xT_residue)

    def _add(self, **kw) -> int:
        self.nodes.append(kw)
        return len(self.nodes) - 1

    def deltagen(self, eps, dilate_r=0):
        return self._add(kind="deltagen", **{"in": []}, eps=float(eps), dilate_r=int(dilate_r))

    def conv(self, src, k, stride, cin, cout, depthwise=False, pad=None):
        pad = k // 2 if pad is None else pad
        return self._add(kind="conv", **{"in": [src]}, k=k, stride=stride, pad=pad, cin=cin, cout=cout,
                         depthwise=bool(depthwise))

    def act(self, src, f, eps):
        nd = dict(kind="act", **{"in": [src]}, f=f, eps=float(eps))
        if self.no_xT:
            nd["no_xT"] = True                                     # activations keep no buffer of truncated values
        if self.xT_residue:
            nd["xT_residue"] = True                                # an update leaves x^A's rounding residue in x^T
        return self._add(**nd)

    def add(self, a, b):
        return self._add(kind="add", **{"in": [a, b]})

    def concat(self, a, b):
        return self._add(kind="concat", **{"in": [a, b]})

    def maxpool(self, src, k=3, stride=2, pad=1):
        return self._add(kind="maxpool", **{"in": [src]}, k=k, stride=stride, pad=pad)

    def upsample(self, src, factor):
        return self._add(kind="upsample", **{"in": [src]}, factor=int(factor))

    def upsample_bilinear(self, src, factor):
        return self._add(kind="upsample_bilinear", **{"in": [src]}, factor=int(factor))

    def gavgpool(self, src):
        return self._add(kind="gavgpool", **{"in": [src]})

    def accum(self, src):
        return self._add(kind="accum", **{"in": [src]})


def _net(name, dtype, h, w, c, video, b: _B):
    return {"name": name, "dtype": dtype, "h": h, "w": w, "c": c, "video": video, "nodes": b.nodes}


def single_conv_relu(eps=0.05, eps0=None, h=64, w=64, c=32, frames=4, dtype="f32", no_xT=False, xT_residue=False):
    """3x3 s1 conv + ReLU on a C-channel map (the smallest configuration)."""
    eps0 = eps if eps0 is None else eps0
    b = _B(no_xT, xT_residue)
    x = b.deltagen(eps0)
    x = b.conv(x, 3, 1, c, c)
    x = b.act(x, "relu", eps)
    b.accum(x)
    video = VideoSpec(h=h, w=w, c=c, frames=frames, n_objects=2, obj_kind="rect", obj_size=12, noise_sigma=0.01)
    return _net("conv3x3_relu", dtype, h, w, c, video, b)


def bottleneck_block(eps=0.05, eps0=None, h=128, w=128, cin=64, mid=64, cout=256, frames=16, dtype="f16",
                     n_objects=4, dilate_r=0, no_xT=False, xT_residue=False):
    """ResNet bottleneck with a projection shortcut: 1x1 cin->mid, 3x3 mid->mid,
    1x1 mid->cout, shortcut 1x1 cin->cout, add, ReLU."""
    eps0 = eps if eps0 is None else eps0
    b = _B(no_xT, xT_residue)
    x0 = b.deltagen(eps0, dilate_r)
    x = b.act(b.conv(x0, 1, 1, cin, mid), "relu", eps)
    x = b.act(b.conv(x, 3, 1, mid, mid), "relu", eps)
    x = b.conv(x, 1, 1, mid, cout)
    s = b.conv(x0, 1, 1, cin, cout)
    x = b.act(b.add(x, s), "relu", eps)
    b.accum(x)
    video = VideoSpec(h=h, w=w, c=cin, frames=frames, n_objects=n_objects, obj_kind="rect", obj_size=12,
                      noise_sigma=0.01)
    return _net("resnet_bottleneck", dtype, h, w, cin, video, b)


def mobilenet_stack(eps=0.05, eps0=None, h=224, w=224, frames=32, dtype="f16"):
    """Stem 3x3 s2 3->32 + ReLU6, then 7 inverted-residual blocks (expansion 6,
    depthwise 3x3): (32->32 s1) (32->48 s2) (48->48 s1) (48->64 s2) (64->96 s1)
    (96->160 s2) (160->160 s1); residual add when stride 1 and cin == cout."""
    eps0 = eps if eps0 is None else eps0
    b = _B()
    x = b.deltagen(eps0)
    x = b.act(b.conv(x, 3, 2, 3, 32), "relu6", eps)
    table = [(32, 32, 1), (32, 48, 2), (48, 48, 1), (48, 64, 2), (64, 96, 1), (96, 160, 2), (160, 160, 1)]
    for cin, cout, s in table:
        e = cin * 6
        y = b.act(b.conv(x, 1, 1, cin, e), "relu6", eps)
        y = b.act(b.conv(y, 3, s, e, e, depthwise=True), "relu6", eps)
        y = b.conv(y, 1, 1, e, cout)
        x = b.add(x, y) if (s == 1 and cin == cout) else y
    b.accum(x)
    video = VideoSpec(h=h, w=w, c=3, frames=frames, n_objects=8, obj_kind="rect", obj_size=28, noise_sigma=0.01)
    return _net("mobilenetv2_stack", dtype, h, w, 3, video, b)


def _bottleneck(b: _B, x, cin, mid, cout, stride, eps, project):
    y = b.act(b.conv(x, 1, 1, cin, mid), "relu", eps)
    y = b.act(b.conv(y, 3, stride, mid, mid), "relu", eps)
    y = b.conv(y, 1, 1, mid, cout)
    s = b.conv(x, 1, stride, cin, cout, pad=0) if project else x
    return b.act(b.add(y, s), "relu", eps)


def resnet50_backbone(eps=0.05, eps0=None, h=256, w=256, frames=64, dtype="f16", stages=(3, 4, 6, 3)):
    """conv1 7x7 s2 3->64 + ReLU, max-pool 3x3 s2, four bottleneck stages."""
    eps0 = eps if eps0 is None else eps0
    b = _B()
    x = b.deltagen(eps0)
    x = b.act(b.conv(x, 7, 2, 3, 64), "relu", eps)
    x = b.maxpool(x, 3, 2, 1)
    cin = 64
    for si, nblk in enumerate(stages):
        mid = 64 << si
        for bi in range(nblk):
            stride = 2 if (bi == 0 and si > 0) else 1
            x = _bottleneck(b, x, cin, mid, mid * 4, stride, eps, project=(bi == 0))
            cin = mid * 4
    b.accum(x)
    video = VideoSpec(h=h, w=w, c=3, frames=frames, n_objects=6, obj_kind="blob", obj_size=16, noise_sigma=0.02,
                      drift=0.002)
    return _net("resnet50_backbone", dtype, h, w, 3, video, b)


def _basic(b: _B, x, c, eps):
    y = b.act(b.conv(x, 3, 1, c, c), "relu", eps)
    y = b.conv(y, 3, 1, c, c)
    return b.act(b.add(y, x), "relu", eps)


def hrnet_like(eps=0.05, eps0=None, h=384, w=288, frames=128, dtype="f16", blocks_per_stage=1):
    """Multi-resolution network: stem of two 3x3 s2 convs, then stages with
    2, 3 and 4 parallel branches of widths 32/64/128/256 at 1/4 .. 1/32
    resolution.  Each stage runs residual 3x3 blocks per branch and then fuses
    every branch into every other: 1x1 conv + nearest upsample towards finer
    branches, chains of 3x3 s2 convs towards coarser ones, add, ReLU."""
    eps0 = eps if eps0 is None else eps0
    widths = [32, 64, 128, 256]
    b = _B()
    x = b.deltagen(eps0)
    x = b.act(b.conv(x, 3, 2, 3, 64), "relu", eps)
    x = b.act(b.conv(x, 3, 2, 64, 64), "relu", eps)
    branches = [b.act(b.conv(x, 3, 1, 64, widths[0]), "relu", eps),
                b.act(b.conv(x, 3, 2, 64, widths[1]), "relu", eps)]
    for stage in range(3):
        nb = len(branches)
        for _ in range(blocks_per_stage):
            branches = [_basic(b, branches[i], widths[i], eps) for i in range(nb)]
        fused = []
        for i in range(nb):                      # target branch
            acc = None
            for j in range(nb):                  # source branch
                if j == i:
                    t = branches[j]
                elif j > i:                      # coarser -> finer
                    t = b.upsample(b.conv(branches[j], 1, 1, widths[j], widths[i]), 2 ** (j - i))
                else:                            # finer -> coarser
                    t = branches[j]
                    cj = widths[j]
                    for step in range(i - j):
                        last = step == i - j - 1
                        co = widths[i] if last else cj
                        t = b.conv(t, 3, 2, cj, co)
                        if not last:
                            t = b.act(t, "relu", eps)
                        cj = co
                acc = t if acc is None else b.add(acc, t)
            fused.append(b.act(acc, "relu", eps))
        branches = fused
        if nb < 4:                               # open the next, coarser branch
            branches.append(b.act(b.conv(branches[-1], 3, 2, widths[nb - 1], widths[nb]), "relu", eps))
    # head: fuse everything into the finest branch, then a 1x1 to 16 heat-map channels
    acc = branches[0]
    for j in range(1, len(branches)):
        acc = b.add(acc, b.upsample(b.conv(branches[j], 1, 1, widths[j], widths[0]), 2 ** j))
    x = b.act(acc, "relu", eps)
    x = b.conv(x, 1, 1, widths[0], 16)
    b.accum(x)
    video = VideoSpec(h=h, w=w, c=3, frames=frames, n_objects=1, obj_kind="stick", obj_size=120, noise_sigma=0.01)
    return _net("hrnet_like", dtype, h, w, 3, video, b)


def node_shapes(net):
    """Output (h, w, c) of every node."""
    shapes = []
    for nd in net["nodes"]:
        k = nd["kind"]
        if k == "deltagen":
            shapes.append((net["h"], net["w"], net["c"]))
            continue
        h, w, c = shapes[nd["in"][0]]
        if k == "conv":
            ho = (h + 2 * nd["pad"] - nd["k"]) // nd["stride"] + 1
            wo = (w + 2 * nd["pad"] - nd["k"]) // nd["stride"] + 1
            shapes.append((ho, wo, nd["cout"]))
        elif k == "maxpool":
            ho = (h + 2 * nd["pad"] - nd["k"]) // nd["stride"] + 1
            wo = (w + 2 * nd["pad"] - nd["k"]) // nd["stride"] + 1
            shapes.append((ho, wo, c))
        elif k in ("upsample", "upsample_bilinear"):
            shapes.append((h * nd["factor"], w * nd["factor"], c))
        elif k == "gavgpool":
            shapes.append((1, 1, c))
        elif k == "concat":
            shapes.append((h, w, c + shapes[nd["in"][1]][2]))
        else:
            shapes.append((h, w, c))
    return shapes


def make_weights(net, seed: int):
    """He-normal (fan-in) conv weights and N(0, 0.01) biases, float64, keyed by node index."""
    rng = np.random.default_rng(seed + 1000)
    out = {}
    for i, nd in enumerate(net["nodes"]):
        if nd["kind"] != "conv":
            continue
        k, cin, cout = nd["k"], nd["cin"], nd["cout"]
        if nd["depthwise"]:
            wgt = rng.standard_normal((k, k, cout)) * np.sqrt(2.0 / (k * k))
        else:
            wgt = rng.standard_normal((k, k, cin, cout)) * np.sqrt(2.0 / (k * k * cin))
        out[i] = (wgt, rng.normal(0.0, 0.01, size=cout))
    return out


def dense_flops(net) -> int:
    """FLOPs of ordinary dense inference of one frame (1 multiply-add = 2 FLOP, convs only)."""
    shapes = node_shapes(net)
    total = 0
    for i, nd in enumerate(net["nodes"]):
        if nd["kind"] != "conv":
            continue
        ho, wo, co = shapes[i]
        per_out = nd["k"] * nd["k"] * (1 if nd["depthwise"] else nd["cin"])
        total += 2 * ho * wo * co * per_out
    return total


def tiny_concat_net(eps=0.05, eps0=None, h=20, w=24, c=8, frames=6, dtype="f32"):
    """Two branches of different widths joined by a channel concatenation (tests only)."""
    eps0 = eps if eps0 is None else eps0
    b = _B()
    x0 = b.deltagen(eps0)
    a = b.act(b.conv(x0, 3, 1, c, 16), "relu", eps)
    z = b.act(b.conv(x0, 1, 1, c, 8), "relu6", eps)
    q = b.concat(a, z)                                          # 24 channels
    q = b.act(b.conv(q, 3, 1, 24, 16), "relu", eps)
    q = b.concat(q, x0)                                         # joins the raw input delta as well
    q = b.conv(q, 1, 1, 16 + c, 8)
    b.accum(q)
    video = VideoSpec(h=h, w=w, c=c, frames=frames, n_objects=2, obj_kind="rect", obj_size=5, noise_sigma=0.01)
    return _net("tiny_concat", dtype, h, w, c, video, b)


def tiny_pool_net(eps=0.05, eps0=None, h=18, w=22, c=8, frames=6, dtype="f32"):
    """Bilinear upsampling of a coarser branch and a global-average-pooled head (tests only)."""
    eps0 = eps if eps0 is None else eps0
    b = _B()
    x0 = b.deltagen(eps0)
    x = b.act(b.conv(x0, 3, 2, c, 16), "relu", eps)             # h/2
    u = b.upsample_bilinear(b.conv(x, 1, 1, 16, 8), 2)          # back to h
    q = b.act(b.conv(b.add(u, x0), 3, 1, 8, 16), "relu", eps)
    g = b.gavgpool(q)                                           # [1, 1, 16]
    b.accum(b.conv(g, 1, 1, 16, 10))                            # a fully connected head
    video = VideoSpec(h=h, w=w, c=c, frames=frames, n_objects=2, obj_kind="rect", obj_size=5, noise_sigma=0.01)
    return _net("tiny_pool", dtype, h, w, c, video, b)


def tiny_mixed_net(eps=0.05, eps0=None, h=24, w=20, c=8, frames=6, dtype="f32", no_xT=False, xT_residue=False):
    """A small network that touches every node kind once (tests only): strided and
    depthwise convs, ReLU and ReLU6, max-pool, a coarser branch that is upsampled
    back, two adds."""
    eps0 = eps if eps0 is None else eps0
    b = _B(no_xT, xT_residue)
    x0 = b.deltagen(eps0)
    x = b.act(b.conv(x0, 3, 1, c, 16), "relu", eps)
    p = b.maxpool(x, 3, 2, 1)                                   # h/2
    y = b.act(b.conv(p, 3, 1, 16, 16, depthwise=True), "relu6", eps)
    y = b.conv(y, 1, 1, 16, 16)
    z = b.act(b.conv(p, 3, 2, 16, 32), "relu", eps)             # h/4
    z = b.upsample(b.conv(z, 1, 1, 32, 16), 2)                  # back to h/2
    q = b.act(b.add(b.add(y, z), p), "relu", eps)
    q = b.conv(q, 3, 1, 16, 8)
    b.accum(q)
    video = VideoSpec(h=h, w=w, c=c, frames=frames, n_objects=2, obj_kind="rect", obj_size=5, noise_sigma=0.01)
    return _net("tiny_mixed", dtype, h, w, c, video, b)

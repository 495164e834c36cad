"""CPU oracle for sparse frame-difference CNN inference (DeltaCNN, arXiv 2203.03996).

THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct numpy
implementation of what the HIP library computes, written from the paper and
sharing no code with the library.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product never does.

What follows the paper, passage by passage
------------------------------------------
* Linear layers consume deltas directly, c(x + dx) = c(x) + c(dx)   (Section 3.1, Eq. 1).
  Biases are applied in the first (dense) frame only                (Section 3.1, "Nonlinear layers").
* Non-linear layers keep their accumulated input and emit
  dy = f(x + dx) - f(x)                                             (Section 3.1, Eq. 3).
* Activation + truncation with the two buffers x^A and x^T:
  dy = f(x^A + x^T + dx) - f(x^A); a pixel is truncated (marked
  unchanged) iff max_k |dy_k| < eps, in which case dx is added onto
  x^T; otherwise x^A <- x^A + x^T + dx and x^T <- 0                 (Section 3.1, Eqs. 4-6).
* Every feature map travels with a per-pixel update mask; values at
  unflagged pixels are undefined and never read                     (Section 3.2 "Update mask";
                                                                     supplementary Section 1.3).
* A convolution flags every output pixel whose window holds a flagged
  input ("1 pixel -> 49 after three 3x3 convolutions")              (Section 3.3).
* Frame 1 is dense and initialises every buffer; from frame 2 on the
  input layer turns the camera frame into (delta, mask) and the last
  layer accumulates deltas into the dense output                    (Fig. 2 caption; Section 4).
* Negative thresholds force every pixel to be updated (dense mode)  (Section 5, overhead discussion).
* Buffers can be reset, after which the next frame is a first frame (supplementary Section 1.4).

Readings taken where the paper is silent or ambiguous
-----------------------------------------------------
* update iff max_k |dy_k| >= eps (the formula's "< eps truncates").
* the thresholded quantity is the activation's delta *output*.
* the input layer compares against the last *propagated* input per
  pixel (Eqs. 5/6 with f = identity), so slow drift is not lost.
* input-mask dilation is a (2r+1)^2 square.
* a convolution's / pooling's output mask is the exact per-pixel
  footprint of the in-bounds window, independent of any tiling.
* pooling does not truncate; add is stateless.
* storage precision S in {f64, f32, f16}: element-wise arithmetic runs
  in float32 for S in {f32, f16} and float64 for S = f64, with one
  round-to-nearest-even at every store.  Convolution sums are formed
  in float64 and rounded once to S.

Pinned by tests/test_oracle_pins.py (no function here is "parity unpinned").
"""
from __future__ import annotations

import numpy as np

_STORE = {"f64": np.float64, "f32": np.float32, "f16": np.float16}
_MATH = {"f64": np.float64, "f32": np.float32, "f16": np.float32}


# --------------------------------------------------------------------------------------
# small helpers
# --------------------------------------------------------------------------------------
def act_fn(name: str, x: np.ndarray) -> np.ndarray:
    """ReLU (Section 3.1, Eq. 2) or ReLU6, in the dtype of x."""
    if name == "relu":
        return np.maximum(x, x.dtype.type(0))
    if name == "relu6":
        return np.minimum(np.maximum(x, x.dtype.type(0)), x.dtype.type(6))
    if name == "none":
        return x
    raise ValueError(name)


def compact(mask: np.ndarray):
    """Ascending linear indices (n*H + y)*W + x of the flagged pixels, and their count."""
    idx = np.flatnonzero(mask.reshape(-1)).astype(np.int32)
    return idx, int(idx.size)


def window_mask(mask: np.ndarray, k: int, stride: int, pad: int) -> np.ndarray:
    """Output mask of a k x k window op: OR of the input mask over the in-bounds
    taps of every output pixel (Section 3.3: masks dilate through convolutions)."""
    n, h, w = mask.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    mp = np.zeros((n, h + 2 * pad + stride, w + 2 * pad + stride), dtype=bool)
    mp[:, pad:pad + h, pad:pad + w] = mask.astype(bool)
    out = np.zeros((n, ho, wo), dtype=bool)
    for ky in range(k):
        for kx in range(k):
            out |= mp[:, ky:ky + (ho - 1) * stride + 1:stride, kx:kx + (wo - 1) * stride + 1:stride]
    return out.astype(np.uint8)


def dilate_square(mask: np.ndarray, r: int) -> np.ndarray:
    """Dilation by the (2r+1)^2 square (input-mask dilation, Section 4)."""
    if r <= 0:
        return mask.astype(np.uint8)
    return window_mask(mask, 2 * r + 1, 1, r)


def conv_dense(x: np.ndarray, wgt: np.ndarray, stride: int, pad: int, depthwise: bool) -> np.ndarray:
    """Textbook zero-padded cross-correlation in float64.

    x [N,H,W,Cin]; wgt [k,k,Cin,Cout] (or [k,k,C] depthwise);
    y[n,oy,ox,:] = sum_{ky,kx} x[n, oy*s - pad + ky, ox*s - pad + kx, :] (.) wgt[ky,kx]
    """
    x = np.asarray(x, dtype=np.float64)
    wgt = np.asarray(wgt, dtype=np.float64)
    n, h, w, cin = x.shape
    k = wgt.shape[0]
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    xp = np.zeros((n, h + 2 * pad, w + 2 * pad, cin))
    xp[:, pad:pad + h, pad:pad + w, :] = x
    cout = wgt.shape[-1]
    y = np.zeros((n, ho, wo, cout))
    for ky in range(k):
        for kx in range(k):
            win = xp[:, ky:ky + (ho - 1) * stride + 1:stride, kx:kx + (wo - 1) * stride + 1:stride, :]
            if depthwise:
                y += win * wgt[ky, kx]
            else:
                y += win @ wgt[ky, kx]
    return y


def maxpool_dense(x: np.ndarray, k: int, stride: int, pad: int) -> np.ndarray:
    """Max over the in-bounds part of each k x k window (-inf padding), dtype of x."""
    n, h, w, c = x.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    xp = np.full((n, h + 2 * pad, w + 2 * pad, c), -np.inf, dtype=x.dtype)
    xp[:, pad:pad + h, pad:pad + w, :] = x
    y = np.full((n, ho, wo, c), -np.inf, dtype=x.dtype)
    for ky in range(k):
        for kx in range(k):
            y = np.maximum(y, xp[:, ky:ky + (ho - 1) * stride + 1:stride, kx:kx + (wo - 1) * stride + 1:stride, :])
    return y


class Delta:
    """A sparse update: `data` [N,H,W,C] is defined only where `mask` [N,H,W] == 1."""

    def __init__(self, data: np.ndarray, mask: np.ndarray):
        self.data = data
        self.mask = mask.astype(np.uint8)

    def poisoned(self) -> "Delta":
        """Copy with NaN at every unflagged pixel: nothing downstream may read those."""
        d = self.data.copy()
        d[self.mask == 0] = np.nan
        return Delta(d, self.mask)

    def zero_filled(self) -> np.ndarray:
        return np.where(self.mask[..., None] != 0, self.data, self.data.dtype.type(0))

    @property
    def idx(self):
        return compact(self.mask)[0]

    @property
    def count(self):
        return int(self.mask.sum())


# --------------------------------------------------------------------------------------
# layers.  Every layer has init(dense input(s)) -> dense output   (frame 1)
#                      and step(Delta input(s))  -> Delta output   (frames >= 2)
# --------------------------------------------------------------------------------------
class DeltaGen:
    """Input layer (Fig. 2 "Delta Generation"; Section 4: the first truncation
    threshold, optionally followed by a dilation of the mask).  State P holds,
    per pixel, the input value that was last propagated."""

    def __init__(self, eps: float, dilate_r: int = 0, S: str = "f32"):
        self.S, self.eps, self.r = S, eps, int(dilate_r)
        self.P = None

    def init(self, frame: np.ndarray) -> np.ndarray:
        self.P = frame.astype(_STORE[self.S]).copy()
        return self.P.copy()

    def step(self, frame: np.ndarray) -> Delta:
        st, mt = _STORE[self.S], _MATH[self.S]
        cur = frame.astype(st)
        d = cur.astype(mt) - self.P.astype(mt)
        u = np.abs(d).max(axis=-1)
        m = dilate_square((u >= mt(self.eps)).astype(np.uint8), self.r)
        sel = m != 0
        out = np.full(cur.shape, np.nan, dtype=st)
        out[sel] = d[sel].astype(st)
        self.P[sel] = cur[sel]
        return Delta(out, m)


class Conv:
    """Convolution on deltas (Section 3.1, Eq. 1).  Stateless; bias only in frame 1."""

    def __init__(self, wgt, bias, stride: int, pad: int, depthwise: bool = False, S: str = "f32"):
        st = _STORE[S]
        self.S = S
        self.w = np.asarray(wgt).astype(st)          # weights live in storage precision
        self.b = None if bias is None else np.asarray(bias).astype(st)
        self.k, self.stride, self.pad, self.dw = self.w.shape[0], stride, pad, depthwise

    def init(self, x: np.ndarray) -> np.ndarray:
        y = conv_dense(x, self.w, self.stride, self.pad, self.dw)
        if self.b is not None:
            y = y + self.b.astype(np.float64)
        return y.astype(_STORE[self.S])

    def step(self, d: Delta) -> Delta:
        m_out = window_mask(d.mask, self.k, self.stride, self.pad)
        y = conv_dense(d.zero_filled(), self.w, self.stride, self.pad, self.dw).astype(_STORE[self.S])
        y[m_out == 0] = np.nan
        return Delta(y, m_out)


class ActTrunc:
    """Activation fused with truncation (Section 3.1, Eqs. 4-6; Fig. 3).

    use_xT=False gives the variant without the truncated-values buffer
    (Section 6, memory remark): truncated input is simply dropped.

    carry=True is an option beyond the paper for reduced-precision storage (supplementary
    Section 1.4 accepts that floating-point error accumulates in the buffers and resets them
    periodically): on an update x^A <- round_S(s) loses s - round_S(s); instead of x^T <- 0 the
    layer keeps that rounding residue, x^T <- round_S(s - x^A), so that x^A + x^T still equals
    everything received (Eq. 6) to the precision of the arithmetic, not of the storage type.
    The emitted delta and the threshold test are unchanged.  With S = f64 the residue is 0."""

    def __init__(self, f: str, eps: float, S: str = "f32", use_xT: bool = True, carry: bool = False):
        self.f, self.eps, self.S, self.use_xT, self.carry = f, eps, S, use_xT, bool(carry)
        if self.carry and not self.use_xT:
            raise ValueError("the rounding residue lives in x^T")
        self.xA = self.xT = self.last_u = None

    def init(self, x: np.ndarray) -> np.ndarray:
        st = _STORE[self.S]
        self.xA = x.astype(st).copy()
        self.xT = np.zeros_like(self.xA)
        return act_fn(self.f, self.xA.astype(_MATH[self.S])).astype(st)

    def step(self, d: Delta) -> Delta:
        st, mt = _STORE[self.S], _MATH[self.S]
        out = np.full(d.data.shape, np.nan, dtype=st)
        m_out = np.zeros_like(d.mask)
        self.last_u = np.full(d.mask.shape, np.nan)   # max_k |dy_k| of the visited pixels (inspection only)
        sel = np.nonzero(d.mask)                      # only flagged pixels are touched
        if sel[0].size:
            xa = self.xA[sel].astype(mt)
            xt = self.xT[sel].astype(mt)
            dx = d.data[sel].astype(mt)
            s = (xa + xt) + dx
            dy = act_fn(self.f, s) - act_fn(self.f, xa)
            u = np.abs(dy).max(axis=-1)
            self.last_u[sel] = u
            upd = u >= mt(self.eps)
            new_xa = np.where(upd[:, None], s.astype(st), self.xA[sel])
            if self.use_xT:
                kept = (s - s.astype(st).astype(mt)).astype(st) if self.carry else st(0)
                new_xt = np.where(upd[:, None], kept, (xt + dx).astype(st))
            else:
                new_xt = np.zeros_like(new_xa)
            self.xA[sel] = new_xa
            self.xT[sel] = new_xt
            o = np.where(upd[:, None], dy.astype(st), st(np.nan))
            out[sel] = o
            m_out[sel] = upd.astype(np.uint8)
        return Delta(out, m_out)


class Add:
    """Sum of two delta streams: linear, stateless; mask is the OR."""

    def __init__(self, S: str = "f32"):
        self.S = S

    def init(self, a: np.ndarray, b: np.ndarray) -> np.ndarray:
        mt = _MATH[self.S]
        return (a.astype(mt) + b.astype(mt)).astype(_STORE[self.S])

    def step(self, a: Delta, b: Delta) -> Delta:
        st, mt = _STORE[self.S], _MATH[self.S]
        m = (a.mask | b.mask).astype(np.uint8)
        s = (a.zero_filled().astype(mt) + b.zero_filled().astype(mt)).astype(st)
        s[m == 0] = np.nan
        return Delta(s, m)


class Concat:
    """Channel concatenation of two delta streams (Section 3.4 lists it with the other
    linear, stateless layers): mask is the OR; a stream that is not flagged at a pixel
    contributes zeros there (its delta is zero by definition)."""

    def __init__(self, S: str = "f32"):
        self.S = S

    def init(self, a: np.ndarray, b: np.ndarray) -> np.ndarray:
        return np.concatenate([a, b], axis=-1).astype(_STORE[self.S])

    def step(self, a: Delta, b: Delta) -> Delta:
        st = _STORE[self.S]
        m = (a.mask | b.mask).astype(np.uint8)
        s = np.concatenate([a.zero_filled(), b.zero_filled()], axis=-1).astype(st)
        s[m == 0] = np.nan
        return Delta(s, m)


class MaxPool:
    """Max pooling on deltas (Section 3.1, Eq. 3 with f = pooling): the layer keeps
    its accumulated dense input x^A; dy = pool(x^A + dx) - pool(x^A); no truncation."""

    def __init__(self, k: int, stride: int, pad: int, S: str = "f32"):
        self.k, self.stride, self.pad, self.S = k, stride, pad, S
        self.xA = None

    def init(self, x: np.ndarray) -> np.ndarray:
        self.xA = x.astype(_STORE[self.S]).copy()
        return maxpool_dense(self.xA, self.k, self.stride, self.pad)

    def step(self, d: Delta) -> Delta:
        st, mt = _STORE[self.S], _MATH[self.S]
        sel = d.mask != 0
        x_new = self.xA.copy()
        x_new[sel] = (self.xA[sel].astype(mt) + d.data[sel].astype(mt)).astype(st)
        m_out = window_mask(d.mask, self.k, self.stride, self.pad)
        p_new = maxpool_dense(x_new, self.k, self.stride, self.pad).astype(mt)
        p_old = maxpool_dense(self.xA, self.k, self.stride, self.pad).astype(mt)
        with np.errstate(invalid="ignore"):
            dy = (p_new - p_old).astype(st)
        dy[m_out == 0] = np.nan
        self.xA = x_new
        return Delta(dy, m_out)


class Upsample:
    """Nearest-neighbour upsampling by an integer factor: linear, stateless."""

    def __init__(self, factor: int, S: str = "f32"):
        self.r, self.S = int(factor), S

    def init(self, x: np.ndarray) -> np.ndarray:
        return np.repeat(np.repeat(x, self.r, axis=1), self.r, axis=2)

    def step(self, d: Delta) -> Delta:
        return Delta(self.init(d.data), np.repeat(np.repeat(d.mask, self.r, axis=1), self.r, axis=2))


def bilinear_taps(o: int, r: int, size: int):
    """Source indices and weights of output coordinate `o` of a bilinear upsampling by the
    integer factor r with half-pixel centres: the sample position is (o + 0.5) / r - 0.5 =
    (2o + 1 - r) / 2r, clamped to the map.  Integer arithmetic decides which sources carry
    weight, so "weight is zero" is exact."""
    num, den = 2 * o + 1 - r, 2 * r
    if num <= 0:
        return [(0, 1.0)]
    i0, rem = divmod(num, den)
    if i0 >= size - 1:
        return [(size - 1, 1.0)]
    if rem == 0:
        return [(i0, 1.0)]
    w1 = rem / den
    return [(i0, 1.0 - w1), (i0 + 1, w1)]


class UpsampleBilinear:
    """Bilinear upsampling by an integer factor (half-pixel centres): linear, stateless
    (Section 3.4 lists bilinear upsampling with the supported layers).  An output pixel is
    flagged iff a source pixel that carries weight is flagged; unflagged sources contribute
    zeros."""

    def __init__(self, factor: int, S: str = "f32"):
        self.r, self.S = int(factor), S

    def _apply(self, x: np.ndarray, mask):
        n, h, w, c = x.shape
        r = self.r
        out = np.zeros((n, h * r, w * r, c), np.float64)
        m = np.zeros((n, h * r, w * r), np.uint8)
        for oy in range(h * r):
            ty = bilinear_taps(oy, r, h)
            for ox in range(w * r):
                tx = bilinear_taps(ox, r, w)
                for iy, wy in ty:
                    for ix, wx in tx:
                        out[:, oy, ox, :] += wy * wx * x[:, iy, ix, :]
                        if mask is not None:
                            m[:, oy, ox] |= mask[:, iy, ix]
        return out, m

    def init(self, x: np.ndarray) -> np.ndarray:
        return self._apply(x.astype(np.float64), None)[0].astype(_STORE[self.S])

    def step(self, d: Delta) -> Delta:
        out, m = self._apply(d.zero_filled().astype(np.float64), d.mask)
        o = out.astype(_STORE[self.S])
        o[m == 0] = np.nan
        return Delta(o, m)


class GlobalAvgPool:
    """Global average pooling to a 1x1 map (linear, stateless; Section 3.4 lists average pooling
    with the supported layers): the output pixel of a stream is flagged iff any of its input
    pixels is; unflagged inputs contribute zeros."""

    def __init__(self, S: str = "f32"):
        self.S = S

    def init(self, x: np.ndarray) -> np.ndarray:
        return x.astype(np.float64).mean(axis=(1, 2), keepdims=True).astype(_STORE[self.S])

    def step(self, d: Delta) -> Delta:
        n, h, w, c = d.data.shape
        m = d.mask.reshape(n, -1).any(axis=1).astype(np.uint8).reshape(n, 1, 1)
        o = (d.zero_filled().astype(np.float64).sum(axis=(1, 2), keepdims=True) / (h * w)).astype(_STORE[self.S])
        o[m == 0] = np.nan
        return Delta(o, m)


class Accumulate:
    """Output layer (Fig. 2: deltas are accumulated onto the previous dense output)."""

    def __init__(self, S: str = "f32"):
        self.S = S
        self.O = None

    def init(self, y: np.ndarray) -> np.ndarray:
        self.O = y.astype(_STORE[self.S]).copy()
        return self.O.copy()

    def step(self, d: Delta) -> np.ndarray:
        st, mt = _STORE[self.S], _MATH[self.S]
        sel = d.mask != 0
        self.O[sel] = (self.O[sel].astype(mt) + d.data[sel].astype(mt)).astype(st)
        return self.O.copy()


# --------------------------------------------------------------------------------------
# whole networks
# --------------------------------------------------------------------------------------
def build_layers(net: dict, weights: dict, S: str, use_xT: bool = True):
    layers = []
    for i, nd in enumerate(net["nodes"]):
        k = nd["kind"]
        if k == "deltagen":
            layers.append(DeltaGen(nd["eps"], nd.get("dilate_r", 0), S))
        elif k == "conv":
            wgt, bias = weights[i]
            layers.append(Conv(wgt, bias, nd["stride"], nd["pad"], nd["depthwise"], S))
        elif k == "act":
            layers.append(ActTrunc(nd["f"], nd["eps"], S, use_xT and not nd.get("no_xT", False), nd.get("xT_residue", False)))
        elif k == "add":
            layers.append(Add(S))
        elif k == "concat":
            layers.append(Concat(S))
        elif k == "maxpool":
            layers.append(MaxPool(nd["k"], nd["stride"], nd["pad"], S))
        elif k == "upsample":
            layers.append(Upsample(nd["factor"], S))
        elif k == "upsample_bilinear":
            layers.append(UpsampleBilinear(nd["factor"], S))
        elif k == "gavgpool":
            layers.append(GlobalAvgPool(S))
        elif k == "accum":
            layers.append(Accumulate(S))
        else:
            raise ValueError(k)
    return layers


class OracleNet:
    """Runs a topology table frame by frame: `frame(x)` is dense for the first frame
    after construction or reset() and sparse afterwards.  `outs[i]` keeps node i's
    latest output (dense array in frame 1, poisoned Delta later) for inspection."""

    def __init__(self, net: dict, weights: dict, S: str = "f32", use_xT: bool = True):
        self.net, self.S = net, S
        self.layers = build_layers(net, weights, S, use_xT)
        self.started = False
        self.outs = [None] * len(self.layers)

    def reset(self):
        self.started = False

    def frame(self, x: np.ndarray) -> np.ndarray:
        x = np.asarray(x)
        first = not self.started
        for i, (nd, ly) in enumerate(zip(self.net["nodes"], self.layers)):
            if nd["kind"] == "deltagen":
                self.outs[i] = ly.init(x) if first else ly.step(x).poisoned()
                continue
            ins = [self.outs[j] for j in nd["in"]]
            if first:
                self.outs[i] = ly.init(*ins)
            else:
                o = ly.step(*ins)
                self.outs[i] = o.poisoned() if isinstance(o, Delta) else o
        self.started = True
        return self.outs[-1]

    # statistics the paper reports per network (Section 5: fraction of updated
    # conv-input pixels) -- valid after a sparse frame
    def conv_input_density(self):
        dens = []
        for i, nd in enumerate(self.net["nodes"]):
            if nd["kind"] == "conv":
                src = self.outs[nd["in"][0]]
                if isinstance(src, Delta):
                    dens.append(float(src.mask.mean()))
        return dens


def tune_thresholds(onet: "OracleNet", video: np.ndarray, target: float, lo: float = 1e-4, hi: float = 16.0,
                    iters: int = 10) -> dict:
    """Density-budget analogue of the front-to-back threshold tuning of Section 4 (which needs a
    dataset and a loss): for every node with a threshold (input layer, activations) in
    topological order, earlier thresholds fixed, bisect on a geometric scale for the smallest
    threshold at which the node flags at most `target` of its output pixels, averaged over the
    sparse frames of `video` ([T, N, H, W, C]).  Returns {node: threshold} and leaves them set."""
    found = {}
    for v, (nd, ly) in enumerate(zip(onet.net["nodes"], onet.layers)):
        if nd["kind"] not in ("deltagen", "act"):
            continue
        a, b = lo, hi
        for _ in range(iters):
            mid = float(np.sqrt(a * b))
            ly.eps = mid
            onet.reset()
            onet.frame(video[0])
            dens = []
            for t in range(1, video.shape[0]):
                onet.frame(video[t])
                dens.append(float(onet.outs[v].mask.mean()))
            if sum(dens) / len(dens) > target:
                a = mid
            else:
                b = mid
        ly.eps = b
        found[v] = b
    onet.reset()
    return found


def dense_reference(net: dict, weights: dict, x: np.ndarray) -> np.ndarray:
    """Ordinary per-frame inference in float64 (what the method must reproduce
    when nothing is truncated)."""
    outs = []
    for i, nd in enumerate(net["nodes"]):
        k = nd["kind"]
        ins = [outs[j] for j in nd["in"]]
        if k == "deltagen":
            y = np.asarray(x, dtype=np.float64)
        elif k == "conv":
            wgt, bias = weights[i]
            y = conv_dense(ins[0], wgt, nd["stride"], nd["pad"], nd["depthwise"]) + np.asarray(bias, np.float64)
        elif k == "act":
            y = act_fn(nd["f"], ins[0])
        elif k == "add":
            y = ins[0] + ins[1]
        elif k == "concat":
            y = np.concatenate([ins[0], ins[1]], axis=-1)
        elif k == "maxpool":
            y = maxpool_dense(ins[0], nd["k"], nd["stride"], nd["pad"])
        elif k == "upsample":
            y = np.repeat(np.repeat(ins[0], nd["factor"], axis=1), nd["factor"], axis=2)
        elif k == "upsample_bilinear":
            y = UpsampleBilinear(nd["factor"], "f64").init(ins[0])
        elif k == "gavgpool":
            y = ins[0].mean(axis=(1, 2), keepdims=True)
        elif k == "accum":
            y = ins[0]
        else:
            raise ValueError(k)
        outs.append(y)
    return outs[-1]


# --------------------------------------------------------------------------------------
# cost counters (Section 3.2 tile example: inputs, filter parameters, multiplications)
# --------------------------------------------------------------------------------------
def conv_tile_cost(tile_h: int, tile_w: int, k: int, stride: int, cin: int, cout: int) -> dict:
    """Loads and multiplications of one dense output tile of a k x k convolution."""
    ih = (tile_h - 1) * stride + k
    iw = (tile_w - 1) * stride + k
    return {"inputs": ih * iw * cin, "weights": k * k * cin * cout,
            "multiplications": tile_h * tile_w * k * k * cin * cout}


def conv_sparse_macs(mask_in: np.ndarray, k: int, stride: int, pad: int, cin: int, cout: int,
                     depthwise: bool = False) -> int:
    """Multiply-adds a sparse step really needs: every flagged input contributes to
    each output pixel whose in-bounds window contains it."""
    n, h, w = mask_in.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    pairs = 0
    ys, xs = np.nonzero(mask_in.reshape(-1, w))[0] % h, np.nonzero(mask_in.reshape(-1, w))[1]
    for ky in range(k):
        for kx in range(k):
            oy_num, ox_num = ys + pad - ky, xs + pad - kx
            ok = (oy_num % stride == 0) & (ox_num % stride == 0)
            oy, ox = oy_num // stride, ox_num // stride
            ok &= (oy >= 0) & (oy < ho) & (ox >= 0) & (ox < wo)
            pairs += int(ok.sum())
    return pairs * (cout if depthwise else cin * cout)

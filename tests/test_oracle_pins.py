"""Pins for the CPU oracle: facts the paper and the mathematics fix, none of which
is a retyping of the oracle's own formulae.  CPU only."""
import itertools

import numpy as np
import pytest
import scipy.ndimage as ndi
import torch
import torch.nn.functional as F

import workloads as wl
from oracle import deltacnn_oracle as orc
from oracle.deltacnn_oracle import Delta

INF = float("inf")


def _video(net, seed, n_streams=1):
    v = wl.make_batch(net["video"], seed, n_streams)          # [T,N,H,W,C]
    return v


def _run(net, S, seed=3, n_streams=1, use_xT=True):
    wts = wl.make_weights(net, seed)
    on = orc.OracleNet(net, wts, S, use_xT)
    vid = _video(net, seed, n_streams)
    return on, wts, vid


NETS_DENSE_MODE = {
    "conv3x3": lambda e: wl.single_conv_relu(eps=e, h=16, w=12, c=4, frames=4),
    "bottleneck": lambda e: wl.bottleneck_block(eps=e, h=12, w=12, cin=8, mid=8, cout=16, frames=4, n_objects=1),
    "mixed": lambda e: wl.tiny_mixed_net(eps=e, frames=4),
    "concat": lambda e: wl.tiny_concat_net(eps=e, frames=4),
    "pool": lambda e: wl.tiny_pool_net(eps=e, frames=4),
}


# ---- P1: nothing truncated  =>  the method reproduces ordinary per-frame inference -----------
@pytest.mark.parametrize("name", list(NETS_DENSE_MODE))
def test_negative_thresholds_reproduce_dense_inference(name):
    """Section 3.1 Eq. 1 + Eq. 3; Section 5: negative thresholds = dense mode."""
    net = NETS_DENSE_MODE[name](-1.0)
    on, wts, vid = _run(net, "f64", n_streams=2)
    for t in range(vid.shape[0]):
        out = on.frame(vid[t])
        ref = orc.dense_reference(net, wts, vid[t])
        assert np.abs(out - ref).max() <= 1e-10 * max(1.0, np.abs(ref).max()), (name, t)


def test_bias_only_in_first_frame():
    """Zero weights, non-zero bias: every later delta must be exactly zero."""
    net = wl.single_conv_relu(eps=-1.0, h=8, w=8, c=4, frames=3)
    wts = wl.make_weights(net, 5)
    wts = {i: (np.zeros_like(w), np.full_like(b, 0.7)) for i, (w, b) in wts.items()}
    on = orc.OracleNet(net, wts, "f64")
    vid = _video(net, 5)
    o1 = on.frame(vid[0])
    assert np.allclose(o1, 0.7)
    o2 = on.frame(vid[1])
    assert np.array_equal(o1, o2)
    assert np.all(on.outs[1].zero_filled() == 0)


# ---- P2/P3: bookkeeping invariants of Eqs. 5 and 6 ------------------------------------------
@pytest.mark.parametrize("f", ["relu", "relu6"])
@pytest.mark.parametrize("eps", [0.3, 1.5])
def test_state_invariants(f, eps):
    rng = np.random.default_rng(11)
    shape = (2, 6, 5, 4)
    layer = orc.ActTrunc(f, eps, "f64")
    x0 = rng.normal(0, 2, shape)
    y0 = layer.init(x0)
    total_in = x0.copy()
    total_out = y0.copy()
    xa_init = x0.copy()
    fn = {"relu": lambda v: np.maximum(v, 0), "relu6": lambda v: np.clip(v, 0, 6)}[f]
    saw_trunc = saw_upd = False
    for _ in range(12):
        mask = (rng.random(shape[:3]) < 0.6).astype(np.uint8)
        dx = rng.normal(0, 0.4, shape)
        d = Delta(dx, mask).poisoned()
        o = layer.step(d)
        total_in += np.where(mask[..., None] != 0, dx, 0)
        total_out += o.zero_filled()
        saw_upd |= bool(o.mask.any())
        saw_trunc |= bool(((mask == 1) & (o.mask == 0)).any())
        assert np.all(o.mask <= mask)
        # x^A + x^T is the sum of everything received
        assert np.abs(layer.xA + layer.xT - total_in).max() < 1e-12
        # the emitted deltas telescope to f(x^A_now) - f(x^A_init)
        assert np.abs(total_out - y0 - (fn(layer.xA) - fn(xa_init))).max() < 1e-12
        # x^T is zero wherever the pixel was just updated
        assert np.all(layer.xT[o.mask == 1] == 0)
        # un-propagated residue stays below the threshold
        assert np.abs(fn(layer.xA + layer.xT) - fn(layer.xA)).max(axis=-1).max() < eps
        assert not np.isnan(layer.xA).any() and not np.isnan(layer.xT).any()
        assert not np.isnan(o.data[o.mask == 1]).any()
    assert saw_trunc and saw_upd


# ---- P4: slow drift -- the reason x^T exists -------------------------------------------------
def test_slow_drift_fires_with_xT_and_is_lost_without():
    """Section 3.1 ("sun slowly rising"): per-frame change eps/10; with x^T an update fires
    within about ten frames and the output error never reaches eps; without x^T it never fires."""
    eps = 0.5
    shape = (1, 2, 2, 3)
    step = np.full(shape, eps / 10)
    mask = np.ones(shape[:3], np.uint8)
    for use_xT in (True, False):
        layer = orc.ActTrunc("relu", eps, "f64", use_xT=use_xT)
        x0 = np.full(shape, 1.0)
        y = layer.init(x0).copy()
        fired_at = None
        worst = 0.0
        for t in range(1, 31):
            o = layer.step(Delta(step.copy(), mask))
            y = y + o.zero_filled()
            truth = np.maximum(x0 + t * step, 0)
            worst = max(worst, np.abs(y - truth).max())
            if fired_at is None and o.mask.any():
                fired_at = t
        if use_xT:
            assert fired_at is not None and 9 <= fired_at <= 11
            assert worst < eps
        else:
            assert fired_at is None
            assert worst > 2 * eps          # the error keeps growing: the negative control


def test_input_layer_keeps_last_propagated_value():
    """Same drift at the input layer: the frame is compared with the last propagated
    input, so a drift of eps0/4 per frame is flagged every fourth frame."""
    eps0 = 0.4
    g = orc.DeltaGen(eps0, 0, "f64")
    base = np.zeros((1, 3, 3, 2))
    g.init(base)
    flagged = []
    for t in range(1, 13):
        d = g.step(base + t * eps0 / 4 + 1e-12)
        flagged.append(int(d.mask.all()))
        if d.mask.all():
            assert np.allclose(d.data, eps0, atol=1e-9)
    assert flagged == [0, 0, 0, 1] * 3


# ---- P5: nothing changes => nothing happens ---------------------------------------------------
@pytest.mark.parametrize("S", ["f32", "f16"])
def test_identical_frames_give_empty_masks(S):
    net = wl.tiny_mixed_net(eps=0.05)
    on, wts, vid = _run(net, S)
    o1 = on.frame(vid[0]).copy()
    state = [(getattr(l, "xA", None), getattr(l, "xT", None)) for l in on.layers]
    state = [(None if a is None else a.copy(), None if b is None else b.copy()) for a, b in state]
    o2 = on.frame(vid[0])
    assert np.array_equal(o1, o2)
    for i, o in enumerate(on.outs[:-1]):
        assert o.count == 0 and o.idx.size == 0, i
    for l, (a, b) in zip(on.layers, state):
        if a is not None:
            assert np.array_equal(l.xA, a)
        if b is not None:
            assert np.array_equal(l.xT, b)


def test_infinite_threshold_freezes_output():
    """Table 1's eps = infinity row: no update propagates after frame 1."""
    net = wl.single_conv_relu(eps=INF, eps0=INF, h=16, w=16, c=4)
    on, wts, vid = _run(net, "f32")
    o1 = on.frame(vid[0]).copy()
    for t in range(1, 4):
        assert np.array_equal(on.frame(vid[t]), o1)
        assert on.outs[0].count == 0


def test_threshold_equality_updates():
    """max |dy| == eps counts as an update (only strictly smaller values truncate);
    eps = 0 therefore propagates every visited pixel, even with dy = 0."""
    layer = orc.ActTrunc("relu", 0.5, "f64")
    layer.init(np.array([[[[1.0, 2.0]]]]))
    o = layer.step(Delta(np.array([[[[0.5, 0.25]]]]), np.ones((1, 1, 1), np.uint8)))
    assert o.mask[0, 0, 0] == 1
    o = layer.step(Delta(np.array([[[[0.4999, 0.25]]]]), np.ones((1, 1, 1), np.uint8)))
    assert o.mask[0, 0, 0] == 0
    z = orc.ActTrunc("relu", 0.0, "f64")
    z.init(np.array([[[[-3.0]]]]))
    o = z.step(Delta(np.array([[[[1.0]]]]), np.ones((1, 1, 1), np.uint8)))
    assert o.mask[0, 0, 0] == 1 and o.data[0, 0, 0, 0] == 0.0


# ---- P6: mask dilation -----------------------------------------------------------------------
def test_one_pixel_becomes_49_after_three_3x3(golden):
    c = 2
    net_nodes = wl.nets._B()
    x = net_nodes.deltagen(0.5)
    for _ in range(3):
        x = net_nodes.conv(x, 3, 1, c, c)
    net_nodes.accum(x)
    net = {"name": "t", "dtype": "f32", "h": 15, "w": 15, "c": c, "video": None, "nodes": net_nodes.nodes}
    wts = wl.make_weights(net, 1)
    on = orc.OracleNet(net, wts, "f64")
    f0 = np.zeros((1, 15, 15, c))
    on.frame(f0)
    f1 = f0.copy()
    f1[0, 7, 7, :] = 1.0
    on.frame(f1)
    counts = [on.outs[i].count for i in range(4)]
    assert counts == [1, 9, 25, golden["dilation_after_three_3x3"]]
    m = np.zeros((15, 15), bool)
    m[7, 7] = True
    for i in range(1, 4):
        m = ndi.binary_dilation(m, structure=np.ones((3, 3), bool))
        assert np.array_equal(on.outs[i].mask[0].astype(bool), m)
        assert np.array_equal(on.outs[i].idx, np.flatnonzero(m))


@pytest.mark.parametrize("k,stride,pad", [(3, 1, 1), (3, 2, 1), (1, 1, 0), (1, 2, 0), (7, 2, 3), (5, 1, 2), (3, 2, 0)])
def test_window_mask_brute_force(k, stride, pad):
    rng = np.random.default_rng(k * 100 + stride * 10 + pad)
    m = (rng.random((2, 11, 9)) < 0.08).astype(np.uint8)
    got = orc.window_mask(m, k, stride, pad)
    ho = (11 + 2 * pad - k) // stride + 1
    wo = (9 + 2 * pad - k) // stride + 1
    ref = np.zeros((2, ho, wo), np.uint8)
    for n, oy, ox, ky, kx in itertools.product(range(2), range(ho), range(wo), range(k), range(k)):
        iy, ix = oy * stride - pad + ky, ox * stride - pad + kx
        if 0 <= iy < 11 and 0 <= ix < 9 and m[n, iy, ix]:
            ref[n, oy, ox] = 1
    assert np.array_equal(got, ref)
    if stride == 1 and 2 * pad == k - 1:
        for n in range(2):
            assert np.array_equal(got[n].astype(bool),
                                  ndi.binary_dilation(m[n].astype(bool), structure=np.ones((k, k), bool)))


def test_input_mask_dilation_is_a_square():
    m = np.zeros((1, 21, 21), np.uint8)
    m[0, 10, 10] = 1
    out = orc.dilate_square(m, 7)
    assert out.sum() == 15 * 15 and out[0, 3, 3] == 1 and out[0, 2, 3] == 0


def test_input_layer_with_dilation_updates_the_whole_square():
    """Section 4 (high input threshold + dilated input mask): a single pixel that crosses the threshold flags
    the (2r+1)^2 square around it, and the delta AND the stored input are updated on that whole square --
    also at pixels whose own change is below the threshold -- and nowhere else.  By hand on a 9x9 map."""
    r, eps = 2, 0.3
    rng = np.random.default_rng(4)
    f0 = rng.normal(0, 1, (1, 9, 9, 2))
    small = rng.uniform(0.01, 0.05, (1, 9, 9, 2))            # every pixel changes a little (below the threshold)
    f1 = f0 + small
    f1[0, 4, 5, 1] += 1.0                                    # ... and one pixel a lot
    layer = orc.DeltaGen(eps, r, "f64")
    layer.init(f0)
    out = layer.step(f1)
    square = np.zeros((1, 9, 9), bool)
    square[0, 2:7, 3:8] = True
    assert np.array_equal(out.mask.astype(bool), square) and out.count == 25
    assert np.array_equal(out.data[square], (f1 - f0)[square])           # delta on the whole square, own change only
    assert np.all(np.abs(out.data[square]).max(axis=-1)[:12] < eps)      # most of it below the threshold by itself
    assert np.array_equal(layer.P[square], f1[square])                   # stored input follows on the whole square
    assert np.array_equal(layer.P[~square], f0[~square])                 # and is untouched elsewhere
    # the change that was not propagated is not lost: it is still pending against the stored input
    out2 = layer.step(f1)
    assert out2.count == 0
    f2 = f1.copy()
    f2[0, 0, 0, 0] += 0.3 - small[0, 0, 0, 0] + 1e-9                     # frame-to-frame change below eps, total above
    out3 = layer.step(f2)
    assert out3.mask[0, 0, 0] == 1 and out3.data[0, 0, 0, 0] == f2[0, 0, 0, 0] - f0[0, 0, 0, 0]
    # r = 0 flags the one pixel only
    plain = orc.DeltaGen(eps, 0, "f64")
    plain.init(f0)
    assert plain.step(f1).count == 1


def test_dilated_input_mask_with_dense_layers_behind_equals_dense_inference_of_the_stored_input():
    """With every later threshold negative the network output is dense inference of the input layer's stored
    frame P, whatever the input threshold and dilation (Eq. 1 + Eq. 3): an input layer that emitted deltas at
    other pixels than it updated P at -- thresholded pixels only, say, instead of the dilated set -- breaks it."""
    net = wl.tiny_mixed_net(eps=-1.0, eps0=0.4, frames=5)
    net["nodes"][0]["dilate_r"] = 2
    wts = wl.make_weights(net, 6)
    vid = _video(net, 6)
    onet = orc.OracleNet(net, wts, "f64")
    saw_partial = False
    for t in range(vid.shape[0]):
        out = onet.frame(vid[t])
        P = onet.layers[0].P
        dense = orc.dense_reference(net, wts, P)
        assert np.abs(out - dense).max() <= 1e-10 * max(1.0, np.abs(dense).max()), f"frame {t}"
        if t:
            m = onet.outs[0].mask
            saw_partial |= 0 < m.sum() < m.size and not np.array_equal(P, vid[t])
    assert saw_partial, "the input threshold must hold some pixels back for this pin to bite"


# ---- x^T that carries the rounding residue of x^A (option for reduced-precision storage) ---------
def test_residue_in_xT_keeps_the_accumulated_input_to_arithmetic_precision():
    """Eq. 6 says x^A + x^T is everything the layer has received.  In fp16 storage an update rounds x^A to 11
    bits and, with x^T <- 0, loses the rest; with the residue kept in x^T the pair still holds the fp32 sum
    (to one rounding of the residue itself).  Checked against the float64 sum of the very inputs."""
    rng = np.random.default_rng(21)
    shape = (1, 6, 7, 16)
    x0 = rng.normal(0, 2, shape).astype(np.float16)
    plain, carry = orc.ActTrunc("relu", -1.0, "f16"), orc.ActTrunc("relu", -1.0, "f16", carry=True)
    plain.init(x0), carry.init(x0)
    total = x0.astype(np.float64)
    m = np.ones(shape[:3], np.uint8)
    worst_plain = worst_carry = 0.0
    for t in range(400):
        d = rng.normal(0, 0.01, shape).astype(np.float16)           # far below one unit in the last place of x^A
        total = total + d.astype(np.float64)
        op, oc = plain.step(Delta(d, m)), carry.step(Delta(d, m))
        assert op.count == oc.count == m.size                       # eps < 0: every pixel updates, every frame
        acc_p = plain.xA.astype(np.float64) + plain.xT.astype(np.float64)
        acc_c = carry.xA.astype(np.float64) + carry.xT.astype(np.float64)
        worst_plain = max(worst_plain, np.abs(acc_p - total).max())
        worst_carry = max(worst_carry, np.abs(acc_c - total).max())
        # one step: x^A + x^T is the fp32 sum s up to the rounding of the residue (<= 2^-11 of half a unit of x^A)
        assert np.all(np.abs(carry.xT.astype(np.float64)) <= 0.5 * np.spacing(np.abs(carry.xA)).astype(np.float64) + 1e-12)
    scale = np.abs(total).max()
    assert worst_carry <= 2.0 ** -16 * scale, worst_carry           # 400 fp32 + residue roundings (measured 4e-6 at scale 6)
    assert worst_plain >= 20 * worst_carry and worst_plain >= 2.0 ** -11 * scale / 4, (worst_plain, worst_carry)
    # what is emitted is the same rule, f(s) - f(x^A): with identical state the deltas are identical
    a, b = orc.ActTrunc("relu", 0.3, "f16"), orc.ActTrunc("relu", 0.3, "f16", carry=True)
    a.init(x0), b.init(x0)
    d = rng.normal(0, 0.5, shape).astype(np.float16)
    oa, ob = a.step(Delta(d, m)), b.step(Delta(d, m))
    assert np.array_equal(oa.mask, ob.mask) and np.array_equal(oa.data[oa.mask == 1], ob.data[ob.mask == 1])
    assert np.array_equal(a.xA, b.xA) and np.array_equal(a.xT[oa.mask == 0], b.xT[oa.mask == 0])
    assert np.any(b.xT[ob.mask == 1] != 0) and not np.any(a.xT[oa.mask == 1] != 0)
    with pytest.raises(ValueError):
        orc.ActTrunc("relu", 0.3, "f16", use_xT=False, carry=True)


@pytest.mark.parametrize("S", ["f64", "f32"])
def test_residue_option_changes_nothing_where_storage_is_the_arithmetic_type(S):
    """f64 / f32 storage: s is stored as computed, the residue is exactly zero, both variants are bit-identical."""
    net_a = wl.tiny_mixed_net(eps=0.05, frames=5)
    net_b = wl.tiny_mixed_net(eps=0.05, frames=5, xT_residue=True)
    wts = wl.make_weights(net_a, 8)
    vid = _video(net_a, 8)
    a, b = orc.OracleNet(net_a, wts, S), orc.OracleNet(net_b, wts, S)
    for t in range(vid.shape[0]):
        assert np.array_equal(a.frame(vid[t]), b.frame(vid[t]))
    for la, lb in zip(a.layers, b.layers):
        if isinstance(la, orc.ActTrunc):
            assert lb.carry and np.array_equal(la.xA, lb.xA) and np.array_equal(la.xT, lb.xT)


def test_residue_option_tracks_dense_inference_closer_over_a_long_run():
    """fp16 bottleneck-shaped block, 150 frames of slow brightness drift over a static scene, every threshold
    negative so that nothing is truncated: what is left is the rounding of the buffers (supplementary Section
    1.4).  With the residue carried the output stays closer to float64 dense inference of the same frame."""
    net_p = wl.bottleneck_block(eps=-1.0, h=12, w=12, cin=8, mid=8, cout=16, frames=2, n_objects=1)
    net_c = wl.bottleneck_block(eps=-1.0, h=12, w=12, cin=8, mid=8, cout=16, frames=2, n_objects=1, xT_residue=True)
    wts = wl.make_weights(net_p, 31)
    base = _video(net_p, 31)[0].astype(np.float16)
    wts_s = {i: (w.astype(np.float16).astype(np.float64), b.astype(np.float16).astype(np.float64)) for i, (w, b) in wts.items()}
    p, c = orc.OracleNet(net_p, wts, "f16"), orc.OracleNet(net_c, wts, "f16")
    err_p = err_c = 0.0
    for t in range(150):
        fr = (base.astype(np.float64) + 0.0007 * t).astype(np.float16)
        op, oc = p.frame(fr), c.frame(fr)
        if t >= 100:
            dense = orc.dense_reference(net_p, wts_s, fr.astype(np.float64))
            sc = np.abs(dense).max()
            err_p = max(err_p, np.abs(op - dense).max() / sc)
            err_c = max(err_c, np.abs(oc - dense).max() / sc)
    assert err_c < 0.5 * err_p and err_c < 4e-3, (err_p, err_c)


# ---- P7: the paper's scalar example -----------------------------------------------------------
def test_relu_scalar_example(golden):
    prev, dlt = float(golden["relu_prev"]), float(golden["relu_delta"])
    layer = orc.ActTrunc("relu", -1.0, "f64")
    layer.init(np.array([[[[prev]]]]))
    o = layer.step(Delta(np.array([[[[dlt]]]]), np.ones((1, 1, 1), np.uint8)))
    assert o.data[0, 0, 0, 0] == golden["relu_correct_delta"] != golden["relu_wrong_sum"]
    layer = orc.ActTrunc("relu", -1.0, "f64")
    layer.init(np.array([[[[1.0]]]]))
    o = layer.step(Delta(np.array([[[[-3.0]]]]), np.ones((1, 1, 1), np.uint8)))
    assert o.data[0, 0, 0, 0] == -1.0


# ---- P8: convolution / pooling / upsampling against brute force and a library -----------------
CONV_CASES = [(3, 1, 1, False), (3, 2, 1, False), (1, 1, 0, False), (1, 2, 0, False), (7, 2, 3, False),
              (3, 1, 1, True), (3, 2, 1, True), (3, 1, 0, False),
              # depthwise 1x1 (an unfused batch-norm scale) and even windows (average pooling as a depthwise layer)
              (1, 1, 0, True), (2, 2, 0, True), (5, 1, 2, False)]


@pytest.mark.parametrize("k,stride,pad,dw", CONV_CASES)
def test_conv_dense_brute_force_and_torch(k, stride, pad, dw):
    rng = np.random.default_rng(k + 10 * stride + 100 * pad + 1000 * dw)
    n, h, w, cin = 2, 9, 8, 3
    cout = cin if dw else 4
    x = rng.normal(size=(n, h, w, cin))
    wgt = rng.normal(size=(k, k, cin) if dw else (k, k, cin, cout))
    got = orc.conv_dense(x, wgt, stride, pad, dw)
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    ref = np.zeros((n, ho, wo, cout))
    for b, oy, ox, co in itertools.product(range(n), range(ho), range(wo), range(cout)):
        acc = 0.0
        for ky, kx in itertools.product(range(k), range(k)):
            iy, ix = oy * stride - pad + ky, ox * stride - pad + kx
            if not (0 <= iy < h and 0 <= ix < w):
                continue
            if dw:
                acc += x[b, iy, ix, co] * wgt[ky, kx, co]
            else:
                for ci in range(cin):
                    acc += x[b, iy, ix, ci] * wgt[ky, kx, ci, co]
        ref[b, oy, ox, co] = acc
    assert got.shape == ref.shape
    assert np.abs(got - ref).max() < 1e-12
    xt = torch.from_numpy(x).permute(0, 3, 1, 2)
    if dw:
        wt = torch.from_numpy(wgt).permute(2, 0, 1).unsqueeze(1)            # [C,1,k,k]
        yt = F.conv2d(xt, wt, stride=stride, padding=pad, groups=cin)
    else:
        wt = torch.from_numpy(wgt).permute(3, 2, 0, 1)                       # [Cout,Cin,k,k]
        yt = F.conv2d(xt, wt, stride=stride, padding=pad)
    assert np.abs(got - yt.permute(0, 2, 3, 1).numpy()).max() < 1e-12


@pytest.mark.parametrize("k,stride,pad,dw", CONV_CASES)
def test_sparse_conv_step_equals_conv_of_zero_filled_delta(k, stride, pad, dw):
    """Linearity (Eq. 1): the step equals the dense conv of the delta with zeros at unflagged
    pixels -- computed here through torch, with NaN poison proving unflagged values are not used."""
    rng = np.random.default_rng(7 + k)
    n, h, w, cin = 1, 10, 9, 4
    cout = cin if dw else 6
    wgt = rng.normal(size=(k, k, cin) if dw else (k, k, cin, cout))
    layer = orc.Conv(wgt, rng.normal(size=cout), stride, pad, dw, "f64")
    mask = (rng.random((n, h, w)) < 0.15).astype(np.uint8)
    data = rng.normal(size=(n, h, w, cin))
    out = layer.step(Delta(data, mask).poisoned())
    zf = np.where(mask[..., None] != 0, data, 0.0)
    xt = torch.from_numpy(zf).permute(0, 3, 1, 2)
    if dw:
        yt = F.conv2d(xt, torch.from_numpy(wgt).permute(2, 0, 1).unsqueeze(1), stride=stride, padding=pad, groups=cin)
    else:
        yt = F.conv2d(xt, torch.from_numpy(wgt).permute(3, 2, 0, 1), stride=stride, padding=pad)
    ref = yt.permute(0, 2, 3, 1).numpy()
    sel = out.mask != 0
    assert sel.any()
    assert not np.isnan(out.data[sel]).any()
    assert np.abs(out.data[sel] - ref[sel]).max() < 1e-12
    assert not (~sel).any() or np.abs(ref[~sel]).max() == 0.0   # nothing outside the mask is non-zero
    assert np.isnan(out.data[~sel]).all()


def test_maxpool_and_upsample_against_torch():
    rng = np.random.default_rng(2)
    x = rng.normal(size=(2, 9, 11, 3))
    got = orc.maxpool_dense(x, 3, 2, 1)
    ref = F.max_pool2d(torch.from_numpy(x).permute(0, 3, 1, 2), 3, 2, 1).permute(0, 2, 3, 1).numpy()
    assert np.array_equal(got, ref)
    up = orc.Upsample(2, "f64").init(x)
    ref = F.interpolate(torch.from_numpy(x).permute(0, 3, 1, 2), scale_factor=2, mode="nearest")
    assert np.array_equal(up, ref.permute(0, 2, 3, 1).numpy())


def test_maxpool_step_tracks_dense_pooling():
    """dy = pool(x + dx) - pool(x): summed deltas equal pooling of the summed input."""
    rng = np.random.default_rng(4)
    layer = orc.MaxPool(3, 2, 1, "f64")
    x = rng.normal(size=(1, 8, 8, 2))
    y = layer.init(x).copy()
    for _ in range(5):
        mask = (rng.random((1, 8, 8)) < 0.2).astype(np.uint8)
        dx = rng.normal(size=x.shape)
        o = layer.step(Delta(dx, mask).poisoned())
        x = x + np.where(mask[..., None] != 0, dx, 0)
        y = y + o.zero_filled()
        assert np.abs(y - orc.maxpool_dense(x, 3, 2, 1)).max() < 1e-12
        assert np.array_equal(o.mask, orc.window_mask(mask, 3, 2, 1))
        assert not np.isnan(o.data[o.mask == 1]).any()


def test_add_and_accumulate():
    rng = np.random.default_rng(9)
    a = Delta(rng.normal(size=(1, 4, 4, 2)), (rng.random((1, 4, 4)) < 0.5).astype(np.uint8)).poisoned()
    b = Delta(rng.normal(size=(1, 4, 4, 2)), (rng.random((1, 4, 4)) < 0.5).astype(np.uint8)).poisoned()
    s = orc.Add("f64").step(a, b)
    assert np.array_equal(s.mask, a.mask | b.mask)
    for y, x in itertools.product(range(4), range(4)):
        exp = np.zeros(2)
        if a.mask[0, y, x]:
            exp = exp + a.data[0, y, x]
        if b.mask[0, y, x]:
            exp = exp + b.data[0, y, x]
        if s.mask[0, y, x]:
            assert np.allclose(s.data[0, y, x], exp, atol=1e-15)
        else:
            assert np.isnan(s.data[0, y, x]).all()
    acc = orc.Accumulate("f64")
    base = rng.normal(size=(1, 4, 4, 2))
    acc.init(base)
    out = acc.step(s)
    assert np.allclose(out, base + s.zero_filled(), atol=1e-15)


# ---- P9: compaction ---------------------------------------------------------------------------
def test_compaction_is_flatnonzero():
    rng = np.random.default_rng(1)
    m = (rng.random((3, 7, 5)) < 0.3).astype(np.uint8)
    idx, cnt = orc.compact(m)
    assert idx.dtype == np.int32 and cnt == int(m.sum())
    assert np.all(np.diff(idx) > 0)
    n, y, x = np.unravel_index(idx, m.shape)
    assert np.all(m[n, y, x] == 1)
    e_idx, e_cnt = orc.compact(np.zeros((1, 4, 4), np.uint8))
    assert e_cnt == 0 and e_idx.size == 0


# ---- P10: the never-read rule, end to end -----------------------------------------------------
@pytest.mark.parametrize("S", ["f64", "f32", "f16"])
def test_no_nan_reaches_outputs_or_state(S):
    net = wl.tiny_mixed_net(eps=0.05)
    on, wts, vid = _run(net, S, n_streams=2)
    for t in range(vid.shape[0]):
        out = on.frame(vid[t])
        assert not np.isnan(out).any()
        for ly, o in zip(on.layers, on.outs):
            for nm in ("xA", "xT", "P", "O"):
                v = getattr(ly, nm, None)
                if v is not None:
                    assert not np.isnan(v).any()
            if isinstance(o, Delta):
                assert not np.isnan(o.data[o.mask == 1]).any()
                assert np.isnan(o.data[o.mask == 0]).all()


# ---- P11: the paper's tile arithmetic ---------------------------------------------------------
def test_tile_cost_matches_paper(golden):
    c = golden["tile_channels"]
    cost = orc.conv_tile_cost(golden["tile_out"], golden["tile_out"], golden["tile_k"], 1, c, c)
    assert cost["inputs"] == golden["tile_inputs"]
    assert cost["weights"] == golden["tile_weights"]
    assert cost["multiplications"] == golden["tile_multiplications"]


def test_sparse_mac_count_brute_force():
    rng = np.random.default_rng(3)
    m = (rng.random((2, 7, 6)) < 0.3).astype(np.uint8)
    for k, s, p in [(3, 1, 1), (3, 2, 1), (1, 1, 0), (7, 2, 3)]:
        ho, wo = (7 + 2 * p - k) // s + 1, (6 + 2 * p - k) // s + 1
        pairs = 0
        for n, oy, ox, ky, kx in itertools.product(range(2), range(ho), range(wo), range(k), range(k)):
            iy, ix = oy * s - p + ky, ox * s - p + kx
            if 0 <= iy < 7 and 0 <= ix < 6 and m[n, iy, ix]:
                pairs += 1
        assert orc.conv_sparse_macs(m, k, s, p, 5, 3) == pairs * 15
    full = np.ones((1, 8, 8), np.uint8)
    assert orc.conv_sparse_macs(full, 1, 1, 0, 4, 4) == 64 * 16


# ---- storage precisions -----------------------------------------------------------------------
@pytest.mark.parametrize("S,tol", [("f32", 2e-5), ("f16", 3e-2)])
def test_reduced_precision_tracks_f64(S, tol):
    """The f32 / f16 runs stay close to the f64 run in dense mode (no threshold decisions)."""
    net = wl.tiny_mixed_net(eps=-1.0)
    wts = wl.make_weights(net, 3)
    a = orc.OracleNet(net, wts, "f64")
    b = orc.OracleNet(net, wts, S)
    vid = _video(net, 3)
    for t in range(vid.shape[0]):
        ya, yb = a.frame(vid[t]), b.frame(vid[t])
        assert yb.dtype == {"f32": np.float32, "f16": np.float16}[S]
        assert np.abs(ya - yb.astype(np.float64)).max() <= tol * np.abs(ya).max()


def test_reset_restarts_from_a_dense_frame():
    net = wl.single_conv_relu(eps=0.05, h=16, w=16, c=4)
    on, wts, vid = _run(net, "f32")
    for t in range(3):
        on.frame(vid[t])
    on.reset()
    out = on.frame(vid[3])
    fresh = orc.OracleNet(net, wts, "f32").frame(vid[3])
    assert np.array_equal(out, fresh)


def test_truncation_error_is_bounded_not_accumulating():
    """With eps > 0 the accumulated output differs from dense inference, but the difference
    does not grow with the number of frames (Section 3.1, last sentence)."""
    net = wl.single_conv_relu(eps=0.05, h=32, w=32, c=8, frames=40)
    on, wts, vid = _run(net, "f64")
    errs = []
    for t in range(vid.shape[0]):
        out = on.frame(vid[t])
        errs.append(np.abs(out - orc.dense_reference(net, wts, vid[t])).max())
    assert errs[0] < 1e-12
    assert max(errs[20:]) < 2.0 * max(errs[1:20]) + 1e-9
    assert max(errs) < 1.0


def test_concat_by_hand():
    """Channel concatenation of two updates: mask = OR, a stream that is not flagged at a pixel contributes
    zeros (its delta there is zero by definition), nothing is defined where neither is flagged."""
    a = orc.Delta(np.array([[[[1.0, 2.0]], [[3.0, 4.0]], [[5.0, 6.0]]]]), np.array([[[1], [0], [0]]], np.uint8)).poisoned()
    b = orc.Delta(np.array([[[[7.0]], [[8.0]], [[9.0]]]]), np.array([[[1], [1], [0]]], np.uint8)).poisoned()
    out = orc.Concat("f64").step(a, b)
    assert out.mask.tolist() == [[[1], [1], [0]]]
    assert out.data[0, 0, 0].tolist() == [1.0, 2.0, 7.0]
    assert out.data[0, 1, 0].tolist() == [0.0, 0.0, 8.0]
    assert np.isnan(out.data[0, 2, 0]).all()
    dense = orc.Concat("f64").init(np.ones((1, 2, 2, 3)), np.zeros((1, 2, 2, 1)))
    assert dense.shape == (1, 2, 2, 4) and dense[0, 1, 1].tolist() == [1.0, 1.0, 1.0, 0.0]


def test_density_budget_tuner_meets_the_budget_with_the_smallest_probed_threshold():
    """Front-to-back tuning on a density budget (dataset-free analogue of Section 4): after tuning, every
    node with a threshold emits at most `target` of its pixels on the clip, and one bisection step below the
    threshold found (earlier thresholds unchanged) the budget is exceeded -- unless the search ended at its
    lower bound."""
    spec = wl.tiny_mixed_net(eps=0.05, frames=5)
    wts = wl.make_weights(spec, 3)
    vid = wl.make_batch(spec["video"], 3, 1).astype(np.float32)
    net = orc.OracleNet(spec, wts, "f32")
    target, lo, hi, iters = 0.3, 1e-4, 16.0, 8
    found = orc.tune_thresholds(net, vid, target, lo, hi, iters)
    assert sorted(found) == [i for i, nd in enumerate(spec["nodes"]) if nd["kind"] in ("deltagen", "act")]

    def density(v):
        net.reset()
        net.frame(vid[0])
        d = []
        for t in range(1, vid.shape[0]):
            net.frame(vid[t])
            d.append(float(net.outs[v].mask.mean()))
        return sum(d) / len(d)

    step = (hi / lo) ** (2.0 ** -iters)                          # ratio between the last two probes of a bisection
    for v in sorted(found):
        for u, e in found.items():
            net.layers[u].eps = e
        assert density(v) <= target
        if found[v] / step > lo * step:
            net.layers[v].eps = found[v] / step
            # later thresholds do not influence node v; earlier ones are as they were during the search
            assert density(v) > target, f"node {v}: a smaller threshold also meets the budget"
    # a looser budget never needs larger thresholds at the input layer
    net2 = orc.OracleNet(spec, wts, "f32")
    found2 = orc.tune_thresholds(net2, vid, 0.6, lo, hi, iters)
    assert found2[0] <= found[0]


@pytest.mark.parametrize("r", [2, 3, 4])
def test_bilinear_upsampling_against_torch(r):
    """Half-pixel-centre bilinear upsampling: dense values equal torch's (align_corners=False); a sparse step
    is the same operator on the zero-filled delta, and the output mask is exactly the support of the
    interpolated 0/1 mask (a source flags an output pixel iff it carries weight there)."""
    rng = np.random.default_rng(r)
    x = rng.normal(size=(2, 5, 7, 3))
    up = orc.UpsampleBilinear(r, "f64")
    tx = torch.from_numpy(x).permute(0, 3, 1, 2)
    ref = F.interpolate(tx, scale_factor=r, mode="bilinear", align_corners=False).permute(0, 2, 3, 1).numpy()
    assert np.abs(up.init(x) - ref).max() < 1e-13
    mask = (rng.random((2, 5, 7)) < 0.2).astype(np.uint8)
    d = Delta(np.where(mask[..., None] > 0, x, np.nan), mask)
    out = up.step(d)
    zf = torch.from_numpy(np.where(mask[..., None] > 0, x, 0.0)).permute(0, 3, 1, 2)
    ref_d = F.interpolate(zf, scale_factor=r, mode="bilinear", align_corners=False).permute(0, 2, 3, 1).numpy()
    ref_m = F.interpolate(torch.from_numpy(mask.astype(np.float64))[:, None], scale_factor=r, mode="bilinear",
                          align_corners=False)[:, 0].numpy() > 0
    assert np.array_equal(out.mask.astype(bool), ref_m)
    assert np.abs(out.zero_filled() - np.where(ref_m[..., None], ref_d, 0.0)).max() < 1e-13
    assert np.isnan(out.data[out.mask == 0]).all()
    # the tap rule by hand: factor 2, output 0 sits on source 0; output 1 = 3/4 * s0 + 1/4 * s1
    assert orc.bilinear_taps(0, 2, 5) == [(0, 1.0)]
    assert orc.bilinear_taps(1, 2, 5) == [(0, 0.75), (1, 0.25)]
    assert orc.bilinear_taps(9, 2, 5) == [(4, 1.0)]
    assert orc.bilinear_taps(1, 3, 5) == [(0, 1.0)]             # sample position exactly on source 0: source 1 carries no weight


def test_global_average_pooling_against_torch_and_by_hand():
    rng = np.random.default_rng(4)
    x = rng.normal(size=(3, 4, 6, 5))
    gap = orc.GlobalAvgPool("f64")
    ref = F.adaptive_avg_pool2d(torch.from_numpy(x).permute(0, 3, 1, 2), 1).permute(0, 2, 3, 1).numpy()
    assert np.abs(gap.init(x) - ref).max() < 1e-14
    mask = np.zeros((3, 4, 6), np.uint8)
    mask[0, 1, 2] = mask[0, 3, 5] = 1                           # stream 0: two updates; stream 1: none; stream 2: one
    mask[2, 0, 0] = 1
    d = Delta(np.where(mask[..., None] > 0, x, np.nan), mask)
    out = gap.step(d)
    assert out.mask.reshape(-1).tolist() == [1, 0, 1]
    assert np.allclose(out.data[0, 0, 0], (x[0, 1, 2] + x[0, 3, 5]) / 24.0, rtol=0, atol=1e-15)
    assert np.allclose(out.data[2, 0, 0], x[2, 0, 0] / 24.0, rtol=0, atol=1e-15)
    assert np.isnan(out.data[1]).all()

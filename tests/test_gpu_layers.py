"""GPU parity, layer by layer (teacher-forced): every HIP layer is fed the oracle's inputs and
state for a frame and must reproduce the oracle's outputs and state -- masks, index lists and
all element-wise arithmetic bit-exactly, convolution sums within the stated tolerance.
All calls go through the C ABI (ctypes binding)."""
import numpy as np
import pytest
import torch

import paper_2203_03996_amd as pkg
from oracle import deltacnn_oracle as orc
from oracle.deltacnn_oracle import Delta as ODelta
from tests.helpers import NP_DTYPE, TOL, U32, check_delta, rel_err, sum_slack, to_np, ulp, upload_delta

pytestmark = pytest.mark.gpu
DT = {"f32": pkg.F32, "f16": pkg.F16}
TDT = {"f32": torch.float32, "f16": torch.float16}


def _rand_delta(rng, shape, density, S, scale=1.0):
    """Random delta whose unflagged pixels are NaN (reading them would poison the result)."""
    n, h, w, c = shape
    mask = (rng.random((n, h, w)) < density).astype(np.uint8)
    data = (rng.normal(0, scale, shape)).astype(NP_DTYPE[S])
    return ODelta(data, mask).poisoned()


def _upload(d: ODelta):
    return upload_delta(d.data, d.mask)


# ---- mask propagation + compaction (bit-exact) --------------------------------------------------
@pytest.mark.parametrize("n,h,w", [(1, 64, 64), (3, 37, 53), (2, 128, 128), (1, 7, 5)])
@pytest.mark.parametrize("k,stride,pad", [(1, 1, 0), (3, 1, 1), (3, 2, 1), (7, 2, 3), (1, 2, 0)])
@pytest.mark.parametrize("density", [0.0, 0.03, 0.5, 1.0])
def test_mask_compact(n, h, w, k, stride, pad, density):
    rng = np.random.default_rng(n * 1000 + h + k * 7 + int(density * 100))
    m = (rng.random((n, h, w)) < density).astype(np.uint8)
    ctx = pkg.Context(n * h * w)
    mo, idx, cnt = ctx.mask_compact(torch.from_numpy(m).cuda(), k, stride, pad)
    ctx.sync()
    ref = orc.window_mask(m, k, stride, pad)
    assert np.array_equal(to_np(mo), ref)
    ridx, rcnt = orc.compact(ref)
    assert int(to_np(cnt)[0]) == rcnt
    assert np.array_equal(to_np(idx)[:rcnt], ridx)


def test_mask_union():
    rng = np.random.default_rng(5)
    a = (rng.random((2, 33, 47)) < 0.1).astype(np.uint8)
    b = (rng.random((2, 33, 47)) < 0.1).astype(np.uint8)
    ctx = pkg.Context(a.size)
    mo, idx, cnt = ctx.mask_compact(torch.from_numpy(a).cuda(), 1, 1, 0, mask_b=torch.from_numpy(b).cuda())
    ctx.sync()
    assert np.array_equal(to_np(mo), a | b)
    assert np.array_equal(to_np(idx)[:int(to_np(cnt)[0])], np.flatnonzero((a | b).reshape(-1)))


# ---- input delta generation (bit-exact) ---------------------------------------------------------
@pytest.mark.parametrize("S", ["f32", "f16"])
@pytest.mark.parametrize("shape,r", [((1, 64, 64, 32), 0), ((2, 45, 31, 64), 0), ((1, 40, 56, 3), 0), ((1, 9, 9, 17), 0),
                                     ((1, 16, 16, 1024), 0),
                                     # input-mask dilation by the (2r+1)^2 square (Section 4)
                                     ((2, 45, 31, 64), 1), ((1, 64, 72, 16), 7), ((1, 9, 9, 17), 3), ((3, 20, 20, 8), 15)])
def test_deltagen(S, shape, r):
    rng = np.random.default_rng(sum(shape) + r)
    n, h, w, c = shape
    ref = orc.DeltaGen(0.3, r, S)
    ctx = pkg.Context(n * h * w)
    layer = pkg.Layer(ctx, pkg.make_desc(pkg.DELTAGEN, DT[S], n, h, w, c, eps=0.3, dilate_r=r))
    f0 = rng.normal(0, 1, shape).astype(NP_DTYPE[S])
    r0 = ref.init(f0)
    g0 = layer.init([torch.from_numpy(f0).cuda()])
    ctx.sync()
    assert np.array_equal(to_np(g0), r0)
    frame = f0.astype(np.float64)
    for t in range(4):
        frame = frame + (rng.random((n, h, w, 1)) < (0.2 if r == 0 else 0.02)) * rng.normal(0, 0.4, shape)
        fr = frame.astype(NP_DTYPE[S])
        want = ref.step(fr).poisoned()
        out = layer.step([pkg.Delta(torch.from_numpy(fr).cuda(), None, None, None)])
        ctx.sync()
        check_delta(out, want, S, f"deltagen frame {t}", exact_values=True)
        assert np.array_equal(to_np(layer.state_tensor(0)), ref.P)
    st = layer.stats()
    assert st["pixels_out"] == want.count and st["pixels_total"] == n * h * w


# ---- activation + truncation (bit-exact) ---------------------------------------------------------
@pytest.mark.parametrize("S", ["f32", "f16"])
@pytest.mark.parametrize("f,carry", [("relu", False), ("relu6", False), ("relu", True)])
@pytest.mark.parametrize("shape", [(1, 64, 64, 32), (2, 33, 29, 64), (1, 24, 24, 256), (1, 12, 12, 960),
                                   (1, 10, 10, 2048), (1, 9, 11, 3), (1, 9, 11, 17), (1, 8, 8, 100),
                                   # wide pixels on short lists: the channels of a pixel are split over a workgroup's waves
                                   (2, 9, 7, 1024), (1, 5, 5, 1536), (3, 6, 7, 512)])
def test_act_trunc(S, f, carry, shape):
    """carry: the variant that leaves the rounding residue of x^A in x^T on an update (bit-exact like the rest)."""
    rng = np.random.default_rng(sum(shape) + len(f))
    n, h, w, c = shape
    eps = 0.35
    ref = orc.ActTrunc(f, eps, S, carry=carry)
    ctx = pkg.Context(n * h * w)
    layer = pkg.Layer(ctx, pkg.make_desc(pkg.ACT, DT[S], n, h, w, c, act=pkg.ACT_CODES[f], eps=eps, xT_residue=int(carry)))
    x0 = rng.normal(0, 2, shape).astype(NP_DTYPE[S])
    r0 = ref.init(x0)
    g0 = layer.init([torch.from_numpy(x0).cuda()])
    ctx.sync()
    assert np.array_equal(to_np(g0), r0)
    assert np.array_equal(to_np(layer.state_tensor(0)), ref.xA)
    saw = set()
    for t in range(4):
        d = _rand_delta(rng, shape, [0.3, 0.05, 1.0, 0.0][t], S, scale=0.3)
        want = ref.step(d).poisoned()
        out = layer.step([_upload(d)])
        ctx.sync()
        check_delta(out, want, S, f"act frame {t}", exact_values=True)
        assert np.array_equal(to_np(layer.state_tensor(0)), ref.xA)
        assert np.array_equal(to_np(layer.state_tensor(1)), ref.xT)
        if want.count:
            saw.add("upd")
        if want.count < d.count:
            saw.add("trunc")
    assert "upd" in saw and ("trunc" in saw or c > 64)     # wide pixels always exceed the threshold
    if carry and S == "f16":
        assert np.any(ref.xT[want.mask == 1] != 0) if want.count else True


@pytest.mark.parametrize("shape", [(2, 40, 37, 64), (1, 9, 7, 1024)])
def test_layer_whose_list_nobody_walks_keeps_no_count_and_alternates_its_masks(shape):
    """want_idx = 0: the view hands out no count (nothing on a step's path keeps one) and dcnn_layer_stats counts
    the mask instead; the layer walks its input's list, so it alternates between two output masks, each cleared a
    step ahead -- frames whose lists are disjoint, full and empty in turn must leave no stale flag behind."""
    S, f, eps = "f16", "relu", 0.35
    rng = np.random.default_rng(shape[3])
    n, h, w, c = shape
    ref = orc.ActTrunc(f, eps, S)
    ctx = pkg.Context(n * h * w)
    layer = pkg.Layer(ctx, pkg.make_desc(pkg.ACT, DT[S], n, h, w, c, act=pkg.ACT_CODES[f], eps=eps, want_idx=0))
    x0 = rng.normal(0, 2, shape).astype(NP_DTYPE[S])
    ref.init(x0)
    layer.init([torch.from_numpy(x0).cuda()])
    masks = set()
    for t, dens in enumerate([0.4, 0.4, 1.0, 0.0, 0.1, 0.0, 0.6]):
        d = _rand_delta(rng, shape, dens, S, scale=0.3)
        want = ref.step(d).poisoned()
        out = layer.step([_upload(d)])
        ctx.sync()
        assert out.count is None
        masks.add(out.mask.data_ptr())
        assert np.array_equal(to_np(out.mask), want.mask), f"frame {t}"
        assert layer.stats()["pixels_out"] == want.count and layer.stats()["pixels_in"] == d.count
        sel = want.mask.astype(bool)
        assert np.array_equal(to_np(out.data)[sel], want.data[sel])
    assert len(masks) == 2


@pytest.mark.parametrize("S", ["f32", "f16"])
@pytest.mark.parametrize("act", ["relu", "none"])
@pytest.mark.parametrize("shape", [(2, 31, 30, 64), (2, 11, 9, 2048), (1, 13, 5, 1024)])
def test_add_act(S, act, shape):
    rng = np.random.default_rng(17)
    n, h, w, c = shape
    eps = 0.4
    radd, ract = orc.Add(S), orc.ActTrunc(act, eps, S)
    ctx = pkg.Context(n * h * w)
    layer = pkg.Layer(ctx, pkg.make_desc(pkg.ACT, DT[S], n, h, w, c, act=pkg.ACT_CODES[act], eps=eps, n_in=2))
    a0 = rng.normal(0, 1, shape).astype(NP_DTYPE[S])
    b0 = rng.normal(0, 1, shape).astype(NP_DTYPE[S])
    r0 = radd.init(a0, b0)
    if act != "none":
        r0 = ract.init(r0)
    g0 = layer.init([torch.from_numpy(a0).cuda(), torch.from_numpy(b0).cuda()])
    ctx.sync()
    assert np.array_equal(to_np(g0), r0)
    for t in range(3):
        da = _rand_delta(rng, shape, 0.2, S, 0.3)
        db = _rand_delta(rng, shape, 0.1, S, 0.3)
        want = radd.step(da, db).poisoned()
        if act != "none":
            want = ract.step(want).poisoned()
        out = layer.step([_upload(da), _upload(db)])
        ctx.sync()
        check_delta(out, want, S, f"add+{act} frame {t}", exact_values=True)
        if act != "none":
            assert np.array_equal(to_np(layer.state_tensor(0)), ract.xA)
            assert np.array_equal(to_np(layer.state_tensor(1)), ract.xT)


# ---- convolution: linear (values within tolerance; masks and lists bit-exact) -------------------
CONV_CASES = [
    # S, k, stride, pad, cin, cout, (n,h,w)
    ("f32", 3, 1, 1, 32, 32, (1, 64, 64)),
    ("f32", 1, 1, 0, 32, 64, (2, 20, 23)),
    ("f32", 3, 2, 1, 16, 48, (1, 31, 33)),
    ("f32", 3, 1, 1, 3, 32, (1, 30, 30)),
    ("f16", 1, 1, 0, 64, 64, (2, 40, 40)),
    ("f16", 3, 1, 1, 64, 64, (2, 40, 37)),
    ("f16", 1, 1, 0, 64, 256, (1, 48, 48)),
    ("f16", 3, 2, 1, 3, 32, (1, 50, 50)),
    ("f16", 7, 2, 3, 3, 64, (1, 40, 40)),
    # few input channels: the window's (tap, channel) pairs are one flat K dimension
    ("f16", 5, 1, 2, 6, 32, (1, 18, 20)),
    ("f32", 5, 2, 2, 3, 16, (2, 17, 19)),
    ("f16", 3, 1, 1, 1, 8, (1, 12, 16)),
    ("f16", 7, 1, 3, 5, 40, (1, 15, 15)),
    ("f16", 1, 1, 0, 48, 96, (1, 25, 25)),
    ("f16", 3, 1, 1, 32, 160, (1, 21, 20)),
    ("f16", 1, 2, 0, 64, 128, (1, 30, 30)),
    ("f16", 3, 1, 1, 64, 16, (1, 24, 24)),
    # weights too large for LDS: streamed in slices; the last two are wider than one staging tile
    ("f16", 3, 2, 1, 64, 128, (1, 30, 30)),
    ("f16", 3, 1, 1, 256, 256, (1, 20, 20)),
    ("f16", 1, 1, 0, 160, 960, (1, 14, 14)),
    ("f16", 1, 1, 0, 512, 2048, (1, 9, 8)),
    ("f32", 3, 1, 1, 128, 128, (1, 16, 16)),
    ("f32", 1, 1, 0, 64, 1024, (1, 12, 12)),
    # long work lists on streamed weights (sparse steps: several pixel tiles per wave share the weight operands):
    # two / four waves per tile, an input's own list, a strided window, fp32, and two passes over the channels
    ("f16", 3, 1, 1, 128, 128, (6, 128, 128)),
    ("f16", 1, 1, 0, 256, 512, (4, 96, 96)),
    ("f16", 3, 2, 1, 128, 256, (8, 128, 128)),
    ("f32", 3, 1, 1, 64, 128, (6, 96, 96)),
    ("f16", 1, 1, 0, 256, 1024, (4, 80, 80)),
]


def _near_tie(ract, eps, slack):
    """Pixels whose decision the arithmetic leaves open: the oracle's max-norm lies within the value
    tolerance of the threshold, or within what the pixel's own intermediates may differ by."""
    u = np.nan_to_num(ract.last_u, nan=np.inf)
    return np.abs(u - eps) <= TOL[ract.S] * abs(eps) + np.asarray(slack).max(axis=-1)


def _conv_layers(S, k, stride, pad, cin, cout, nhw, rng, act=pkg.ACT_NONE, eps=0.0, n_in=1, depthwise=False):
    n, h, w = nhw
    if depthwise:
        wgt = (rng.normal(0, 1, (k, k, cin)) * np.sqrt(2.0 / (k * k))).astype(NP_DTYPE[S])
    else:
        wgt = (rng.normal(0, 1, (k, k, cin, cout)) * np.sqrt(2.0 / (k * k * cin))).astype(NP_DTYPE[S])
    bias = rng.normal(0, 0.1, cout).astype(NP_DTYPE[S])
    ref = orc.Conv(wgt, bias, stride, pad, depthwise, S)
    ctx = pkg.Context(n * h * w)
    desc = pkg.make_desc(pkg.DWCONV if depthwise else pkg.CONV, DT[S], n, h, w, cin, k=k, stride=stride, pad=pad,
                         cout=cout, act=act, eps=eps, n_in=n_in)
    layer = pkg.Layer(ctx, desc, torch.from_numpy(wgt).cuda(), torch.from_numpy(bias).cuda())
    return ctx, layer, ref


@pytest.mark.parametrize("S,k,stride,pad,cin,cout,nhw", CONV_CASES)
def test_conv_linear(S, k, stride, pad, cin, cout, nhw):
    rng = np.random.default_rng(k * 100 + cin + cout)
    n, h, w = nhw
    ctx, layer, ref = _conv_layers(S, k, stride, pad, cin, cout, nhw, rng)
    x0 = rng.normal(0, 1, (n, h, w, cin)).astype(NP_DTYPE[S])
    r0 = ref.init(x0)
    g0 = layer.init([torch.from_numpy(x0).cuda()])
    ctx.sync()
    assert rel_err(to_np(g0), r0, slack=sum_slack(ref, x0, bias=True)) <= TOL[S], "dense first frame"
    for t, dens in enumerate([0.05, 0.4, 1.0, 0.0]):
        d = _rand_delta(rng, (n, h, w, cin), dens, S)
        want = ref.step(d).poisoned()
        out = layer.step([_upload(d)])
        ctx.sync()
        check_delta(out, want, S, f"conv frame {t} density {dens}", slack=sum_slack(ref, d.zero_filled()))
        st = layer.stats()
        assert st["pixels_in"] == d.count and st["pixels_out"] == want.count


@pytest.mark.parametrize("pattern", ["columns3", "rows3", "diagonal", "holes", "border"])
@pytest.mark.parametrize("nhw", [(2, 40, 37), (1, 33, 64)])
def test_conv3x3_row_gathers_on_structured_masks(pattern, nhw):
    """3x3 / stride 1 / padding 1 on a resident-weight layer with masks that list (nearly) the whole map while
    every pixel has only some taps flagged: the kernel then fetches one centre column per window row and takes the
    left / right taps from neighbouring lanes -- across tile boundaries, row ends and images."""
    S, cin, cout = "f16", 64, 64
    rng = np.random.default_rng(len(pattern) * 7 + nhw[1])
    n, h, w = nhw
    ctx, layer, ref = _conv_layers(S, 3, 1, 1, cin, cout, nhw, rng)
    x0 = rng.normal(0, 1, (n, h, w, cin)).astype(NP_DTYPE[S])
    ref.init(x0)
    layer.init([torch.from_numpy(x0).cuda()])
    yy, xx = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    mask2d = {"columns3": xx % 3 == 0, "rows3": yy % 3 == 1, "diagonal": (xx + yy) % 3 == 0,
              "holes": (xx * 7 + yy * 13) % 11 != 0, "border": (xx == 0) | (xx == w - 1) | (yy % 2 == 0)}[pattern]
    mask = np.broadcast_to(mask2d, (n, h, w)).astype(np.uint8).copy()
    mask[-1, h // 2:, : w // 3] = 0                      # a corner of the last image without any flag
    data = rng.normal(0, 1, (n, h, w, cin)).astype(NP_DTYPE[S])
    d = ODelta(data, mask).poisoned()
    want = ref.step(d).poisoned()
    out = layer.step([_upload(d)])
    ctx.sync()
    assert want.count * 4 >= n * h * w * 3, "the pattern must list at least three quarters of the map"
    check_delta(out, want, S, f"row gathers, {pattern}", slack=sum_slack(ref, d.zero_filled()))


@pytest.mark.parametrize("pattern", ["all", "holes", "sevenths"])
@pytest.mark.parametrize("S,cin,cout", [("f16", 128, 128), ("f32", 64, 128)])
def test_conv3x3_row_gathers_on_the_register_blocked_kernel(S, cin, cout, pattern):
    """The same window-row gathers on a layer whose weights do not fit LDS, with a list long enough for several
    pixel tiles per wave (more than 65,536 entries) and at least three quarters of all window taps flagged: three
    tiles per wave, left / right taps from neighbouring lanes, the tiles' edge columns fetched separately."""
    nhw = (5, 128, 136)
    rng = np.random.default_rng(len(pattern) * 11 + cin)
    n, h, w = nhw
    ctx, layer, ref = _conv_layers(S, 3, 1, 1, cin, cout, nhw, rng)
    x0 = rng.normal(0, 1, (n, h, w, cin)).astype(NP_DTYPE[S])
    ref.init(x0)
    layer.init([torch.from_numpy(x0).cuda()])
    yy, xx = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    mask2d = {"all": xx >= 0, "holes": (xx * 7 + yy * 13) % 11 != 0, "sevenths": (xx * 5 + yy * 3) % 7 != 0}[pattern]
    mask = np.broadcast_to(mask2d, (n, h, w)).astype(np.uint8).copy()
    mask[-1, h - 9:, : w // 3] = 0                       # a corner of the last image without any flag
    data = rng.normal(0, 1, (n, h, w, cin)).astype(NP_DTYPE[S])
    d = ODelta(data, mask).poisoned()
    want = ref.step(d).poisoned()
    out = layer.step([_upload(d)])
    ctx.sync()
    assert want.count > 65536 and d.count * 4 >= want.count * 3, "long list, at least three quarters of the taps flagged"
    check_delta(out, want, S, f"row gathers, register-blocked, {pattern}", slack=sum_slack(ref, d.zero_filled()))


@pytest.mark.parametrize("S,k,stride,cin,cout,nhw,res", [
    # streamed weights, long lists, fused tail: two waves per tile with a residual, four waves per tile, three
    # column blocks per wave in fp32
    ("f16", 3, 1, 128, 128, (5, 128, 136), True),
    ("f16", 1, 1, 256, 256, (4, 96, 96), True),
    ("f32", 3, 1, 64, 96, (6, 96, 96), True),
    ("f32", 3, 1, 32, 32, (1, 64, 64), False),
    ("f16", 1, 1, 64, 64, (2, 32, 32), False),
    ("f16", 3, 1, 64, 64, (2, 33, 35), False),
    ("f16", 1, 1, 64, 256, (1, 40, 40), True),
    ("f16", 3, 2, 64, 128, (1, 30, 30), False),
    ("f16", 3, 2, 3, 32, (1, 40, 40), False),
    ("f32", 1, 1, 16, 16, (1, 20, 20), True),
    # further shapes of the wave-specialised kernel: strided resident 3x3, channels that do not fill the
    # last K-step, three column blocks per wave, two and four waves per tile with a residual, fp32 wide
    ("f16", 3, 2, 32, 32, (2, 41, 37), False),
    ("f16", 1, 1, 24, 96, (1, 33, 31), False),
    ("f16", 3, 1, 16, 96, (1, 31, 29), True),
    ("f16", 1, 1, 64, 128, (1, 45, 40), True),
    ("f16", 1, 2, 32, 256, (1, 50, 44), True),
    ("f32", 1, 1, 32, 64, (1, 37, 30), True),
    ("f32", 3, 1, 16, 64, (3, 21, 22), False),
    ("f16", 1, 1, 64, 64, (4, 96, 96), False),
    # output channels that do not fill the last column block (padded lanes must stay out of the maximum)
    ("f16", 1, 1, 32, 72, (1, 29, 33), True),
    ("f16", 3, 1, 32, 40, (1, 23, 27), False),
    ("f32", 1, 1, 16, 44, (1, 23, 27), False),
])
def test_conv_fused_act(S, k, stride, cin, cout, nhw, res):
    """conv (+ residual) + activation/truncation in one layer == oracle conv -> add -> act."""
    rng = np.random.default_rng(k + cin * 3 + cout)
    n, h, w = nhw
    eps = 0.3
    pad = k // 2
    ctx, layer, rconv = _conv_layers(S, k, stride, pad, cin, cout, nhw, rng, act=pkg.ACT_RELU, eps=eps,
                                     n_in=2 if res else 1)
    radd, ract = orc.Add(S), orc.ActTrunc("relu", eps, S)
    oh, ow = layer.out_shape[1:3]
    x0 = rng.normal(0, 1, (n, h, w, cin)).astype(NP_DTYPE[S])
    y0 = rconv.init(x0)
    # what the arithmetic leaves open, per element: the fp32 sum, and one unit in the last place of every
    # intermediate the two sides round independently (convolution sum; sum with the residual)
    sl0 = sum_slack(rconv, x0, bias=True) + ulp(y0, S)
    ins0 = [torch.from_numpy(x0).cuda()]
    if res:
        s0 = rng.normal(0, 1, (n, oh, ow, cout)).astype(NP_DTYPE[S])
        y0 = radd.init(y0, s0)
        sl0 = sl0 + ulp(y0, S)
        ins0.append(torch.from_numpy(s0).cuda())
    r0 = ract.init(y0)
    g0 = layer.init(ins0)
    ctx.sync()
    assert rel_err(to_np(g0), r0, slack=sl0) <= TOL[S]
    assert rel_err(to_np(layer.state_tensor(0)), ract.xA, slack=sl0) <= TOL[S]
    ties = 0
    for t, dens in enumerate([0.05, 0.3, 1.0, 0.0, 0.1]):
        # teacher forcing: the layer starts every frame from the oracle's state
        layer.state_tensor(0).copy_(torch.from_numpy(ract.xA).cuda())
        layer.state_tensor(1).copy_(torch.from_numpy(ract.xT).cuda())
        d = _rand_delta(rng, (n, h, w, cin), dens, S, 0.5)
        mid = rconv.step(d).poisoned()
        sl = sum_slack(rconv, d.zero_filled()) + ulp(mid.data, S)
        ins = [_upload(d)]
        if res:
            ds = _rand_delta(rng, (n, oh, ow, cout), dens / 2, S, 0.5)
            mid = radd.step(mid, ds).poisoned()
            sl = sl + ulp(mid.data, S)
            ins.append(_upload(ds))
        want = ract.step(mid).poisoned()
        out = layer.step(ins)
        ctx.sync()
        near = _near_tie(ract, eps, sl)
        ties += check_delta(out, want, S, f"fused frame {t}", allow_mask_diff=near, slack=sl)
        # state: equal to the oracle's where the decision agreed
        agree = to_np(out.mask) == want.mask
        assert rel_err(to_np(layer.state_tensor(0))[agree], ract.xA[agree], slack=sl[agree]) <= TOL[S]
        assert rel_err(to_np(layer.state_tensor(1))[agree], ract.xT[agree], slack=sl[agree]) <= TOL[S]
    assert ties <= 3


@pytest.mark.parametrize("S,k,cin,cout,nhw,res", [
    ("f16", 1, 64, 64, (2, 30, 30), False),       # wave-specialised kernel
    ("f16", 3, 32, 96, (1, 21, 24), True),        # three column blocks, residual
    ("f16", 3, 256, 256, (1, 12, 12), False),     # streamed weights: plain kernel tail
    ("f32", 3, 16, 32, (1, 20, 22), False),
    ("f16", 0, 0, 576, (2, 9, 11), False),        # k = 0: a stand-alone activation layer (wide pixels)
    ("f32", 0, 0, 2048, (1, 6, 6), False),        # eight vectors per lane: the pointer-addressed kernel
])
def test_layers_without_truncated_value_buffer(S, k, cin, cout, nhw, res):
    """no_xT = 1 (Section 6, memory remark): a truncated update is dropped, an update is x^A <- x^A + dx;
    teacher-forced against the oracle's ActTrunc(use_xT=False).  Buffer 1 does not exist."""
    rng = np.random.default_rng(k * 7 + cout)
    n, h, w = nhw
    eps = 1.6 if k else 0.3                                     # of the order of a pixel's largest change: both branches occur
    ract = orc.ActTrunc("relu", eps, S, use_xT=False)
    if k:
        wgt = (rng.normal(0, 1, (k, k, cin, cout)) * np.sqrt(2.0 / (k * k * cin))).astype(NP_DTYPE[S])
        bias = rng.normal(0, 0.1, cout).astype(NP_DTYPE[S])
        rconv, radd = orc.Conv(wgt, bias, 1, k // 2, False, S), orc.Add(S)
        ctx = pkg.Context(n * h * w)
        desc = pkg.make_desc(pkg.CONV, DT[S], n, h, w, cin, k=k, stride=1, pad=k // 2, cout=cout, act=pkg.ACT_RELU, eps=eps,
                             n_in=2 if res else 1, no_xT=1)
        layer = pkg.Layer(ctx, desc, torch.from_numpy(wgt).cuda(), torch.from_numpy(bias).cuda())
    else:
        cin = cout
        ctx = pkg.Context(n * h * w)
        layer = pkg.Layer(ctx, pkg.make_desc(pkg.ACT, DT[S], n, h, w, cout, act=pkg.ACT_RELU, eps=eps, no_xT=1))
    with pytest.raises(pkg.DcnnError):
        layer.state_tensor(1)
    x0 = rng.normal(0, 1, (n, h, w, cin)).astype(NP_DTYPE[S])
    y0 = rconv.init(x0) if k else x0
    ins0 = [torch.from_numpy(x0).cuda()]
    if res:
        s0 = rng.normal(0, 1, (n, h, w, cout)).astype(NP_DTYPE[S])
        y0 = radd.init(y0, s0)
        ins0.append(torch.from_numpy(s0).cuda())
    r0 = ract.init(y0)
    g0 = layer.init(ins0)
    ctx.sync()
    sl0 = (sum_slack(rconv, x0, bias=True) + ulp(rconv.init(x0), S) + (ulp(y0, S) if res else 0.0)) if k else 0.0
    assert rel_err(to_np(g0), r0, slack=sl0) <= TOL[S]
    ties = 0
    saw_trunc = False
    for t, dens in enumerate([0.1, 0.5, 1.0, 0.0, 0.2]):
        layer.state_tensor(0).copy_(torch.from_numpy(ract.xA).cuda())
        d = _rand_delta(rng, (n, h, w, cin), dens, S, 0.05 if not k else 0.5)
        mid = rconv.step(d).poisoned() if k else d
        sl = (sum_slack(rconv, d.zero_filled()) + ulp(mid.data, S)) if k else np.zeros(mid.data.shape)
        ins = [_upload(d)]
        if res:
            ds = _rand_delta(rng, (n, h, w, cout), dens / 2, S, 0.5)
            mid = radd.step(mid, ds).poisoned()
            sl = sl + ulp(mid.data, S)
            ins.append(_upload(ds))
        xa_before = ract.xA.copy()
        want = ract.step(mid).poisoned()
        out = layer.step(ins)
        ctx.sync()
        near = _near_tie(ract, eps, sl)
        ties += check_delta(out, want, S, f"no-xT frame {t}", allow_mask_diff=near, exact_values=not k, slack=sl)
        agree = to_np(out.mask) == want.mask
        assert rel_err(to_np(layer.state_tensor(0))[agree], ract.xA[agree], slack=sl[agree]) <= TOL[S]
        trunc = (mid.mask == 1) & (want.mask == 0)
        saw_trunc |= bool(trunc.any())
        assert np.array_equal(ract.xA[trunc], xa_before[trunc])       # the oracle really dropped those updates
    assert ties <= 3 and (saw_trunc or cout > 96)


@pytest.mark.parametrize("S,k,cin,cin2,cout,nhw,stride2", [
    ("f16", 1, 64, 64, 256, (2, 24, 40), 1),
    ("f16", 1, 64, 32, 128, (1, 19, 23), 2),
    ("f16", 3, 32, 48, 64, (1, 33, 35), 1),
    ("f32", 1, 16, 8, 32, (1, 20, 20), 1),
    ("f32", 3, 16, 16, 32, (1, 17, 21), 2),
])
def test_conv_fused_projection(S, k, cin, cin2, cout, nhw, stride2):
    """conv_a(x) + conv_b(z) + activation/truncation in one layer (the 1x1 projection conv_b of the other
    arm of a residual add runs inside the same kernel) == oracle conv, conv, add, act."""
    rng = np.random.default_rng(7 * k + cin + cin2 + cout + stride2)
    n, oh, ow = nhw
    h, w = oh, ow                                           # main convolution: stride 1, same padding
    h2, w2 = (oh - 1) * stride2 + 1 + (stride2 - 1), (ow - 1) * stride2 + 1      # ragged: an unused last row
    if (h2 - 1) // stride2 + 1 != oh:
        h2 = (oh - 1) * stride2 + 1
    eps = 0.3
    wa = (rng.normal(0, 1, (k, k, cin, cout)) * np.sqrt(2.0 / (k * k * cin))).astype(NP_DTYPE[S])
    wb = (rng.normal(0, 1, (1, 1, cin2, cout)) * np.sqrt(2.0 / cin2)).astype(NP_DTYPE[S])
    ba = rng.normal(0, 0.1, cout).astype(NP_DTYPE[S])
    bb = rng.normal(0, 0.1, cout).astype(NP_DTYPE[S])
    ra, rb = orc.Conv(wa, ba, 1, k // 2, False, S), orc.Conv(wb, bb, stride2, 0, False, S)
    radd, ract = orc.Add(S), orc.ActTrunc("relu", eps, S)
    ctx = pkg.Context(n * max(h * w, h2 * w2))
    desc = pkg.make_desc(pkg.CONV, DT[S], n, h, w, cin, k=k, stride=1, pad=k // 2, cout=cout, act=pkg.ACT_RELU, eps=eps,
                         n_in=2, proj=(cin2, h2, w2, stride2))
    wcat = torch.from_numpy(np.concatenate([wa.ravel(), wb.ravel()])).cuda()
    bcat = torch.from_numpy(np.concatenate([ba, bb])).cuda()
    layer = pkg.Layer(ctx, desc, wcat, bcat)
    assert layer.out_shape == (n, oh, ow, cout)
    x0 = rng.normal(0, 1, (n, h, w, cin)).astype(NP_DTYPE[S])
    z0 = rng.normal(0, 1, (n, h2, w2, cin2)).astype(NP_DTYPE[S])
    ya0, yb0 = ra.init(x0), rb.init(z0)
    y0 = radd.init(ya0, yb0)
    r0 = ract.init(y0)
    g0 = layer.init([torch.from_numpy(x0).cuda(), torch.from_numpy(z0).cuda()])
    ctx.sync()
    # both convolution sums and their sum are intermediates each side rounds on its own
    sl0 = sum_slack(ra, x0, bias=True) + sum_slack(rb, z0, bias=True) + ulp(ya0, S) + ulp(yb0, S) + ulp(y0, S)
    assert rel_err(to_np(g0), r0, slack=sl0) <= TOL[S], "dense first frame"
    assert rel_err(to_np(layer.state_tensor(0)), ract.xA, slack=sl0) <= TOL[S]
    ties = 0
    for t, (dx, dz) in enumerate([(0.05, 0.1), (0.3, 0.0), (0.0, 0.2), (1.0, 1.0), (0.0, 0.0), (0.1, 0.02)]):
        layer.state_tensor(0).copy_(torch.from_numpy(ract.xA).cuda())
        layer.state_tensor(1).copy_(torch.from_numpy(ract.xT).cuda())
        d = _rand_delta(rng, (n, h, w, cin), dx, S, 0.5)
        z = _rand_delta(rng, (n, h2, w2, cin2), dz, S, 0.5)
        ma, mb = ra.step(d).poisoned(), rb.step(z).poisoned()
        mid = radd.step(ma, mb).poisoned()
        sl = (sum_slack(ra, d.zero_filled()) + sum_slack(rb, z.zero_filled()) + ulp(ma.data, S) + ulp(mb.data, S)
              + ulp(mid.data, S))
        want = ract.step(mid).poisoned()
        out = layer.step([_upload(d), _upload(z)])
        ctx.sync()
        near = _near_tie(ract, eps, sl)
        ties += check_delta(out, want, S, f"projection frame {t}", allow_mask_diff=near, slack=sl)
        agree = to_np(out.mask) == want.mask
        assert rel_err(to_np(layer.state_tensor(0))[agree], ract.xA[agree], slack=sl[agree]) <= TOL[S]
        assert rel_err(to_np(layer.state_tensor(1))[agree], ract.xT[agree], slack=sl[agree]) <= TOL[S]
        st = layer.stats()
        assert st["pixels_in"] == d.count and st["pixels_in2"] == z.count and st["pixels_work"] == mid.count
    assert ties <= 3


@pytest.mark.parametrize("S,k,cin,cout,nhw,proj", [
    ("f16", 1, 64, 256, (2, 24, 40), True),
    ("f16", 3, 32, 64, (1, 33, 35), False),
    ("f32", 1, 16, 32, (1, 20, 21), False),
    ("f32", 3, 16, 32, (1, 17, 21), True),
])
def test_conv_fused_accumulate(S, k, cin, cout, nhw, proj):
    """The network's output layer folded into the last convolution + activation: the layer keeps the dense
    accumulated output O and adds every emitted delta to it == oracle conv (, conv, add), act, accumulate."""
    rng = np.random.default_rng(11 * k + cin + cout + int(proj))
    n, h, w = nhw
    cin2 = 16
    eps = 0.3
    wa = (rng.normal(0, 1, (k, k, cin, cout)) * np.sqrt(2.0 / (k * k * cin))).astype(NP_DTYPE[S])
    wb = (rng.normal(0, 1, (1, 1, cin2, cout)) * np.sqrt(2.0 / cin2)).astype(NP_DTYPE[S])
    ba = rng.normal(0, 0.1, cout).astype(NP_DTYPE[S])
    bb = rng.normal(0, 0.1, cout).astype(NP_DTYPE[S])
    ra, rb = orc.Conv(wa, ba, 1, k // 2, False, S), orc.Conv(wb, bb, 1, 0, False, S)
    radd, ract, racc = orc.Add(S), orc.ActTrunc("relu", eps, S), orc.Accumulate(S)
    ctx = pkg.Context(n * h * w)
    desc = pkg.make_desc(pkg.CONV, DT[S], n, h, w, cin, k=k, stride=1, pad=k // 2, cout=cout, act=pkg.ACT_RELU, eps=eps,
                         n_in=2 if proj else 1, proj=(cin2, h, w, 1) if proj else None, fuse_accum=1, want_idx=0)
    wcat = np.concatenate([wa.ravel(), wb.ravel()]) if proj else wa
    bcat = np.concatenate([ba, bb]) if proj else ba
    layer = pkg.Layer(ctx, desc, torch.from_numpy(wcat).cuda(), torch.from_numpy(bcat).cuda())
    x0 = rng.normal(0, 1, (n, h, w, cin)).astype(NP_DTYPE[S])
    z0 = rng.normal(0, 1, (n, h, w, cin2)).astype(NP_DTYPE[S])
    y0 = ra.init(x0)
    sl0 = sum_slack(ra, x0, bias=True) + ulp(y0, S)
    if proj:
        yb0 = rb.init(z0)
        y0 = radd.init(y0, yb0)
        sl0 = sl0 + sum_slack(rb, z0, bias=True) + ulp(yb0, S) + ulp(y0, S)
    r0 = racc.init(ract.init(y0))
    g0 = layer.init([torch.from_numpy(x0).cuda()] + ([torch.from_numpy(z0).cuda()] if proj else []))
    ctx.sync()
    assert rel_err(to_np(g0), r0, slack=sl0) <= TOL[S]
    assert np.array_equal(to_np(layer.state_tensor(2)), to_np(g0)), "O starts as the dense first output"
    for t, dens in enumerate([0.05, 0.3, 1.0, 0.0, 0.1]):
        layer.state_tensor(0).copy_(torch.from_numpy(ract.xA).cuda())
        layer.state_tensor(1).copy_(torch.from_numpy(ract.xT).cuda())
        layer.state_tensor(2).copy_(torch.from_numpy(racc.O).cuda())
        d = _rand_delta(rng, (n, h, w, cin), dens, S, 0.5)
        mid = ra.step(d).poisoned()
        sl = sum_slack(ra, d.zero_filled()) + ulp(mid.data, S)
        ins = [_upload(d)]
        if proj:
            z = _rand_delta(rng, (n, h, w, cin2), dens / 2, S, 0.5)
            mb = rb.step(z).poisoned()
            mid = radd.step(mid, mb).poisoned()
            sl = sl + sum_slack(rb, z.zero_filled()) + ulp(mb.data, S) + ulp(mid.data, S)
            ins.append(_upload(z))
        o_before = racc.O.copy()
        want = ract.step(mid).poisoned()
        o_ref = racc.step(want)
        out = layer.step(ins)
        ctx.sync()
        gm = to_np(out.mask)
        near = _near_tie(ract, eps, sl)
        assert np.all(near[gm != want.mask]), f"frame {t}: mask mismatch away from a threshold tie"
        agree = gm == want.mask
        got_o = to_np(layer.state_tensor(2)).reshape(o_ref.shape)
        assert not np.isnan(got_o.astype(np.float64)).any()
        # the folded layer writes O = f(new x^A), the oracle's output layer adds the rounded delta onto O:
        # one more independent rounding, of the delta
        sl_o = sl + ulp(want.data, S)
        assert rel_err(got_o[agree], o_ref[agree], slack=sl_o[agree]) <= TOL[S], f"frame {t}: accumulated output"
        untouched = want.mask == 0
        assert np.array_equal(got_o[untouched & agree], o_before[untouched & agree]), "O changes only where a delta was emitted"
        assert out.data.data_ptr() == layer.state_tensor(2).data_ptr(), "the layer's output data is O"


@pytest.mark.parametrize("S", ["f32", "f16"])
@pytest.mark.parametrize("stride,c", [(1, 32), (2, 192), (1, 960), (2, 20)])
def test_depthwise(S, stride, c):
    rng = np.random.default_rng(stride + c)
    nhw = (1, 28, 27)
    eps = 0.3
    ctx, layer, rconv = _conv_layers(S, 3, stride, 1, c, c, nhw, rng, act=pkg.ACT_RELU6, eps=eps, depthwise=True)
    ract = orc.ActTrunc("relu6", eps, S)
    x0 = rng.normal(0, 1, nhw + (c,)).astype(NP_DTYPE[S])
    y0 = rconv.init(x0)
    r0 = ract.init(y0)
    g0 = layer.init([torch.from_numpy(x0).cuda()])
    ctx.sync()
    assert rel_err(to_np(g0), r0, slack=sum_slack(rconv, x0, bias=True) + ulp(y0, S)) <= TOL[S]
    ties = 0
    for t, dens in enumerate([0.1, 0.5, 0.0]):
        layer.state_tensor(0).copy_(torch.from_numpy(ract.xA).cuda())
        layer.state_tensor(1).copy_(torch.from_numpy(ract.xT).cuda())
        d = _rand_delta(rng, nhw + (c,), dens, S, 0.5)
        mid = rconv.step(d).poisoned()
        sl = sum_slack(rconv, d.zero_filled()) + ulp(mid.data, S)
        want = ract.step(mid).poisoned()
        out = layer.step([_upload(d)])
        ctx.sync()
        near = _near_tie(ract, eps, sl)
        ties += check_delta(out, want, S, f"depthwise frame {t}", allow_mask_diff=near, slack=sl)
    assert ties <= 3


@pytest.mark.parametrize("S", ["f32", "f16"])
@pytest.mark.parametrize("k,stride,pad,what", [(1, 1, 0, "batchnorm"), (2, 2, 0, "avgpool"), (3, 2, 1, "avgpool")])
def test_depthwise_as_batchnorm_and_average_pooling(S, k, stride, pad, what):
    """The remaining linear per-channel layers are depthwise convolutions: an unfused batch norm is a 1x1
    depthwise layer (scale on the delta, shift only in the first frame -- Section 3.1: biases enter once),
    average pooling a k x k depthwise layer with weights 1/k^2 (zero padding counted)."""
    rng = np.random.default_rng(k * 10 + stride)
    n, h, w, c = 2, 26, 22, 48
    if what == "batchnorm":
        wgt = rng.uniform(0.5, 1.5, (1, 1, c)).astype(NP_DTYPE[S])
        bias = rng.normal(0, 0.5, c).astype(NP_DTYPE[S])
    else:
        wgt = np.full((k, k, c), 1.0 / (k * k)).astype(NP_DTYPE[S])
        bias = np.zeros(c, NP_DTYPE[S])
    ref = orc.Conv(wgt, bias, stride, pad, True, S)
    ctx = pkg.Context(n * h * w)
    desc = pkg.make_desc(pkg.DWCONV, DT[S], n, h, w, c, k=k, stride=stride, pad=pad, cout=c)
    layer = pkg.Layer(ctx, desc, torch.from_numpy(wgt).cuda(), torch.from_numpy(bias).cuda())
    x0 = rng.normal(0, 1, (n, h, w, c)).astype(NP_DTYPE[S])
    r0 = ref.init(x0)
    g0 = layer.init([torch.from_numpy(x0).cuda()])
    ctx.sync()
    assert rel_err(to_np(g0), r0, slack=sum_slack(ref, x0, bias=True)) <= TOL[S]
    for t, dens in enumerate([0.1, 0.6, 0.0]):
        d = _rand_delta(rng, (n, h, w, c), dens, S)
        want = ref.step(d).poisoned()
        out = layer.step([_upload(d)])
        ctx.sync()
        check_delta(out, want, S, f"{what} frame {t}", slack=sum_slack(ref, d.zero_filled()))


# ---- pooling, upsampling, accumulation (bit-exact) -----------------------------------------------
@pytest.mark.parametrize("S", ["f32", "f16"])
def test_maxpool(S):
    rng = np.random.default_rng(3)
    shape = (2, 33, 30, 64)
    n, h, w, c = shape
    ref = orc.MaxPool(3, 2, 1, S)
    ctx = pkg.Context(n * h * w)
    layer = pkg.Layer(ctx, pkg.make_desc(pkg.MAXPOOL, DT[S], n, h, w, c, k=3, stride=2, pad=1))
    x0 = rng.normal(0, 1, shape).astype(NP_DTYPE[S])
    r0 = ref.init(x0)
    g0 = layer.init([torch.from_numpy(x0).cuda()])
    ctx.sync()
    assert np.array_equal(to_np(g0), r0)
    for t, dens in enumerate([0.1, 0.6, 0.0]):
        d = _rand_delta(rng, shape, dens, S, 0.7)
        want = ref.step(d).poisoned()
        out = layer.step([_upload(d)])
        ctx.sync()
        check_delta(out, want, S, f"maxpool frame {t}", exact_values=True)
        assert np.array_equal(to_np(layer.state_tensor(0)), ref.xA)


@pytest.mark.parametrize("S", ["f32", "f16"])
@pytest.mark.parametrize("factor", [2, 4])
def test_upsample(S, factor):
    rng = np.random.default_rng(factor)
    shape = (2, 9, 12, 32)
    n, h, w, c = shape
    ref = orc.Upsample(factor, S)
    ctx = pkg.Context(n * h * w * factor * factor)
    layer = pkg.Layer(ctx, pkg.make_desc(pkg.UPSAMPLE, DT[S], n, h, w, c, factor=factor))
    x0 = rng.normal(0, 1, shape).astype(NP_DTYPE[S])
    g0 = layer.init([torch.from_numpy(x0).cuda()])
    ctx.sync()
    assert np.array_equal(to_np(g0), ref.init(x0))
    for t, dens in enumerate([0.1, 1.0, 0.0]):
        d = _rand_delta(rng, shape, dens, S)
        want = ref.step(d).poisoned()
        out = layer.step([_upload(d)])
        ctx.sync()
        check_delta(out, want, S, f"upsample frame {t}", exact_values=True)


@pytest.mark.parametrize("S", ["f32", "f16"])
@pytest.mark.parametrize("factor,c", [(2, 32), (3, 5), (4, 16)])
def test_upsample_bilinear(S, factor, c):
    """Masks and lists bit-exact (integer tap rule); values within tolerance (fp32 weights vs float64)."""
    rng = np.random.default_rng(factor * 10 + c)
    shape = (2, 7, 9, c)
    n, h, w, _ = shape
    ref = orc.UpsampleBilinear(factor, S)
    ctx = pkg.Context(n * h * w * factor * factor)
    layer = pkg.Layer(ctx, pkg.make_desc(pkg.UPSAMPLE_BILINEAR, DT[S], n, h, w, c, factor=factor))
    assert layer.out_shape == (n, h * factor, w * factor, c)
    x0 = rng.normal(0, 1, shape).astype(NP_DTYPE[S])
    g0 = layer.init([torch.from_numpy(x0).cuda()])
    ctx.sync()
    # a weighted sum of up to four sources in fp32 against the oracle's float64: same allowance as a convolution sum
    mag = orc.UpsampleBilinear(factor, "f64")
    assert rel_err(to_np(g0), ref.init(x0), slack=8 * U32 * mag.init(np.abs(x0))) <= TOL[S]
    for t, dens in enumerate([0.1, 1.0, 0.02, 0.0]):
        d = _rand_delta(rng, shape, dens, S)
        want = ref.step(d).poisoned()
        out = layer.step([_upload(d)])
        ctx.sync()
        check_delta(out, want, S, f"bilinear x{factor} frame {t}", slack=8 * U32 * mag.init(np.abs(d.zero_filled())))


@pytest.mark.parametrize("S", ["f32", "f16"])
@pytest.mark.parametrize("shape", [(3, 7, 7, 64), (2, 13, 10, 20), (5, 4, 6, 3), (1, 1, 1, 8), (2, 24, 24, 1280)])
def test_global_average_pooling(S, shape):
    rng = np.random.default_rng(sum(shape))
    n, h, w, c = shape
    ref = orc.GlobalAvgPool(S)
    ctx = pkg.Context(n * h * w)
    layer = pkg.Layer(ctx, pkg.make_desc(pkg.GAVGPOOL, DT[S], n, h, w, c))
    assert layer.out_shape == (n, 1, 1, c)
    x0 = rng.normal(0, 1, shape).astype(NP_DTYPE[S])
    g0 = layer.init([torch.from_numpy(x0).cuda()])
    ctx.sync()
    mag = orc.GlobalAvgPool("f64")
    assert rel_err(to_np(g0), ref.init(x0), slack=8 * U32 * mag.init(np.abs(x0))) <= TOL[S]
    for t, dens in enumerate([0.1, 1.0, 0.0]):
        d = _rand_delta(rng, shape, dens, S)
        if t == 0 and n > 1:
            d.mask[1] = 0                                       # one stream without any update
            d.data[1] = np.nan
        want = ref.step(d).poisoned()
        out = layer.step([_upload(d)])
        ctx.sync()
        check_delta(out, want, S, f"global average pool frame {t}",
                    slack=8 * U32 * mag.init(np.abs(d.zero_filled().astype(np.float64))))


@pytest.mark.parametrize("S", ["f32", "f16"])
@pytest.mark.parametrize("ca,cb", [(32, 64), (16, 3), (5, 7)])
def test_concat(S, ca, cb):
    """Channel concatenation: values are copies (bit-exact); an unflagged stream contributes zeros."""
    rng = np.random.default_rng(ca * 100 + cb)
    n, h, w = 2, 23, 19
    ref = orc.Concat(S)
    ctx = pkg.Context(n * h * w)
    layer = pkg.Layer(ctx, pkg.make_desc(pkg.CONCAT, DT[S], n, h, w, ca, cout=ca + cb, n_in=2))
    assert layer.out_shape == (n, h, w, ca + cb)
    a0 = rng.normal(0, 1, (n, h, w, ca)).astype(NP_DTYPE[S])
    b0 = rng.normal(0, 1, (n, h, w, cb)).astype(NP_DTYPE[S])
    g0 = layer.init([torch.from_numpy(a0).cuda(), torch.from_numpy(b0).cuda()])
    ctx.sync()
    assert np.array_equal(to_np(g0), ref.init(a0, b0))
    for t, (da_, db_) in enumerate([(0.2, 0.1), (1.0, 0.0), (0.0, 0.3), (0.0, 0.0)]):
        da = _rand_delta(rng, (n, h, w, ca), da_, S)
        db = _rand_delta(rng, (n, h, w, cb), db_, S)
        want = ref.step(da, db).poisoned()
        out = layer.step([_upload(da), _upload(db)])
        ctx.sync()
        check_delta(out, want, S, f"concat frame {t}", exact_values=True)


@pytest.mark.parametrize("S", ["f32", "f16"])
def test_accumulate(S):
    rng = np.random.default_rng(8)
    shape = (2, 21, 19, 256)
    n, h, w, c = shape
    ref = orc.Accumulate(S)
    ctx = pkg.Context(n * h * w)
    layer = pkg.Layer(ctx, pkg.make_desc(pkg.ACCUM, DT[S], n, h, w, c))
    y0 = rng.normal(0, 1, shape).astype(NP_DTYPE[S])
    ref.init(y0)
    layer.init([torch.from_numpy(y0).cuda()])
    for t, dens in enumerate([0.1, 0.7, 0.0]):
        d = _rand_delta(rng, shape, dens, S)
        want = ref.step(d)
        out = layer.step([_upload(d)])
        ctx.sync()
        assert np.array_equal(to_np(out.data), want)


# ---- error paths through the ABI ------------------------------------------------------------------
def test_error_paths():
    ctx = pkg.Context(16 * 16)
    layer = pkg.Layer(ctx, pkg.make_desc(pkg.ACT, pkg.F32, 1, 16, 16, 8, act=pkg.ACT_RELU, eps=0.1))
    d = _upload(ODelta(np.zeros((1, 16, 16, 8), np.float32), np.zeros((1, 16, 16), np.uint8)))
    with pytest.raises(pkg.DcnnError) as e:
        layer.step([d])                                   # step before the first frame
    assert e.value.status == 4
    layer.init([torch.zeros((1, 16, 16, 8), device="cuda")])
    bad = _upload(ODelta(np.zeros((1, 8, 16, 8), np.float32), np.zeros((1, 8, 16), np.uint8)))
    with pytest.raises(pkg.DcnnError) as e:
        layer.step([bad])
    assert e.value.status == 2
    half = _upload(ODelta(np.zeros((1, 16, 16, 8), np.float16), np.zeros((1, 16, 16), np.uint8)))
    with pytest.raises(pkg.DcnnError) as e:
        layer.step([half])
    assert e.value.status == 3
    layer.reset()
    with pytest.raises(pkg.DcnnError):
        layer.step([d])
    small = pkg.Context(64)                               # workspace too small for this layer
    l2 = pkg.Layer(small, pkg.make_desc(pkg.ACT, pkg.F32, 1, 64, 64, 8, act=pkg.ACT_RELU, eps=0.1, n_in=2))
    l2.init([torch.zeros((1, 64, 64, 8), device="cuda")] * 2)
    big = _upload(ODelta(np.zeros((1, 64, 64, 8), np.float32), np.zeros((1, 64, 64), np.uint8)))
    with pytest.raises(pkg.DcnnError) as e:
        l2.step([big, big])
    assert e.value.status == 5
    with pytest.raises(pkg.DcnnError) as e:               # a fused activation needs the whole pixel in one LDS tile
        pkg.Layer(ctx, pkg.make_desc(pkg.CONV, pkg.F16, 1, 16, 16, 64, k=1, stride=1, pad=0, cout=2048,
                                     act=pkg.ACT_RELU, eps=0.1),
                  torch.zeros((1, 1, 64, 2048), dtype=torch.float16, device="cuda"))
    assert e.value.status == 7

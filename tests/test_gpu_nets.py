"""GPU parity of whole networks run free (no teacher forcing) through dcnn_net_*.

The library's convolution sums differ from the oracle's in rounding order, so a pixel whose
max |dy| lands within rounding of the threshold may be decided differently ("threshold tie");
from then on the two delta streams legitimately differ while both keep tracking dense
inference.  The checks are therefore:
  * until the first tie: every mask identical, every index list the oracle's, the dense
    output within the value tolerance;
  * a mask difference is only accepted at pixels whose oracle max-norm is within the value
    tolerance of the threshold;
  * always: the dense output stays as close to plain dense inference as the oracle's does
    (truncation error does not accumulate), and with negative thresholds it equals it.
"""
import numpy as np
import pytest
import torch

import paper_2203_03996_amd as pkg
import workloads as wl
from oracle import deltacnn_oracle as orc
from oracle.deltacnn_oracle import Delta as ODelta
from tests.helpers import NP_DTYPE, TOL, rel_err, to_np

pytestmark = pytest.mark.gpu


def _run_net(spec, seed, n_streams, flags=3, frames=None, check_dense=True):
    S = spec["dtype"]
    wts = wl.make_weights(spec, seed)
    vid = wl.make_batch(spec["video"], seed, n_streams)
    if frames:
        vid = vid[:frames]
    oracle = orc.OracleNet(spec, wts, S)
    # dense reference uses the weights as stored (rounded to S), like both implementations
    wts_s = {i: (w.astype(NP_DTYPE[S]).astype(np.float64), b.astype(NP_DTYPE[S]).astype(np.float64))
             for i, (w, b) in wts.items()}
    shapes = wl.node_shapes(spec)
    max_px = n_streams * max(h * w for h, w, _ in shapes)
    ctx = pkg.Context(max_px)
    net = pkg.Net(ctx, spec, wts, n_streams, flags)
    oh, ow, oc = shapes[-1]
    out = torch.empty((n_streams, oh, ow, oc), dtype=torch.float16 if S == "f16" else torch.float32, device="cuda")
    eps_of = {i: nd["eps"] for i, nd in enumerate(spec["nodes"]) if nd["kind"] in ("act", "deltagen")}
    # Free-running, every stored intermediate is rounded independently by the two implementations
    # (fp32 vs float64 convolution sums), and these differences random-walk through the layers: the
    # single-operation tolerance is widened with the square root of the depth (1x up to 4 convolutions).
    n_conv = sum(1 for nd in spec["nodes"] if nd["kind"] == "conv")
    tol = TOL[S] * max(1.0, (n_conv ** 0.5) / 2.0)
    diverged = False
    ties = 0
    report = []
    for t in range(vid.shape[0]):
        fr = vid[t].astype(NP_DTYPE[S])
        frame = torch.from_numpy(fr).cuda()
        (net.init if t == 0 else net.step)(frame, out)
        ctx.sync()
        ref = oracle.frame(fr)
        got = to_np(out)
        assert not np.isnan(got.astype(np.float64)).any(), f"frame {t}: NaN in the dense output"
        if t > 0:
            for li in range(net.num_layers):
                nid, view, _ = net.layer_output(li)
                o = oracle.outs[nid]
                if not isinstance(o, ODelta) or view.mask is None:
                    continue
                gm = to_np(view.mask)
                diff = gm != o.mask
                if diff.any() and not diverged:
                    # the first difference of the run must sit on a threshold tie of this very layer
                    ly = oracle.layers[nid]
                    assert getattr(ly, "last_u", None) is not None, f"frame {t} node {nid}: mask differs"
                    eps = eps_of[nid]
                    near = np.abs(np.nan_to_num(ly.last_u, nan=np.inf) - eps) <= tol * abs(eps)
                    assert np.all(near[diff]), f"frame {t} node {nid}: mask differs away from a threshold tie"
                    ties += int(diff.sum())
                    diverged = True
                if not diverged:
                    if view.count is not None and (flags & 2):
                        cnt = int(to_np(view.count)[0])
                        assert cnt == o.count, f"frame {t} node {nid}: count {cnt} vs {o.count}"
                        assert np.array_equal(to_np(view.idx)[:cnt], o.idx), f"frame {t} node {nid}: index list"
                    # free-running, the delta streams themselves are small differences of rounded
                    # accumulated values; what must agree is the accumulated input of every
                    # non-linear layer, x^A + x^T (deltas are compared teacher-forced in test_gpu_layers)
                    ly = oracle.layers[nid]
                    xa, xt = net.layer_state(li, 0), net.layer_state(li, 1)
                    if xa is not None and getattr(ly, "xT", None) is not None:
                        # (a layer without a buffer of truncated values has x^T = 0 on both sides)
                        got_acc = to_np(xa).astype(np.float64) + (to_np(xt).astype(np.float64) if xt is not None else 0.0)
                        ref_acc = ly.xA.astype(np.float64).reshape(-1) + ly.xT.astype(np.float64).reshape(-1)
                        e = rel_err(got_acc, ref_acc, floor=0.1)
                        assert e <= tol, f"frame {t} node {nid}: accumulated input off by {e:.2e}"
                else:
                    assert diff.mean() < 0.02, f"frame {t} node {nid}: masks drifted apart ({diff.mean():.3f})"
        if not diverged:
            e = rel_err(got, ref)
            assert e <= tol, f"frame {t}: dense output off by {e:.2e}"
        if check_dense:
            dense = orc.dense_reference(spec, wts_s, fr.astype(np.float64))
            scale = np.abs(dense).max()
            err_o = np.abs(ref.astype(np.float64) - dense).max() / scale
            err_g = np.abs(got.astype(np.float64) - dense).max() / scale
            report.append((err_o, err_g))
            assert err_g <= 2.0 * err_o + 4 * tol, f"frame {t}: library drifts from dense inference ({err_g:.2e} vs oracle {err_o:.2e})"
    return {"ties": ties, "diverged": diverged, "errs": report, "net": net, "ctx": ctx, "oracle": oracle}


def test_config1_single_conv_fp32_full_size():
    """BASELINE config 1: 3x3 conv + ReLU, 32 channels, 64x64, fp32, 4 frames, eps 0.05."""
    r = _run_net(wl.single_conv_relu(), wl.CONFIG_SEEDS[1], 1)
    assert r["ties"] == 0


@pytest.mark.parametrize("flags", [1, 3, 2])
def test_config2_bottleneck_fp16_full_size(flags):
    """BASELINE config 2 at its real size (128x128, 64->64->256, fp16), 6 of its 16 frames."""
    r = _run_net(wl.bottleneck_block(eps=0.1), wl.CONFIG_SEEDS[2], 1, flags=flags, frames=6)
    assert r["ties"] <= 20


def test_config2_batched_streams():
    _run_net(wl.bottleneck_block(eps=0.1, h=64, w=48), wl.CONFIG_SEEDS[2], 3, frames=5)


def test_input_mask_dilation_in_a_network():
    """High input threshold with a dilated input mask (Section 4)."""
    _run_net(wl.bottleneck_block(eps=0.1, eps0=0.3, h=64, w=48, dilate_r=3), wl.CONFIG_SEEDS[2], 2, frames=5)


@pytest.mark.parametrize("S", ["f32", "f16"])
@pytest.mark.parametrize("flags", [3, 2])
def test_tiny_mixed_net_all_layer_kinds(S, flags):
    _run_net(wl.tiny_mixed_net(eps=0.05, dtype=S), 11, 2, flags=flags)


@pytest.mark.parametrize("S", ["f32", "f16"])
@pytest.mark.parametrize("flags", [3, 2])
def test_tiny_concat_net(S, flags):
    """Branches of different widths joined by channel concatenation, one of them the raw input delta."""
    _run_net(wl.tiny_concat_net(eps=0.05, dtype=S), 13, 2, flags=flags)


@pytest.mark.parametrize("S", ["f32", "f16"])
def test_tiny_pool_net(S):
    """Bilinear upsampling of a coarser branch and a global-average-pooled, fully connected head."""
    _run_net(wl.tiny_pool_net(eps=0.05, dtype=S), 17, 2)


@pytest.mark.parametrize("spec_fn", [lambda: wl.single_conv_relu(eps=-1.0), lambda: wl.bottleneck_block(eps=-1.0, h=32, w=32, frames=4),
                                     lambda: wl.tiny_mixed_net(eps=-1.0, dtype="f16"), lambda: wl.tiny_concat_net(eps=-1.0), lambda: wl.tiny_pool_net(eps=-1.0)])
def test_dense_mode_matches_dense_inference(spec_fn):
    """Negative thresholds: every pixel is reprocessed and the output is plain dense inference."""
    spec = spec_fn()
    r = _run_net(spec, 5, 1)
    assert not r["diverged"]
    for err_o, err_g in r["errs"]:
        assert err_g <= 8 * TOL[spec["dtype"]]


def test_identical_frames_and_infinite_threshold_do_nothing():
    spec = wl.bottleneck_block(eps=0.05, h=32, w=32, frames=3)
    wts = wl.make_weights(spec, 2)
    vid = wl.make_batch(spec["video"], 2, 1).astype(np.float16)
    ctx = pkg.Context(32 * 32)
    net = pkg.Net(ctx, spec, wts, 1, 3)
    out = torch.empty((1, 32, 32, 256), dtype=torch.float16, device="cuda")
    f0 = torch.from_numpy(vid[0]).cuda()
    net.init(f0, out)
    ctx.sync()
    o1 = out.clone()
    arena1 = net.arena.clone()
    net.step(f0, out)
    ctx.sync()
    assert torch.equal(out, o1)
    for s in net.stats():
        assert s["pixels_out"] == 0 and s["pixels_work"] == 0
    spec_inf = wl.bottleneck_block(eps=float("inf"), h=32, w=32, frames=3)
    net2 = pkg.Net(ctx, spec_inf, wts, 1, 3)
    net2.init(f0, out)
    net2.step(torch.from_numpy(vid[1]).cuda(), out)
    ctx.sync()
    assert torch.equal(out, o1)
    assert all(s["pixels_out"] == 0 for s in net2.stats())
    del arena1


def test_reset_restarts_from_a_dense_frame():
    spec = wl.single_conv_relu(h=32, w=32)
    wts = wl.make_weights(spec, 3)
    vid = wl.make_batch(spec["video"], 3, 1).astype(np.float32)
    ctx = pkg.Context(32 * 32)
    net = pkg.Net(ctx, spec, wts, 1)
    out = torch.empty((1, 32, 32, 32), device="cuda")
    with pytest.raises(pkg.DcnnError):
        net.step(torch.from_numpy(vid[0]).cuda(), out)
    net.init(torch.from_numpy(vid[0]).cuda(), out)
    net.step(torch.from_numpy(vid[1]).cuda(), out)
    net.reset()
    with pytest.raises(pkg.DcnnError):
        net.step(torch.from_numpy(vid[2]).cuda(), out)
    net.init(torch.from_numpy(vid[3]).cuda(), out)
    ctx.sync()
    fresh = pkg.Net(ctx, spec, wts, 1)
    out2 = torch.empty_like(out)
    fresh.init(torch.from_numpy(vid[3]).cuda(), out2)
    ctx.sync()
    assert torch.equal(out, out2)


def test_run_to_run_determinism():
    spec = wl.bottleneck_block(eps=0.1, h=64, w=64, frames=4)
    wts = wl.make_weights(spec, 9)
    vid = wl.make_batch(spec["video"], 9, 2).astype(np.float16)
    outs = []
    for _ in range(2):
        ctx = pkg.Context(2 * 64 * 64)
        net = pkg.Net(ctx, spec, wts, 2)
        out = torch.empty((2, 64, 64, 256), dtype=torch.float16, device="cuda")
        for t in range(4):
            (net.init if t == 0 else net.step)(torch.from_numpy(vid[t]).cuda(), out)
        ctx.sync()
        outs.append(out.clone())
    assert torch.equal(outs[0], outs[1])


def test_config2_bench_configuration_sampled_streams():
    """The launch configuration bench.py times: 64 independent streams of BASELINE config 2 at full
    size through the fused plan.  Streams do not interact, so sampled streams must match a
    single-stream oracle run fed that stream's frames; masks, states and the dense output of every
    stream must also equal what the same library computes for that stream alone."""
    spec = wl.bottleneck_block(eps=0.0443)
    S, seed, B, T = spec["dtype"], wl.CONFIG_SEEDS[2], 64, 4
    wts = wl.make_weights(spec, seed)
    vid = wl.make_batch(spec["video"], seed, B)[:T].astype(NP_DTYPE[S])        # [T, B, H, W, C]
    ctx = pkg.Context(B * 128 * 128)
    net = pkg.Net(ctx, spec, wts, B, 1)
    out = torch.empty((B, 128, 128, 256), dtype=torch.float16, device="cuda")
    sampled = [0, 37, 63]
    oracles = {b: orc.OracleNet(spec, wts, S) for b in sampled}
    solo_ctx = pkg.Context(128 * 128)
    solo = {b: pkg.Net(solo_ctx, spec, wts, 1, 1) for b in (5, 63)}
    solo_out = torch.empty((1, 128, 128, 256), dtype=torch.float16, device="cuda")
    tol = TOL[S] * 1.0
    for t in range(T):
        frame = torch.from_numpy(vid[t]).cuda()
        (net.init if t == 0 else net.step)(frame, out)
        ctx.sync()
        got = to_np(out)
        assert not np.isnan(got.astype(np.float64)).any()
        for b in sampled:
            ref = oracles[b].frame(vid[t, b:b + 1])
            assert rel_err(got[b:b + 1], ref) <= tol, f"frame {t} stream {b}: dense output vs oracle"
        for b, sn in solo.items():
            (sn.init if t == 0 else sn.step)(frame[b:b + 1].contiguous(), solo_out)
            solo_ctx.sync()
            assert np.array_equal(to_np(solo_out)[0], got[b]), f"frame {t} stream {b}: batched run differs from the stream alone"
        if t > 0:
            st = net.stats()
            total = sum(s["pixels_work"] for s in st)
            assert total > 0 and all(s["pixels_out"] <= s["pixels_work"] <= s["pixels_total"] for s in st if s["kind"] != pkg.DELTAGEN)


def test_tensors_beyond_2gib_take_the_plain_kernels():
    """Buffer addressing limits the wave-specialised convolution to tensors below 2 GiB; a batch whose
    256-channel maps exceed that must fall back (per layer) and still give, for every sampled stream,
    what the stream gives alone."""
    spec = wl.bottleneck_block(eps=0.0443)
    S, seed, B, T = spec["dtype"], wl.CONFIG_SEEDS[2], 260, 3          # 260 * 128*128*256 * 2 B = 2.18 GB
    wts = wl.make_weights(spec, seed)
    base = wl.make_batch(spec["video"], seed, 4)[:T].astype(NP_DTYPE[S])    # 4 distinct streams, tiled
    ctx = pkg.Context(B * 128 * 128)
    net = pkg.Net(ctx, spec, wts, B, 1)
    solo_ctx = pkg.Context(128 * 128)
    picks = {0: 0, 129: 1, 259: 3}                                    # stream index -> which base stream it shows
    solo = {b: pkg.Net(solo_ctx, spec, wts, 1, 1) for b in picks}
    solo_out = torch.empty((1, 128, 128, 256), dtype=torch.float16, device="cuda")
    layout = np.array([picks.get(b, b % 4) for b in range(B)])
    for t in range(T):
        frame = torch.from_numpy(base[t]).cuda()[torch.from_numpy(layout).cuda()].contiguous()
        (net.init if t == 0 else net.step)(frame)
        ctx.sync()
        view = net.output()
        for b, src in picks.items():
            sn = solo[b]
            (sn.init if t == 0 else sn.step)(frame[b:b + 1].contiguous(), solo_out)
            solo_ctx.sync()
            # same numbers up to the rounding of the output layer: the stand-alone one (large batch) adds rounded
            # deltas to O, the folded one (single stream) writes f(x^A); one fp16 ulp per update at most
            e = rel_err(to_np(view.data[b]), to_np(solo_out[0]))
            assert e <= 3e-3, f"frame {t} stream {b}: differs from the stream alone ({e:.2e})"


def test_density_budget_tuner_matches_the_oracle():
    """Thresholds found front to back on a density budget: the library's tuner (every frame through the HIP
    kernels) and the oracle's arrive at the same threshold for every layer, and the densities they were
    decided on are equal."""
    from paper_2203_03996_amd import tuner
    spec = wl.tiny_mixed_net(eps=0.05, frames=5)
    seed, n_streams = 3, 2
    wts = wl.make_weights(spec, seed)
    vid = wl.make_batch(spec["video"], seed, n_streams).astype(np.float32)
    target, lo, hi, iters = 0.3, 1e-4, 16.0, 8
    onet = orc.OracleNet(spec, wts, "f32")
    want = orc.tune_thresholds(onet, vid, target, lo, hi, iters)

    shapes = wl.node_shapes(spec)
    ctx = pkg.Context(n_streams * max(h * w for h, w, _ in shapes))
    net = pkg.Net(ctx, spec, wts, n_streams, 3)
    frames = [torch.from_numpy(vid[t]).cuda() for t in range(vid.shape[0])]
    # stats need one step to exist
    net.init(frames[0]); net.step(frames[1])
    layers = tuner.tunable_layers(net)
    assert [net.layer_node(i) for i in layers] == sorted(want)
    got = tuner.tune_thresholds(net, frames, target, lo, hi, iters)
    for i in layers:
        assert got[i] == pytest.approx(want[net.layer_node(i)], rel=1e-12), f"layer {i} (node {net.layer_node(i)})"
    # with the tuned thresholds both sides flag the same number of pixels in every tuned layer
    net.reset(); onet.reset()
    net.init(frames[0]); onet.frame(vid[0])
    for t in range(1, vid.shape[0]):
        net.step(frames[t]); onet.frame(vid[t])
        st = net.stats()
        for i in layers:
            assert st[i]["pixels_out"] == int(onet.outs[net.layer_node(i)].mask.sum()), f"frame {t} layer {i}"
    with pytest.raises(pkg.DcnnError):
        net.set_eps(1, float("nan"))


@pytest.mark.parametrize("spec_fn", [lambda: wl.bottleneck_block(eps=0.08, h=48, w=40, frames=6, no_xT=True),
                                     lambda: wl.tiny_mixed_net(eps=0.05, dtype="f32", no_xT=True),
                                     lambda: wl.tiny_mixed_net(eps=0.05, dtype="f16", no_xT=True)])
def test_networks_without_truncated_value_buffers(spec_fn):
    """Memory-lean variant (Section 6): activations keep no x^T; a truncated update is dropped.  Same
    frame-by-frame comparison as every other network, against the oracle run in the same mode; the layers
    report no buffer 1 and need less state memory."""
    spec = spec_fn()
    r = _run_net(spec, 23, 2, check_dense=False)
    net = r["net"]
    acts = [li for li in range(net.num_layers) if net.stats()[li]["act"] != pkg.ACT_NONE]
    assert acts and all(net.layer_state(li, 1) is None and net.layer_state(li, 0) is not None for li in acts)
    with_xt = pkg.Net(r["ctx"], dict(spec, nodes=[{k: v for k, v in nd.items() if k != "no_xT"} for nd in spec["nodes"]]),
                      wl.make_weights(spec, 23), 2, 3)
    assert net.arena.numel() < with_xt.arena.numel()


@pytest.mark.parametrize("eps", [0.05, 0.3])
def test_free_running_without_touching_the_state(eps):
    """The library keeps, per pixel, whether a layer's x^T row is all zero (such rows are not read).  Reading
    the state through the ABI makes it rebuild those flags, so this run never does until the end: dense
    outputs are compared every frame, the accumulated buffers after the last one."""
    spec = wl.bottleneck_block(eps=eps, h=40, w=48, frames=8)
    seed, n_streams = 29, 2
    wts = wl.make_weights(spec, seed)
    vid = wl.make_batch(spec["video"], seed, n_streams)
    oracle = orc.OracleNet(spec, wts, "f16")
    shapes = wl.node_shapes(spec)
    ctx = pkg.Context(n_streams * max(h * w for h, w, _ in shapes))
    net = pkg.Net(ctx, spec, wts, n_streams, 1)
    oh, ow, oc = shapes[-1]
    out = torch.empty((n_streams, oh, ow, oc), dtype=torch.float16, device="cuda")
    tol = TOL["f16"]
    for t in range(vid.shape[0]):
        fr = vid[t].astype(np.float16)
        (net.init if t == 0 else net.step)(torch.from_numpy(fr).cuda(), out)
        ctx.sync()
        ref = oracle.frame(fr)
        assert rel_err(to_np(out), ref) <= 2 * tol, f"frame {t}"
    checked = 0
    for li in range(net.num_layers):
        nid = net.layer_node(li)
        ly = oracle.layers[nid]
        xa, xt = net.layer_state(li, 0), net.layer_state(li, 1)
        if xa is None or xt is None or getattr(ly, "xT", None) is None:
            continue
        got = to_np(xa).astype(np.float64) + to_np(xt).astype(np.float64)
        want = ly.xA.astype(np.float64).reshape(-1) + ly.xT.astype(np.float64).reshape(-1)
        assert rel_err(got, want, floor=0.1) <= 2 * tol, f"layer {li}"
        checked += 1
    assert checked >= 3
    # one more frame after the state was handed out (flags rebuilt from x^T)
    fr = vid[-2].astype(np.float16)
    net.step(torch.from_numpy(fr).cuda(), out)
    ctx.sync()
    assert rel_err(to_np(out), oracle.frame(fr)) <= 2 * tol


def test_frames_of_the_wrong_shape_are_refused_before_any_launch():
    """The ABI takes bare pointers; the binding refuses a frame whose shape or type does not match the network."""
    spec = wl.single_conv_relu(h=16, w=16, c=8, frames=2)
    wts = wl.make_weights(spec, 1)
    ctx = pkg.Context(2 * 16 * 16)
    net = pkg.Net(ctx, spec, wts, 2, 1)
    good = torch.zeros((2, 16, 16, 8), dtype=torch.float32, device="cuda")
    net.init(good)
    for bad in (good[:1], good.half(), good.permute(0, 2, 1, 3), good.cpu()):
        with pytest.raises(ValueError):
            net.step(bad)
    net.step(good)
    ctx.sync()

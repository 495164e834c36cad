"""GPU parity of whole networks run free (no teacher forcing) through dcnn_net_*.

The library's convolution sums differ from the oracle's in rounding order, so a pixel whose
max |dy| lands within rounding of the threshold may be decided differently ("threshold tie").
From then on the two sides legitimately differ, but only inside the tie's dependence cone: the
pixels of later layers (and later frames) whose windows reach a tied pixel.  The checks are:
  * outside the cone, every frame: every mask identical, every index list the ordered
    compaction (and the oracle's list when the whole mask agrees), every accumulated input
    x^A + x^T, every pooling buffer, the stored input frame and the dense output equal to the
    oracle's within the value tolerance;
  * a mask difference outside the cone is only accepted at a layer with a threshold, at pixels
    whose oracle max-norm is within rounding of the threshold; these ties are counted per frame
    and reported, and their cone is excluded from then on;
  * everywhere, cone included: the dense output stays as close to plain dense inference as the
    oracle's does (truncation error does not accumulate), and with negative thresholds it equals it.
"""
import numpy as np
import pytest
import torch

import paper_2203_03996_amd as pkg
import workloads as wl
from oracle import deltacnn_oracle as orc
from oracle.deltacnn_oracle import Delta as ODelta
from tests.helpers import NP_DTYPE, TOL, U32, rel_err, sum_slack, to_np, ulp, worst

pytestmark = pytest.mark.gpu

# Free-running, both sides round every stored intermediate on their own (fp32 against float64
# convolution sums): a layer's accumulated input differs between two correct implementations by a few
# units in the last place of the tensor's largest magnitude -- not of the element: a small element is a
# sum of large rounded ones -- and these differences random-walk through the layers.  The free-running
# comparison with the independent oracle run therefore allows, per tensor, QUANTA * sqrt(depth) units in
# the last place of its scale on top of the relative tolerance (depth = rounding stages on the longest
# path from the input; measured need on the five configurations: below 2).  The TIGHT per-layer gate at
# network scale is the replay below, which has no such term.
QUANTA = 4.0


def _spread(nd, taints):
    """Which output pixels of node `nd` depend on the given pixels of its inputs (structural)."""
    k = nd["kind"]
    ins = [taints[j] for j in nd["in"]]
    if k in ("conv", "maxpool"):
        return orc.window_mask(ins[0], nd["k"], nd["stride"], nd["pad"]).astype(bool)
    if k in ("add", "concat"):
        return ins[0] | ins[1]
    if k == "upsample":
        return np.repeat(np.repeat(ins[0], nd["factor"], axis=1), nd["factor"], axis=2)
    if k == "upsample_bilinear":
        # a dependence is a tap with weight: the oracle's own mask rule gives it
        n, h, w = ins[0].shape
        return orc.UpsampleBilinear(nd["factor"], "f64")._apply(np.zeros((n, h, w, 1)), ins[0].astype(np.uint8))[1].astype(bool)
    if k == "gavgpool":
        return ins[0].reshape(ins[0].shape[0], -1).any(axis=1).reshape(-1, 1, 1)
    return ins[0]                                                    # act, accum: pixel-local


_ROUNDS = ("conv", "add", "upsample_bilinear", "gavgpool")           # kinds whose result each side rounds on its own


def _depths(nodes):
    d = []
    for nd in nodes:
        d.append(max([d[j] for j in nd["in"]], default=0) + (1 if nd["kind"] in _ROUNDS else 0))
    return d


def free_running_slack(spec, ref, S):
    """Absolute allowance of a network's dense output in a free-running comparison (see QUANTA)."""
    return QUANTA * max(1.0, _depths(spec["nodes"])[-1]) ** 0.5 * float(ulp(float(np.abs(ref).max(initial=0)), S))


# ---- replay: every planned layer of the running network against the oracle's definition of that layer ----
def _snapshot(net):
    """Host copies of every layer's buffers (x^A / stored frame / pooling buffer / O, x^T, folded O)."""
    snap = {}
    for li in range(net.num_layers):
        snap[li] = tuple(None if (b := net.layer_state(li, which)) is None else to_np(b).copy() for which in (0, 1, 2))
    return snap


def _replay_layers(net, spec, oracle, layer_of, pre, S, t):
    """Teacher forcing by the library's own stream: for every planned layer, the oracle's layers of the nodes
    it covers are run on the inputs the library's producer layers left in memory this frame and on the
    library's buffers from before the step; the library's output and buffers after the step must equal the
    result to single-operation tolerance.  No compounding over depth or frames, no dependence cone: a
    threshold tie is a property of one pixel of one layer in one frame.  Returns the ties it saw."""
    nodes = spec["nodes"]
    tol = TOL[S]
    st = NP_DTYPE[S]
    stats = net.stats()
    cache = {}

    def produced(j):                                               # output of a planned layer, as the library left it
        if j not in cache:
            _, view, _ = net.layer_output(layer_of[j])
            cache[j] = ODelta(to_np(view.data).copy(), to_np(view.mask)).poisoned()
        return cache[j]

    ties = 0
    for li in range(net.num_layers):
        nid = net.layer_node(li)
        group = []

        def walk(j):
            for a in nodes[j]["in"]:
                if a not in layer_of and a not in group:
                    walk(a)
            group.append(j)
        walk(nid)
        folded = bool(stats[li]["fuse_accum"])
        vals, slk = {}, {}

        def val(j):
            return vals[j] if j in vals else produced(j)

        def slack(j):
            return slk.get(j, 0.0)

        xa0, xt0, o0 = pre[li]
        what = f"frame {t} layer {li} (nodes {group})"
        act_ly = None
        for j in group:
            nd = nodes[j]
            k = nd["kind"]
            ly = oracle.layers[j]
            if k == "deltagen":
                continue
            ins = [val(a) for a in nd["in"]]
            if k == "conv":
                vals[j] = ly.step(ins[0]).poisoned()                # stateless: the oracle's own object serves
                slk[j] = sum_slack(ly, ins[0].zero_filled()) + ulp(vals[j].data, S)
            elif k == "add":
                vals[j] = ly.step(*ins).poisoned()
                sa, sb = slack(nd["in"][0]), slack(nd["in"][1])
                # the sum of two stored streams is one exact fp32 addition and one rounding on both sides
                slk[j] = (sa + sb + ulp(vals[j].data, S)) if (np.any(sa) or np.any(sb)) else 0.0
            elif k == "act":
                act_ly = orc.ActTrunc(ly.f, ly.eps, S, ly.use_xT, ly.carry)
                act_ly.xA = xa0.reshape(ins[0].data.shape).copy()
                act_ly.xT = np.zeros_like(act_ly.xA) if xt0 is None else xt0.reshape(ins[0].data.shape).copy()
                vals[j] = act_ly.step(ins[0]).poisoned()
                slk[j] = slack(nd["in"][0])
            elif k == "maxpool":
                sh = orc.MaxPool(ly.k, ly.stride, ly.pad, S)
                sh.xA = xa0.reshape(ins[0].data.shape).copy()
                vals[j] = sh.step(ins[0]).poisoned()
                act_ly = sh
            elif k == "accum":
                sh = orc.Accumulate(S)
                sh.O = xa0.reshape(ins[0].data.shape).copy()
                vals[j] = sh.step(ins[0])
            elif k in ("upsample", "concat"):
                vals[j] = ly.step(*ins).poisoned()
            elif k == "upsample_bilinear":
                vals[j] = ly.step(ins[0]).poisoned()
                slk[j] = 8 * U32 * orc.UpsampleBilinear(nd["factor"], "f64").init(np.abs(ins[0].zero_filled().astype(np.float64)))
            elif k == "gavgpool":
                vals[j] = ly.step(ins[0]).poisoned()
                slk[j] = 8 * U32 * orc.GlobalAvgPool("f64").init(np.abs(ins[0].zero_filled().astype(np.float64)))
            else:
                raise ValueError(k)
        kind = nodes[nid]["kind"]
        _, view, _ = net.layer_output(li)
        xa1, xt1, o1 = (None if (b := net.layer_state(li, w)) is None else to_np(b) for w in (0, 1, 2))
        if kind == "deltagen":
            # the input layer is replayed from the frame itself by the free-running comparison (bit-exact there)
            continue
        if kind == "accum":
            assert np.array_equal(xa1.reshape(vals[nid].shape), vals[nid]), f"{what}: accumulated output"
            continue
        want = vals[nid]
        sl = np.broadcast_to(np.asarray(slack(nid), np.float64), want.data.shape)
        gm = to_np(view.mask)
        diff = gm != want.mask
        if diff.any():
            assert isinstance(act_ly, orc.ActTrunc), f"{what}: {int(diff.sum())} mask differences in a layer without a threshold"
            gap = np.abs(np.nan_to_num(act_ly.last_u, nan=np.inf) - act_ly.eps)
            room = tol * abs(act_ly.eps) + sl.max(axis=-1)
            assert np.all(gap[diff] <= room[diff]), f"{what}: mask differs away from a threshold tie (gap {gap[diff].max():.3e})"
            ties += int(diff.sum())
        agree = ~diff
        exact = not np.any(sl)
        both = (gm == 1) & (want.mask == 1)
        if not folded:
            g, r = to_np(view.data)[both], want.data[both]
            assert not np.isnan(g.astype(np.float64)).any(), f"{what}: NaN in a flagged output"
            if exact:
                assert np.array_equal(g, r), f"{what}: values differ"
            else:
                e = rel_err(g, r, slack=sl[both])
                assert e <= tol, f"{what}: output off by {e:.2e}; {worst(g, r, slack=sl[both])}"
        if isinstance(act_ly, (orc.ActTrunc, orc.MaxPool)):
            shape = act_ly.xA.shape
            sl_state = sl if isinstance(act_ly, orc.ActTrunc) else 0.0 * act_ly.xA.astype(np.float64)
            ag = agree if isinstance(act_ly, orc.ActTrunc) else np.ones(shape[:3], bool)
            e = rel_err(xa1.reshape(shape)[ag], act_ly.xA[ag], slack=sl_state[ag])
            assert e <= (0.0 if exact else tol), f"{what}: x^A off by {e:.2e}; {worst(xa1.reshape(shape)[ag], act_ly.xA[ag], slack=sl_state[ag])}"
            if xt1 is not None and getattr(act_ly, "carry", False) and not exact:
                # a kept residue s - round(s) flips with the last bit of s; what both sides must agree on is
                # x^A + x^T, i.e. s itself (and x^A, above) -- to within what s may differ by, not a relative term
                got_s = xa1.reshape(shape).astype(np.float64) + xt1.reshape(shape).astype(np.float64)
                ref_s = act_ly.xA.astype(np.float64) + act_ly.xT.astype(np.float64)
                over = np.abs(got_s - ref_s)[ag] - (sl_state + 2 * ulp(act_ly.xT, S) + 2 * ulp(ref_s, "f32"))[ag]
                assert over.max(initial=0) <= 0, f"{what}: x^A + x^T off by {over.max():.2e} beyond the intermediates' rounding"
            elif xt1 is not None:
                e = rel_err(xt1.reshape(shape)[ag], act_ly.xT[ag], slack=sl_state[ag])
                assert e <= (0.0 if exact else tol), f"{what}: x^T off by {e:.2e}; {worst(xt1.reshape(shape)[ag], act_ly.xT[ag], slack=sl_state[ag])}"
        if folded:
            # the folded output layer writes O = f(new x^A) where the oracle's adds the rounded delta onto O
            acc = orc.Accumulate(S)
            acc.O = o0.reshape(want.data.shape).copy()
            o_ref = acc.step(want)
            e = rel_err(o1.reshape(o_ref.shape)[agree], o_ref[agree], slack=(sl + ulp(want.data, S))[agree])
            assert e <= tol, f"{what}: dense output off by {e:.2e}"
    return ties


def _run_net(spec, seed, n_streams, flags=3, frames=None, check_dense=True, replay=True, diag=None):
    S = spec["dtype"]
    wts = wl.make_weights(spec, seed)
    vid = wl.make_batch(spec["video"], seed, n_streams)
    if frames:
        vid = vid[:frames]
    oracle = orc.OracleNet(spec, wts, S)
    # dense reference uses the weights as stored (rounded to S), like both implementations
    wts_s = {i: (w.astype(NP_DTYPE[S]).astype(np.float64), b.astype(NP_DTYPE[S]).astype(np.float64))
             for i, (w, b) in wts.items()}
    nodes = spec["nodes"]
    shapes = wl.node_shapes(spec)
    depth = _depths(nodes)
    max_px = n_streams * max(h * w for h, w, _ in shapes)
    ctx = pkg.Context(max_px)
    net = pkg.Net(ctx, spec, wts, n_streams, flags)
    oh, ow, oc = shapes[-1]
    out = torch.empty((n_streams, oh, ow, oc), dtype=torch.float16 if S == "f16" else torch.float32, device="cuda")
    tol = TOL[S]
    layer_of = {net.layer_node(li): li for li in range(net.num_layers)}
    # cone[i]: pixels of node i's output that a threshold tie has reached so far (persistent: state differs there)
    cone = [np.zeros((n_streams, h, w), bool) for h, w, _ in shapes]
    scale = {}                                                       # running largest magnitude per compared tensor

    sum_unit = [0.0]                                                 # fp32 storage: largest fp32-summation allowance of any convolution so far

    def allowance(key, ref_t, d):
        # rounding unit of a stage: one unit in the last place of the tensor's scale, plus -- it only matters next to
        # fp32's own unit -- what an fp32 sum may differ by from the exact one (sum_slack)
        scale[key] = max(scale.get(key, 0.0), float(np.abs(ref_t).max(initial=0)))
        return QUANTA * max(1.0, d) ** 0.5 * (float(ulp(scale[key], S)) + sum_unit[0])

    ties_per_frame, replay_ties = [], []
    report = []
    for t in range(vid.shape[0]):
        fr = vid[t].astype(NP_DTYPE[S])
        frame = torch.from_numpy(fr).cuda()
        do_replay = t > 0 and (replay is True or (replay and t in replay))
        pre = _snapshot(net) if do_replay else None
        (net.init if t == 0 else net.step)(frame, out)
        ctx.sync()
        ref = oracle.frame(fr)
        got = to_np(out)
        assert not np.isnan(got.astype(np.float64)).any(), f"frame {t}: NaN in the dense output"
        if S == "f32":
            for j, ndj in enumerate(nodes):
                if ndj["kind"] == "conv":
                    xin = oracle.outs[ndj["in"][0]]
                    xin = xin.zero_filled() if isinstance(xin, ODelta) else xin
                    sum_unit[0] = max(sum_unit[0], float(sum_slack(oracle.layers[j], xin, bias=(t == 0)).max(initial=0)))
        ties = 0
        if do_replay:
            replay_ties.append(_replay_layers(net, spec, oracle, layer_of, pre, S, t))
        if t > 0:
            for i, nd in enumerate(nodes):
                if nd["in"]:
                    cone[i] |= _spread(nd, cone)
                li = layer_of.get(i)
                if li is None:
                    continue                                        # fused into a later layer
                _, view, _ = net.layer_output(li)
                o = oracle.outs[i]
                ly = oracle.layers[i]
                clean = ~cone[i]
                if isinstance(o, ODelta) and view.mask is not None:
                    gm = to_np(view.mask)
                    diff = gm != o.mask
                    new = diff & clean
                    if new.any():
                        assert getattr(ly, "last_u", None) is not None, \
                            f"frame {t} node {i} ({nd['kind']}): {int(new.sum())} mask differences outside any tie's cone"
                        # free-running, what decides is the delta path (x^T + dx): its rounding quanta, this frame's
                        # and -- through x^T -- earlier frames'
                        # free-running, the two sides' accumulated inputs s and x^A of this layer agree to within the
                        # tensor's allowance (checked below), so their max-norms of f(s) - f(x^A) to within twice that;
                        # the replay above decides the same pixel at single-operation tolerance
                        al = allowance(i, ly.xA.astype(np.float64) + ly.xT.astype(np.float64), depth[i])
                        room = tol * abs(ly.eps) + 2.0 * al
                        gap = np.abs(np.nan_to_num(ly.last_u, nan=np.inf) - ly.eps)
                        if diag is not None:
                            diag.setdefault("tie_need", []).append(float((gap[new].max() - tol * abs(ly.eps)) / al))
                        else:
                            assert np.all(gap[new] <= room), \
                                f"frame {t} node {i}: mask differs away from a threshold tie (gap {gap[new].max():.3e}, room {room:.3e})"
                        ties += int(new.sum())
                        cone[i] |= new
                        clean = ~cone[i]
                    if view.count is not None and view.idx is not None and (flags & 2):
                        cnt = int(to_np(view.count)[0])
                        assert cnt == int(gm.sum()), f"frame {t} node {i}: count {cnt} vs mask {int(gm.sum())}"
                        assert np.array_equal(to_np(view.idx)[:cnt], np.flatnonzero(gm.reshape(-1))), f"frame {t} node {i}: index list"
                        if not diff.any():
                            assert np.array_equal(to_np(view.idx)[:cnt], o.idx), f"frame {t} node {i}: index list vs oracle"
        # buffers and dense output, outside the cone of every tie so far (frame 0: everywhere)
        for i, nd in enumerate(nodes):
            li = layer_of.get(i)
            if li is None:
                continue
            ly = oracle.layers[i]
            xa, xt = net.layer_state(li, 0), net.layer_state(li, 1)
            if nd["kind"] == "deltagen":
                assert np.array_equal(to_np(xa).reshape(ly.P.shape), ly.P), f"frame {t}: stored input frame"
            elif nd["kind"] == "maxpool":
                cl = ~cone[nd["in"][0]]
                e = rel_err(to_np(xa).reshape(ly.xA.shape)[cl], ly.xA[cl], slack=allowance(i, ly.xA, depth[i]))
                if diag is None:
                    assert e <= tol, f"frame {t} node {i}: pooling buffer off by {e:.2e} outside the ties' cone"
            elif xa is not None and getattr(ly, "xT", None) is not None:
                # x^A + x^T = everything received so far (Eqs. 5, 6); (a layer without x^T keeps zeros)
                clean = ~cone[i]
                ref_acc = ly.xA.astype(np.float64) + ly.xT.astype(np.float64)
                got_acc = (to_np(xa).astype(np.float64) + (to_np(xt).astype(np.float64) if xt is not None else 0.0)).reshape(ref_acc.shape)
                al = allowance(i, ref_acc, depth[i])
                if diag is not None:
                    err = np.abs(got_acc - ref_acc)[clean]
                    den = np.maximum(np.abs(ref_acc), 1e-3 * np.abs(ref_acc).max())[clean]
                    diag.setdefault("acc_need", []).append((t, i, float((err - tol * den).max(initial=0) / (al / QUANTA)), float(clean.mean())))
                else:
                    e = rel_err(got_acc[clean], ref_acc[clean], slack=al)
                    assert e <= tol, f"frame {t} node {i}: accumulated input off by {e:.2e} outside the ties' cone"
        clean = ~cone[-1]
        al = allowance("out", ref, depth[-1])
        if diag is not None:
            err = np.abs(got.astype(np.float64) - ref)[clean]
            den = np.maximum(np.abs(ref), 1e-3 * np.abs(ref).max())[clean]
            diag.setdefault("out_need", []).append((t, float((err - tol * den).max(initial=0) / (al / QUANTA)), float(clean.mean())))
        else:
            e = rel_err(got[clean], ref[clean], slack=al)
            assert e <= tol, f"frame {t}: dense output off by {e:.2e} outside the ties' cone"
        ties_per_frame.append(ties)
        if check_dense:
            dense = orc.dense_reference(spec, wts_s, fr.astype(np.float64))
            sc = np.abs(dense).max()
            err_o = np.abs(ref.astype(np.float64) - dense).max() / sc
            err_g = np.abs(got.astype(np.float64) - dense).max() / sc
            report.append((err_o, err_g))
            assert err_g <= 2.0 * err_o + 4 * tol, f"frame {t}: library drifts from dense inference ({err_g:.2e} vs oracle {err_o:.2e})"
    first = next((t for t, n in enumerate(ties_per_frame) if n), None)
    summary = {"ties": sum(ties_per_frame), "ties_per_frame": ties_per_frame, "first_tie_frame": first,
               "replay_ties": replay_ties, "diverged": first is not None,
               "compared_output_fraction": float((~cone[-1]).mean()),
               "errs": report, "net": net, "ctx": ctx, "oracle": oracle}
    print(f"[{spec['name']} {S} x{n_streams}] frames {vid.shape[0]}: free-running ties per frame {ties_per_frame} "
          f"(first at frame {first}), output pixels still outside every cone {summary['compared_output_fraction']:.3f}; "
          f"replayed frames {len(replay_ties)}, ties in replay {replay_ties}")
    return summary


def test_config1_single_conv_fp32_full_size():
    """BASELINE config 1: 3x3 conv + ReLU, 32 channels, 64x64, fp32, 4 frames, eps 0.05."""
    r = _run_net(wl.single_conv_relu(), wl.CONFIG_SEEDS[1], 1)
    assert r["ties"] == 0 and sum(r["replay_ties"]) == 0


@pytest.mark.parametrize("flags", [1, 3, 2])
def test_config2_bottleneck_fp16_full_size(flags):
    """BASELINE config 2 at its real size (128x128, 64->64->256, fp16), all 16 frames of its clip."""
    r = _run_net(wl.bottleneck_block(eps=0.1), wl.CONFIG_SEEDS[2], 1, flags=flags)
    assert r["ties"] <= 20 and sum(r["replay_ties"]) <= 20, f"ties per frame {r['ties_per_frame']}, in replay {r['replay_ties']}"


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
            e = rel_err(got[b:b + 1], ref, slack=free_running_slack(spec, ref, S))
            assert e <= tol, f"frame {t} stream {b}: dense output vs oracle ({e:.2e})"
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
            # two kernel families (plain / wave-specialised, stand-alone / folded output layer): the same numbers up to
            # where each rounds its intermediates, i.e. two free-running implementations of the same network
            want = to_np(solo_out[0])
            e = rel_err(to_np(view.data[b]), want, slack=free_running_slack(spec, want, S))
            assert e <= TOL[S], f"frame {t} stream {b}: differs from the stream alone ({e:.2e})"


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


@pytest.mark.parametrize("spec_fn", [lambda: wl.bottleneck_block(eps=0.08, h=48, w=40, frames=8, xT_residue=True),
                                     lambda: wl.single_conv_relu(eps=0.05, h=40, w=36, dtype="f16", xT_residue=True),
                                     lambda: wl.tiny_mixed_net(eps=0.05, dtype="f16", xT_residue=True),
                                     lambda: wl.tiny_mixed_net(eps=0.05, dtype="f32", xT_residue=True)])
@pytest.mark.parametrize("flags", [1, 2])
def test_networks_that_keep_the_rounding_residue_in_xT(spec_fn, flags):
    """xT_residue = 1: an update leaves s - round(s) in x^T instead of 0.  Same frame-by-frame comparison and layer
    replay as every other network, against the oracle run in the same mode (fused and unfused plans: the
    wave-specialised convolution, the plain one, the stand-alone activation and the depthwise kernel)."""
    spec = spec_fn()
    r = _run_net(spec, 37, 2, flags=flags)
    net, onet = r["net"], r["oracle"]
    seen = 0
    for li in range(net.num_layers):
        ly = onet.layers[net.layer_node(li)]
        if isinstance(ly, orc.ActTrunc):
            assert ly.carry
            xt = net.layer_state(li, 1)
            if spec["dtype"] == "f16":
                assert bool((xt != 0).any()), f"layer {li}: no residue was kept"
            seen += 1
    assert seen >= 1


def test_long_run_error_with_and_without_truncated_values_and_residue():
    """Supplementary Section 1.4 / Section 3.1 (Eqs. 5, 6) over a few hundred frames: a looped clip with a slow global
    brightness drift (per frame far below the thresholds).  Against float64 dense inference of the same frame:
    with x^T the error stays bounded (truncated changes accumulate and eventually propagate); without x^T the
    drift is lost and the error grows with the number of frames; with the rounding residue kept in x^T the
    error is no larger than with plain x^T (the growth that remains there is the rounding of x^A)."""
    T, frames, B = 8, 320, 2
    mk = lambda **kw: wl.bottleneck_block(eps=0.05, h=32, w=32, frames=T, n_objects=2, **kw)
    specs = {"xT": mk(), "no_xT": mk(no_xT=True), "residue": mk(xT_residue=True)}
    seed = 41
    wts = wl.make_weights(specs["xT"], seed)
    wts_s = {i: (w.astype(np.float16).astype(np.float64), b.astype(np.float16).astype(np.float64)) for i, (w, b) in wts.items()}
    clip = wl.make_batch(specs["xT"]["video"], seed, B).astype(np.float64)              # [T, B, H, W, C]
    order = list(range(1, T)) + list(range(T - 2, -1, -1))
    drift = 0.0008

    def frame(t):
        return (clip[order[t % len(order)] if t else 0] + drift * t).astype(np.float16)

    ctx = pkg.Context(B * 32 * 32)
    nets = {k: pkg.Net(ctx, sp, wts, B, 1) for k, sp in specs.items()}
    out = torch.empty((B, 32, 32, 256), dtype=torch.float16, device="cuda")
    checks = (40, 80, 160, 240, 320)
    err = {k: {} for k in nets}
    for t in range(frames + 1):
        fr = frame(t)
        dense = orc.dense_reference(specs["xT"], wts_s, fr.astype(np.float64)) if t in checks else None
        for k, net in nets.items():
            (net.init if t == 0 else net.step)(torch.from_numpy(fr).cuda(), out)
            if dense is not None:
                ctx.sync()
                err[k][t] = float(np.abs(to_np(out).astype(np.float64) - dense).max() / np.abs(dense).max())
    print("long run, max |out - dense| / max |dense| at frames", checks, {k: [round(v, 4) for v in e.values()] for k, e in err.items()})
    assert max(err["xT"].values()) < 0.05, err["xT"]                       # bounded by the thresholds, not by the run length
    assert err["no_xT"][320] > 3 * err["xT"][320] and err["no_xT"][320] > 1.5 * err["no_xT"][80], err["no_xT"]
    assert err["residue"][320] <= 1.1 * err["xT"][320] + 1e-3, (err["residue"], err["xT"])


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
        assert rel_err(to_np(out), ref, slack=free_running_slack(spec, ref, "f16")) <= tol, f"frame {t}"
    checked = 0
    for li in range(net.num_layers):
        nid = net.layer_node(li)
        ly = oracle.layers[nid]
        xa, xt = net.layer_state(li, 0), net.layer_state(li, 1)
        if xa is None or xt is None or getattr(ly, "xT", None) is None:
            continue
        got = to_np(xa).astype(np.float64) + to_np(xt).astype(np.float64)
        want = ly.xA.astype(np.float64).reshape(-1) + ly.xT.astype(np.float64).reshape(-1)
        depth = _depths(spec["nodes"])[nid]
        assert rel_err(got, want, slack=QUANTA * depth ** 0.5 * float(ulp(float(np.abs(want).max()), "f16"))) <= tol, f"layer {li}"
        checked += 1
    assert checked >= 3
    # one more frame after the state was handed out (flags rebuilt from x^T)
    fr = vid[-2].astype(np.float16)
    net.step(torch.from_numpy(fr).cuda(), out)
    ctx.sync()
    ref = oracle.frame(fr)
    assert rel_err(to_np(out), ref, slack=free_running_slack(spec, ref, "f16")) <= tol


def _small_hrnet():
    spec = wl.hrnet_like(eps=0.05, h=96, w=64, frames=4)
    spec["video"] = wl.VideoSpec(h=96, w=64, c=3, frames=4, n_objects=1, obj_kind="stick", obj_size=40, noise_sigma=0.01)
    return spec


def _small_resnet():
    spec = wl.resnet50_backbone(eps=0.05, h=64, w=64, frames=4, stages=(2, 1, 1, 1))
    spec["video"] = wl.VideoSpec(h=64, w=64, c=3, frames=4, n_objects=2, obj_kind="blob", obj_size=12, noise_sigma=0.02, drift=0.002)
    return spec


@pytest.mark.parametrize("spec_fn", [_small_hrnet, _small_resnet, lambda: wl.tiny_mixed_net(eps=0.05, dtype="f16"),
                                     lambda: wl.tiny_concat_net(eps=0.05), lambda: wl.bottleneck_block(eps=0.08, h=40, w=48, frames=5)])
@pytest.mark.parametrize("flags", [5, 6])
def test_independent_branches_on_streams_of_their_own(spec_fn, flags):
    """Finalize flag bit 2: independent branches run on up to three HIP streams with event dependencies.  The
    same checks against the oracle as every other network (fused and unfused plans), and bit-identical dense
    outputs and buffers to the single-stream run of the same plan -- a missing dependency shows as a difference."""
    spec = spec_fn()
    seed, B = 47, 2
    r = _run_net(spec, seed, B, flags=flags)
    lanes, wts = r["net"], wl.make_weights(spec, seed)
    vid = wl.make_batch(spec["video"], seed, B).astype(NP_DTYPE[spec["dtype"]])
    shapes = wl.node_shapes(spec)
    ctx = pkg.Context(B * max(h * w for h, w, _ in shapes))
    tdt = torch.float16 if spec["dtype"] == "f16" else torch.float32
    outs = []
    for fl in (flags, flags & 3):
        for rep_ in range(2 if fl == flags else 1):               # the lanes twice: run-to-run identical as well
            net = pkg.Net(ctx, spec, wts, B, fl)
            out = torch.empty((B,) + shapes[-1], dtype=tdt, device="cuda")
            per_frame = []
            for t in range(vid.shape[0]):
                (net.init if t == 0 else net.step)(torch.from_numpy(vid[t]).cuda(), out)
                ctx.sync()
                per_frame.append(out.clone())
            states = [net.layer_state(li, w) for li in range(net.num_layers) for w in (0, 1)]
            outs.append((per_frame, [None if s_ is None else s_.clone() for s_ in states]))
    for other in outs[1:]:
        for a, b in zip(outs[0][0], other[0]):
            assert torch.equal(a, b), "dense outputs differ between stream layouts / runs"
        for a, b in zip(outs[0][1], other[1]):
            assert (a is None) == (b is None) and (a is None or torch.equal(a, b)), "buffers differ between stream layouts / runs"
    del lanes


def test_statistics_mode_counts_the_truncated_value_rows_a_step_touches():
    """dcnn_layer_set_counting: convolutions whose sparse steps skip all-zero x^T rows report the rows they read and
    wrote.  With negative thresholds every visited pixel updates, x^T stays zero: nothing is read or written.  With
    thresholds that truncate, rows read are rows that held values, rows written at least those; both are bounded
    by the visited pixels, and the counts equal what the x^T buffers themselves show before and after the step."""
    def run(eps, steps):
        spec = wl.bottleneck_block(eps=eps, eps0=0.05, h=40, w=48, frames=6)
        wts = wl.make_weights(spec, 43)
        vid = wl.make_batch(spec["video"], 43, 2).astype(np.float16)
        ctx = pkg.Context(2 * 40 * 48)
        net = pkg.Net(ctx, spec, wts, 2, 1)
        net.init(torch.from_numpy(vid[0]).cuda())
        rows = []
        for t in range(1, steps + 1):
            if t == steps:
                net.set_counting(True)
                before = {li: to_np(net.layer_state(li, 1)).copy() for li in range(net.num_layers) if net.layer_state(li, 1) is not None}
            net.step(torch.from_numpy(vid[t]).cuda())
        st = net.stats()
        for li, s in enumerate(st):
            if s["xT_bytes_read"] >= 0:
                c = s["c_out"]
                b4 = (before[li].reshape(-1, c) != 0).any(axis=1)
                now = (to_np(net.layer_state(li, 1)).reshape(-1, c) != 0).any(axis=1)
                rows.append((s, int(b4.sum()), int((b4 | now).sum())))
        return rows
    dense = run(-1.0, 3)
    assert len(dense) >= 2
    for s, _, _ in dense:
        assert s["xT_bytes_read"] == 0 and s["xT_bytes_written"] == 0, s
    mixed = run(0.3, 4)
    saw = 0
    for s, held_before, held_any in mixed:
        row = s["c_out"] * 2
        assert 0 <= s["xT_bytes_read"] <= s["xT_bytes_written"] <= s["pixels_work"] * row, s
        # rows that held values and were visited were read; no more than all rows that held values
        assert s["xT_bytes_read"] <= held_before * row and s["xT_bytes_written"] <= held_any * row, (s, held_before, held_any)
        saw += s["xT_bytes_written"] > 0
    assert saw >= 1


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

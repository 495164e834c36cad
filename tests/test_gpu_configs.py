"""GPU parity on the remaining BASELINE configurations (reduced spatial sizes / frame counts so the
CPU oracle finishes in seconds; channel counts, strides, kernel sizes and topology are the real
ones).  These exercise depthwise and strided convolutions, ReLU6, max pooling, weight streaming,
multi-branch adds and nearest upsampling through dcnn_net_*."""
import pytest

import workloads as wl
from tests.test_gpu_nets import _run_net

pytestmark = pytest.mark.gpu


def test_config3_mobilenet_stack():
    """7 inverted-residual blocks, expansion 6, depthwise 3x3, channels 32 -> 160, fp16."""
    spec = wl.mobilenet_stack(eps=0.05, h=96, w=96, frames=4)
    spec["video"] = wl.VideoSpec(h=96, w=96, c=3, frames=4, n_objects=3, obj_kind="rect", obj_size=20, noise_sigma=0.01)
    r = _run_net(spec, wl.CONFIG_SEEDS[3], 1)
    assert r["ties"] <= 40


def test_config4_resnet50_backbone():
    """conv1 7x7 s2, max-pool, bottleneck stages [3,4,6,3] (here [2,2,2,2] to bound oracle time), fp16."""
    spec = wl.resnet50_backbone(eps=0.05, h=64, w=64, frames=3, stages=(2, 2, 2, 2))
    spec["video"] = wl.VideoSpec(h=64, w=64, c=3, frames=3, n_objects=2, obj_kind="blob", obj_size=12, noise_sigma=0.02,
                                 drift=0.002)
    r = _run_net(spec, wl.CONFIG_SEEDS[4], 1)
    assert r["ties"] <= 40


def test_config5_hrnet_like():
    """Four-resolution multi-branch network with cross-branch up/down-sampling adds, fp16."""
    spec = wl.hrnet_like(eps=0.05, h=96, w=64, frames=3)
    spec["video"] = wl.VideoSpec(h=96, w=64, c=3, frames=3, n_objects=1, obj_kind="stick", obj_size=40, noise_sigma=0.01)
    r = _run_net(spec, wl.CONFIG_SEEDS[5], 1)
    assert r["ties"] <= 40

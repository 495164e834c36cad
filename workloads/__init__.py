"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package holds input generators (video frames, weights) and network
topology tables only.  It contains none of the method's arithmetic: no delta
rule, no masks, no convolution.  Both `oracle/` and `paper_2203_03996_amd/`
consume what it produces; neither is imported here.
"""
from .video import VideoSpec, make_video, make_batch          # noqa: F401
from .nets import (                                            # noqa: F401
    single_conv_relu, bottleneck_block, mobilenet_stack, resnet50_backbone,
    hrnet_like, tiny_mixed_net, tiny_concat_net, tiny_pool_net, make_weights, dense_flops, node_shapes, CONFIG_SEEDS,
)

"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package only draws random numbers and describes shapes: static-camera style video
(fixed background, moving textured rectangles, per-frame sensor noise), network layer
lists and He-normal weights.  It contains none of the method's arithmetic (no
thresholding, no index lists, no convolution), so both sides can consume it without
sharing any part of what is being compared.
"""
from .video import SyntheticVideo, MovingObject
from .networks import (LayerSpec, conv, pool, single_layer_net, scene_labeling_net, strided_net,
                       vgg10_net, make_weights, out_shape, dense_flops)
from .configs import Config, get_config, SEED_BASE

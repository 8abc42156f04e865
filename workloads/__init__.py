"""Seeded synthetic inputs and layer lists for the benchmark workloads.

This package holds *data descriptions only*: layer lists (plain dicts) and a
counter-based random generator.  It contains none of the method's arithmetic and
is the only module imported by both the CPU oracle's tests and the GPU binding's
tests, so that both sides see identical inputs.
"""
from .rng import normal, uniform, integers, round_to_bf16          # noqa: F401
from .configs import (lenet, vgg16_cifar, resnet18_cifar, r50_conv4x, vgg16_224,   # noqa: F401
                      tiny_lenet, tiny_resnet, tiny_vgg, tiny_linear, tiny_fc, tiny_wide, tiny_deep_pool, resnet34_cifar, resattnet18_3d, tiny_conv3d, tiny_conv3d_mfma, CONFIGS, EXTRA_CONFIGS, out_shape, out_dhw, in_shape,
                      param_shapes, make_params, make_batch, tensor_shapes)

"""Seeded synthetic workloads shared by the CPU oracle's tests and the HIP path's tests.

This package holds network descriptions (layer lists) and seeded input generators only.
It contains none of the training step's arithmetic: no convolution, normalisation, loss
or update code lives here, and it imports neither the oracle nor the HIP binding.
"""
from .nets import (Net, tiny_cnn, vgg_style, resnet18, resnet50, wrn28_10, mini_resnet,
                   mini_preact, CONFIGS, build_config)
from .gen import make_inputs, to_bf16_representable, rng_for, make_dataset, epoch_orders
from .vit import ViT, vit_b16, vit_mini, make_vit_inputs, make_vit_dataset

__all__ = ["Net", "tiny_cnn", "vgg_style", "resnet18", "resnet50", "wrn28_10", "mini_resnet",
           "mini_preact", "CONFIGS", "build_config", "make_inputs", "to_bf16_representable",
           "rng_for", "make_dataset", "epoch_orders", "ViT", "vit_b16", "vit_mini", "make_vit_inputs", "make_vit_dataset"]

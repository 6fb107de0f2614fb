"""Seeded synthetic inputs shared by the CPU checker's tests and the GPU tests."""
from . import rng
from .layers import (PSET8, PSET16, Layer, mask_taps, random_pruned_layer, random_pruned_layer_k, random_pattern_set, dense_layer, magnitude_pruned_layer,
                     config1, config2, config3, config4, config5, RESNET_SHAPES, VGG16_CHANNELS, VGG16_POOL_AFTER)
from .block_layers import BlockLayer, random_block_layer, transformer_block_layer
from .reuse_layers import ReuseLayer, random_reuse_layer, conv_shaped_reuse_layer

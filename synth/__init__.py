"""Seeded synthetic inputs and workload graphs.

This package is the only code shared by the CPU oracle's tests and the GPU
harness.  It holds no arithmetic of the method itself: it draws random arrays
from a counter-based generator and lists the shapes, byte sizes and dependency
structure of the benchmark networks.
"""
from .rng import (splitmix64, stream_seed, uniform01, normal, uniform,  # noqa: F401
                  integers, f32_to_bf16_bits, bf16_bits_to_f32)
from .resnet import (LayerSpec, bottleneck_stack, identity_block, resnet_layers, make_params,  # noqa: F401
                     make_input, make_labels, fused_graph, opgranular_graph, config_graph,
                     transformer_graph, Graph, master_seed, cost_model_ns)
from .transformer import encoder_layers, make_layer_params, make_encoder_params, LN_EPS  # noqa: F401

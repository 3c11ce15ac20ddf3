"""Seeded synthetic workloads for the integer-only ASR encoder path.

This package holds ONLY input generation and network *shape* tables: a counter-based
64-bit generator, the tensor value distributions, and the op lists (layer geometry and
activation-slot wiring) of the five benchmark configurations.  It contains none of the
method's arithmetic (no convolution, no requantization), so that both the CPU oracle's
tests and the HIP path's tests can draw identical inputs from it without sharing any
computational code.
"""
from .rng import splitmix64_stream, randint_array, tensor_seed  # noqa: F401
from .nets import (  # noqa: F401
    OpSpec, NetSpec, FLAG_RELU,
    separable_module, quartznet, jasper, conformer_shaped, build_config, tiny_config,
    draw_net_params, draw_input, out_len, net_macs, net_weight_count,
)

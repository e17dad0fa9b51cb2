"""Seeded synthetic workloads: tensors and layer tables only.

This package describes WHAT is run (shapes, seeds, value distributions, layer
sequences, explicit paddings) and holds none of the layers' arithmetic. Both the
CPU oracle and the HIP library consume it; neither of those imports the other.
"""
from .nets import Layer, Network, residual_cnn, dsep_cnn, audio_cnn, dense_autoencoder, single_conv_relu, block_of  # noqa: F401
from .gen import (BASE_SEED, uniform_pm1, normal, he_normal, network_tensors, u8_codes, u8_multiplier, quantized_network_tensors,  # noqa: F401
                  sweep_shapes, SWEEP_N)

"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's
tests and benchmark.  Nothing here is part of the proof system: it produces
uniformly random field elements as raw little-endian limbs, and runs a
quantised fully connected network forward and backward in plain integers to
obtain the tensors that a prover would be handed."""
from .tables import uniform_fr_limbs, CONFIG_SEED
from .fcnn import quantise, fcnn_window, fc_relu_layer

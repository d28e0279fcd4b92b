"""Seeded synthetic inputs and workload descriptions shared by the CPU oracle and the HIP path.

This package holds no arithmetic of the method itself: it only produces input
tensors (a counter-based generator, so any element can be regenerated from
(seed, tensor id, flat index) alone) and plain-data descriptions of the einsum
graphs that stand in for the paper's workloads (Section 9: matrix chain, FFNN
training step, LLaMA-like decoder block).  Neither the oracle nor the library
is imported from here.
"""
from .prng import (hash_u64, uniform_pm1, normal, small_ints, onehot, causal_mask,
                   f32_to_bf16_bits, bf16_bits_to_f32, HostTensor, make_tensor)
from .workloads import Vertex, Workload, CONFIGS, build_config

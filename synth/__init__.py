"""Seeded synthetic inputs shared by the oracle-side tests and the HIP-side tests/bench.

This package holds input generation and memory layout only: random draws, rounding of
the drawn values to the storage type, and the packing of round segments into flat
buffers.  None of the method's arithmetic (logits, softmax, round scores, selection,
attention) lives here.
"""
from .workloads import Workload, make_workload, CONFIGS, to_bf16_bits, bf16_bits_to_f32  # noqa: F401
from .layout import pack_layer, pack_round_host, round_host_elems, PackedLayer  # noqa: F401

"""Seeded synthetic activation workloads (shapes, value distributions and bit-width
assignments of the five benchmark configurations).

This module serves both the CPU oracle's tests and the HIP path's tests/bench.  It holds
none of the method's arithmetic: no quantization, no rounding, no packing, no RNG of the
method.  The only statistic it computes is a per-group value range, used to *rank* groups
for the benchmark's stand-in bit-width policy (the paper's own controller, a greedy
knapsack over importance scores, is outside this build and `bits[]` is an input to it).

Everything is generated on the host with a seeded torch.Generator so the oracle and the
GPU see the same bytes on any machine.  The tensors stand in for the ResNet / RoBERTa /
GPT-2 activations the paper trains on; no dataset or trained weight is involved.
"""
from .workloads import (BF16, F16, F32, CONFIG_NAMES, Workload, bits_by_range_quantiles,
                        make_config, to_numpy_bits, torch_dtype)

__all__ = ["F32", "F16", "BF16", "CONFIG_NAMES", "Workload", "bits_by_range_quantiles",
           "make_config", "to_numpy_bits", "torch_dtype"]

"""Layer-shape tables and seeded synthetic input generators for the benchmark configurations.

This package is shared by the tests (which feed the same arrays to the CPU oracle and to
the GPU library) and by the benchmark.  It contains none of the method's arithmetic: the
quantizer-parameter helpers it needs (choose_qparams, quantize_multipliers, act_range,
pack_int4, quantize_weights) are passed in by the caller -- the oracle's in the tests, the
library's own host helpers in the benchmark.
"""
from .shapes import Layer, fuse_adds, gemm_sweep, mobilenet_v1, mobilenet_v2, resnet50, single_conv  # noqa: F401
from .synth import SEED_BASE, conv_case, gemm_case, qadd_case, quantize_case, seed_for  # noqa: F401

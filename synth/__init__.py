"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU tests.

This package only draws numbers and names workload shapes.  It contains none of
the arithmetic of convolution, matrix multiplication, layout blocking or the
reuse model, and imports neither the oracle nor the HIP library.
"""
from .rng import (uniform_pm1, normal, small_ints, to_bf16_bits, bf16_bits_to_f32,
                  splitmix64)
from .workloads import (ConvShape, RESNET50_SUITE, HELDOUT_SUITE, CONFIG1, CONFIG4, SGEMM_SIZES,
                        PAPER_GEMM_SIZES, conv_inputs, sgemm_inputs, out_hw)

__all__ = ["uniform_pm1", "normal", "small_ints", "to_bf16_bits", "bf16_bits_to_f32",
           "splitmix64", "ConvShape", "RESNET50_SUITE", "HELDOUT_SUITE", "CONFIG1", "CONFIG4",
           "SGEMM_SIZES", "PAPER_GEMM_SIZES", "conv_inputs", "sgemm_inputs", "out_hw"]

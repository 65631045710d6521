"""CPU oracle of the Hadamard-quantised layer.  TEST INFRASTRUCTURE ONLY:
imported by tests/, by the smoke check and by the benchmark's CPU-baseline leg,
never by the product package."""
from .hq_oracle import (  # noqa: F401
    act_hadamard_quant,
    act_hadamard_quant_static,
    act_width_quant_static,
    block_hadamard,
    build,
    hadamard_raw,
    int_conv2d,
    int_conv2d_static,
    int_conv2d_width,
    int_gemm,
    int_gemm_single,
    int_linear,
    int_linear_single,
    int_linear_static,
    max_threads,
    quantize_rows,
    quantize_static,
    quantize_weights,
    quantize_weights_single,
)

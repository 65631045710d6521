"""CPU oracle of the Hadamard-quantised layer.  TEST INFRASTRUCTURE ONLY:
imported by tests/, by the smoke check and by the benchmark's CPU-baseline leg,
never by the product package."""
from .hq_oracle import (  # noqa: F401
    act_hadamard_quant,
    block_hadamard,
    build,
    hadamard_raw,
    int_conv2d,
    int_gemm,
    int_linear,
    max_threads,
    quantize_rows,
    quantize_weights,
)

"""MI355X-native Hadamard-quantised layer of HQ-DM: thin Python face of libhq.so."""
from .binding import (  # noqa: F401
    HqError,
    hq_act_hadamard_quant,
    hq_act_hadamard_quant_static,
    hq_act_hadamard_quant_width,
    hq_int_conv2d,
    hq_int_conv2d_i8,
    hq_int_conv2d_static,
    hq_int_conv2d_width,
    hq_int_linear,
    hq_int_linear_i8,
    hq_int_linear_single,
    hq_int_linear_static,
    hq_quantize_weights,
    hq_quantize_weights_single,
    load_library,
    status_string,
)

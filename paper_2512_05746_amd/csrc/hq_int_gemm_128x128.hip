// Integer GEMM / convolution kernels, workgroup tile 128x128 (output channels x pixels).
#include "hq_int_gemm_kernel.h"

hq_status hq_gemm_launch_128x128(const GemmArgs &a, int taps, hq_dtype y_dtype, hipStream_t stream) {
    return launch_config<2, 2, 2, 2, 2, true>(a, taps, y_dtype, stream);
}

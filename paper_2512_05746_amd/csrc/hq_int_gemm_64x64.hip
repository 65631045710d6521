// Integer GEMM / convolution kernels, workgroup tile 64x64 (output channels x pixels).
#include "hq_int_gemm_kernel.h"

hq_status hq_gemm_launch_64x64(const GemmArgs &a, int taps, hq_dtype y_dtype, hipStream_t stream) {
    return launch_config<1, 1, 2, 2, 4, false, 2, true>(a, taps, y_dtype, stream);
}

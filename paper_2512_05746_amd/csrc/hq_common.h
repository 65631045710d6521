// Internal helpers shared by the HIP translation units of libhq (host side only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hq.h"

namespace hq {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool pow2_upto_128(int v) { return v >= 1 && v <= 128 && (v & (v - 1)) == 0; }

inline int ilog2(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

// Compute units of the current device (queried once per device; 256 on MI355X).
inline int compute_units() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

// Maps the sticky launch error (if any) of the calling thread to a status.
inline hq_status launch_status() {
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_ERR_LAUNCH;
}

}  // namespace hq

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

// Maps the sticky launch error (if any) of the calling thread to a status.
inline hq_status launch_status() {
    return hipGetLastError() == hipSuccess ? HQ_OK : HQ_ERR_LAUNCH;
}

}  // namespace hq

// Internal helpers shared by the HIP translation units of libhq.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

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
    static std::atomic<int> cached[64];   // zero-initialised; host threads may race to fill an entry with the same value
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Exact division of n < 2^31 by a run-time constant d >= 2: n / d == umulhi(n, m) >> s.
// (d == 1 is handled where the quotient is taken.)
struct Magic31 {
    uint32_t m, s;
};

inline Magic31 magic31(uint32_t d) {
    if (d <= 1) return {0, 0};
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    const uint64_t m = ((1ull << (31 + l)) + d - 1) / d;   // l <= 31: no overflow
    return {static_cast<uint32_t>(m), l - 1};
}

__device__ __forceinline__ uint32_t div_magic31(uint32_t n, uint32_t d, uint32_t m, uint32_t s) {
    return d == 1 ? n : (__umulhi(n, m) >> s);
}

// Signed base-16 digits of v, least significant first: v = d[0] + 16 d[1] + 256 d[2] with every
// digit in [-8, 7] (|v| <= 1911).  The format of the digit planes of wide integers.
__device__ __forceinline__ void digits16(int v, int (&d)[3]) {
    d[0] = ((v + 8) & 15) - 8;
    v = (v - d[0]) >> 4;
    d[1] = ((v + 8) & 15) - 8;
    d[2] = (v - d[1]) >> 4;
}

// Status of the launches made while an object of this class lives.  Kernel launches report
// failures through the calling thread's "last error", which an earlier call of the caller may
// already have set: the state is sampled BEFORE the launches, and an error that was pending then
// is neither reported as the library's nor cleared (it stays for the caller to find).  Only when
// the state was clean is a new error taken (and cleared) as the launch's own.
class LaunchCheck {
public:
    LaunchCheck() : prior_(hipPeekAtLastError()) {}
    hq_status status() const {
        if (prior_ != hipSuccess) return hipPeekAtLastError() == prior_ ? HQ_OK : HQ_ERR_LAUNCH;
        return hipGetLastError() == hipSuccess ? HQ_OK : HQ_ERR_LAUNCH;
    }

private:
    hipError_t prior_;
};

}  // namespace hq

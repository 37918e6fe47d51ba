// adaptra_internal.h -- host-side helpers shared by the library's source files (not part of
// the C ABI).
#ifndef ADAPTRA_INTERNAL_H
#define ADAPTRA_INTERNAL_H

#include <hip/hip_runtime.h>

namespace adaptra_detail {

constexpr int kThreadsPerBlock = 256;

// Records the hipError_t for adaptra_last_hip_error and returns ADAPTRA_EHIP.
int hip_fail(hipError_t e);

inline int blocks_for(long long n, long long cap) {
    long long g = (n + kThreadsPerBlock - 1) / kThreadsPerBlock;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

}  // namespace adaptra_detail

#define ADAPTRA_CHECK_LAUNCH()                                             \
    do {                                                                   \
        hipError_t e_ = hipGetLastError();                                 \
        if (e_ != hipSuccess) return adaptra_detail::hip_fail(e_);         \
    } while (0)

#endif  // ADAPTRA_INTERNAL_H

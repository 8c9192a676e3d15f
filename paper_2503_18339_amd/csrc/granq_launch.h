// Kernel launches whose status is that of the launch itself.
//
// hipGetLastError() returns, and clears, whatever error any earlier HIP call of
// the thread left behind (the caller's own, or another library's), so it can
// blame a launch that succeeded and then hide the error from its owner.
// hipLaunchKernel returns the status of the launch it makes and leaves the
// thread's sticky error alone.  launch_kernel() forwards to it and remembers the
// first failure of the current entry point in a thread-local; launched() hands
// that status out and clears it.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>

#include "granq.h"

namespace granq {

template <typename T>
struct launch_arg { using type = T; };

inline hipError_t &launch_error_slot() {
    static thread_local hipError_t first_failure = hipSuccess;
    return first_failure;
}

// Arguments are converted to the kernel's parameter types (deduced from the kernel
// alone) and passed by address, as hipLaunchKernel expects.
template <typename... P>
inline void launch_kernel(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds_bytes,
                          hipStream_t stream, typename launch_arg<P>::type... args) {
    void *ptrs[sizeof...(P) + 1] = {(void *)&args..., nullptr};
    const hipError_t e = hipLaunchKernel((const void *)kernel, grid, block, ptrs, lds_bytes, stream);
    if (e != hipSuccess && launch_error_slot() == hipSuccess) launch_error_slot() = e;
}

// Status of the launches made by this thread since the last call of launched().
inline granq_status_t launched() {
    const hipError_t e = launch_error_slot();
    launch_error_slot() = hipSuccess;
    return e == hipSuccess ? GRANQ_OK : GRANQ_ERR_HIP;
}

}  // namespace granq

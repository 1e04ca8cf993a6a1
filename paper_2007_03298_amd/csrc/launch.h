// Kernel launch that hands back the launch's own status (hipGetLastError
// would also report, and clear, an error left by an unrelated earlier call).
#pragma once

#include <hip/hip_runtime.h>

namespace ds {

template <typename T>
struct exactly { typedef T type; };

// The arguments are converted to the kernel's parameter types before their
// addresses are taken, so a call site cannot pass a narrower or wider value
// than the kernel reads.
template <typename... Params>
hipError_t launch_kernel(void (*kernel)(Params...), dim3 grid, dim3 block, unsigned dynamic_lds, hipStream_t stream,
                         typename exactly<Params>::type... args) {
    void* slots[] = {const_cast<void*>(static_cast<const volatile void*>(&args))...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, slots, dynamic_lds, stream);
}

}  // namespace ds

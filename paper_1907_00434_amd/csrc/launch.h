// Kernel launch helper and device queries shared by the kernel sources of the library.
#ifndef MLF_LAUNCH_H
#define MLF_LAUNCH_H

#include <hip/hip_runtime.h>

#include <stddef.h>

#include <atomic>
#include <tuple>
#include <utility>

namespace mlf_detail {

template <typename... PARAMS, size_t... I>
bool launch_with(void (*kernel)(PARAMS...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                 std::tuple<PARAMS...> &values, std::index_sequence<I...>)
{
    void *params[] = {static_cast<void *>(&std::get<I>(values))...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, params, lds, stream) ==
           hipSuccess;
}

}  // namespace mlf_detail

// Launches `kernel` and returns the status of this launch itself, so that a
// sticky error left by an earlier, unrelated HIP call is not mistaken for a
// failure here.  The arguments are converted to the kernel's parameter types.
template <typename... PARAMS, typename... ARGS>
bool launch_kernel(void (*kernel)(PARAMS...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                   ARGS &&...args)
{
    static_assert(sizeof...(PARAMS) == sizeof...(ARGS), "one argument per kernel parameter");
    std::tuple<PARAMS...> values{static_cast<PARAMS>(args)...};
    return mlf_detail::launch_with(kernel, grid, block, lds, stream, values,
                                   std::index_sequence_for<PARAMS...>{});
}

// Compute units of the current device, looked up once per device (0 when the
// runtime cannot tell).
inline unsigned cu_count()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cached[kMaxDevices];
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return 0;
    int n = cached[device].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n < 1) return 0;
        cached[device].store(n, std::memory_order_relaxed);
    }
    return static_cast<unsigned>(n);
}

#endif  // MLF_LAUNCH_H

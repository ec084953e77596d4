// Shared host-side helpers of the HIP entry points (kernel launches with their own status).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <utility>

#include "agentsam.h"

namespace agentsam {
constexpr int kWave = 64;

template <class Tuple, size_t... I>
inline hipError_t launch_tuple(const void *fn, dim3 grid, dim3 block, hipStream_t st, Tuple &t, std::index_sequence<I...>) {
    void *argv[] = {(void *)&std::get<I>(t)...};
    return hipLaunchKernel(fn, grid, block, argv, 0, st);
}

// Launches kernel(args...) and returns the status of THIS launch (hipGetLastError would also report, and
// clear, whatever an unrelated earlier call of the thread left behind).  The arguments are converted
// to the kernel's parameter types first.
template <class... KArgs, class... Args>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t st, Args &&...args) {
    static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count");
    std::tuple<KArgs...> t(std::forward<Args>(args)...);
    return launch_tuple((const void *)kernel, grid, block, st, t, std::index_sequence_for<KArgs...>{});
}
}  // namespace agentsam

#define AGENTSAM_LAUNCH(kernel, grid, block, st, ...)                                                   \
    do {                                                                                                \
        if (agentsam::launch(kernel, grid, block, st, __VA_ARGS__) != hipSuccess) return AGENTSAM_ERR_HIP; \
    } while (0)

// Internal: kernel launch that hands back the launch's own status.
//
// The <<<...>>> syntax drops what the runtime returns, and asking afterwards with
// hipGetLastError() would also fetch -- and clear -- an error that the caller's
// earlier, unrelated work left behind, and report it as this library's.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdio>
#include <tuple>
#include <utility>

#include "plan.h"

namespace covap {

template <typename... P, size_t... I>
inline hipError_t launch_impl(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds, hipStream_t st,
                              std::tuple<P...> &params, std::index_sequence<I...>)
{
    void *ptrs[] = {(void *)&std::get<I>(params)...};
    return hipLaunchKernel((const void *)kernel, grid, block, ptrs, lds, st);
}

// Launches kernel<<<grid, block, lds, st>>>(args...); every argument is converted to
// the kernel's own parameter type first.
template <typename... P, typename... A>
inline hipError_t launch(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds, hipStream_t st, A &&...args)
{
    static_assert(sizeof...(P) == sizeof...(A), "one argument per kernel parameter");
    std::tuple<P...> params{static_cast<P>(std::forward<A>(args))...};
    return launch_impl(kernel, grid, block, lds, st, params, std::index_sequence_for<P...>{});
}

// What a call's launches returned: the first failure, if any.
struct launch_status {
    hipError_t err = hipSuccess;
    void operator+=(hipError_t e)
    {
        if (err == hipSuccess) err = e;
    }
    covap_status_t report(const char *what) const
    {
        if (err == hipSuccess) return COVAP_OK;
        char msg[200];
        std::snprintf(msg, sizeof msg, "%s: %s", what, hipGetErrorString(err));
        return fail(COVAP_EHIP, msg);
    }
};

}  // namespace covap

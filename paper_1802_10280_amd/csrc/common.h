// Internal helpers shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <tuple>
#include <utility>

#include "escoin.h"

namespace escoin {

struct Dims {
    int N, C, H, W, M, R, S, stride, pad;
    int Hp, Wp, E, F;
};

// Fills `d` from a checked descriptor; returns an ESCOIN_* code.
int make_dims(const escoin_conv_desc* desc, Dims* d);

inline int hip_status(hipError_t e) { return e == hipSuccess ? ESCOIN_OK : ESCOIN_EHIP; }

// Launches `kernel` and reports the status of this launch alone: hipLaunchKernel's own return
// value, not the thread's sticky last-error slot (which other users of the runtime in the same
// process may have left set).
template <typename... Params, typename... Args, size_t... I>
inline int launch_impl(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds,
                       hipStream_t stream, std::index_sequence<I...>, Args... args) {
    std::tuple<Params...> a{static_cast<Params>(args)...};
    void* ptrs[] = {(void*)&std::get<I>(a)...};
    return hip_status(hipLaunchKernel((const void*)kernel, grid, block, ptrs, lds, stream));
}

template <typename... Params, typename... Args>
inline int launch(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                  Args... args) {
    static_assert(sizeof...(Params) == sizeof...(Args), "kernel argument count mismatch");
    return launch_impl(kernel, grid, block, lds, stream, std::index_sequence_for<Params...>{},
                       args...);
}

}  // namespace escoin

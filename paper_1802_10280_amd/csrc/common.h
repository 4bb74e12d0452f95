// Internal helpers shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "escoin.h"

namespace escoin {

struct Dims {
    int N, C, H, W, M, R, S, stride, pad;
    int Hp, Wp, E, F;
};

// Fills `d` from a checked descriptor; returns an ESCOIN_* code.
int make_dims(const escoin_conv_desc* desc, Dims* d);

inline int hip_status(hipError_t e) { return e == hipSuccess ? ESCOIN_OK : ESCOIN_EHIP; }

}  // namespace escoin

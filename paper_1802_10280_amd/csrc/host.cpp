// Host-side entry points: descriptor checks, size queries and weight stretching.
#include <limits.h>

#include "common.h"

namespace escoin {

int make_dims(const escoin_conv_desc* desc, Dims* d) {
    if (!desc || !d) return ESCOIN_EINVAL;
    const escoin_conv_desc& p = *desc;
    if (p.N <= 0 || p.C <= 0 || p.H <= 0 || p.W <= 0 || p.M <= 0 || p.R <= 0 || p.S <= 0 ||
        p.stride < 1 || p.pad < 0)
        return ESCOIN_EINVAL;
    // guard the additions below against int32 overflow
    if (p.pad > (1 << 20) || p.H > (1 << 28) || p.W > (1 << 28)) return ESCOIN_ERANGE;
    const int64_t Hp = (int64_t)p.H + 2 * p.pad, Wp = (int64_t)p.W + 2 * p.pad;
    if (Hp < p.R || Wp < p.S) return ESCOIN_EINVAL;
    const int64_t E = (Hp - p.R) / p.stride + 1, F = (Wp - p.S) / p.stride + 1;
    // per-image offsets are int32 inside the kernels (Section 2.3 counts 4-byte indices)
    if ((int64_t)p.C * Hp * Wp >= (int64_t)INT32_MAX) return ESCOIN_ERANGE;
    if ((int64_t)p.M * E * F >= (int64_t)INT32_MAX) return ESCOIN_ERANGE;
    if ((int64_t)p.C * p.R * p.S >= (int64_t)INT32_MAX) return ESCOIN_ERANGE;
    d->N = p.N; d->C = p.C; d->H = p.H; d->W = p.W; d->M = p.M; d->R = p.R; d->S = p.S;
    d->stride = p.stride; d->pad = p.pad;
    d->Hp = (int)Hp; d->Wp = (int)Wp; d->E = (int)E; d->F = (int)F;
    return ESCOIN_OK;
}

}  // namespace escoin

using escoin::Dims;

extern "C" {

const char* escoin_strerror(int code) {
    switch (code) {
        case ESCOIN_OK: return "ok";
        case ESCOIN_EINVAL: return "invalid argument (null pointer, bad dimension, malformed CSR or flags)";
        case ESCOIN_ERANGE: return "index range exceeds int32";
        case ESCOIN_EHIP: return "HIP runtime call failed";
        case ESCOIN_ESIZE: return "caller-provided buffer too small";
        default: return "unknown escoin error code";
    }
}

int escoin_check_desc(const escoin_conv_desc* desc) {
    Dims d;
    return escoin::make_dims(desc, &d);
}

int escoin_output_dims(const escoin_conv_desc* desc, int32_t* E, int32_t* F) {
    Dims d;
    int rc = escoin::make_dims(desc, &d);
    if (rc != ESCOIN_OK) return rc;
    if (E) *E = d.E;
    if (F) *F = d.F;
    return ESCOIN_OK;
}

size_t escoin_padded_elems(const escoin_conv_desc* desc) {
    Dims d;
    if (escoin::make_dims(desc, &d) != ESCOIN_OK) return 0;
    return (size_t)d.N * d.C * d.Hp * d.Wp;
}

size_t escoin_output_elems(const escoin_conv_desc* desc) {
    Dims d;
    if (escoin::make_dims(desc, &d) != ESCOIN_OK) return 0;
    return (size_t)d.N * d.M * d.E * d.F;
}

// Weight stretching (Section 3.1): column j=(c*R+r)*S+s -> f(c,r,s)=(c*Hp+r)*Wp+s.
int escoin_sconv_pack(const escoin_conv_desc* desc, const int32_t* rowptr, const int32_t* colidx,
                      int32_t* colidx_stretched) {
    Dims d;
    int rc = escoin::make_dims(desc, &d);
    if (rc != ESCOIN_OK) return rc;
    if (!rowptr) return ESCOIN_EINVAL;
    if (rowptr[0] != 0) return ESCOIN_EINVAL;
    for (int m = 0; m < d.M; ++m)
        if (rowptr[m + 1] < rowptr[m]) return ESCOIN_EINVAL;
    const int32_t nnz = rowptr[d.M];
    if (nnz > 0 && (!colidx || !colidx_stretched)) return ESCOIN_EINVAL;
    const int32_t cols = d.C * d.R * d.S;
    // validate first so that a failing call leaves the output untouched (it may alias colidx)
    for (int32_t j = 0; j < nnz; ++j)
        if (colidx[j] < 0 || colidx[j] >= cols) return ESCOIN_EINVAL;
    const int32_t RS = d.R * d.S;
    const int32_t plane = d.Hp * d.Wp;
    for (int32_t j = 0; j < nnz; ++j) {
        const int32_t col = colidx[j];
        const int32_t c = col / RS;
        const int32_t rs = col - c * RS;
        const int32_t r = rs / d.S;
        const int32_t s = rs - r * d.S;
        colidx_stretched[j] = c * plane + r * d.Wp + s;
    }
    return ESCOIN_OK;
}

}  // extern "C"

// sconv, general form: Algorithm 2 on the stretched CSR and the padded input array, with the
// data-to-thread mapping of Section 3.2 (consecutive lanes own consecutive output positions)
// and a workgroup per output channel (Section 3.3).  It accepts any filter size, stride and
// CSR entry order.  The CSR row is wave-uniform, so its (offset, value) pairs travel through
// the scalar data path instead of being staged in LDS; the input window is read through the
// vector L1/L2, which plays the part of the read-only cache of Section 3.3.
#include "common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kPix = 4;  // output positions per lane, kThreads apart (independent FMA chains)

__global__ __launch_bounds__(kThreads) void sconv_direct_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
    const float* __restrict__ value, const float* __restrict__ padded, float* __restrict__ out,
    const float* __restrict__ bias, uint32_t flags, int M, int E, int F, int Wp, int stride,
    int img_elems /* C*Hp*Wp */) {
    const int m = blockIdx.y;
    const int EF = E * F;
    const int j0 = rowptr[m], j1 = rowptr[m + 1];
    const float b = (flags & ESCOIN_F_BIAS) ? bias[m] : 0.0f;
    {
        const int n = blockIdx.z;
        const float* __restrict__ img = padded + (size_t)n * img_elems;
        int p[kPix];
        int base[kPix];
        float acc[kPix];
#pragma unroll
        for (int k = 0; k < kPix; ++k) {
            p[k] = (blockIdx.x * kPix + k) * kThreads + threadIdx.x;
            const int pc = p[k] < EF ? p[k] : 0;  // clamp: out-of-range lanes read a valid pixel
            const int h = pc / F;
            const int w = pc - h * F;
            base[k] = h * stride * Wp + w * stride;  // f(0, h, w) on the padded pitch
            acc[k] = b;
        }
        for (int j = j0; j < j1; ++j) {
            const int off = colidx[j];
            const float val = value[j];
#pragma unroll
            for (int k = 0; k < kPix; ++k) acc[k] = fmaf(val, img[off + base[k]], acc[k]);
        }
        float* __restrict__ o = out + ((size_t)n * M + m) * EF;
#pragma unroll
        for (int k = 0; k < kPix; ++k) {
            float v = acc[k];
            if (flags & ESCOIN_F_RELU) v = v > 0.0f ? v : 0.0f;
            if (p[k] < EF) o[p[k]] = v;
        }
    }
}

}  // namespace

namespace escoin {

int launch_sconv_direct(const Dims& d, const int32_t* d_rowptr, const int32_t* d_colidx,
                        const float* d_value, const float* d_padded, float* d_out,
                        const float* d_bias, uint32_t flags, hipStream_t stream) {
    const int EF = d.E * d.F;
    const int per_block = kThreads * kPix;
    // grid.y / grid.z carry M and N; both are far below the 65535 limit for any layer whose
    // indices fit int32 here, but reject rather than fold silently
    if (d.M > 65535 || d.N > 65535) return ESCOIN_ERANGE;
    dim3 grid((EF + per_block - 1) / per_block, d.M, d.N);
    return launch(sconv_direct_kernel, grid, dim3(kThreads), 0, stream, d_rowptr, d_colidx, d_value,
                  d_padded, d_out, d_bias, flags, d.M, d.E, d.F, d.Wp, d.stride,
                  d.C * d.Hp * d.Wp);
}

}  // namespace escoin

extern "C" int escoin_sconv_forward(const escoin_conv_desc* desc, const int32_t* d_rowptr,
                                    const int32_t* d_colidx_stretched, const float* d_value,
                                    const float* d_padded, float* d_out, const float* d_bias,
                                    uint32_t flags, void* hip_stream) {
    escoin::Dims d;
    int rc = escoin::make_dims(desc, &d);
    if (rc != ESCOIN_OK) return rc;
    if (!d_rowptr || !d_padded || !d_out) return ESCOIN_EINVAL;
    if (flags & ~(uint32_t)(ESCOIN_F_BIAS | ESCOIN_F_RELU)) return ESCOIN_EINVAL;
    if ((flags & ESCOIN_F_BIAS) && !d_bias) return ESCOIN_EINVAL;
    return escoin::launch_sconv_direct(d, d_rowptr, d_colidx_stretched, d_value, d_padded, d_out,
                                       d_bias, flags, (hipStream_t)hip_stream);
}

// pad_in: the zero-padded 1-D input array of Section 3.1 (the pad_in step of Section 4.2).
#include "common.h"

namespace {

// One thread per padded element of a plane; planes are walked with a grid-stride over y.
// Interior elements copy the input bit for bit, the frame is +0.0f.
__global__ __launch_bounds__(256) void pad_in_kernel(const float* __restrict__ in,
                                                     float* __restrict__ padded, int planes,
                                                     int H, int W, int Hp, int Wp, int pad) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= Hp * Wp) return;
    const int yp = i / Wp;
    const int xp = i - yp * Wp;
    const int y = yp - pad, x = xp - pad;
    const bool inside = (unsigned)y < (unsigned)H && (unsigned)x < (unsigned)W;
    const int src = y * W + x;
    for (int p = blockIdx.y; p < planes; p += gridDim.y) {
        float v = 0.0f;
        if (inside) v = in[(size_t)p * H * W + src];
        padded[(size_t)p * Hp * Wp + i] = v;
    }
}

}  // namespace

extern "C" int escoin_pad_in(const escoin_conv_desc* desc, const float* d_in, float* d_padded,
                             void* hip_stream) {
    escoin::Dims d;
    int rc = escoin::make_dims(desc, &d);
    if (rc != ESCOIN_OK) return rc;
    if (!d_in || !d_padded) return ESCOIN_EINVAL;
    const long long planes = (long long)d.N * d.C;
    if (planes >= INT32_MAX) return ESCOIN_ERANGE;
    const int plane = d.Hp * d.Wp;
    dim3 grid((plane + 255) / 256, (unsigned)(planes < 32768 ? planes : 32768));
    return escoin::launch(pad_in_kernel, grid, dim3(256), 0, (hipStream_t)hip_stream, d_in, d_padded,
                          (int)planes, d.H, d.W, d.Hp, d.Wp, d.pad);
}

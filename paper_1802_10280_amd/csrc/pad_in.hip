// pad_in: the zero-padded 1-D input array of Section 3.1 (the pad_in step of Section 4.2).
#include "common.h"

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

// floor(i / d) and the remainder, for i below 2^52, from the reciprocal rounded to double: the
// product is at most one off, which the remainder shows.
__device__ __forceinline__ void divmod(uint64_t i, uint32_t d, double inv_d, uint64_t* q, uint32_t* r) {
    uint64_t qq = (uint64_t)((double)i * inv_d);
    int64_t rr = (int64_t)(i - qq * d);
    if (rr < 0) { --qq; rr += d; }
    else if (rr >= (int64_t)d) { ++qq; rr -= d; }
    *q = qq;
    *r = (uint32_t)rr;
}

// The padded array is produced four consecutive floats per thread (one 16-byte store where the
// destination allows it), a grid-stride loop over those groups: the kernel is bound by HBM, and
// what it needs is few, long-running workgroups with wide, contiguous stores.  Interior elements
// copy the input bit for bit, the frame is +0.0f.
__global__ __launch_bounds__(256) void pad_in_kernel(const float* __restrict__ in, float* __restrict__ padded,
                                                     uint64_t total, int H, int W, int Hp, int Wp, int pad,
                                                     double inv_plane, double inv_wp, int wide) {
    const uint32_t plane = (uint32_t)Hp * (uint32_t)Wp;
    const uint64_t groups = (total + 3) / 4;
    for (uint64_t g = (uint64_t)blockIdx.x * 256 + threadIdx.x; g < groups; g += (uint64_t)gridDim.x * 256) {
        const uint64_t i0 = 4 * g;
        uint64_t p;
        uint32_t rem, xp;
        uint64_t ypq;
        divmod(i0, plane, inv_plane, &p, &rem);
        divmod(rem, (uint32_t)Wp, inv_wp, &ypq, &xp);
        int yp = (int)ypq, x = (int)xp;
        float v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int y = yp - pad, xx = x - pad;
            const bool inside = (unsigned)y < (unsigned)H && (unsigned)xx < (unsigned)W && i0 + k < total;
            v[k] = inside ? in[p * (uint64_t)(H * W) + (uint32_t)(y * W + xx)] : 0.0f;
            if (++x == Wp) {
                x = 0;
                if (++yp == Hp) { yp = 0; ++p; }
            }
        }
        if (wide && i0 + 3 < total) {
            *(f4*)__builtin_assume_aligned(padded + i0, 16) = (f4){v[0], v[1], v[2], v[3]};
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (i0 + k < total) padded[i0 + k] = v[k];
        }
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
    const uint64_t plane = (uint64_t)d.Hp * d.Wp;
    const uint64_t total = (uint64_t)planes * plane;
    if (total >= (1ull << 50)) return ESCOIN_ERANGE;
    const uint64_t groups = (total + 3) / 4;
    // enough workgroups to fill the compute units several times over, each with a long loop
    const unsigned blocks = (unsigned)std::min<uint64_t>((groups + 255) / 256, 256 * 16);
    return escoin::launch(pad_in_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, d_in, d_padded,
                          total, d.H, d.W, d.Hp, d.Wp, d.pad, 1.0 / (double)plane, 1.0 / (double)d.Wp,
                          (int)(((uintptr_t)d_padded & 15) == 0));
}

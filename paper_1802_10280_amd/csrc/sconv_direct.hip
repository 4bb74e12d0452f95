// sconv, general form: Algorithm 2 on the stretched CSR and the padded input array, with the
// data-to-thread mapping of Section 3.2 (consecutive lanes own consecutive output positions,
// numbered through the images of the batch) and a workgroup per output channel (Section 3.3).  It accepts any filter size, stride and
// CSR entry order.  The CSR row is wave-uniform, so its (offset, value) pairs travel through
// the scalar data path instead of being staged in LDS; the input window is read through the
// vector L1/L2, which plays the part of the read-only cache of Section 3.3.
#include "common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kPix = 4;  // output positions per lane, kThreads apart (independent FMA chains)

// A workgroup owns one output channel and kThreads * kPix output positions of a group of images:
// the positions of the group's images are numbered through (image, h, w), so that small maps
// fill the lanes as well as large ones.  Offsets inside a group fit 32 bits (the launch sizes the
// groups for that).
__global__ __launch_bounds__(kThreads) void sconv_direct_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
    const float* __restrict__ value, const float* __restrict__ padded, float* __restrict__ out,
    const float* __restrict__ bias, uint32_t flags, int N, int M, int E, int F, int Wp, int stride,
    int img_elems /* C*Hp*Wp */, int group_images, int n_groups, int bx, int deal) {
    // Workgroup -> (image group, output channel, block of positions), all channels of a group
    // before the next group.  Consecutive workgroup ids land on different XCDs (id mod 8), each
    // with an L2 of its own.  Small images: the XCDs share every group (plain order).  Large
    // images (`deal`): the groups are dealt to the XCDs in turn and an XCD walks its own groups
    // one after the other, so that the few groups it has in flight stay in its L2.
    const uint32_t per_group = (uint32_t)bx * (uint32_t)M;
    uint32_t group, rest;
    if (deal) {
        const uint32_t xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        group = (slot / per_group) * 8 + xcd;
        rest = slot % per_group;
    } else {
        group = blockIdx.x / per_group;
        rest = blockIdx.x % per_group;
    }
    if (group >= (uint32_t)n_groups) return;
    const int m = (int)(rest / (uint32_t)bx);
    const uint32_t xblk = rest % (uint32_t)bx;
    const int EF = E * F;
    const int j0 = rowptr[m], j1 = rowptr[m + 1];
    const float b = (flags & ESCOIN_F_BIAS) ? bias[m] : 0.0f;
    const int n_first = (int)group * group_images;
    const int n_here = min(group_images, N - n_first);
    const uint32_t positions = (uint32_t)n_here * (uint32_t)EF;
    const float* __restrict__ grp = padded + (size_t)n_first * img_elems;
    uint32_t p[kPix], base[kPix];
    float acc[kPix];
#pragma unroll
    for (int k = 0; k < kPix; ++k) {
        p[k] = (xblk * kPix + k) * kThreads + threadIdx.x;
        const uint32_t pc = p[k] < positions ? p[k] : 0;  // clamp: out-of-range lanes read a valid pixel
        const uint32_t n = pc / (uint32_t)EF, pp = pc - n * (uint32_t)EF;
        const uint32_t h = pp / (uint32_t)F, w = pp - h * (uint32_t)F;
        base[k] = n * (uint32_t)img_elems + h * (uint32_t)(stride * Wp) + w * (uint32_t)stride;  // f(0, h, w) of image n
        acc[k] = b;
    }
    for (int j = j0; j < j1; ++j) {
        const uint32_t off = (uint32_t)colidx[j];
        const float val = value[j];
#pragma unroll
        for (int k = 0; k < kPix; ++k) acc[k] = fmaf(val, grp[off + base[k]], acc[k]);
    }
#pragma unroll
    for (int k = 0; k < kPix; ++k) {
        float v = acc[k];
        if (flags & ESCOIN_F_RELU) v = v > 0.0f ? v : 0.0f;
        if (p[k] < positions) {
            const uint32_t n = p[k] / (uint32_t)EF, pp = p[k] - n * (uint32_t)EF;
            out[((size_t)(n_first + n) * M + m) * EF + pp] = v;
        }
    }
}

}  // namespace

namespace escoin {

int launch_sconv_direct(const Dims& d, const int32_t* d_rowptr, const int32_t* d_colidx,
                        const float* d_value, const float* d_padded, float* d_out,
                        const float* d_bias, uint32_t flags, hipStream_t stream) {
    const long long EF = (long long)d.E * d.F;
    const long long img_elems = (long long)d.C * d.Hp * d.Wp;
    // images per group: offsets inside a group (below group * img_elems, plus a nonzero's own
    // offset below img_elems) and position numbers stay under 2^32
    long long limit = std::max<long long>(1, std::min<long long>(d.N, ((1ll << 31) / img_elems)));
    limit = std::max<long long>(1, std::min<long long>(limit, (1ll << 30) / EF));
    // A group's padded input should stay in an L2 (4 MB per XCD) while all M output channels
    // walk over it, and its positions should fill the lanes of whole workgroups.  Images of
    // more than 512 KB (eight of them in flight overflow an L2) are dealt to the XCDs, and the
    // groups should then come in multiples of 8.  Among the sizes that split the batch evenly
    // and hold at most 6 MB of input: the best lane fill (x XCD balance), ties to the smaller.
    const long long per_block = kThreads * kPix;
    const bool deal = img_elems * 4 > (512ll << 10);
    const long long most = std::max<long long>(1, std::min<long long>(limit, (6ll << 20) / (img_elems * 4)));
    long long group = 1;
    double best = 0.0;
    for (long long g = 1; g <= most; ++g) {
        const long long n_g = (d.N + g - 1) / g, even = (d.N + n_g - 1) / n_g;
        if (even != g) continue;
        const double fill = (double)(g * EF) / (double)(((g * EF + per_block - 1) / per_block) * per_block);
        const double balance = deal ? (double)n_g / (double)(((n_g + 7) / 8) * 8) : 1.0;
        if (fill * balance > best * 1.03) { best = fill * balance; group = g; }
    }
    const long long groups = (d.N + group - 1) / group;
    const long long bx = (group * EF + per_block - 1) / per_block;
    // one-dimensional grid: 8 XCDs x (groups per XCD) x M x blocks of positions
    const long long blocks = (deal ? 8 * ((groups + 7) / 8) : groups) * bx * d.M;
    if (blocks > 0x7FFFFFFFll || bx * d.M > 0x7FFFFFFFll) return ESCOIN_ERANGE;
    return launch(sconv_direct_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, d_rowptr, d_colidx,
                  d_value, d_padded, d_out, d_bias, flags, d.N, d.M, d.E, d.F, d.Wp, d.stride,
                  (int)img_elems, (int)group, (int)groups, (int)bx, (int)deal);
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

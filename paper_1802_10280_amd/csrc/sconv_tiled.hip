// LDS-tiled sconv for gfx950.
//
// One workgroup owns a tile of output positions (a band of rows of one image, or several
// small images) and a group of output channels, and walks the input channels in chunks:
//   stage   the chunk's input window is copied from the UNPADDED input into LDS through a
//           lookup table that also supplies the zero frame (pad_in fused into the staging);
//           the window is the flat padded array of Section 3.1, split into stride phases
//           and stored once per 16-byte alignment class ("slot") of the filter taps;
//   compute Algorithm 2 on that window: every wave streams the (LDS offset, value) records
//           of its K CSR rows through the scalar data path; a lane owns 4*Q consecutive
//           positions of the flat array, fetches them with one aligned 16-byte LDS read per
//           record and position group and accumulates val * in[off + f(0,h,w)] in registers;
//   store   positions that are real outputs go to out[n][m][h][w] through the second table,
//           with the optional bias + ReLU epilogue.
// Consecutive lanes own consecutive positions (the data-to-thread mapping of Section 3.2), so
// LDS reads are conflict-free and output stores are contiguous along w.
#include "common.h"
#include "plan.h"

namespace escoin {

typedef float f4 __attribute__((ext_vector_type(4)));

struct TiledArgs {
    const float* in;
    float* out;
    const float* bias;
    const int32_t* src_lut;
    const int32_t* dst_lut;
    const int32_t* perm;
    const uint32_t* seg;
    const uint32_t* rec;
    int N, C, HW, M, EF;
    int WM, WQ, CC, NB;
    int n_tiles, n_mgroups, n_chunks, n_in_tiles;
    int plane_stride, P4, lut_entries;
    uint32_t flags;
};

namespace {

template <int B>
struct Batch {
    uint32_t w[2 * B];  // B x {LDS byte offset, value bits}
};

template <int B>
__device__ __forceinline__ Batch<B> load_batch(const uint32_t* __restrict__ p) {
    Batch<B> b;
#pragma unroll
    for (int i = 0; i < 2 * B; ++i) b.w[i] = p[i];  // uniform address: merged scalar loads
    return b;
}

template <int K, int Q, int B>
__global__ __launch_bounds__(512) void sconv_tiled_kernel(const TiledArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wq = wave % a.WQ, wm = wave / a.WQ;

    // Workgroup -> (input tile, output-channel group).  Consecutive workgroup ids land on
    // different XCDs, so all channel groups of one input tile are given ids that are equal
    // mod 8: they run on the same XCD and share the tile through its L2.
    const int xcd = blockIdx.x & 7, slot_j = blockIdx.x >> 3;
    const int mg = slot_j % a.n_mgroups;
    const int t_in = (slot_j / a.n_mgroups) * 8 + xcd;
    if (t_in >= a.n_in_tiles) return;  // whole workgroup leaves before any barrier
    const int tile = t_in % a.n_tiles;
    const int n0 = (t_in / a.n_tiles) * a.NB;

    const int gpi = a.P4 >> 2;  // position groups per image
    int base_bytes[Q], nloc[Q], pos0[Q];
    bool active[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int g = (wq * Q + q) * 64 + lane;
        active[q] = g < a.NB * gpi;
        const int gg = active[q] ? g : 0;  // idle lanes shadow group 0 (reads stay in range)
        nloc[q] = gg / gpi;
        pos0[q] = (gg - nloc[q] * gpi) * 4;
        base_bytes[q] = (nloc[q] * a.plane_stride + pos0[q]) * 4;
    }

    f4 acc[K][Q];
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
        for (int q = 0; q < Q; ++q) acc[k][q] = (f4)(0.0f);

    const int bin = mg * a.WM + wm;
    const uint32_t* __restrict__ segp = a.seg + (size_t)bin * a.n_chunks * (1 + K);
    const int32_t* __restrict__ lut = a.src_lut + (size_t)tile * a.lut_entries;
    const int nthreads = blockDim.x;

    for (int ch = 0; ch < a.n_chunks; ++ch) {
        __syncthreads();  // every wave is done reading the previous chunk
        // ---- stage: LDS[slot][c][n][e] = in[n][c0+c][src_lut[slot][e]], 0 where the table says -1
        const int c0 = ch * a.CC;
        const int ccur = min(a.CC, a.C - c0);
        for (int idx = tid; idx < a.lut_entries; idx += nthreads) {
            const int s = lut[idx];
            const int slot = idx / a.plane_stride;
            const int e = idx - slot * a.plane_stride;
            float* __restrict__ dst = lds + (size_t)slot * a.CC * a.NB * a.plane_stride + e;
            const float* __restrict__ src = a.in + ((size_t)n0 * a.C + c0) * a.HW + (s >= 0 ? s : 0);
            for (int nl = 0; nl < a.NB; ++nl) {
                const bool ok = s >= 0 && n0 + nl < a.N;
#pragma unroll 4
                for (int cl = 0; cl < ccur; ++cl) {
                    float v = 0.0f;
                    if (ok) v = src[((size_t)nl * a.C + cl) * a.HW];
                    dst[(cl * a.NB + nl) * a.plane_stride] = v;
                }
            }
        }
        __syncthreads();

        // ---- compute: Algorithm 2 over this chunk's nonzeros of the wave's K rows
        const uint32_t* __restrict__ sg = segp + (size_t)ch * (1 + K);
        const uint32_t* __restrict__ rp = a.rec + (size_t)sg[0] * (2 * B);
        Batch<B> nxt = load_batch<B>(rp);
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int cnt = (int)sg[1 + k];
            for (int b = 0; b < cnt; ++b) {
                const Batch<B> cur = nxt;
                rp += 2 * B;
                nxt = load_batch<B>(rp);  // the stream has two spare batches at its end
                f4 x[B][Q];
#pragma unroll
                for (int u = 0; u < B; ++u)
#pragma unroll
                    for (int q = 0; q < Q; ++q)
                        x[u][q] = *(const f4*)__builtin_assume_aligned(
                            (const char*)lds + (base_bytes[q] + (int)cur.w[2 * u]), 16);
#pragma unroll
                for (int u = 0; u < B; ++u)
#pragma unroll
                    for (int q = 0; q < Q; ++q)
                        acc[k][q] += __uint_as_float(cur.w[2 * u + 1]) * x[u][q];
            }
        }
    }

    // ---- store
    const int32_t* __restrict__ dlut = a.dst_lut + (size_t)tile * a.P4;
    int dofs[Q][4];
#pragma unroll
    for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int d = dlut[pos0[q] + i];
            dofs[q][i] = (active[q] && n0 + nloc[q] < a.N) ? d : -1;
        }
    const int32_t* __restrict__ pm = a.perm + (size_t)bin * K;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int m = pm[k];
        if (m < 0) continue;  // uniform: padding row of the last group
        const float bv = (a.flags & ESCOIN_F_BIAS) ? a.bias[m] : 0.0f;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            float* __restrict__ o = a.out + ((size_t)(n0 + nloc[q]) * a.M + m) * a.EF;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float v = acc[k][q][i] + bv;
                if (a.flags & ESCOIN_F_RELU) v = v > 0.0f ? v : 0.0f;
                if (dofs[q][i] >= 0) o[dofs[q][i]] = v;
            }
        }
    }
}

typedef void (*TiledKernel)(const TiledArgs);

template <int K, int Q, int B>
TiledKernel instance() {
    return sconv_tiled_kernel<K, Q, B>;
}

TiledKernel pick(int K, int Q, int B) {
#define ESCOIN_PICK(KK)                                                   \
    if (K == KK) {                                                        \
        if (Q == 1) return B == 4 ? instance<KK, 1, 4>() : instance<KK, 1, 8>(); \
        return B == 4 ? instance<KK, 2, 4>() : instance<KK, 2, 8>();      \
    }
    ESCOIN_PICK(2)
    ESCOIN_PICK(4)
    ESCOIN_PICK(8)
    ESCOIN_PICK(16)
#undef ESCOIN_PICK
    return nullptr;
}

}  // namespace

bool tiled_variant_exists(int K, int Q, int B) {
    return (K == 2 || K == 4 || K == 8 || K == 16) && (Q == 1 || Q == 2) && (B == 4 || B == 8);
}

}  // namespace escoin

extern "C" int escoin_sconv_forward_tiled(const escoin_conv_desc* desc, const void* plan_host,
                                          const void* d_plan, const float* d_in, float* d_out,
                                          const float* d_bias, uint32_t flags, void* hip_stream) {
    using namespace escoin;
    Dims d;
    int rc = make_dims(desc, &d);
    if (rc != ESCOIN_OK) return rc;
    if (!plan_host || !d_plan || !d_in || !d_out) return ESCOIN_EINVAL;
    if (flags & ~(uint32_t)(ESCOIN_F_BIAS | ESCOIN_F_RELU)) return ESCOIN_EINVAL;
    if ((flags & ESCOIN_F_BIAS) && !d_bias) return ESCOIN_EINVAL;
    PlanHeader h;
    h = *(const PlanHeader*)plan_host;
    if (h.magic != kPlanMagic || h.version != kPlanVersion) return ESCOIN_EINVAL;
    if (h.C != d.C || h.H != d.H || h.W != d.W || h.M != d.M || h.R != d.R || h.S != d.S ||
        h.stride != d.stride || h.pad != d.pad || h.E != d.E || h.F != d.F)
        return ESCOIN_EINVAL;
    TiledKernel kern = pick(h.K, h.Q, h.B);
    if (!kern) return ESCOIN_EINVAL;
    const int threads = 64 * h.WQ * h.WM;
    if (threads > 512 || threads <= 0) return ESCOIN_EINVAL;
    // the kernel's index arithmetic relies on these plan invariants
    if (h.P4 % 4 || h.plane_stride % 4 || h.P4 > h.plane_stride || h.NB < 1 || h.CC < 1 ||
        h.lut_entries != h.n_slots * h.plane_stride || h.WQ * 64 * h.Q * 4 < h.NB * h.P4)
        return ESCOIN_EINVAL;

    const char* base = (const char*)d_plan;
    TiledArgs a;
    a.in = d_in; a.out = d_out; a.bias = d_bias;
    a.src_lut = (const int32_t*)(base + h.off_src_lut);
    a.dst_lut = (const int32_t*)(base + h.off_dst_lut);
    a.perm = (const int32_t*)(base + h.off_perm);
    a.seg = (const uint32_t*)(base + h.off_seg);
    a.rec = (const uint32_t*)(base + h.off_rec);
    a.N = d.N; a.C = d.C; a.HW = d.H * d.W; a.M = d.M; a.EF = d.E * d.F;
    a.WM = h.WM; a.WQ = h.WQ; a.CC = h.CC; a.NB = h.NB;
    a.n_tiles = h.n_tiles; a.n_mgroups = h.n_mgroups; a.n_chunks = h.n_chunks;
    const long long n_in_tiles = (long long)h.n_tiles * ((d.N + h.NB - 1) / h.NB);
    const long long blocks = (n_in_tiles + 7) / 8 * 8 * h.n_mgroups;
    if (blocks > 0x7FFFFFFFll) return ESCOIN_ERANGE;
    a.n_in_tiles = (int)n_in_tiles;
    a.plane_stride = h.plane_stride; a.P4 = h.P4; a.lut_entries = h.lut_entries;
    a.flags = flags;

    const size_t lds_bytes = (size_t)h.lds_floats * 4;
    if (lds_bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)kern,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return ESCOIN_EHIP;
    }
    return launch(kern, dim3((unsigned)blocks), dim3(threads), lds_bytes, (hipStream_t)hip_stream, a);
}

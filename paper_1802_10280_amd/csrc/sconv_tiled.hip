// LDS-tiled sconv for gfx950.
//
// One workgroup owns a tile of output positions (a band of rows of one image, or several
// small images) and a group of accumulator rows, and walks the input channels in chunks:
//   stage   the chunk's input window goes from the UNPADDED input to LDS: the window is the flat
//           padded array of Section 3.1, one plane per stride phase, and its frame of zeros is
//           never fetched, so pad_in is folded into the staging.  Either through registers and
//           a table of (input word -> LDS word), the frame being cleared once at kernel start;
//           or, where every run of four input words lands on one aligned 16-byte LDS slot, by
//           global -> LDS copies that fill every slot with input or with zeros.  The chunk's CSR
//           records (LDS offset, value) of the workgroup's rows are copied to LDS as well
//           (Section 3.3 keeps colidx/value on chip).  Both are double-buffered: chunk i+1 is on
//           its way while chunk i is consumed, with one barrier per chunk;
//   compute Algorithm 2 on that window: a wave walks the records of its K accumulator rows
//           (every lane reads the same record: an LDS broadcast); a lane owns 4 consecutive
//           positions of the flat array per position run.  For each record it fetches the
//           aligned 16 bytes that hold most of the four words val multiplies; the words that
//           fall into the neighbouring 16-byte group are taken from the neighbouring lane,
//           which has just fetched them, with a lane shift (DPP) instead of a second LDS
//           read.  Records are grouped by that alignment class so the shift is static code;
//   store   positions that are real outputs go to out[n][m][h][w] through the second table,
//           with the optional bias + ReLU epilogue: a row that is whole in its wave as soon as
//           the wave has finished it in the last chunk; an output channel whose nonzeros are
//           split over several accumulator rows (of different waves) after its partial sums
//           have met in LDS.
// Consecutive lanes own consecutive positions (the data-to-thread mapping of Section 3.2), so
// LDS reads are conflict-free and output stores are contiguous along w.
#include <algorithm>
#include <mutex>
#include <vector>

#include "common.h"
#include "plan.h"

namespace escoin {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

struct TiledArgs {
    const float* in;
    float* out;
    const float* bias;
    const StageSlot* stage;
    const DmaSlot* dma;
    const float* zero16;
    const LaneSlot* lanes;
    const int32_t* dst_lut;
    const RowSlot* slots;
    const int32_t* group_regions;
    const uint32_t* blk;
    const uint32_t* seg;
    const uint32_t* rec;
    int N, C, HW, M, EF;
    int WM, WQ, CC, CC0, NB, CS, WW, MB;
    int n_tiles, n_mgroups, n_chunks, n_in_tiles;
    int plane_stride, P4, n_items, buf_floats, tail_floats, rec_buf_bytes, region_floats, used_slots, n_dma, win_slots;
    uint32_t flags;
};

namespace {

// Plan data that is wave-uniform and read-only for the whole launch is viewed through the
// constant address space, which keeps those loads on the scalar data path.
typedef const uint32_t __attribute__((address_space(4))) * cu32p;
typedef const int32_t __attribute__((address_space(4))) * ci32p;
__device__ __forceinline__ cu32p as_const(const uint32_t* p) { return (cu32p)(uintptr_t)p; }
__device__ __forceinline__ ci32p as_const(const int32_t* p) { return (ci32p)(uintptr_t)p; }

// acc += w * (x of the next lane) / (x of the previous lane): the lane shift rides on the
// multiply-add itself (its DPP form), so the neighbour's word costs no instruction of its own.
// A lane with no such neighbour (63, resp. 0) multiplies a zero.  The shifted operand comes
// straight from an LDS read; nothing here writes it with a vector instruction, which that form
// would need two idle issue slots after.
__device__ __forceinline__ float fma_next_lane(float acc, float x, float w) {
    asm("v_fmac_f32_dpp %0, %1, %2 wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:0" : "+v"(acc) : "v"(x), "v"(w));
    return acc;
}
__device__ __forceinline__ float fma_prev_lane(float acc, float x, float w) {
    asm("v_fmac_f32_dpp %0, %1, %2 wave_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:0" : "+v"(acc) : "v"(x), "v"(w));
    return acc;
}

// acc += w * (the four words a record of alignment class CLS multiplies), given the aligned
// group `x` this lane fetched (its neighbours fetched the adjacent groups at the same time).
template <int CLS>
__device__ __forceinline__ void fma_window(f4& acc, f4 x, float w) {
    if (CLS == 0) {
        acc += w * x;
    } else if (CLS == 1) {
        acc[0] += w * x[1]; acc[1] += w * x[2]; acc[2] += w * x[3];
        acc[3] = fma_next_lane(acc[3], x[0], w);
    } else if (CLS == 2) {
        acc[0] += w * x[2]; acc[1] += w * x[3];
        acc[2] = fma_next_lane(acc[2], x[0], w);
        acc[3] = fma_next_lane(acc[3], x[1], w);
    } else {
        acc[0] = fma_prev_lane(acc[0], x[3], w);
        acc[1] += w * x[0]; acc[2] += w * x[1]; acc[3] += w * x[2];
    }
}

// Issue priority of this wave (0..3, higher is served first); `p` folds to a constant once the
// calling loop is unrolled, and the instruction takes an immediate.
__device__ __forceinline__ void set_prio(int p) {
    switch (p) {
        case 0: __builtin_amdgcn_s_setprio(0); break;
        case 1: __builtin_amdgcn_s_setprio(1); break;
        case 2: __builtin_amdgcn_s_setprio(2); break;
        default: __builtin_amdgcn_s_setprio(3); break;
    }
}

constexpr uint32_t kKeyOffsetMask = (1u << kKeyOffsetBits) - 1;

// Waits until at most n vector-memory operations of this wave are outstanding (and for every
// LDS / scalar operation); n is wave-uniform.  The instruction takes an immediate.
__device__ __forceinline__ void wait_vmcnt_at_most(int n) {
    // simm16: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14; expcnt is left alone (7)
#define ESCOIN_WAIT(N) case N: __builtin_amdgcn_s_waitcnt(((N) & 15) | (7 << 4) | (((N) >> 4) << 14)); break;
    switch (n) {
        ESCOIN_WAIT(1) ESCOIN_WAIT(2) ESCOIN_WAIT(3) ESCOIN_WAIT(4) ESCOIN_WAIT(5) ESCOIN_WAIT(6) ESCOIN_WAIT(7)
        ESCOIN_WAIT(8) ESCOIN_WAIT(9) ESCOIN_WAIT(10) ESCOIN_WAIT(11) ESCOIN_WAIT(12)
        default: __builtin_amdgcn_s_waitcnt(0 | (7 << 4)); break;  // 0, or more than listed: everything
    }
#undef ESCOIN_WAIT
}

template <int B>
struct Batch {
    u4 w[B / 2];  // B x {LDS byte offset, value bits}, two records per 16 bytes
};

// Every lane reads the same 8*B bytes: an LDS broadcast.
template <int B>
__device__ __forceinline__ Batch<B> read_batch(const char* lds_bytes, int addr) {
    Batch<B> b;
#pragma unroll
    for (int i = 0; i < B / 2; ++i)
        b.w[i] = *(const u4*)__builtin_assume_aligned(lds_bytes + addr + 16 * i, 16);
    return b;
}

// byte distance between the groups one lane reads in consecutive position runs of a tile that
// holds a single image (62 groups of 16 bytes)
constexpr int kRunStrideBytes = 62 * 16;

// A tile's groups are consecutive in LDS whatever image they belong to, so a lane's groups in
// consecutive position runs are kRunStrideBytes apart and the second LDS read of a record needs no
// address arithmetic of its own (an immediate offset).
// VW: input words per staging load (4: the plan dealt the window words in runs of four
// consecutive, 16-byte aligned input words and the input pointer is 16-byte aligned; 1: any plan).
// VW = 16: the window is not staged through registers at all; every 16-byte slot of a window
// buffer is filled by a global -> LDS copy (a run of four input words, or zeros), which needs
// the plan's DmaSlot table.
template <int K, int Q, int B, int VW>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(4, 4))) void sconv_tiled_kernel(const TiledArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    char* const lds_bytes = (char*)lds;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wq = wave % a.WQ, wm = wave / a.WQ;
    const int nthreads = blockDim.x;

    // Workgroup -> (input tile, output-channel group, channel split).  Consecutive workgroup
    // ids land on different XCDs (id mod 8).  The jobs, ordered tile-major, are cut into 8
    // contiguous, equally long ranges, one per XCD: every XCD gets the same number of
    // workgroups, and the workgroups that read one input tile mostly run on one XCD, one after
    // the other, sharing the tile through its L2.
    const int xcd = blockIdx.x & 7, slot_j = blockIdx.x >> 3;
    const int jobs = a.n_in_tiles * a.n_mgroups * a.CS;
    const int jq = jobs >> 3, jr = jobs & 7;
    if (slot_j >= jq + (xcd < jr ? 1 : 0)) return;  // whole workgroup leaves before any barrier
    const int job = xcd * jq + (xcd < jr ? xcd : jr) + slot_j;
    // Job order: (block of channel groups, input tile, group inside the block, channel split).
    // With one block this is tile-major; with MB blocks an XCD's range spans 1/MB of the groups,
    // hence of the records, which matters where the records outweigh the input.
    const int per_block = (a.n_mgroups + a.MB - 1) / a.MB;           // groups of a full block
    const int block_jobs = a.n_in_tiles * per_block * a.CS;
    const int blk_i = job / block_jobs;
    const int in_block = min(per_block, a.n_mgroups - blk_i * per_block);  // the last block may be short
    const int rj = job - blk_i * block_jobs;
    const int cs = rj % a.CS;
    const int t_in = (rj / a.CS) / in_block;
    const int mg = blk_i * per_block + (rj / a.CS) - t_in * in_block;
    const int tile = t_in % a.n_tiles;
    const int n0 = (t_in / a.n_tiles) * a.NB;

    // ---- this lane's group and positions in each of the wave's position runs
    int base_bytes[Q], nloc[Q], pos0[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const LaneSlot ls = a.lanes[((size_t)(wq * Q + q)) * 64 + lane];
        base_bytes[q] = ls.base_word * 4;
        nloc[q] = ls.nloc;
        pos0[q] = ls.pos0;
    }
    const int base0 = base_bytes[0];

    // ---- this thread's share of the staging work (the same for every chunk), from the plan
    constexpr bool DMA = VW == 16;
    constexpr int kRuns = DMA ? 1 : kMaxItemsPerThread / VW;
    int st_src[kRuns];  // per run of VW words: offset from the chunk's first input word, -1 = none
    // bits 0..17: LDS byte offset of the word inside a window buffer; 18..31: channel in the chunk
    uint32_t st_key[kMaxItemsPerThread];
    // DMA staging: this wave issues the copies wave, wave + nwaves, ...; per copy, this lane's
    // slot: where its four words come from (-1: zeros) and their channel inside the chunk
    int dma_src[kMaxDmaPerWave], dma_chan[kMaxDmaPerWave];
    const int nwaves = nthreads >> 6;
    if (DMA) {
        const int src_end = min(a.NB, a.N - n0) * a.C * a.HW;
#pragma unroll
        for (int i = 0; i < kMaxDmaPerWave; ++i) {
            const int j = wave + i * nwaves;
            DmaSlot v;
            v.src = -1;
            v.chan = 0;
            if (j < a.n_dma) v = a.dma[((size_t)tile * a.n_dma + j) * 64 + lane];
            dma_src[i] = v.src < src_end ? v.src : -1;
            dma_chan[i] = v.chan;
        }
    } else {
        const StageSlot* __restrict__ sl = a.stage + (size_t)tile * kMaxItemsPerThread * nthreads + tid;
        // words of images past the end of the batch (ragged last image group) are not staged
        const int src_end = min(a.NB, a.N - n0) * a.C * a.HW;
        // Only the slots the tile uses are read, and where every run of four words is
        // committed with one 16-byte LDS write only the run's first slot matters: the table is
        // read by every workgroup, so for layers of few chunks it weighs as much as the input.
        const bool run_heads_only = VW == 4 && a.WW == 4;
#pragma unroll
        for (int j = 0; j < kMaxItemsPerThread; ++j) {
            StageSlot v;
            v.src = -1;
            v.key = 0;
            if (j < a.used_slots && (j % 4 == 0 || !run_heads_only)) v = sl[(size_t)j * nthreads];
            if (j % VW == 0) st_src[j / VW] = v.src < src_end ? v.src : -1;
            st_key[j] = v.key;
        }
    }
    const int win_bytes = a.buf_floats * 4;
    const int rec_base = (2 * a.buf_floats + a.tail_floats) * 4;  // first record buffer
    cu32p blkp = as_const(a.blk) + (size_t)mg * a.n_chunks * 2;
    constexpr int kSeg = 1 + K * kClasses;
    cu32p segp = as_const(a.seg) + ((size_t)mg * a.WM + wm) * a.n_chunks * kSeg;

    float st_val[kMaxItemsPerThread];

    // Issue the global loads of chunk `ch`: window words into registers, the record block
    // straight into record buffer `buf` (global_load ... lds, 16 bytes per lane, no registers).
    // chunk `ch` holds the channels c0 .. c0 + ccur - 1: the first chunk CC0 of them, the others CC
    auto chunk_c0 = [&](int ch) { return ch == 0 ? 0 : a.CC0 + (ch - 1) * a.CC; };
    auto chunk_len = [&](int ch) { return ch == 0 ? a.CC0 : min(a.CC, a.C - chunk_c0(ch)); };
    auto fetch = [&](int ch, int buf) {
        const int c0 = chunk_c0(ch);
        const int ccur = chunk_len(ch);
        const float* __restrict__ src = a.in + ((size_t)n0 * a.C + c0) * a.HW;
        if (DMA) {
            char* const win = lds_bytes + buf * win_bytes;
#pragma unroll
            for (int i = 0; i < kMaxDmaPerWave; ++i) {
                const int j = wave + i * nwaves;  // wave-uniform
                if (j < a.n_dma) {
                    const bool has = dma_src[i] >= 0 && dma_chan[i] < ccur;
                    const float* g = has ? src + dma_src[i] : a.zero16;
                    if (j * 64 + lane < a.win_slots)  // lane 0 always passes: the copy is always issued
                        __builtin_amdgcn_global_load_lds((const void*)g,
                                                         (void __attribute__((address_space(3)))*)(win + 1024 * j), 16, 0, 0);
                }
            }
        }
#pragma unroll
        for (int r = 0; r < (DMA ? 0 : kRuns); ++r)
            if (st_src[r] >= 0 && (int)(st_key[r * VW] >> kKeyOffsetBits) < ccur) {
                if (VW == 4) {
                    const f4 v = *(const f4*)__builtin_assume_aligned(src + st_src[r], 16);
                    st_val[4 * r] = v[0]; st_val[4 * r + 1] = v[1]; st_val[4 * r + 2] = v[2]; st_val[4 * r + 3] = v[3];
                } else {
                    st_val[r] = src[st_src[r]];
                }
            }
        const char* rsrc = (const char*)(a.rec + (size_t)blkp[2 * ch] * (2 * B));
        const int units = (int)blkp[2 * ch + 1] * (B / 2);  // 16-byte units in the block
        char* const rb = lds_bytes + rec_base + buf * a.rec_buf_bytes;
        for (int u0 = wave * 64; u0 < units; u0 += nthreads) {  // u0: wave-uniform
            if (u0 + lane < units)
                __builtin_amdgcn_global_load_lds((const void*)(rsrc + 16 * (size_t)(u0 + lane)),
                                                 (void __attribute__((address_space(3)))*)(rb + 16 * u0), 16, 0, 0);
        }
    };
    // Write the window words fetch(ch) loaded into window buffer `buf`.
    auto commit = [&](int ch, int buf) {
        if (DMA) return;
        const int ccur = chunk_len(ch);
        char* const win = lds_bytes + buf * win_bytes;
        if (VW == 4 && a.WW == 4) {  // every run lands on 16 aligned, consecutive LDS bytes
#pragma unroll
            for (int r = 0; r < kRuns; ++r)
                if (st_src[r] >= 0 && (int)(st_key[4 * r] >> kKeyOffsetBits) < ccur) {
                    f4 v;
                    v[0] = st_val[4 * r]; v[1] = st_val[4 * r + 1]; v[2] = st_val[4 * r + 2]; v[3] = st_val[4 * r + 3];
                    *(f4*)__builtin_assume_aligned(win + (st_key[4 * r] & kKeyOffsetMask), 16) = v;
                }
            return;
        }
#pragma unroll
        for (int j = 0; j < kMaxItemsPerThread; ++j)
            if (st_src[j / VW] >= 0 && (int)(st_key[j] >> kKeyOffsetBits) < ccur)
                *(float*)(win + (st_key[j] & kKeyOffsetMask)) = st_val[j];
    };

    // This workgroup's chunks: cs, cs + CS, ... (all of them unless the channels are split).
    fetch(cs, 0);
    // With a single chunk to do, the output offsets are asked for now, next to the first
    // fetch, instead of after it: one memory round trip less in a short launch.
    const bool single_chunk = cs + a.CS >= a.n_chunks;
    int early_dst[Q][4];
    if (single_chunk) {
#pragma unroll
        for (int q = 0; q < Q; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int dd = -1;
                if (pos0[q] >= 0 && n0 + nloc[q] < a.N) dd = a.dst_lut[(size_t)tile * a.P4 + pos0[q] + i];
                early_dst[q][i] = dd;
            }
    }
    if (DMA) {
        // The copies need no registers, so the second chunk is asked for right away as well:
        // two chunks are on their way before the first FMA.  Every slot of the channel planes
        // is rewritten by every chunk's copies (input or zeros); only the stretches behind
        // them are cleared here, once.
        if (!single_chunk) fetch(cs + a.CS, 1);
        for (int i = 4 * a.win_slots + 4 * tid; i < a.buf_floats; i += 4 * nthreads)
            *(f4*)__builtin_assume_aligned(&lds[i], 16) = (f4)(0.0f);
        for (int i = a.buf_floats + 4 * a.win_slots + 4 * tid; i < 2 * a.buf_floats + a.tail_floats; i += 4 * nthreads)
            *(f4*)__builtin_assume_aligned(&lds[i], 16) = (f4)(0.0f);
        // Wait for the first chunk only.  The vector-memory counter counts down in issue order,
        // so the first chunk is complete once no more operations are outstanding than this wave
        // issued after it: its copies of the second chunk (window, then records), each of which
        // is issued whatever the lanes do (lane 0 always takes part).
        int later = 0;
        if (!single_chunk) {
            const int units = (int)blkp[2 * (cs + a.CS) + 1] * (B / 2);
            later = (wave < a.n_dma ? (a.n_dma - wave + nwaves - 1) / nwaves : 0) +
                    (units > wave * 64 ? (units - wave * 64 + nthreads - 1) / nthreads : 0);
        }
        wait_vmcnt_at_most(later);
    } else {
        // The frame of zeros never changes: clear the window buffers and the tail once; from
        // here on only words that hold input are rewritten, chunk after chunk.
        for (int i = 4 * tid; i < 2 * a.buf_floats + a.tail_floats; i += 4 * nthreads)  // both are multiples of 4
            *(f4*)__builtin_assume_aligned(&lds[i], 16) = (f4)(0.0f);
        __syncthreads();
        commit(cs, 0);
        __builtin_amdgcn_s_waitcnt(0);  // this wave's record copies have landed
    }
    if (single_chunk) {  // the staging registers are free for good: they take the output offsets
#pragma unroll
        for (int q = 0; q < Q; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) st_val[q * 4 + i] = __int_as_float(early_dst[q][i]);
    }
    __syncthreads();

    f4 acc[K][Q];
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
        for (int q = 0; q < Q; ++q) acc[k][q] = (f4)(0.0f);

    // The wave's K accumulator rows: output channel, and how a channel whose nonzeros are
    // split over several accumulator rows of the workgroup is put together after the last chunk.
    const int bin = mg * a.WM + wm;
    RowSlot rs[K];
    {
        ci32p sp = as_const((const int32_t*)a.slots) + (size_t)bin * K * 4;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            rs[k].m = sp[4 * k];
            rs[k].my_region = sp[4 * k + 1];
            rs[k].first_region = sp[4 * k + 2];
            rs[k].n_partials = sp[4 * k + 3];
        }
    }
    // With split channels every workgroup adds its partial sums to an output that was cleared
    // before the launch; the first split brings the bias and the clamp is a pass of its own.
    const bool split = a.CS > 1;
    const int32_t* __restrict__ dlut = a.dst_lut + (size_t)tile * a.P4;
    // Where this lane's positions go inside an E*F output plane (-1: not an output).  The
    // offsets are fetched at the start of the last chunk, when the staging registers are free
    // (nothing is fetched any more), and live there until the stores.
    auto load_dst = [&]() {
#pragma unroll
        for (int q = 0; q < Q; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int dd = -1;
                if (pos0[q] >= 0 && n0 + nloc[q] < a.N) dd = dlut[pos0[q] + i];
                st_val[q * 4 + i] = __int_as_float(dd);
            }
    };
    static_assert(Q * 4 <= kMaxItemsPerThread, "the output offsets borrow the staging registers");
    // Row k of this wave is complete: epilogue and store (or atomic add with split channels).
    auto store_row = [&](int k, const f4(&ak)[Q]) {
        const int m = rs[k].m;
        const float bv = ((a.flags & ESCOIN_F_BIAS) && cs == 0) ? a.bias[m] : 0.0f;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            int dofs[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) dofs[i] = __float_as_int(st_val[q * 4 + i]);
            float* __restrict__ o = a.out + ((size_t)(n0 + nloc[q]) * a.M + m) * a.EF;
            f4 v = ak[q] + bv;
            if (split) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (dofs[i] >= 0) unsafeAtomicAdd(o + dofs[i], v[i]);
                continue;
            }
            if (a.flags & ESCOIN_F_RELU) {
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = v[i] > 0.0f ? v[i] : 0.0f;
            }
            // A lane whose four positions are four consecutive, 16-byte aligned output words
            // stores them at once.
            const bool quad = (a.EF & 3) == 0 && ((uintptr_t)a.out & 15) == 0 && dofs[0] >= 0 && (dofs[0] & 3) == 0 &&
                              dofs[1] == dofs[0] + 1 && dofs[2] == dofs[0] + 2 && dofs[3] == dofs[0] + 3;
            if (quad) {
                *(f4*)__builtin_assume_aligned(o + dofs[0], 16) = v;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (dofs[i] >= 0) o[dofs[i]] = v[i];
            }
        }
    };

    // Algorithm 2 over chunk `ch`'s nonzeros of the wave's K rows, on window buffer `buf`.
    // LAST: the workgroup's last chunk, after which a row that is whole in this wave is stored.
    auto compute = [&](int ch, int buf, auto last_tag) {
        constexpr bool LAST = decltype(last_tag)::value;
        const int bufb = buf * win_bytes;
        cu32p sg = segp + (size_t)ch * kSeg;
        // all segment lengths of the chunk in one scalar load, not one load per segment
        uint32_t cnts[kSeg];
#pragma unroll
        for (int i = 0; i < kSeg; ++i) cnts[i] = sg[i];
        int rptr = rec_base + buf * a.rec_buf_bytes + (int)cnts[0] * (8 * B);
        // Two record batches ping-pong between `ra` and `rb`: while one is consumed the next
        // one is already being read, and no register copies are needed to rotate them.
        Batch<B> ra = read_batch<B>(lds_bytes, rptr), rb;
        auto step = [&](auto cls_tag, f4(&ak)[Q], const Batch<B>& cur, Batch<B>& nxt) {
            constexpr int CLS = decltype(cls_tag)::value;
            rptr += 8 * B;
            nxt = read_batch<B>(lds_bytes, rptr);  // at worst the spare batch after the block
            f4 x[B][Q];
#pragma unroll
            for (int u = 0; u < B; ++u) {
                const int at = base0 + bufb + (int)cur.w[u >> 1][(u & 1) * 2];
#pragma unroll
                for (int q = 0; q < Q; ++q)
                    x[u][q] = *(const f4*)__builtin_assume_aligned(lds_bytes + at + q * kRunStrideBytes, 16);
            }
#pragma unroll
            for (int u = 0; u < B; ++u)
#pragma unroll
                for (int q = 0; q < Q; ++q)
                    fma_window<CLS>(ak[q], x[u][q], __uint_as_float(cur.w[u >> 1][(u & 1) * 2 + 1]));
        };
        auto run_class = [&](auto cls_tag, f4(&ak)[Q], int cnt) {
            int b = 0;
#pragma unroll 1
            for (; b + 2 <= cnt; b += 2) {
                step(cls_tag, ak, ra, rb);
                step(cls_tag, ak, rb, ra);
            }
            if (b < cnt) {
                step(cls_tag, ak, ra, rb);
                ra = rb;
            }
        };
        // The SIMD's arbiter favours its oldest wave, so without a hint the youngest waves of
        // the workgroup reach the chunk's barrier long after the oldest ones, which then idle.
        // A wave lowers its issue priority as it advances through its segments: whoever is
        // behind gets served first, and the waves arrive together.
#pragma unroll
        for (int k = 0; k < K; ++k) {
            set_prio(3 - (k * kClasses + 0) / K);
            run_class(std::integral_constant<int, 0>{}, acc[k], (int)cnts[1 + k * kClasses + 0]);
            set_prio(3 - (k * kClasses + 1) / K);
            run_class(std::integral_constant<int, 1>{}, acc[k], (int)cnts[1 + k * kClasses + 1]);
            set_prio(3 - (k * kClasses + 2) / K);
            run_class(std::integral_constant<int, 2>{}, acc[k], (int)cnts[1 + k * kClasses + 2]);
            set_prio(3 - (k * kClasses + 3) / K);
            run_class(std::integral_constant<int, 3>{}, acc[k], (int)cnts[1 + k * kClasses + 3]);
            // The stores of rows 0 .. K-2 run under the arithmetic of the rows after them
            // instead of all workgroups storing at once at the end of the launch.
            if (LAST && rs[k].m >= 0 && rs[k].my_region < 0 && rs[k].n_partials == 0) store_row(k, acc[k]);
        }
        set_prio(3);
    };

    int ch = cs, it = 0;
    for (; ch + a.CS < a.n_chunks; ch += a.CS, ++it) {
        const int buf = it & 1;
        if (!DMA || it > 0) fetch(ch + a.CS, buf ^ 1);  // (the copies of the second chunk are on their way)
        compute(ch, buf, std::false_type{});
        // The other buffers were last read in the previous iteration, which every wave left
        // through the barrier below: they can be rewritten now.
        commit(ch + a.CS, buf ^ 1);
        __builtin_amdgcn_s_waitcnt(0);  // this wave's record copies have landed
        __syncthreads();
    }
    // the last chunk: nothing to fetch any more, so the staging registers take the output offsets
    // (a workgroup with a single chunk has had them since its prologue)
    if (it > 0) load_dst();
    compute(ch, it & 1, std::true_type{});

    // ---- channels split over several accumulator rows: the lending rows put their partial
    // sums into LDS (the window is no longer needed once every wave has left the last chunk),
    // the owning row adds them up and stores.
    if (as_const(a.group_regions)[mg] > 0) {
        __syncthreads();  // every wave is done with the window and the records
        const int mine = ((wq * Q) * 64 + lane) * 4;  // floats; run q sits q * 256 floats further
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (rs[k].my_region >= 0) {
#pragma unroll
                for (int q = 0; q < Q; ++q)
                    *(f4*)__builtin_assume_aligned(&lds[(size_t)rs[k].my_region * a.region_floats + mine + q * 256], 16) = acc[k][q];
            }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (rs[k].m >= 0 && rs[k].n_partials > 0) {
                for (int i = 0; i < rs[k].n_partials; ++i)
#pragma unroll
                    for (int q = 0; q < Q; ++q)
                        acc[k][q] += *(const f4*)__builtin_assume_aligned(
                            &lds[(size_t)(rs[k].first_region + i) * a.region_floats + mine + q * 256], 16);
                store_row(k, acc[k]);
            }
    }
}

// out[i] = 0 / out[i] = max(out[i], 0): the passes before and after a launch with split channels.
__global__ __launch_bounds__(256) void fill_zero_kernel(float* __restrict__ p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0.0f;
}
__global__ __launch_bounds__(256) void relu_kernel(float* __restrict__ p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float v = p[i];
        p[i] = v > 0.0f ? v : 0.0f;
    }
}

typedef void (*TiledKernel)(const TiledArgs);

// A kernel that wants more than 64 KB of dynamic LDS has to be told so once per device; the
// largest size granted so far is remembered, so that later launches skip the runtime call.
int allow_dynamic_lds(const void* kernel, int bytes) {
    struct Granted { int device; const void* kernel; int bytes; };
    static std::mutex mu;
    static std::vector<Granted> granted;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return ESCOIN_EHIP;
    std::lock_guard<std::mutex> lock(mu);
    for (Granted& gr : granted)
        if (gr.device == dev && gr.kernel == kernel) {
            if (gr.bytes >= bytes) return ESCOIN_OK;
            if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return ESCOIN_EHIP;
            gr.bytes = bytes;
            return ESCOIN_OK;
        }
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return ESCOIN_EHIP;
    granted.push_back({dev, kernel, bytes});
    return ESCOIN_OK;
}

// (K, Q, B) instantiations: the ones that fit 128 VGPRs (four waves per SIMD) without spilling.
#define ESCOIN_TILED_VARIANTS(X) \
    X(1, 1, 2) X(1, 2, 2) X(2, 1, 2) X(2, 1, 4) X(2, 2, 2) X(2, 2, 4) X(4, 1, 2) X(4, 1, 4) X(4, 2, 2) X(8, 1, 2) X(8, 1, 4)

// The instantiations that also exist with 16-byte staging loads (fewer load instructions and
// nine registers less; the ones the layers with W % 4 == 0 of the bundled workloads use).
#define ESCOIN_TILED_WIDE_STAGING(X) X(1, 1, 2) X(2, 1, 2) X(4, 1, 2) X(2, 2, 2) X(4, 2, 2)

TiledKernel pick(int K, int Q, int B, bool wide_staging, bool dma_staging) {
    if (dma_staging) {
#define ESCOIN_PICK(KK, QQ, BB) \
    if (K == KK && Q == QQ && B == BB) return sconv_tiled_kernel<KK, QQ, BB, 16>;
        ESCOIN_TILED_WIDE_STAGING(ESCOIN_PICK)
#undef ESCOIN_PICK
    }
    if (wide_staging) {
#define ESCOIN_PICK(KK, QQ, BB) \
    if (K == KK && Q == QQ && B == BB) return sconv_tiled_kernel<KK, QQ, BB, 4>;
        ESCOIN_TILED_WIDE_STAGING(ESCOIN_PICK)
#undef ESCOIN_PICK
    }
#define ESCOIN_PICK(KK, QQ, BB) \
    if (K == KK && Q == QQ && B == BB) return sconv_tiled_kernel<KK, QQ, BB, 1>;
    ESCOIN_TILED_VARIANTS(ESCOIN_PICK)
#undef ESCOIN_PICK
    return nullptr;
}

}  // namespace

bool tiled_wide_staging_exists(int K, int Q, int B) {
#define ESCOIN_HAS(KK, QQ, BB) \
    if (K == KK && Q == QQ && B == BB) return true;
    ESCOIN_TILED_WIDE_STAGING(ESCOIN_HAS)
#undef ESCOIN_HAS
    return false;
}

// the same instantiations exist with global -> LDS staging
bool tiled_dma_staging_exists(int K, int Q, int B) { return tiled_wide_staging_exists(K, Q, B); }

bool tiled_variant_exists(int K, int Q, int B) {
#define ESCOIN_HAS(KK, QQ, BB) \
    if (K == KK && Q == QQ && B == BB) return true;
    ESCOIN_TILED_VARIANTS(ESCOIN_HAS)
#undef ESCOIN_HAS
    return false;
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
    // 16-byte staging loads need the plan's runs of four words and a 16-byte aligned input
    const bool aligned_in = ((uintptr_t)d_in & 15) == 0 && ((uintptr_t)d_plan & 15) == 0;
    TiledKernel kern = pick(h.K, h.Q, h.B, h.VW == 4 && aligned_in, h.n_dma > 0 && h.VW == 4 && h.WW == 4 && aligned_in);
    if (!kern) return ESCOIN_EINVAL;
    const int threads = 64 * h.WQ * h.WM;
    if (threads > 1024 || threads <= 0) return ESCOIN_EINVAL;
    // the kernel's index arithmetic relies on these plan invariants
    const long long region_bytes = (long long)h.WQ * h.Q * 64 * 16;
    if (h.P4 % 4 || h.plane_stride % 4 || (long long)h.P4 > (long long)h.NB * h.plane_stride || h.NB < 1 || h.CC < 1 ||
        h.CC > kMaxChunkChannels || h.CC0 < 1 || h.CC0 > h.CC ||
        h.n_chunks != (d.C <= h.CC0 ? 1 : 1 + (d.C - h.CC0 + h.CC - 1) / h.CC) ||
        h.WQ < 1 || h.WM < 1 || h.WS < 1 || h.WS > h.WM || h.tail_floats % 4 || h.rec_buf_bytes % 16 || h.front < 4 ||
        h.n_phases < 1 || h.n_phases > kMaxPhases || (h.VW != 1 && h.VW != 4) || (h.WW != 1 && h.WW != 4) || (h.WW == 4 && h.VW != 4) || h.CS < 1 || h.CS > h.n_chunks ||
        h.zero_floats % 4 || h.zero_floats < h.P4 + 16 || h.n_dma < 0 ||
        (h.n_dma > 0 && (h.n_dma != ((h.buf_floats - h.zero_floats) / 4 + 63) / 64 || h.n_dma > kMaxDmaPerWave * (threads / 64))) || h.MB < 1 || h.MB > 8 || h.MB > h.n_mgroups ||
        (long long)h.buf_floats != (long long)h.n_phases * h.CC * h.NB * h.plane_stride + h.zero_floats ||
        (long long)h.n_items * h.CC * h.NB > (long long)kMaxItemsPerThread * threads ||
        (long long)h.buf_floats * 4 >= (1 << kKeyOffsetBits) || h.max_regions < 0 ||
        h.lds_bytes != std::max((long long)(2 * h.buf_floats + h.tail_floats) * 4 + 2 * h.rec_buf_bytes,
                                h.max_regions * region_bytes) ||
        h.lds_bytes > 160 * 1024)
        return ESCOIN_EINVAL;

    const char* base = (const char*)d_plan;
    TiledArgs a;
    a.in = d_in; a.out = d_out; a.bias = d_bias;
    a.stage = (const StageSlot*)(base + h.off_items);
    a.dma = (const DmaSlot*)(base + h.off_dma);
    a.zero16 = (const float*)(base + h.off_zero);
    a.n_dma = h.n_dma;
    a.win_slots = (h.buf_floats - h.zero_floats) / 4;
    a.lanes = (const LaneSlot*)(base + h.off_lanes);
    a.dst_lut = (const int32_t*)(base + h.off_dst_lut);
    a.slots = (const RowSlot*)(base + h.off_perm);
    a.group_regions = (const int32_t*)(base + h.off_perm + (size_t)h.n_mgroups * h.WM * h.K * sizeof(RowSlot));
    a.blk = (const uint32_t*)(base + h.off_blk);
    a.seg = (const uint32_t*)(base + h.off_seg);
    a.rec = (const uint32_t*)(base + h.off_rec);
    a.N = d.N; a.C = d.C; a.HW = d.H * d.W; a.M = d.M; a.EF = d.E * d.F;
    a.WM = h.WM; a.WQ = h.WQ; a.CC = h.CC; a.CC0 = h.CC0; a.NB = h.NB; a.CS = h.CS; a.WW = h.WW; a.MB = h.MB;
    a.n_tiles = h.n_tiles; a.n_mgroups = h.n_mgroups; a.n_chunks = h.n_chunks;
    const long long n_in_tiles = (long long)h.n_tiles * ((d.N + h.NB - 1) / h.NB);
    const long long blocks = (n_in_tiles * h.n_mgroups * h.CS + 7) / 8 * 8;
    if (blocks > 0x7FFFFFFFll) return ESCOIN_ERANGE;
    a.n_in_tiles = (int)n_in_tiles;
    a.plane_stride = h.plane_stride; a.P4 = h.P4; a.n_items = h.n_items;
    a.buf_floats = h.buf_floats; a.tail_floats = h.tail_floats; a.rec_buf_bytes = h.rec_buf_bytes;
    a.region_floats = h.WQ * h.Q * 256;
    {   // staging slots in use: the tile's runs of VW words are dealt to the threads in turn
        const long long runs = ((long long)h.n_items * h.CC * h.NB + h.VW - 1) / h.VW;
        a.used_slots = (int)std::min<long long>(kMaxItemsPerThread, (runs + threads - 1) / threads * h.VW);
    }
    a.flags = flags;

    const size_t lds_bytes = (size_t)h.lds_bytes;
    if (lds_bytes > 64 * 1024) {
        rc = allow_dynamic_lds((const void*)kern, (int)lds_bytes);
        if (rc != ESCOIN_OK) return rc;
    }
    if (h.CS == 1)
        return launch(kern, dim3((unsigned)blocks), dim3(threads), lds_bytes, (hipStream_t)hip_stream, a);
    const size_t n_out = (size_t)d.N * d.M * d.E * d.F;
    const unsigned sweep_blocks = (unsigned)std::min<size_t>((n_out + 255) / 256, 256 * 8);
    rc = launch(fill_zero_kernel, dim3(sweep_blocks), dim3(256), 0, (hipStream_t)hip_stream, d_out, n_out);
    if (rc != ESCOIN_OK) return rc;
    rc = launch(kern, dim3((unsigned)blocks), dim3(threads), lds_bytes, (hipStream_t)hip_stream, a);
    if (rc != ESCOIN_OK || !(flags & ESCOIN_F_RELU)) return rc;
    return launch(relu_kernel, dim3(sweep_blocks), dim3(256), 0, (hipStream_t)hip_stream, d_out, n_out);
}

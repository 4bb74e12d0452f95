// Layout of the tiled-sconv plan blob (internal; the ABI treats it as opaque bytes).
//
// The plan re-encodes the stretched CSR for the LDS-tiled kernel: the input window of a
// workgroup lives in LDS as a flat padded array (the 1-D padded array of Section 3.1, one
// tile at a time), and each nonzero's stretched offset is stretched a second time into a
// byte offset inside that LDS window, so the kernel's inner loop is Algorithm 2's
// "in[off + f(0,h,w)]" with both terms already resolved to LDS addresses.
#pragma once
#include <stdint.h>

namespace escoin {

constexpr uint32_t kPlanMagic = 0x4E4C5045u;  // "EPLN"
constexpr uint32_t kPlanVersion = 13;
constexpr int kMaxPhases = 16;          // stride*stride phase planes
constexpr int kClasses = 4;             // alignment classes of a tap: (LDS offset) mod 4
constexpr int kMaxItemsPerThread = 12;  // staged input words per thread and chunk

// One input word a thread stages per channel chunk: where it comes from and where it goes.
struct StageSlot {
    int32_t src;   // offset from the first input word of the chunk's first channel of the
                   // workgroup's first image: (image*C + channel)*H*W + offset in the plane;
                   // -1 = this thread has nothing to do in this slot
    uint32_t key;  // bits 0..17: LDS byte offset of the word inside a window buffer;
                   // bits 18..31: channel inside the chunk
};
constexpr int kKeyOffsetBits = 18;                   // a window buffer is below 256 KB
constexpr int kMaxChunkChannels = 1 << (32 - kKeyOffsetBits);

// What one lane of a position run does: the 16-byte group it reads and the outputs it owns.
struct LaneSlot {
    int32_t base_word;  // word index of the group inside a (channel 0) plane set
    int32_t pos0;       // first of its 4 positions inside the tile (index into dst_lut), -1 = nothing to store
    int32_t nloc;       // which of the tile's NB images those positions belong to
};

// One accumulator row of a wave: the output channel it works for and, when the channel's
// nonzeros are split over several accumulator rows (of different waves of the workgroup), how
// the partial sums meet in LDS after the last chunk.
struct RowSlot {
    int32_t m;             // output channel, -1 = unused accumulator row
    int32_t my_region;     // >= 0: this row holds a partial sum and writes it to that LDS region
    int32_t first_region;  // owner of a split channel: its partial sums sit in the regions
    int32_t n_partials;    //   first_region .. first_region + n_partials - 1; 0 = nothing to add
};

struct PlanHeader {
    uint32_t magic, version;
    // layer geometry the plan was built for (N is free: it only sets the grid)
    int32_t C, H, W, M, R, S, stride, pad, E, F;
    // tiling
    int32_t K;   // output channels (CSR rows) accumulated per wave
    int32_t Q;   // position runs (one 16-byte group per lane each) per wave
    int32_t B;   // nonzero records per batch
    int32_t WM;  // waves of a workgroup along the output-channel axis (each has K accumulator rows)
    int32_t WQ;  // waves of a workgroup along the position axis
    int32_t CC;  // input channels staged in LDS per chunk (the first chunk holds CC0 <= CC)
    int32_t NB;  // images per workgroup
    int32_t TH;  // output rows per tile (band height)
    int32_t n_tiles, n_mgroups, n_chunks, n_phases;
    int32_t pitch;         // row pitch of a phase plane in LDS (floats): NB images side by side
    int32_t front;         // unused floats in front of every LDS plane
    int32_t rows_in;       // phase-plane rows held per tile
    int32_t plane_stride;  // floats per (phase, channel) plane set in LDS divided by NB (multiple of 4)
    int32_t P4;            // positions of a tile (all its images) on the pitch grid (multiple of 4)
    int32_t n_items;       // input words per (tile, channel, image): the longest tile's count
    int32_t buf_floats;    // floats of one LDS window buffer (two are allocated): the channel
                           // planes of a chunk followed by zero_floats floats nothing ever writes
    int32_t tail_floats;   // zeroed floats after the second window buffer
    int32_t rec_buf_bytes; // bytes of one LDS record buffer (two are allocated)
    int32_t lds_bytes;     // dynamic LDS size
    int32_t nnz, n_records;
    // section offsets in bytes from the start of the blob
    uint64_t off_items;    // StageSlot [n_tiles][kMaxItemsPerThread][threads of a workgroup]
    uint64_t off_lanes;    // LaneSlot [WQ*Q][64]
    uint64_t off_dst_lut;  // int32 [n_tiles][P4]: offset in an E*F plane, or -1
    uint64_t off_perm;     // RowSlot [n_mgroups*WM][K], then int32 [n_mgroups]: LDS regions of the group
    uint64_t off_blk;      // uint32 [n_mgroups][n_chunks][2]: first batch, batches of the group's block
    uint64_t off_seg;      // uint32 [n_mgroups*WM][n_chunks][1+K*kClasses]: first batch inside the
                           // block, then batches per (row, class)
    uint64_t off_rec;      // {uint32 lds_byte_offset, float value} records, B per batch
    uint64_t total_bytes;
    int32_t CS;      // workgroups that share an output tile; each takes every CS-th channel chunk
    int32_t pitch1;  // columns of one image inside a row of `pitch` floats (pitch = NB * pitch1)
    int32_t VW;      // a thread's staging slots come in runs of VW (4 or 1) consecutive input
                     // words whose first is VW-word aligned inside the input tensor
    int32_t WW;      // 4: every run of VW = 4 words also lands on 4 consecutive, 16-byte aligned LDS
                     // words, so one 16-byte LDS write commits it; else 1
    int32_t WS;          // least number of accumulator rows every output channel is split over
    int32_t CC0;         // channels of the first chunk (a short one lets the first FMAs start early)
    int32_t zero_floats; // floats at the end of every window buffer that stay zero: padding records
                         // point there, so they multiply zeros whatever the input holds
    int32_t max_regions; // most LDS regions (of WQ*Q*1024 bytes) a workgroup needs for partial sums
    int32_t MB;          // the channel groups are cut into MB blocks; the launch order is (block,
                         // tile, group in the block), so that an XCD meets 1/MB of the records
    int32_t n_dma;       // > 0: the window can also be staged without registers, by n_dma wave-wide
                         // 16-byte global -> LDS copies per chunk (every 16-byte slot of a window
                         // buffer is a run of four input words or zeros); 0: no such table
    uint64_t off_dma;    // DmaSlot [n_tiles][n_dma][64]
    uint64_t off_zero;   // 64 zero bytes: what the copy of a slot without input reads
};

// One 16-byte slot of a window buffer as the global -> LDS staging sees it: lane l of copy j
// fills slot 64*j + l.
struct DmaSlot {
    int32_t src;    // like StageSlot::src for the slot's four words; -1 = the slot holds zeros
    int32_t chan;   // channel inside the chunk
};
constexpr int kMaxDmaPerWave = 4;  // copies a wave issues per chunk at most (64 KB per chunk with 16 waves)

}  // namespace escoin

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
constexpr uint32_t kPlanVersion = 5;
constexpr int kMaxSlots = 16;
constexpr int kItemDsts = 4;       // a phase plane is stored under at most 4 alignment shifts
constexpr int kMaxItemsPerThread = 8;   // staged input words per thread and chunk
constexpr int kMaxRecLoadsPerThread = 4;  // 16-byte record units per thread and chunk

// One input word of a tile's window and the LDS words (one per alignment slot of its phase
// plane) that hold it, for channel 0 / image 0 of a window buffer; -1 = unused.
struct StageItem {
    int32_t src;              // offset inside an H*W input plane
    int32_t dst[kItemDsts];   // word index inside a window buffer
};

struct PlanHeader {
    uint32_t magic, version;
    // layer geometry the plan was built for (N is free: it only sets the grid)
    int32_t C, H, W, M, R, S, stride, pad, E, F;
    // tiling
    int32_t K;   // output channels (CSR rows) accumulated per wave
    int32_t Q;   // float4 position groups per lane
    int32_t B;   // nonzero records per batch
    int32_t WM;  // waves of a workgroup along the output-channel axis
    int32_t WQ;  // waves of a workgroup along the position axis
    int32_t CC;  // input channels staged in LDS per chunk
    int32_t NB;  // images per workgroup
    int32_t TH;  // output rows per tile (band height)
    int32_t n_tiles, n_mgroups, n_chunks, n_slots;
    int32_t pitch;         // row pitch of a phase plane in LDS (floats, multiple of 4)
    int32_t rows_in;       // phase-plane rows held per tile
    int32_t plane_stride;  // floats per (slot, channel, image) plane in LDS (multiple of 4)
    int32_t P4;            // output positions per image and tile on the pitch grid (multiple of 4)
    int32_t n_items;       // StageItems per tile (shorter tiles are padded with src = -1)
    int32_t buf_floats;    // floats of one LDS window buffer (two are allocated)
    int32_t tail_floats;   // zeroed floats after the second window buffer
    int32_t rec_buf_bytes; // bytes of one LDS record buffer (two are allocated)
    int32_t lds_bytes;     // dynamic LDS size
    int32_t nnz, n_records;
    int32_t reserved0;
    // section offsets in bytes from the start of the blob
    uint64_t off_items;    // StageItem [n_tiles][n_items]
    uint64_t off_dst_lut;  // int32 [n_tiles][P4]: offset in an E*F plane, or -1
    uint64_t off_perm;     // int32 [n_mgroups*WM][K]: output channel of each accumulator row, or -1
    uint64_t off_blk;      // uint32 [n_mgroups][n_chunks][2]: first batch, batches of the group's block
    uint64_t off_seg;      // uint32 [n_mgroups*WM][n_chunks][1+K]: first batch inside the block, batches per row
    uint64_t off_rec;      // {uint32 lds_byte_offset, float value} records, B per batch
    uint64_t total_bytes;
    uint32_t reserved[8];
};

}  // namespace escoin

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
constexpr uint32_t kPlanVersion = 3;
constexpr int kMaxSlots = 16;

struct PlanHeader {
    uint32_t magic, version;
    // layer geometry the plan was built for (N is free: it only sets the grid)
    int32_t C, H, W, M, R, S, stride, pad, E, F;
    // tiling
    int32_t K;   // output channels (CSR rows) accumulated per wave
    int32_t Q;   // float4 position groups per lane
    int32_t B;   // nonzero records per batch (one scalar load)
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
    int32_t lut_entries;   // n_slots * plane_stride
    int32_t lds_floats;    // dynamic LDS size in floats
    int32_t nnz, n_records;
    // section offsets in bytes from the start of the blob
    uint64_t off_src_lut;  // int32 [n_tiles][n_slots][plane_stride]: offset in an H*W plane, or -1
    uint64_t off_dst_lut;  // int32 [n_tiles][P4]: offset in an E*F plane, or -1
    uint64_t off_perm;     // int32 [n_mgroups*WM][K]: output channel of each accumulator row, or -1
    uint64_t off_seg;      // uint32 [n_mgroups*WM][n_chunks][1+K]: first batch, batches per row
    uint64_t off_rec;      // {uint32 lds_byte_offset, float value} records, B per batch
    uint64_t total_bytes;
    uint32_t reserved[8];
};

}  // namespace escoin

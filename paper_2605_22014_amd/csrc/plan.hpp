// Internal structures shared by the host planner, the C ABI and the kernels.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "liver.h"

namespace liver {

// ---- device-side descriptor -------------------------------------------------
// One strided 2-D copy in "units".  A unit is 16 bytes on the vector paths and
// one element on the element paths (unaligned pieces of odd-sized models).
enum DevOp : uint32_t {
    DOP_COPY_V16 = 0,     // 16 B in, 16 B out
    DOP_COPY_E2 = 1,      // one 2-byte element
    DOP_COPY_E4 = 2,      // one 4-byte element
    DOP_CAST_V4 = 3,      // 4 fp32 (16 B) in, 4 bf16 (8 B) out
    DOP_CAST_E = 4,       // one fp32 in, one bf16 out
    DOP_ZERO_V16 = 5,     // 16 B of zeros out
    DOP_ZERO_E2 = 6,
    DOP_ZERO_E4 = 7,
    DOP_COPYCAST_V4 = 8,  // 4 fp32 in; 4 fp32 out to B and 4 bf16 out to C (source read once)
};

struct DevDesc {
    uint64_t a_off;       // byte offset of the piece in its source buffer
    uint64_t b_off;       // byte offset of the piece in its target buffer
    uint64_t c_off;       // second target (COPYCAST only)
    uint32_t a_stride;    // bytes between rows (unused when run == total)
    uint32_t b_stride;
    uint32_t c_stride;
    uint32_t run;         // units per row
    uint32_t total;       // rows * run
    uint32_t tile_begin;  // first tile of this descriptor inside its pass
    uint16_t a_buf;       // index into the pass's buffer table (unused for ZERO)
    uint16_t b_buf;
    uint16_t c_buf;
    uint16_t op;          // DevOp
    uint64_t reserved;
};
static_assert(sizeof(DevDesc) == 64, "descriptor layout is shared with the kernels");

#ifndef LIVER_TILE_UNITS
#define LIVER_TILE_UNITS 4096
#endif
constexpr uint32_t TILE_UNITS = LIVER_TILE_UNITS;  // units per tile: 64 KiB on the 16-byte paths
constexpr int MAX_PASS_BUFS = 400;     // buffer pointers carried in one launch's arguments

struct BufRef {
    int8_t side;  // 0 source world, 1 target world, 2 staging chunk
    int8_t kind;
    int32_t rank;
    bool operator==(const BufRef& o) const { return side == o.side && kind == o.kind && rank == o.rank; }
};

// One kernel launch: a range of descriptors plus the buffers they touch.
struct Pass {
    uint32_t desc_begin = 0, desc_count = 0;  // range in List::dev
    uint32_t n_tiles = 0;
    std::vector<BufRef> bufs;
};

struct List {
    std::vector<liver_desc_t> pub;      // what the planner decided (inspection, tests)
    std::vector<DevDesc> dev;           // lowered for the kernels
    std::vector<Pass> passes;
    std::vector<uint32_t> chunk_pass;   // staged lists: passes of chunk k are [chunk_pass[k], chunk_pass[k+1])
    uint64_t dev_offset = 0;            // byte offset of dev[] inside the plan's device table
    int64_t hbm_read = 0, hbm_written = 0;  // bytes the lowered descriptors read / write
};

struct Bucket {
    int64_t start = 0, padded = 0;  // flat offset and padded size
    int64_t slice = 0;              // padded / DP: what one DP rank holds of it
    int64_t prefix = 0;             // sum of the slices of the buckets before it = offset in a DP rank's buffer
};

struct StageSize {
    int64_t n_local = 0, n_pad = 0, S = 0;  // end of the last parameter, padded size, N_pad / DP
    std::vector<Bucket> buckets;            // the flat buffer is a sequence of buckets (at least one)
    std::vector<int64_t> bounds;            // sorted flat offsets where the owning (bucket, DP rank) changes
};

}  // namespace liver

struct liver_plan {
    liver_model_spec_t spec{};
    liver_layout_t src{}, dst{};
    size_t chunk_bytes = 0;
    std::vector<liver::StageSize> src_stage, dst_stage;  // per pp: the dense buffers (kinds 0..3)
    std::vector<liver::StageSize> src_xstage, dst_xstage;  // per pp: the expert buffers (kinds 4..7); empty if dense
    liver::List direct, pack, unpack;
    liver_plan_info_t info{};
    std::vector<uint8_t> used[2];  // [side][rank*LIVER_NUM_KINDS+kind]
    // device side
    void* dev_table = nullptr;
    int device = -1;
    int n_cu = 0;
    // launch shape
    int grid_blocks = 0, tile_order = -1, cache_hints = -1;  // 0 / -1 / -1 = library defaults
};

namespace liver {
// Fills everything host-side in `plan` (spec/src/dst/chunk_bytes already set).
// Returns LIVER_OK or an error code; `why` gets a short reason.
int build_plan(liver_plan& plan, std::string& why);
}  // namespace liver

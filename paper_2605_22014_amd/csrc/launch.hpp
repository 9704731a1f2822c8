// Launch interface between the C ABI (host) and the kernels.
#pragma once
#include <hip/hip_runtime_api.h>

#include "plan.hpp"

namespace liver {

// Arguments of one launch, passed by value (kernarg segment, < 4 KiB): the
// descriptor range in the plan's device table and the resolved buffer pointers.
struct PassArgs {
    const DevDesc* descs;
    uint32_t n_desc;
    uint32_t n_tiles;
    uint32_t tile_order;  // 0 contiguous ranges, 1 interleaved tiles, 2 scattered groups
    uint32_t group;       // tile_order 2: tiles per group (>= 1)
    uint32_t perm_mul;    // tile_order 2: multiplier of the group permutation, coprime to the group count
    uint32_t reserved;
    char* bufs[MAX_PASS_BUFS];
};
static_assert(sizeof(PassArgs) <= 3584, "kernel arguments must fit the kernarg segment");

// Arguments of a fused launch: two descriptor ranges (segments) whose tiles are numbered through; the
// descriptors of segment i index bufs[buf_base + ...].
struct FusedArgs {
    struct Segment {
        const DevDesc* descs;
        uint32_t n_desc;
        uint32_t n_tiles;
        uint32_t buf_base;
        uint32_t reserved;
    } seg[2];
    char* bufs[MAX_PASS_BUFS];
};
static_assert(sizeof(FusedArgs) <= 3584, "kernel arguments must fit the kernarg segment");
// Enqueue both segments in one launch (unpack policy for segment 0, pack policy for segment 1);
// 1 <= grid <= seg[0].n_tiles + seg[1].n_tiles, both segments non-empty.
hipError_t launch_fused(const FusedArgs& args, uint32_t grid, hipStream_t stream);

// Enqueue one pass on `stream` with `grid` workgroups (1 <= grid <= n_tiles).
hipError_t launch_pass(const PassArgs& args, uint32_t grid, int cache_hints, hipStream_t stream);

// Reference dispatch (read / fill / copy of n_tiles * PROBE_TILE_UNITS contiguous 16-byte units).
constexpr uint32_t PROBE_TILE_UNITS = 2048;  // 32 KiB per workgroup step
hipError_t launch_probe(int mode, const void* src, void* dst, uint64_t n_tiles, uint32_t grid, hipStream_t stream);

// The staging chunk the library itself holds on every device (a file-scope device array of
// STATIC_STAGING_BYTES): *ptr = its address on `device`, which must be the current device the first
// time it is asked for.  Never allocates.
constexpr size_t STATIC_STAGING_BYTES = 64u << 20;
hipError_t static_staging(int device, void** ptr);

}  // namespace liver

// Descriptor-driven copy kernels for gfx950 (CDNA4, wave64).
//
// One kernel serves pack, unpack and the direct reshard (LiveR, Section 4.6.2 and
// Algorithm 1: the sender cuts each task's slice out of its shard, the receiver
// assembles the slices into the new shard): each of the three is a list of
// strided 2-D pieces, rows x run, A -> B (a second kernel runs two such lists
// in one launch for the fused staged pipeline).  The work is pure HBM
// streaming, so the design is about memory, not arithmetic:
//   * a piece is cut into tiles of TILE_UNITS 16-byte units (64 KiB); a tile is
//     what one workgroup moves at a time, so 256 compute units stay evenly loaded
//     whatever the mix of 4 KiB norm vectors and 100 MB matrices;
//   * persistent workgroups: each walks its tiles and advances through the
//     descriptor table by itself (one binary search per workgroup, then
//     sequential), all descriptor reads are wave-uniform;
//   * tiles go to workgroups in teams: a team of 8 or 32 workgroups, all on one
//     XCD (team = workgroup id mod team count, and consecutive ids go round the 8
//     XCDs), owns one contiguous range of tiles and interleaves inside it, so each
//     XCD's L2 sees a few wide sequential streams;
//   * every lane moves 16 bytes per access (global_load/store_dwordx4), 64 lanes
//     cover 1 KiB contiguous, 8 independent loads are in flight per lane before
//     the first store; the fused cast reads 16 B of fp32 once and writes the
//     fp32 copy (16 B) and the bf16 weights (8 B) from the same registers;
//   * runs (row-parallel strips, per-head QKV groups) are multiples of 16 bytes
//     in every real configuration, so strided pieces are linearised over
//     (row, column) and stay fully coalesced on both sides without staging in
//     LDS; pieces of odd-sized toy models that are not 16-byte aligned take the
//     element paths.
#include <hip/hip_runtime.h>

#include "launch.hpp"

namespace liver {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#ifndef LIVER_BLOCK
#define LIVER_BLOCK 256
#endif
#ifndef LIVER_BATCH
#define LIVER_BATCH 8
#endif
constexpr int BLOCK = LIVER_BLOCK;              // threads per workgroup
constexpr int PER_THREAD = TILE_UNITS / BLOCK;  // units per lane per tile
constexpr int BATCH = LIVER_BATCH;              // loads in flight per lane
static_assert(TILE_UNITS % BLOCK == 0 && PER_THREAD % BATCH == 0, "tile must split evenly into batches");

template <bool NTL, bool NTS>
struct Mem {
    template <class T>
    static __device__ __forceinline__ T ld(const T* p) {
        if (NTL) return __builtin_nontemporal_load(p);
        return *p;
    }
    template <class T>
    static __device__ __forceinline__ void st(T* p, T v) {
        if (NTS) __builtin_nontemporal_store(v, p);
        else *p = v;
    }
};

// fp32 bits -> bf16 bits, round to nearest even; NaN keeps sign and upper payload
// and gets the quiet bit; overflow rounds to Inf; denormals round like any value.
__device__ __forceinline__ uint32_t bf16_rne(uint32_t u) {
    uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) r = (u >> 16) | 0x0040u;
    return r & 0xFFFFu;
}

// Unit `u` of a piece sits at row r = u / run, column c = u % run; a dense piece
// (one run) is row 0.  Byte offset in a buffer = r * stride + c * unit_bytes.
struct Geom {
    uint32_t run;
    bool dense;
    __device__ __forceinline__ void locate(uint32_t u, uint32_t& r, uint32_t& c) const {
        if (dense) {
            r = 0;
            c = u;
        } else {
            r = u / run;
            c = u - r * run;
        }
    }
};
__device__ __forceinline__ uint64_t at(uint32_t r, uint32_t c, uint32_t stride, uint32_t unit) {
    return (uint64_t)r * stride + (uint64_t)c * unit;
}

__device__ __forceinline__ u32x2 pack_bf16x4(u32x4 v) {
    u32x2 o;
    o.x = bf16_rne(v.x) | (bf16_rne(v.y) << 16);
    o.y = bf16_rne(v.z) | (bf16_rne(v.w) << 16);
    return o;
}

// FUSE 0: B <- A (16 B units).  FUSE 1: C <- bf16(A).  FUSE 2: B <- A and C <- bf16(A).
template <class M, int FUSE>
__device__ __forceinline__ void tile_v16(const Geom& g, const DevDesc& D, uint32_t u0, uint32_t n, const char* a,
                                         char* b, char* c) {
    const uint32_t tid = threadIdx.x;
    auto out = [&](uint32_t r, uint32_t col, u32x4 v) {
        if (FUSE != 1) M::st((u32x4*)(b + at(r, col, D.b_stride, 16)), v);
        if (FUSE != 0) M::st((u32x2*)(c + at(r, col, D.c_stride, 8)), pack_bf16x4(v));
    };
    if (n == TILE_UNITS) {
#pragma unroll
        for (int k = 0; k < PER_THREAD; k += BATCH) {
            u32x4 v[BATCH];
            uint32_t r[BATCH], col[BATCH];
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                g.locate(u0 + tid + (k + j) * BLOCK, r[j], col[j]);
                v[j] = M::ld((const u32x4*)(a + at(r[j], col[j], D.a_stride, 16)));
            }
#pragma unroll
            for (int j = 0; j < BATCH; ++j) out(r[j], col[j], v[j]);
        }
    } else {
        for (uint32_t i = tid; i < n; i += BLOCK) {
            uint32_t r, col;
            g.locate(u0 + i, r, col);
            out(r, col, M::ld((const u32x4*)(a + at(r, col, D.a_stride, 16))));
        }
    }
}

template <class T>
__device__ __forceinline__ void tile_copy_elem(const Geom& g, const DevDesc& D, uint32_t u0, uint32_t n, const char* a,
                                               char* b) {
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK) {
        uint32_t r, c;
        g.locate(u0 + i, r, c);
        *(T*)(b + at(r, c, D.b_stride, sizeof(T))) = *(const T*)(a + at(r, c, D.a_stride, sizeof(T)));
    }
}

__device__ __forceinline__ void tile_cast_elem(const Geom& g, const DevDesc& D, uint32_t u0, uint32_t n, const char* a,
                                               char* b) {
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK) {
        uint32_t r, c;
        g.locate(u0 + i, r, c);
        *(uint16_t*)(b + at(r, c, D.b_stride, 2)) = (uint16_t)bf16_rne(*(const uint32_t*)(a + at(r, c, D.a_stride, 4)));
    }
}

template <class T>
__device__ __forceinline__ void tile_zero(uint32_t u0, uint32_t n, char* b) {
    T z = {};
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK) *(T*)(b + ((uint64_t)(u0 + i)) * sizeof(T)) = z;
}

// Everything one workgroup does for tiles [t, t_end) with stride `step`: find the descriptor of the
// first tile (binary search), then walk forward through the descriptor table.
// A descriptor range with its tiles and the buffer table its descriptors index into.
struct TileSet {
    const DevDesc* descs;
    uint32_t n_desc, n_tiles;
    char* const* bufs;
};

template <class M>
__device__ __forceinline__ void run_tiles(const TileSet& args, uint32_t t, uint32_t t_end, uint32_t step) {
    const uint32_t n_tiles = args.n_tiles;
    const DevDesc* __restrict__ descs = args.descs;
    // last descriptor whose first tile is <= t  (descs[0].tile_begin == 0)
    uint32_t lo = 0, hi = args.n_desc;
    while (hi - lo > 1) {
        const uint32_t mid = lo + (hi - lo) / 2;
        if (descs[mid].tile_begin <= t) lo = mid;
        else hi = mid;
    }
    uint32_t d = lo;
    DevDesc D = descs[d];
    uint32_t next_begin = d + 1 < args.n_desc ? descs[d + 1].tile_begin : n_tiles;
    for (; t < t_end; t += step) {
        while (t >= next_begin) {  // ends: t < n_tiles == tile_begin past the last descriptor
            ++d;
            D = descs[d];
            next_begin = d + 1 < args.n_desc ? descs[d + 1].tile_begin : n_tiles;
        }
        const uint32_t u0 = (t - D.tile_begin) * TILE_UNITS;
        const uint32_t left = D.total - u0;
        const uint32_t n = left < TILE_UNITS ? left : TILE_UNITS;
        const Geom g{D.run, D.run == D.total};
        const char* a = args.bufs[D.a_buf] + D.a_off;
        char* b = args.bufs[D.b_buf] + D.b_off;
        switch (D.op) {
            case DOP_COPY_V16: tile_v16<M, 0>(g, D, u0, n, a, b, nullptr); break;
            case DOP_CAST_V4: tile_v16<M, 1>(g, D, u0, n, a, nullptr, args.bufs[D.c_buf] + D.c_off); break;
            case DOP_COPYCAST_V4: tile_v16<M, 2>(g, D, u0, n, a, b, args.bufs[D.c_buf] + D.c_off); break;
            case DOP_COPY_E2: tile_copy_elem<uint16_t>(g, D, u0, n, a, b); break;
            case DOP_COPY_E4: tile_copy_elem<uint32_t>(g, D, u0, n, a, b); break;
            case DOP_CAST_E: tile_cast_elem(g, D, u0, n, a, b); break;
            case DOP_ZERO_V16: tile_zero<u32x4>(u0, n, b); break;
            case DOP_ZERO_E2: tile_zero<uint16_t>(u0, n, b); break;
            case DOP_ZERO_E4: tile_zero<uint32_t>(u0, n, b); break;
            default: break;
        }
    }
}

template <bool NTL, bool NTS>
__global__ __launch_bounds__(BLOCK) void liver_copy_kernel(const PassArgs pass) {
    typedef Mem<NTL, NTS> M;
    const TileSet args{pass.descs, pass.n_desc, pass.n_tiles, pass.bufs};
    const uint32_t n_tiles = pass.n_tiles, G = gridDim.x, w = blockIdx.x;
    if (pass.tile_order == 0) {         // one contiguous range of tiles per workgroup
        const uint32_t per = (n_tiles + G - 1) / G;
        const uint32_t t = w * per;     // below 2^32: n_tiles < 2^31 and G <= n_tiles (host checks)
        if (t < n_tiles) run_tiles<M>(args, t, t + per < n_tiles ? t + per : n_tiles, 1);
    } else if (pass.tile_order == 1) {  // workgroups interleave tile by tile
        if (w < n_tiles) run_tiles<M>(args, w, n_tiles, G);
    } else if (pass.tile_order == 3) {  // teams: `group` workgroups share one contiguous range and interleave tile by
                                        // tile inside it; team = w mod n_teams, so a team's members sit on one XCD
        const uint32_t width = pass.group, n_teams = G / width;   // host: G is a multiple of width
        const uint32_t team = w % n_teams, member = w / n_teams;
        const uint32_t per = (n_tiles + n_teams - 1) / n_teams;
        const uint32_t t0 = team * per, t1 = t0 + per < n_tiles ? t0 + per : n_tiles;
        if (t0 + member < t1) run_tiles<M>(args, t0 + member, t1, width);
    } else {                            // scattered: groups of `group` consecutive tiles, visited in the order
                                        // i -> (i * perm_mul) mod n_groups (perm_mul coprime to n_groups)
        const uint32_t group = pass.group, n_groups = (n_tiles + group - 1) / group;
        for (uint32_t i = w; i < n_groups; i += G) {
            const uint32_t gi = (uint32_t)(((uint64_t)i * pass.perm_mul) % n_groups);
            const uint32_t t = gi * group;
            run_tiles<M>(args, t, t + group < n_tiles ? t + group : n_tiles, 1);
        }
    }
}

template <int HINTS>
__device__ __forceinline__ void run_segment(const FusedArgs& f, int i, uint32_t t, uint32_t t_end) {
    const TileSet ts{f.seg[i].descs, f.seg[i].n_desc, f.seg[i].n_tiles, f.bufs + f.seg[i].buf_base};
    run_tiles<Mem<(HINTS & 1) != 0, (HINTS & 2) != 0>>(ts, t, t_end, 1);
}

// Two descriptor ranges in one launch, each with its own cache policy: the staged pipeline's unpack of chunk
// k-1 (segment 0) and pack of chunk k (segment 1), which touch different staging chunks and are independent.
// The tiles of both are numbered through; each workgroup takes one contiguous range of them, so the tail of
// one segment and the head of the other are covered by the same full grid.
template <int HINTS0, int HINTS1>
__global__ __launch_bounds__(BLOCK) void liver_fused_kernel(const FusedArgs f) {
    const uint32_t n0 = f.seg[0].n_tiles, total = n0 + f.seg[1].n_tiles, G = gridDim.x, w = blockIdx.x;
    const uint32_t per = (total + G - 1) / G;
    const uint32_t t0 = w * per;  // below 2^32: total < 2^31 and G <= total (host checks)
    if (t0 >= total) return;
    const uint32_t t1 = t0 + per < total ? t0 + per : total;
    if (t0 < n0) run_segment<HINTS0>(f, 0, t0, t1 < n0 ? t1 : n0);
    if (t1 > n0) run_segment<HINTS1>(f, 1, (t0 > n0 ? t0 : n0) - n0, t1 - n0);
}

}  // namespace

// Reference dispatches for measurement: the plainest streaming kernels the chip can run (grid-stride over
// tiles of PROBE_TILE_UNITS contiguous 16-byte units, PROBE_TILE_UNITS / BLOCK non-temporal accesses in flight per lane).
// MODE 0 reads `a` (and stores one unit per workgroup into `b` so the loads stay), 1 fills `b`, 2 copies a -> b,
// 3 fills BOTH `a` and `b` (n_tiles each) in one launch.
template <int MODE>
__global__ __launch_bounds__(BLOCK) void liver_probe_kernel(u32x4* __restrict__ a, u32x4* __restrict__ b, uint64_t n_tiles) {
    constexpr int U = PROBE_TILE_UNITS / BLOCK;
    u32x4 acc = {1u, 2u, 3u, 4u};
    const uint64_t total = MODE == 3 ? 2 * n_tiles : n_tiles;
    for (uint64_t t = blockIdx.x; t < total; t += gridDim.x) {
        const uint64_t at0 = (MODE == 3 && t >= n_tiles ? t - n_tiles : t) * PROBE_TILE_UNITS + threadIdx.x;
        u32x4* out = MODE == 3 && t < n_tiles ? a : b;
        u32x4 v[U];
#pragma unroll
        for (int i = 0; i < U; ++i) v[i] = MODE == 1 || MODE == 3 ? acc : __builtin_nontemporal_load(a + at0 + (uint64_t)i * BLOCK);
        if (MODE == 0) {
#pragma unroll
            for (int i = 0; i < U; ++i) acc ^= v[i];
        } else {
#pragma unroll
            for (int i = 0; i < U; ++i) __builtin_nontemporal_store(v[i], out + at0 + (uint64_t)i * BLOCK);
        }
    }
    if (MODE == 0 && threadIdx.x == 0) b[blockIdx.x] = acc;  // lane 0's value: enough to keep every lane's loads
}

// Both launchers report the status of THEIR launch (hipLaunchKernel's own return value): an error that
// some earlier call of the thread left behind is neither returned nor cleared here.
hipError_t launch_probe(int mode, const void* src, void* dst, uint64_t n_tiles, uint32_t grid, hipStream_t stream) {
    u32x4* a = (u32x4*)src;  // written by mode 3 only
    u32x4* o = (u32x4*)dst;
    void* kargs[] = {(void*)&a, (void*)&o, (void*)&n_tiles};
    const void* fn = mode == 0   ? (const void*)&liver_probe_kernel<0>
                     : mode == 1 ? (const void*)&liver_probe_kernel<1>
                     : mode == 2 ? (const void*)&liver_probe_kernel<2>
                                 : (const void*)&liver_probe_kernel<3>;
    return hipLaunchKernel(fn, dim3(grid), dim3(BLOCK), kargs, 0, stream);
}

hipError_t launch_pass(const PassArgs& args, uint32_t grid, int cache_hints, hipStream_t stream) {
    if (args.n_tiles == 0 || args.n_desc == 0) return hipSuccess;
    void* kargs[] = {(void*)&args};
    const void* fn;
    switch (cache_hints & 3) {
        case 0: fn = (const void*)&liver_copy_kernel<false, false>; break;
        case 1: fn = (const void*)&liver_copy_kernel<true, false>; break;
        case 2: fn = (const void*)&liver_copy_kernel<false, true>; break;
        default: fn = (const void*)&liver_copy_kernel<true, true>; break;
    }
    return hipLaunchKernel(fn, dim3(grid), dim3(BLOCK), kargs, 0, stream);
}

hipError_t launch_fused(const FusedArgs& args, uint32_t grid, hipStream_t stream) {
    void* kargs[] = {(void*)&args};
    // segment 0 scatters a staging chunk (just written: plain loads) into targets that are streamed (non-temporal
    // stores); segment 1 gathers streamed sources (non-temporal loads) into a staging chunk that is re-read at once
    return hipLaunchKernel((const void*)&liver_fused_kernel<2, 1>, dim3(grid), dim3(BLOCK), kargs, 0, stream);
}

}  // namespace liver

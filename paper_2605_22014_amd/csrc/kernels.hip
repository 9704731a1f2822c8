// Descriptor-driven copy kernels for gfx950 (CDNA4, wave64).
//
// One kernel serves pack, unpack and the direct reshard (LiveR, Algorithm 1:
// "slice <- T[p.bounds]" and "assemble received chunks into T'"; Section 4.6.2):
// each is a list of strided 2-D pieces "rows x run, A -> B".  The work is pure
// HBM streaming, so the design is about memory, not arithmetic:
//   * a piece is cut into tiles of TILE_UNITS 16-byte units (64 KiB); a tile is
//     what one workgroup moves at a time, so 256 compute units stay evenly loaded
//     whatever the mix of 4 KiB norm vectors and 100 MB matrices;
//   * persistent workgroups: each walks its tiles and advances through the
//     descriptor table by itself (one binary search per workgroup, then
//     sequential), all descriptor reads are wave-uniform;
//   * every lane moves 16 bytes per access (global_load/store_dwordx4), 64 lanes
//     cover 1 KiB contiguous, 8 independent loads are in flight per lane before
//     the first store;
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

// Unit `u` of a piece: row r = u / run, column c = u % run.
struct Geom {
    uint32_t run, a_stride, b_stride;
    bool dense;
    __device__ __forceinline__ void locate(uint32_t u, uint64_t a_unit, uint64_t b_unit, uint64_t& ao,
                                           uint64_t& bo) const {
        if (dense) {
            ao = (uint64_t)u * a_unit;
            bo = (uint64_t)u * b_unit;
        } else {
            const uint32_t r = u / run, c = u - r * run;
            ao = (uint64_t)r * a_stride + (uint64_t)c * a_unit;
            bo = (uint64_t)r * b_stride + (uint64_t)c * b_unit;
        }
    }
};

template <class M>
__device__ __forceinline__ void tile_copy_v16(const Geom& g, uint32_t u0, uint32_t n, const char* a, char* b) {
    const uint32_t tid = threadIdx.x;
    if (n == TILE_UNITS) {
#pragma unroll
        for (int k = 0; k < PER_THREAD; k += BATCH) {
            u32x4 v[BATCH];
            uint64_t bo[BATCH];
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                uint64_t ao;
                g.locate(u0 + tid + (k + j) * BLOCK, 16, 16, ao, bo[j]);
                v[j] = M::ld((const u32x4*)(a + ao));
            }
#pragma unroll
            for (int j = 0; j < BATCH; ++j) M::st((u32x4*)(b + bo[j]), v[j]);
        }
    } else {
        for (uint32_t i = tid; i < n; i += BLOCK) {
            uint64_t ao, bo;
            g.locate(u0 + i, 16, 16, ao, bo);
            M::st((u32x4*)(b + bo), M::ld((const u32x4*)(a + ao)));
        }
    }
}

template <class M>
__device__ __forceinline__ void tile_cast_v8(const Geom& g, uint32_t u0, uint32_t n, const char* a, char* b) {
    constexpr int CB = 4;
    for (uint32_t i0 = threadIdx.x; i0 < n; i0 += BLOCK * CB) {
        u32x4 lo[CB], hi[CB];
        uint64_t bo[CB];
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            const uint32_t i = i0 + j * BLOCK;
            if (i < n) {
                uint64_t ao;
                g.locate(u0 + i, 32, 16, ao, bo[j]);
                lo[j] = M::ld((const u32x4*)(a + ao));
                hi[j] = M::ld((const u32x4*)(a + ao + 16));
            }
        }
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            const uint32_t i = i0 + j * BLOCK;
            if (i < n) {
                u32x4 o;
                o.x = bf16_rne(lo[j].x) | (bf16_rne(lo[j].y) << 16);
                o.y = bf16_rne(lo[j].z) | (bf16_rne(lo[j].w) << 16);
                o.z = bf16_rne(hi[j].x) | (bf16_rne(hi[j].y) << 16);
                o.w = bf16_rne(hi[j].z) | (bf16_rne(hi[j].w) << 16);
                M::st((u32x4*)(b + bo[j]), o);
            }
        }
    }
}

template <class T>
__device__ __forceinline__ void tile_copy_elem(const Geom& g, uint32_t u0, uint32_t n, const char* a, char* b) {
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK) {
        uint64_t ao, bo;
        g.locate(u0 + i, sizeof(T), sizeof(T), ao, bo);
        *(T*)(b + bo) = *(const T*)(a + ao);
    }
}

__device__ __forceinline__ void tile_cast_elem(const Geom& g, uint32_t u0, uint32_t n, const char* a, char* b) {
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK) {
        uint64_t ao, bo;
        g.locate(u0 + i, 4, 2, ao, bo);
        *(uint16_t*)(b + bo) = (uint16_t)bf16_rne(*(const uint32_t*)(a + ao));
    }
}

template <class T>
__device__ __forceinline__ void tile_zero(uint32_t u0, uint32_t n, char* b) {
    T z = {};
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK) *(T*)(b + ((uint64_t)(u0 + i)) * sizeof(T)) = z;
}

template <bool NTL, bool NTS>
__global__ __launch_bounds__(BLOCK) void liver_copy_kernel(const PassArgs args) {
    typedef Mem<NTL, NTS> M;
    const uint32_t n_tiles = args.n_tiles, G = gridDim.x, w = blockIdx.x;
    uint32_t t, t_end, step;
    if (args.tile_order == 0) {  // one contiguous range of tiles per workgroup
        const uint32_t per = (n_tiles + G - 1) / G;
        t = w * per;             // w * per <= n_tiles + G: no overflow, both below 2^32 by the host's check
        t_end = t + per < n_tiles ? t + per : n_tiles;
        step = 1;
    } else {                     // workgroups interleave tile by tile
        t = w;
        t_end = n_tiles;
        step = G;
    }
    if (t >= t_end) return;
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
        Geom g{D.run, D.a_stride, D.b_stride, D.run == D.total};
        const char* a = args.bufs[D.a_buf] + D.a_off;
        char* b = args.bufs[D.b_buf] + D.b_off;
        switch (D.op) {
            case DOP_COPY_V16: tile_copy_v16<M>(g, u0, n, a, b); break;
            case DOP_CAST_V8: tile_cast_v8<M>(g, u0, n, a, b); break;
            case DOP_COPY_E2: tile_copy_elem<uint16_t>(g, u0, n, a, b); break;
            case DOP_COPY_E4: tile_copy_elem<uint32_t>(g, u0, n, a, b); break;
            case DOP_CAST_E: tile_cast_elem(g, u0, n, a, b); break;
            case DOP_ZERO_V16: tile_zero<u32x4>(u0, n, b); break;
            case DOP_ZERO_E2: tile_zero<uint16_t>(u0, n, b); break;
            case DOP_ZERO_E4: tile_zero<uint32_t>(u0, n, b); break;
            default: break;
        }
    }
}

}  // namespace

hipError_t launch_pass(const PassArgs& args, uint32_t grid, int cache_hints, hipStream_t stream) {
    if (args.n_tiles == 0 || args.n_desc == 0) return hipSuccess;
    dim3 g(grid), b(BLOCK);
    switch (cache_hints & 3) {
        case 0: hipLaunchKernelGGL((liver_copy_kernel<false, false>), g, b, 0, stream, args); break;
        case 1: hipLaunchKernelGGL((liver_copy_kernel<true, false>), g, b, 0, stream, args); break;
        case 2: hipLaunchKernelGGL((liver_copy_kernel<false, true>), g, b, 0, stream, args); break;
        default: hipLaunchKernelGGL((liver_copy_kernel<true, true>), g, b, 0, stream, args); break;
    }
    return hipGetLastError();
}

}  // namespace liver

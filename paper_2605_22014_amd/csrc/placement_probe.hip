// placement_probe -- measurement aid, a stand-alone program (not part of libliver.so).
//
// Shows how the bandwidth of plain streaming kernels on gfx950 depends on WHERE in device memory the bytes
// sit, which bounds what any copy -- the reshard included -- can reach for a given placement of the caller's
// buffers.  One arena is allocated; windows of it, 32 GiB apart, are read, filled and copied in pairs.
// The kernels are the plainest possible: 256-thread workgroups, 16-byte non-temporal accesses, 8 in flight
// per lane, each workgroup walking one contiguous share of the windows (the reshard's own schedule).
//
//   placement_probe [arena_GiB = 224] [matrix | pairs]
//     matrix  fill / read bandwidth for every pair of windows (a, b), and copy bandwidth window a -> window b
//     pairs   finds, by timing fills, one partner window in the same class as window 0 and one in another
//             class, then runs one labelled fill, read and copy dispatch on each (kernel names carry the
//             label: probe_kernel<MODE, 1> = same class, <MODE, 2> = different class), for counter runs
//             under rocprofv3 --pmc.
//
// Every access is in bounds by construction: window offsets and sizes are checked against the arena on the
// host before each launch, and each workgroup's tile range is clipped to the tile count.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int IN_FLIGHT = 8;
constexpr uint64_t TILE = 256ull * IN_FLIGHT * 16;  // 32 KiB per workgroup step
constexpr uint64_t GiB = 1ull << 30;
enum Mode { READ = 0, FILL = 1, COPY = 2 };

// Tiles [0, n) of window A then tiles [0, n) of window B form one list; workgroup w takes one contiguous
// share of it.  READ reads both windows, FILL fills both, COPY copies window A to window B (n tiles).
template <int MODE, int LABEL>
__global__ __launch_bounds__(256) void probe_kernel(char* a, char* b, uint64_t n, unsigned* sink) {
    const uint64_t total = MODE == COPY ? n : 2 * n;
    const uint64_t per = (total + gridDim.x - 1) / gridDim.x;
    const uint64_t t0 = blockIdx.x * per, t1 = t0 + per < total ? t0 + per : total;
    u32x4 acc = {1, 2, 3, 4};
    for (uint64_t t = t0; t < t1; ++t) {
        char* here = MODE == COPY || t < n ? a + t * TILE : b + (t - n) * TILE;
        u32x4* p = (u32x4*)here + threadIdx.x;
        u32x4* q = (u32x4*)(b + t * TILE) + threadIdx.x;  // used by COPY only (t < n)
        u32x4 v[IN_FLIGHT];
#pragma unroll
        for (int i = 0; i < IN_FLIGHT; ++i) v[i] = MODE == FILL ? acc : __builtin_nontemporal_load(p + i * 256);
        if (MODE == READ) {
#pragma unroll
            for (int i = 0; i < IN_FLIGHT; ++i) acc ^= v[i];
        } else {
#pragma unroll
            for (int i = 0; i < IN_FLIGHT; ++i) __builtin_nontemporal_store(v[i], (MODE == COPY ? q : p) + i * 256);
        }
    }
    if (MODE == READ && (acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[blockIdx.x] = 1;  // keeps the loads
}

char* g_arena = nullptr;
uint64_t g_arena_bytes = 0;
unsigned* g_sink = nullptr;
hipEvent_t g_e0, g_e1;

template <int MODE, int LABEL>
void launch(uint64_t off_a, uint64_t off_b, uint64_t n_tiles) {
    hipLaunchKernelGGL((probe_kernel<MODE, LABEL>), dim3(256), dim3(256), 0, 0, g_arena + off_a, g_arena + off_b, n_tiles, g_sink);
}

// GB/s of `reps` timed launches (best of them, after one untimed); bytes counted: both windows (READ, FILL), or
// the window read plus the window written (COPY).
template <int MODE, int LABEL>
double run(uint64_t off_a, uint64_t off_b, uint64_t win_bytes, int reps = 4) {
    if (win_bytes == 0 || win_bytes % TILE || off_a % 256 || off_b % 256 || off_a + win_bytes > g_arena_bytes ||
        off_b + win_bytes > g_arena_bytes || (off_a < off_b + win_bytes && off_b < off_a + win_bytes)) {
        std::printf("window outside the arena or overlapping: refused\n");
        std::exit(2);
    }
    double best = 0;
    for (int r = 0; r <= reps; ++r) {
        (void)hipEventRecord(g_e0, 0);
        launch<MODE, LABEL>(off_a, off_b, win_bytes / TILE);
        (void)hipEventRecord(g_e1, 0);
        if (hipEventSynchronize(g_e1) != hipSuccess) {
            std::printf("kernel failed\n");
            std::exit(3);
        }
        float ms = 0;
        (void)hipEventElapsedTime(&ms, g_e0, g_e1);
        if (r) best = std::max(best, 2.0 * win_bytes / (ms * 1e-3) / 1e9);
    }
    return best;
}

}  // namespace

int main(int argc, char** argv) {
    const uint64_t arena_gib = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 224;
    const bool pairs = argc > 2 && std::strcmp(argv[2], "pairs") == 0;
    if (arena_gib < 72 || arena_gib > 280) {
        std::printf("arena must be 72..280 GiB\n");
        return 2;
    }
    g_arena_bytes = arena_gib * GiB;
    if (hipMalloc(&g_arena, g_arena_bytes) != hipSuccess || hipMalloc(&g_sink, 4096) != hipSuccess ||
        hipMemset(g_sink, 0, 4096) != hipSuccess || hipEventCreate(&g_e0) != hipSuccess || hipEventCreate(&g_e1) != hipSuccess) {
        std::printf("set-up failed (arena of %llu GiB)\n", (unsigned long long)arena_gib);
        return 1;
    }
    const int n_win = (int)((g_arena_bytes - 16 * GiB) / (32 * GiB)) + 1;  // windows at 8, 40, 72, ... GiB
    auto at = [](int i) { return (uint64_t)i * 32 * GiB + 8 * GiB; };
    const uint64_t W = 2 * GiB;  // window size; a pair partner in the same window index sits 4 GiB further
    std::printf("arena %llu GiB; %d windows of 2 GiB at 8 + 32 i GiB (same-index partner: + 4 GiB)\n", (unsigned long long)arena_gib, n_win);
    for (int i = 0; i < n_win; ++i) (void)run<FILL, 0>(at(i), at(i) + 4 * GiB, W, 1);  // first touch out of the way
    std::fflush(stdout);
    if (!pairs) {
        const char* title[3] = {"READ  both windows (a, b)", "FILL  both windows (a, b)", "COPY  window a -> window b"};
        for (int mode : {FILL, READ, COPY}) {
            std::printf("%s, GB/s; rows a, columns b\n", title[mode]);
            for (int a = 0; a < n_win; ++a) {
                std::printf("  a=%d:", a);
                for (int b = 0; b < n_win; ++b) {
                    const uint64_t ob = at(b) + (a == b ? 4 * GiB : 0);
                    const double g = mode == FILL ? run<FILL, 0>(at(a), ob, W) : mode == READ ? run<READ, 0>(at(a), ob, W) : run<COPY, 0>(at(a), ob, W);
                    std::printf(" %5.0f", g);
                }
                std::printf("\n");
                std::fflush(stdout);
            }
        }
        return 0;
    }
    // pairs: classify the windows against window 0 by fill bandwidth (two groups, split at the midpoint)
    std::vector<double> g(n_win, 0.0);
    for (int b = 1; b < n_win; ++b) g[b] = run<FILL, 0>(at(0), at(b), W);
    const double lo = *std::min_element(g.begin() + 1, g.end()), hi = *std::max_element(g.begin() + 1, g.end());
    int same = -1, other = -1;
    for (int b = 1; b < n_win; ++b) {
        if (g[b] < (lo + hi) / 2 && same < 0) same = b;
        if (g[b] >= (lo + hi) / 2 && other < 0) other = b;
    }
    std::printf("fill of window 0 with window b:");
    for (int b = 1; b < n_win; ++b) std::printf(" b=%d %.0f", b, g[b]);
    std::printf(" GB/s\n");
    if (hi < 1.1 * lo) {
        std::printf("no two classes visible among these windows (fill %0.f..%.0f GB/s): nothing to label\n", lo, hi);
        return 0;
    }
    const uint64_t o0 = at(0), os = same > 0 ? at(same) : at(0) + 4 * GiB, oo = at(other);
    std::printf("same-class partner: window %d; other-class partner: window %d\n", same, other);
    std::printf("labelled dispatches <MODE, 1> (same class):  fill %.0f  read %.0f  copy %.0f GB/s\n", run<FILL, 1>(o0, os, W, 2),
                run<READ, 1>(o0, os, W, 2), run<COPY, 1>(o0, os, W, 2));
    std::printf("labelled dispatches <MODE, 2> (other class): fill %.0f  read %.0f  copy %.0f GB/s\n", run<FILL, 2>(o0, oo, W, 2),
                run<READ, 2>(o0, oo, W, 2), run<COPY, 2>(o0, oo, W, 2));
    return 0;
}

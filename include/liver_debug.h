/*
 * liver_debug.h -- debugging and measurement aids of the resharding library.
 *
 * Not part of the product boundary (include/liver.h): nothing here is called by the data entry points, and
 * there is no CPU fallback behind them.  Tests and the benchmark use these two calls.
 */
#ifndef LIVER_DEBUG_H
#define LIVER_DEBUG_H

#include "liver.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Executes the plan's LOWERED descriptor tables -- what the kernels would run for list `list`
 * (LIVER_LIST_*; `chunk` is ignored for the direct list) -- on HOST memory, unit by unit, and returns
 * LIVER_E_HIP instead of performing any access that is out of bounds or misaligned.  Buffers are host
 * arrays with the sizes liver_plan_buffer_bytes reports; staging has chunk_bytes.  Lets a test prove that
 * a plan's tables stay inside the buffers before the same tables are run on a GPU. */
int liver_debug_emulate_host(const liver_plan_t* plan, int list, int chunk, const void* const* src_bufs,
                             void* const* dst_bufs, void* staging);

/* Enqueues on `hip_stream` the plainest streaming kernel of the library's launch shape (256-thread
 * workgroups, grid-stride over 32 KiB tiles, 16-byte non-temporal accesses) over `bytes` bytes of DEVICE
 * memory, so that a benchmark can quote what a plain read, fill or copy reaches on the same buffers the
 * reshard uses.
 *   mode 0  read src[0, bytes); additionally stores 16 bytes per workgroup into
 *           dst[0, grid*16) (dst must hold at least that; grid*16 <= bytes)
 *   mode 1  fill dst[0, bytes) with a fixed pattern (src is ignored)
 *   mode 2  copy src[0, bytes) to dst[0, bytes)
 *   mode 3  fill BOTH src[0, bytes) and dst[0, bytes) in one launch (src is WRITTEN despite its type): the
 *           rate tells whether the two windows share a class of the device memory (about 5.7 TB/s) or not
 *           (about 7.1 TB/s on MI355X)
 * bytes: positive multiple of 32768; grid: 1..65536 workgroups; pointers 16-byte aligned, owned by the
 * caller, not overlapping.  Asynchronous, allocates nothing.  LIVER_E_INVALID_ARG on a bad argument
 * (nothing is launched), LIVER_E_HIP if the launch fails. */
int liver_debug_bandwidth_probe(int mode, const void* src, void* dst, size_t bytes, int grid, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LIVER_DEBUG_H */

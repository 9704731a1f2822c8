// The C ABI: plan lifetime, inspection, the three data calls and the whole-pipeline forms built on them.
#include <hip/hip_runtime_api.h>

#include <cstring>
#include <new>
#include <string>

#include "launch.hpp"
#include "liver_debug.h"
#include "plan.hpp"

namespace {

thread_local std::string g_last_detail;
thread_local int g_last_code = LIVER_OK;

int fail(int code, const std::string& detail) {
    g_last_detail = detail;
    g_last_code = code;
    return code;
}

int n_ranks(const liver_layout_t& l) { return l.tp * l.pp * l.dp; }

const void* resolve(const liver::BufRef& r, const void* const* src_bufs, void* const* dst_bufs, const void* staging) {
    return r.side == 0   ? (src_bufs ? src_bufs[(size_t)r.rank * LIVER_NUM_KINDS + r.kind] : nullptr)
           : r.side == 1 ? (dst_bufs ? dst_bufs[(size_t)r.rank * LIVER_NUM_KINDS + r.kind] : nullptr)
                         : staging;
}

// Everything that can be refused about passes [p0, p1) of `list`, checked without enqueuing anything.
int check_passes(const liver_plan* plan, const liver::List& list, uint32_t p0, uint32_t p1, const void* const* src_bufs,
                 void* const* dst_bufs, const void* staging) {
    if (plan->device < 0) return fail(LIVER_E_NO_DEVICE, "plan was created without a HIP device");
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess || cur != plan->device)
        return fail(LIVER_E_INVALID_ARG, "current HIP device is not the one the plan was created on");
    for (uint32_t p = p0; p < p1; ++p)
        for (const liver::BufRef& r : list.passes[p].bufs) {
            const void* ptr = resolve(r, src_bufs, dst_bufs, staging);
            if (!ptr) return fail(LIVER_E_INVALID_ARG, "a buffer the plan uses is NULL");
            if ((uintptr_t)ptr % 16) return fail(LIVER_E_INVALID_ARG, "buffers must be 16-byte aligned");
        }
    return LIVER_OK;
}

// Enqueue passes [p0, p1) of `list` in order; check_passes has accepted them.
int launch_passes(const liver_plan* plan, const liver::List& list, uint32_t p0, uint32_t p1, const void* const* src_bufs,
                  void* const* dst_bufs, const void* staging, void* hip_stream, int default_hints) {
    // Default launch shape: one persistent 256-thread workgroup per compute unit.  Measured on MI355X
    // at the 7B shape, 1-2 workgroups per CU reach the same plateau and more only add DRAM page conflicts.
    const uint32_t max_grid = plan->grid_blocks > 0 ? (uint32_t)plan->grid_blocks : (uint32_t)plan->n_cu;
    const int hints = plan->cache_hints >= 0 ? plan->cache_hints : default_hints;
    for (uint32_t p = p0; p < p1; ++p) {
        const liver::Pass& pass = list.passes[p];
        if (pass.n_tiles == 0) continue;
        liver::PassArgs args;
        args.descs = (const liver::DevDesc*)((const char*)plan->dev_table + list.dev_offset) + pass.desc_begin;
        args.n_desc = pass.desc_count;
        args.n_tiles = pass.n_tiles;
        uint32_t grid = pass.n_tiles < max_grid ? pass.n_tiles : max_grid;
        // Tile order.  Default (-1) and order 3: TEAMS.  `width` workgroups share one contiguous tile range and
        // interleave tile by tile inside it; team = workgroup id mod team count, so with a team count that is a
        // multiple of 8 a team's members all sit on one XCD and its stream stays in that XCD's L2.  Measured on
        // MI355X against one range per workgroup (order 0): 7B +0..1 %, 13B share +3..6 %, 70B share +1..2 %,
        // GPT-2-small +-0.5 %; all 256 workgroups interleaving (order 1) loses 4..9 % except when every buffer
        // sits in one 32 GiB region of the HBM.  Big launches run best as 32 teams of 8, small ones as 8 teams
        // (one per XCD) of 32.  100 + w = teams of w (tuning aid).
        const int order = plan->tile_order < 0 ? 3 : plan->tile_order;
        args.tile_order = order >= 3 ? 0u : (uint32_t)order;
        args.reserved = 0;
        // scattered order: groups of up to 64 tiles (4 MiB), at least ~32 groups per workgroup; the groups
        // are visited in a multiplicative permutation with a multiplier near 0.618 * n_groups
        {
            uint32_t group = pass.n_tiles / (max_grid * 32u);
            group = group < 1 ? 1 : group > 64 ? 64 : group;
            const uint32_t n_groups = (pass.n_tiles + group - 1) / group;
            uint32_t mul = (uint32_t)(0.6180339887 * n_groups) | 1u;
            auto gcd = [](uint32_t a, uint32_t b) { while (b) { const uint32_t t = a % b; a = b; b = t; } return a; };
            while (mul > 1 && gcd(mul, n_groups) != 1) mul -= 2;
            if (mul < 1 || n_groups < 3) mul = 1;
            args.group = group, args.perm_mul = mul;
        }
        if (order >= 3) {
            const uint32_t width = order >= 100 ? (uint32_t)order - 100u : pass.n_tiles >= (1u << 20) ? 8u : 32u;
            // the library's own choice wants at least one team per XCD; an explicit width only has to fit the grid
            if (width >= 2 && grid / width >= (order >= 100 ? 1u : 8u)) {  // else: one range per workgroup (order 0)
                grid -= grid % width;
                args.tile_order = 3, args.group = width;
            }
        }
        size_t i = 0;
        for (const liver::BufRef& r : pass.bufs) args.bufs[i++] = (char*)resolve(r, src_bufs, dst_bufs, staging);
        for (; i < (size_t)liver::MAX_PASS_BUFS; ++i) args.bufs[i] = nullptr;
        hipError_t e = liver::launch_pass(args, grid, hints, (hipStream_t)hip_stream);
        if (e != hipSuccess) return fail(LIVER_E_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
    }
    return LIVER_OK;
}

// Validate, then launch: an argument error writes nothing.
int run_passes(const liver_plan* plan, const liver::List& list, uint32_t p0, uint32_t p1, const void* const* src_bufs,
               void* const* dst_bufs, const void* staging, void* hip_stream, int default_hints) {
    const int rc = check_passes(plan, list, p0, p1, src_bufs, dst_bufs, staging);
    if (rc != LIVER_OK) return rc;
    return launch_passes(plan, list, p0, p1, src_bufs, dst_bufs, staging, hip_stream, default_hints);
}

constexpr int HINT_PACK = 1;    // the source is streamed once, the staging chunk is re-read by unpack
constexpr int HINT_UNPACK = 2;  // the staging chunk was just written, the targets are streamed
constexpr int HINT_DIRECT = 3;  // every byte is touched once

}  // namespace

extern "C" {

int liver_plan_create(const liver_model_spec_t* spec, const liver_layout_t* src, const liver_layout_t* dst,
                      size_t chunk_bytes, liver_plan_t** out) {
    if (!spec || !src || !dst || !out) return fail(LIVER_E_INVALID_ARG, "null argument");
    liver_plan* plan = nullptr;
    try {
        plan = new liver_plan;
        plan->spec = *spec, plan->src = *src, plan->dst = *dst, plan->chunk_bytes = chunk_bytes;
        std::string why;
        int rc = liver::build_plan(*plan, why);
        if (rc != LIVER_OK) {
            delete plan;
            return fail(rc, why);
        }
    } catch (const std::bad_alloc&) {
        delete plan;
        return fail(LIVER_E_NOMEM, "host allocation failed");
    }
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) == hipSuccess && n_dev > 0) {
        int dev = 0, cu = 0;
        void* table = nullptr;
        const size_t bytes = (size_t)plan->info.table_bytes_device;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess && bytes) e = hipMalloc(&table, bytes);
        for (const liver::List* l : {&plan->direct, &plan->pack, &plan->unpack})
            if (e == hipSuccess && !l->dev.empty())
                e = hipMemcpy((char*)table + l->dev_offset, l->dev.data(), l->dev.size() * sizeof(liver::DevDesc),
                              hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            if (table) (void)hipFree(table);
            const int code = e == hipErrorOutOfMemory ? LIVER_E_NOMEM : LIVER_E_HIP;
            delete plan;
            return fail(code, std::string("descriptor table upload: ") + hipGetErrorString(e));
        }
        plan->dev_table = table, plan->device = dev, plan->n_cu = cu > 0 ? cu : 256;
        void* unused = nullptr;  // set-up is where the static staging array's address on this device is looked up;
        (void)liver::static_staging(dev, &unused);  // a failure is reported by liver_reshard_static, which needs it
    } else {
        (void)hipGetLastError();  // no device: host-only plan
    }
    *out = plan;
    return LIVER_OK;
}

void liver_plan_destroy(liver_plan_t* plan) {
    if (!plan) return;
    if (plan->dev_table) (void)hipFree(plan->dev_table);
    delete plan;
}

int liver_plan_info(const liver_plan_t* plan, liver_plan_info_t* out) {
    if (!plan || !out) return fail(LIVER_E_INVALID_ARG, "null argument");
    *out = plan->info;
    return LIVER_OK;
}

int liver_plan_buffer_bytes(const liver_plan_t* plan, int side, int rank, int kind, size_t* out) {
    if (!plan || !out || side < 0 || side > 1 || kind < 0 || kind >= LIVER_NUM_KINDS)
        return fail(LIVER_E_INVALID_ARG, "bad argument");
    const liver_layout_t& lay = side ? plan->dst : plan->src;
    if (rank < 0 || rank >= n_ranks(lay)) return fail(LIVER_E_INVALID_ARG, "rank out of range");
    const int pp = rank / (lay.tp * lay.dp);
    const bool expert = kind >= LIVER_EXPERT_PARAM_BF16;
    const std::vector<liver::StageSize>& stages = side ? (expert ? plan->dst_xstage : plan->dst_stage)
                                                       : (expert ? plan->src_xstage : plan->src_stage);
    if (stages.empty()) {  // expert buffers exist only for mixture-of-experts models
        *out = 0;
        return LIVER_OK;
    }
    const liver::StageSize& st = stages[pp];
    *out = kind % 4 == 0 ? (size_t)st.n_pad * 2 : (size_t)st.S * 4;
    return LIVER_OK;
}

int liver_plan_buffer_used(const liver_plan_t* plan, int side, int rank, int kind) {
    if (!plan || side < 0 || side > 1 || kind < 0 || kind >= LIVER_NUM_KINDS)
        return fail(LIVER_E_INVALID_ARG, "bad argument");
    if (rank < 0 || rank >= n_ranks(side ? plan->dst : plan->src)) return fail(LIVER_E_INVALID_ARG, "rank out of range");
    return plan->used[side][(size_t)rank * LIVER_NUM_KINDS + kind];
}

int64_t liver_plan_desc_count(const liver_plan_t* plan, int list) {
    if (!plan || list < 0 || list > 2) return fail(LIVER_E_INVALID_ARG, "bad argument");
    const liver::List& l = list == LIVER_LIST_DIRECT ? plan->direct : list == LIVER_LIST_PACK ? plan->pack : plan->unpack;
    return (int64_t)l.pub.size();
}

int liver_plan_desc(const liver_plan_t* plan, int list, int64_t i, liver_desc_t* out) {
    if (!plan || !out || list < 0 || list > 2) return fail(LIVER_E_INVALID_ARG, "bad argument");
    const liver::List& l = list == LIVER_LIST_DIRECT ? plan->direct : list == LIVER_LIST_PACK ? plan->pack : plan->unpack;
    if (i < 0 || i >= (int64_t)l.pub.size()) return fail(LIVER_E_INVALID_ARG, "descriptor index out of range");
    *out = l.pub[(size_t)i];
    return LIVER_OK;
}

int liver_plan_set_launch(liver_plan_t* plan, int grid_blocks, int tile_order, int cache_hints) {
    if (!plan || grid_blocks < 0 || grid_blocks > 65536 || tile_order < -1 || (tile_order > 3 && (tile_order < 102 || tile_order > 1124)) || cache_hints < -1 ||
        cache_hints > 3)
        return fail(LIVER_E_INVALID_ARG, "bad launch shape");
    plan->grid_blocks = grid_blocks, plan->tile_order = tile_order, plan->cache_hints = cache_hints;
    return LIVER_OK;
}

int liver_pack(const liver_plan_t* plan, int chunk, const void* const* src_bufs, void* staging, void* hip_stream) {
    if (!plan || !src_bufs || !staging) return fail(LIVER_E_INVALID_ARG, "null argument");
    if (chunk < 0 || chunk >= plan->info.n_chunks) return fail(LIVER_E_INVALID_ARG, "chunk index out of range");
    if ((uintptr_t)staging % 256) return fail(LIVER_E_INVALID_ARG, "staging must be 256-byte aligned");
    return run_passes(plan, plan->pack, plan->pack.chunk_pass[chunk], plan->pack.chunk_pass[chunk + 1], src_bufs, nullptr,
                      staging, hip_stream, HINT_PACK);
}

int liver_unpack(const liver_plan_t* plan, int chunk, const void* staging, void* const* dst_bufs, void* hip_stream) {
    if (!plan || !dst_bufs || !staging) return fail(LIVER_E_INVALID_ARG, "null argument");
    if (chunk < 0 || chunk >= plan->info.n_chunks) return fail(LIVER_E_INVALID_ARG, "chunk index out of range");
    if ((uintptr_t)staging % 256) return fail(LIVER_E_INVALID_ARG, "staging must be 256-byte aligned");
    return run_passes(plan, plan->unpack, plan->unpack.chunk_pass[chunk], plan->unpack.chunk_pass[chunk + 1], nullptr,
                      dst_bufs, staging, hip_stream, HINT_UNPACK);
}

int liver_reshard(const liver_plan_t* plan, const void* const* src_bufs, void* const* dst_bufs, void* hip_stream) {
    if (!plan || !src_bufs || !dst_bufs) return fail(LIVER_E_INVALID_ARG, "null argument");
    return run_passes(plan, plan->direct, 0, (uint32_t)plan->direct.passes.size(), src_bufs, dst_bufs, nullptr, hip_stream,
                      HINT_DIRECT);
}

int liver_reshard_staged(const liver_plan_t* plan, const void* const* src_bufs, void* const* dst_bufs,
                         void* const* staging, int n_staging, void* stream_pack, void* stream_unpack) {
    if (!plan || !src_bufs || !dst_bufs || !staging) return fail(LIVER_E_INVALID_ARG, "null argument");
    if (n_staging < 1 || n_staging > 8) return fail(LIVER_E_INVALID_ARG, "n_staging must be 1..8");
    for (int i = 0; i < n_staging; ++i) {
        if (!staging[i] || (uintptr_t)staging[i] % 256) return fail(LIVER_E_INVALID_ARG, "staging chunks must be non-null, 256-byte aligned");
        for (int j = 0; j < i; ++j)
            if (staging[i] == staging[j]) return fail(LIVER_E_INVALID_ARG, "staging chunks must be distinct");
    }
    // every chunk's buffers are checked before the first kernel is enqueued: an argument error writes nothing
    int rc = check_passes(plan, plan->pack, 0, (uint32_t)plan->pack.passes.size(), src_bufs, nullptr, staging[0]);
    if (rc == LIVER_OK)
        rc = check_passes(plan, plan->unpack, 0, (uint32_t)plan->unpack.passes.size(), nullptr, dst_bufs, staging[0]);
    if (rc != LIVER_OK) return rc;
    const int n_chunks = (int)plan->info.n_chunks;
    hipStream_t sp = (hipStream_t)stream_pack, su = (hipStream_t)stream_unpack;
    hipEvent_t packed[8] = {}, unpacked[8] = {};
    hipError_t e = hipSuccess;
    int made = 0;
    for (; made < n_staging && e == hipSuccess; ++made) {
        e = hipEventCreateWithFlags(&packed[made], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&unpacked[made], hipEventDisableTiming);
    }
    for (int k = 0; k < n_chunks && e == hipSuccess && rc == LIVER_OK; ++k) {
        const int slot = k % n_staging;
        if (k >= n_staging) e = hipStreamWaitEvent(sp, unpacked[slot], 0);  // the chunk buffer is free again
        if (e == hipSuccess)
            rc = launch_passes(plan, plan->pack, plan->pack.chunk_pass[k], plan->pack.chunk_pass[k + 1], src_bufs, nullptr,
                               staging[slot], stream_pack, HINT_PACK);
        if (rc != LIVER_OK) break;
        if (e == hipSuccess) e = hipEventRecord(packed[slot], sp);
        if (e == hipSuccess) e = hipStreamWaitEvent(su, packed[slot], 0);
        if (e == hipSuccess)
            rc = launch_passes(plan, plan->unpack, plan->unpack.chunk_pass[k], plan->unpack.chunk_pass[k + 1], nullptr,
                               dst_bufs, staging[slot], stream_unpack, HINT_UNPACK);
        if (rc != LIVER_OK) break;
        if (e == hipSuccess) e = hipEventRecord(unpacked[slot], su);
    }
    for (int i = 0; i < n_staging; ++i) {  // destroying a recorded event is deferred until it has completed
        if (packed[i]) (void)hipEventDestroy(packed[i]);
        if (unpacked[i]) (void)hipEventDestroy(unpacked[i]);
    }
    if (rc != LIVER_OK) return rc;  // a launch the runtime refused (LIVER_E_HIP): earlier chunks may have run
    if (e != hipSuccess) return fail(LIVER_E_HIP, std::string("staged pipeline: ") + hipGetErrorString(e));
    return LIVER_OK;
}

int liver_reshard_staged_fused(const liver_plan_t* plan, const void* const* src_bufs, void* const* dst_bufs,
                               void* staging_even, void* staging_odd, void* hip_stream) {
    if (!plan || !src_bufs || !dst_bufs || !staging_even || !staging_odd) return fail(LIVER_E_INVALID_ARG, "null argument");
    if ((uintptr_t)staging_even % 256 || (uintptr_t)staging_odd % 256)
        return fail(LIVER_E_INVALID_ARG, "staging chunks must be 256-byte aligned");
    if (staging_even == staging_odd) return fail(LIVER_E_INVALID_ARG, "staging chunks must be distinct");
    void* const slot[2] = {staging_even, staging_odd};
    const liver::List &pk = plan->pack, &un = plan->unpack;
    // every chunk's buffers are checked before the first kernel is enqueued: an argument error writes nothing
    int rc = check_passes(plan, pk, 0, (uint32_t)pk.passes.size(), src_bufs, nullptr, staging_even);
    if (rc == LIVER_OK) rc = check_passes(plan, un, 0, (uint32_t)un.passes.size(), nullptr, dst_bufs, staging_even);
    if (rc != LIVER_OK) return rc;
    const int n_chunks = (int)plan->info.n_chunks;
    const uint32_t max_grid = plan->grid_blocks > 0 ? (uint32_t)plan->grid_blocks : (uint32_t)plan->n_cu;
    // launch k = unpack(k - 1) + pack(k): chunk k - 1 leaves its staging chunk while chunk k enters the other one
    for (int k = 0; k <= n_chunks && rc == LIVER_OK; ++k) {
        const bool has_un = k > 0, has_pk = k < n_chunks;
        const uint32_t u0 = has_un ? un.chunk_pass[k - 1] : 0, u1 = has_un ? un.chunk_pass[k] : 0;
        const uint32_t p0 = has_pk ? pk.chunk_pass[k] : 0, p1 = has_pk ? pk.chunk_pass[k + 1] : 0;
        void* s_un = slot[(k + 1) & 1];  // chunk k - 1
        void* s_pk = slot[k & 1];        // chunk k
        const liver::Pass* a = u1 - u0 == 1 ? &un.passes[u0] : nullptr;
        const liver::Pass* b = p1 - p0 == 1 ? &pk.passes[p0] : nullptr;
        const bool fuse = a && b && a->n_tiles > 0 && b->n_tiles > 0 && plan->cache_hints < 0 && plan->tile_order < 0 &&
                          a->bufs.size() + b->bufs.size() <= (size_t)liver::MAX_PASS_BUFS &&
                          (uint64_t)a->n_tiles + b->n_tiles < (1u << 31);
        if (!fuse) {  // a chunk that needs several passes, an empty side, or a non-default launch shape: one after the other
            if (has_un) rc = launch_passes(plan, un, u0, u1, nullptr, dst_bufs, s_un, hip_stream, HINT_UNPACK);
            if (rc == LIVER_OK && has_pk) rc = launch_passes(plan, pk, p0, p1, src_bufs, nullptr, s_pk, hip_stream, HINT_PACK);
            continue;
        }
        liver::FusedArgs args;
        size_t i = 0;
        const liver::Pass* pass[2] = {a, b};
        const liver::List* list[2] = {&un, &pk};
        void* stage[2] = {s_un, s_pk};
        for (int g = 0; g < 2; ++g) {
            args.seg[g].descs = (const liver::DevDesc*)((const char*)plan->dev_table + list[g]->dev_offset) + pass[g]->desc_begin;
            args.seg[g].n_desc = pass[g]->desc_count;
            args.seg[g].n_tiles = pass[g]->n_tiles;
            args.seg[g].buf_base = (uint32_t)i;
            args.seg[g].reserved = 0;
            for (const liver::BufRef& r : pass[g]->bufs) args.bufs[i++] = (char*)resolve(r, src_bufs, dst_bufs, stage[g]);
        }
        for (; i < (size_t)liver::MAX_PASS_BUFS; ++i) args.bufs[i] = nullptr;
        const uint32_t total = a->n_tiles + b->n_tiles;
        const hipError_t e = liver::launch_fused(args, total < max_grid ? total : max_grid, (hipStream_t)hip_stream);
        if (e != hipSuccess) rc = fail(LIVER_E_HIP, std::string("kernel launch: ") + hipGetErrorString(e));
    }
    return rc;
}

size_t liver_static_staging_bytes(void) { return liver::STATIC_STAGING_BYTES; }

int liver_reshard_static(const liver_plan_t* plan, const void* const* src_bufs, void* const* dst_bufs, void* hip_stream) {
    if (!plan || !src_bufs || !dst_bufs) return fail(LIVER_E_INVALID_ARG, "null argument");
    if (plan->chunk_bytes > liver::STATIC_STAGING_BYTES)
        return fail(LIVER_E_INVALID_ARG, "the plan's chunk_bytes (" + std::to_string(plan->chunk_bytes) +
                                             ") exceeds the library's static staging array (" +
                                             std::to_string(liver::STATIC_STAGING_BYTES) +
                                             " bytes): create the plan with a smaller chunk_bytes");
    if (plan->device < 0) return fail(LIVER_E_NO_DEVICE, "plan was created without a HIP device");
    void* staging = nullptr;
    const hipError_t e = liver::static_staging(plan->device, &staging);  // resolved at plan creation; a lookup here
    if (e != hipSuccess) return fail(LIVER_E_HIP, std::string("static staging array: ") + hipGetErrorString(e));
    int rc = check_passes(plan, plan->pack, 0, (uint32_t)plan->pack.passes.size(), src_bufs, nullptr, staging);
    if (rc == LIVER_OK)
        rc = check_passes(plan, plan->unpack, 0, (uint32_t)plan->unpack.passes.size(), nullptr, dst_bufs, staging);
    const int n_chunks = (int)plan->info.n_chunks;
    for (int k = 0; k < n_chunks && rc == LIVER_OK; ++k) {  // one stream: pack(k), unpack(k), pack(k+1) run in order
        rc = launch_passes(plan, plan->pack, plan->pack.chunk_pass[k], plan->pack.chunk_pass[k + 1], src_bufs, nullptr,
                           staging, hip_stream, HINT_PACK);
        if (rc == LIVER_OK)
            rc = launch_passes(plan, plan->unpack, plan->unpack.chunk_pass[k], plan->unpack.chunk_pass[k + 1], nullptr,
                               dst_bufs, staging, hip_stream, HINT_UNPACK);
    }
    return rc;
}

int liver_debug_bandwidth_probe(int mode, const void* src, void* dst, size_t bytes, int grid, void* hip_stream) {
    const size_t tile_bytes = (size_t)liver::PROBE_TILE_UNITS * 16;
    if (mode < 0 || mode > 3) return fail(LIVER_E_INVALID_ARG, "probe mode must be 0 (read), 1 (fill), 2 (copy) or 3 (fill both)");
    if (!dst || (mode != 1 && !src)) return fail(LIVER_E_INVALID_ARG, "probe buffer is NULL");
    if ((uintptr_t)dst % 16 || (uintptr_t)src % 16) return fail(LIVER_E_INVALID_ARG, "buffers must be 16-byte aligned");
    if (bytes == 0 || bytes % tile_bytes) return fail(LIVER_E_INVALID_ARG, "probe size must be a positive multiple of 32 KiB");
    if (grid < 1 || grid > 65536) return fail(LIVER_E_INVALID_ARG, "probe grid must be 1..65536");
    if (mode == 0 && (size_t)grid * 16 > bytes) return fail(LIVER_E_INVALID_ARG, "read probe needs grid*16 <= bytes");
    const uint64_t n_tiles = bytes / tile_bytes;
    const hipError_t e = liver::launch_probe(mode, src, dst, n_tiles, (uint32_t)grid, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(LIVER_E_HIP, std::string("probe launch: ") + hipGetErrorString(e));
    return LIVER_OK;
}

const char* liver_strerror(int code) {
    static thread_local std::string msg;
    const char* base = "unknown error";
    switch (code) {
        case LIVER_OK: return "ok";
        case LIVER_E_INVALID_ARG: base = "invalid argument"; break;
        case LIVER_E_UNSUPPORTED: base = "unsupported configuration"; break;
        case LIVER_E_NOMEM: base = "out of memory"; break;
        case LIVER_E_HIP: base = "HIP error"; break;
        case LIVER_E_NO_DEVICE: base = "no HIP device"; break;
    }
    msg = base;
    if (code == g_last_code && !g_last_detail.empty()) msg += ": " + g_last_detail;  // the detail of this thread's last failure
    return msg.c_str();
}

}  // extern "C"

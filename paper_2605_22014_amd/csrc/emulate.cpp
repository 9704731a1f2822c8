// Host emulation of the LOWERED (device) descriptors, with bounds checks.
//
// A debugging aid: it executes exactly what the kernels would execute -- the same
// DevDesc tables, unit by unit -- but on host memory, and refuses any access
// outside a buffer.  It lets the lowering (ops, units, strides, tiles, passes)
// be validated without a GPU.  The data entry points (liver_pack / liver_unpack /
// liver_reshard) never call it: there is no CPU fallback.
#include <cstring>

#include "liver_debug.h"
#include "plan.hpp"

namespace {

size_t buffer_bytes(const liver_plan* plan, const liver::BufRef& r) {
    if (r.side == 2) return plan->chunk_bytes;
    const liver_layout_t& lay = r.side ? plan->dst : plan->src;
    const bool expert = r.kind >= LIVER_EXPERT_PARAM_BF16;
    const liver::StageSize& st = (r.side ? (expert ? plan->dst_xstage : plan->dst_stage)
                                         : (expert ? plan->src_xstage : plan->src_stage))[r.rank / (lay.tp * lay.dp)];
    return r.kind % 4 == 0 ? (size_t)st.n_pad * 2 : (size_t)st.S * 4;
}

uint32_t bf16_rne(uint32_t u) {
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return ((u >> 16) | 0x0040u) & 0xFFFFu;
    return ((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16) & 0xFFFFu;
}

}  // namespace

extern "C" int liver_debug_emulate_host(const liver_plan_t* plan, int list_id, int chunk, const void* const* src_bufs,
                                        void* const* dst_bufs, void* staging) {
    using namespace liver;
    if (!plan || list_id < 0 || list_id > 2) return LIVER_E_INVALID_ARG;
    const List& list = list_id == LIVER_LIST_DIRECT ? plan->direct : list_id == LIVER_LIST_PACK ? plan->pack : plan->unpack;
    if (list_id == LIVER_LIST_DIRECT) chunk = 0;
    if (chunk < 0 || (size_t)chunk + 1 >= list.chunk_pass.size()) return LIVER_E_INVALID_ARG;
    for (uint32_t pi = list.chunk_pass[chunk]; pi < list.chunk_pass[chunk + 1]; ++pi) {
        const Pass& pass = list.passes[pi];
        if (pass.bufs.size() > (size_t)MAX_PASS_BUFS) return LIVER_E_UNSUPPORTED;
        uint32_t tiles = 0;
        for (uint32_t k = 0; k < pass.desc_count; ++k) {
            const DevDesc& D = list.dev[pass.desc_begin + k];
            if (D.tile_begin != tiles || D.total == 0 || D.run == 0 || D.total % D.run) return LIVER_E_UNSUPPORTED;
            tiles += (D.total + TILE_UNITS - 1) / TILE_UNITS;
            uint32_t a_unit = 0, b_unit = 0, c_unit = 0;
            switch (D.op) {
                case DOP_COPY_V16: a_unit = b_unit = 16; break;
                case DOP_COPY_E2: a_unit = b_unit = 2; break;
                case DOP_COPY_E4: a_unit = b_unit = 4; break;
                case DOP_CAST_V4: a_unit = 16, c_unit = 8; break;
                case DOP_CAST_E: a_unit = 4, b_unit = 2; break;
                case DOP_ZERO_V16: b_unit = 16; break;
                case DOP_ZERO_E2: b_unit = 2; break;
                case DOP_ZERO_E4: b_unit = 4; break;
                case DOP_COPYCAST_V4: a_unit = b_unit = 16, c_unit = 8; break;
                default: return LIVER_E_UNSUPPORTED;
            }
            auto resolve = [&](uint16_t idx, size_t& cap) -> char* {
                if (idx >= pass.bufs.size()) return nullptr;
                const BufRef& r = pass.bufs[idx];
                cap = buffer_bytes(plan, r);
                const void* p = r.side == 0   ? (src_bufs ? src_bufs[(size_t)r.rank * LIVER_NUM_KINDS + r.kind] : nullptr)
                                : r.side == 1 ? (dst_bufs ? dst_bufs[(size_t)r.rank * LIVER_NUM_KINDS + r.kind] : nullptr)
                                              : staging;
                return (char*)p;
            };
            size_t a_cap = 0, b_cap = 0, c_cap = 0;
            char* a = a_unit ? resolve(D.a_buf, a_cap) : nullptr;
            char* b = b_unit ? resolve(D.b_buf, b_cap) : nullptr;
            char* c = c_unit ? resolve(D.c_buf, c_cap) : nullptr;
            if ((a_unit && !a) || (b_unit && !b) || (c_unit && !c)) return LIVER_E_INVALID_ARG;
            const bool dense = D.run == D.total;
            for (uint32_t u = 0; u < D.total; ++u) {
                const uint32_t r = dense ? 0 : u / D.run, col = dense ? u : u % D.run;
                const uint64_t ao = D.a_off + (uint64_t)r * D.a_stride + (uint64_t)col * a_unit;
                const uint64_t bo = D.b_off + (uint64_t)r * D.b_stride + (uint64_t)col * b_unit;
                const uint64_t co = D.c_off + (uint64_t)r * D.c_stride + (uint64_t)col * c_unit;
                if ((a_unit && ao + a_unit > a_cap) || (b_unit && bo + b_unit > b_cap) || (c_unit && co + c_unit > c_cap))
                    return LIVER_E_HIP;  // this access would fault on the device
                if (a_unit >= 16 && ao % 16) return LIVER_E_HIP;  // vector accesses must be aligned
                if (b_unit >= 16 && bo % 16) return LIVER_E_HIP;
                if (c_unit == 8 && co % 8) return LIVER_E_HIP;
                if (!a_unit) {
                    std::memset(b + bo, 0, b_unit);
                    continue;
                }
                if (b_unit && D.op != DOP_CAST_E) std::memcpy(b + bo, a + ao, b_unit);
                if (D.op == DOP_CAST_E) {
                    uint32_t x;
                    std::memcpy(&x, a + ao, 4);
                    const uint16_t y = (uint16_t)bf16_rne(x);
                    std::memcpy(b + bo, &y, 2);
                }
                if (c_unit)
                    for (int e = 0; e < 4; ++e) {
                        uint32_t x;
                        std::memcpy(&x, a + ao + 4 * e, 4);
                        const uint16_t y = (uint16_t)bf16_rne(x);
                        std::memcpy(c + co + 2 * e, &y, 2);
                    }
            }
        }
        if (tiles != pass.n_tiles) return LIVER_E_UNSUPPORTED;
    }
    return LIVER_OK;
}

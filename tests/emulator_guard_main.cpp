// Host-only driver built by tests/test_emulator_guard.py, once from the planner as it is and once from a copy
// with a planted offset error: plans a small world without padding, gives the bounds-checked emulator host
// buffers of exactly the planned sizes and prints what it returns for the direct list and for every chunk.
#include <cstdio>
#include <string>
#include <vector>

#include "liver_debug.h"
#include "plan.hpp"

int main() {
    liver_plan plan;
    plan.spec = liver_model_spec_t{4, 64, 8, 4, 96, 128, 0, LIVER_GLU};
    auto lay = [](int tp, int pp, int dp) {
        liver_layout_t l{};
        l.tp = tp, l.pp = pp, l.dp = dp, l.pad_multiple = 1, l.only_tp = l.only_pp = l.only_dp = -1;
        return l;
    };
    plan.src = lay(4, 2, 1), plan.dst = lay(2, 1, 1), plan.chunk_bytes = 4096;
    std::string why;
    if (liver::build_plan(plan, why) != LIVER_OK) {
        std::printf("build_plan failed: %s\n", why.c_str());
        return 2;
    }
    auto world = [&](const liver_layout_t& l, const std::vector<liver::StageSize>& stages,
                     std::vector<std::vector<unsigned char>>& store, std::vector<void*>& table) {
        const int n = l.tp * l.pp * l.dp;
        table.assign((size_t)n * LIVER_NUM_KINDS, nullptr);
        for (int r = 0; r < n; ++r)
            for (int k = 0; k < 4; ++k) {
                const liver::StageSize& st = stages[r / (l.tp * l.dp)];
                store.emplace_back(k == 0 ? (size_t)st.n_pad * 2 : (size_t)st.S * 4, (unsigned char)(r + k));
                table[(size_t)r * LIVER_NUM_KINDS + k] = store.back().data();
            }
    };
    std::vector<std::vector<unsigned char>> store;
    store.reserve(256);
    std::vector<void*> src, dst;
    world(plan.src, plan.src_stage, store, src);
    world(plan.dst, plan.dst_stage, store, dst);
    std::vector<unsigned char> staging(plan.chunk_bytes);
    int worst = liver_debug_emulate_host(&plan, LIVER_LIST_DIRECT, 0, src.data(), dst.data(), nullptr);
    std::printf("direct: %d\n", worst);
    for (int c = 0; c < (int)plan.info.n_chunks; ++c) {
        const int a = liver_debug_emulate_host(&plan, LIVER_LIST_PACK, c, src.data(), nullptr, staging.data());
        const int b = liver_debug_emulate_host(&plan, LIVER_LIST_UNPACK, c, nullptr, dst.data(), staging.data());
        if (a != LIVER_OK || b != LIVER_OK) {
            std::printf("chunk %d: pack %d unpack %d\n", c, a, b);
            worst = a != LIVER_OK ? a : b;
            break;
        }
    }
    std::printf("verdict: %d\n", worst);
    return 0;
}

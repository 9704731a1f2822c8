// Host-only driver for the planner, built with -fsanitize=address,undefined by
// tests/test_planner_sanitizers.py: plans a set of configurations that exercise every
// layout feature and checks basic invariants of the lowered tables.
#include <cstdio>
#include <string>

#include "plan.hpp"

static int plan_one(const char* name, liver_model_spec_t spec, liver_layout_t src, liver_layout_t dst, size_t chunk) {
    liver_plan plan;
    plan.spec = spec, plan.src = src, plan.dst = dst, plan.chunk_bytes = chunk;
    std::string why;
    const int rc = liver::build_plan(plan, why);
    if (rc != LIVER_OK) {
        std::printf("%s: build_plan failed (%d): %s\n", name, rc, why.c_str());
        return 1;
    }
    for (const liver::List* l : {&plan.direct, &plan.pack, &plan.unpack}) {
        size_t n = 0;
        for (const liver::Pass& p : l->passes) {
            uint32_t tiles = 0;
            for (uint32_t k = 0; k < p.desc_count; ++k) {
                const liver::DevDesc& d = l->dev[p.desc_begin + k];
                if (d.tile_begin != tiles || d.total == 0 || d.a_buf >= p.bufs.size() + 1 || d.b_buf >= p.bufs.size()) {
                    std::printf("%s: inconsistent device descriptor\n", name);
                    return 1;
                }
                tiles += (d.total + liver::TILE_UNITS - 1) / liver::TILE_UNITS;
            }
            if (tiles != p.n_tiles) return 1;
            n += p.desc_count;
        }
        if (n != l->dev.size()) return 1;
    }
    std::printf("%s: ok, %lld direct descriptors, %lld chunks\n", name, (long long)plan.info.n_desc, (long long)plan.info.n_chunks);
    return 0;
}

int main() {
    auto lay = [](int tp, int pp, int dp, int pm) {
        liver_layout_t l{};
        l.tp = tp, l.pp = pp, l.dp = dp, l.pad_multiple = pm, l.only_tp = l.only_pp = l.only_dp = -1;
        return l;
    };
    int bad = 0;
    liver_model_spec_t gpt{2, 256, 4, 4, 1024, 1024, 512, LIVER_NORM_BIAS | LIVER_LINEAR_BIAS | LIVER_TIED_EMBED};
    bad += plan_one("tiny_gpt", gpt, lay(2, 1, 2, 128), lay(1, 2, 2, 128), 1 << 20);
    liver_model_spec_t l7{32, 4096, 32, 32, 11008, 32000, 0, LIVER_GLU};
    bad += plan_one("llama7b", l7, lay(8, 1, 1, 128), lay(4, 2, 1, 128), 256u << 20);
    liver_model_spec_t l70{80, 8192, 64, 8, 28672, 128256, 0, LIVER_GLU};
    liver_layout_t d70 = lay(4, 8, 6, 128);
    d70.only_tp = 1, d70.only_pp = 3, d70.only_dp = 2, d70.flags = LIVER_DERIVE_BF16;
    bad += plan_one("llama70b one rank, derive", l70, lay(8, 8, 4, 128), d70, 512u << 20);
    liver_model_spec_t odd{6, 24, 6, 2, 42, 50, 5, LIVER_GLU | LIVER_NORM_BIAS | LIVER_LINEAR_BIAS | LIVER_TIED_EMBED};
    liver_layout_t a = lay(6, 3, 2, 1), b = lay(2, 2, 3, 4);
    a.vocab_multiple = 4, a.bucket_elems = 700;          // replicated kv heads, padded vocabulary, buckets
    b.vocab_multiple = 8, b.vpp = 3, b.bucket_elems = 300, b.flags = LIVER_DERIVE_BF16;
    bad += plan_one("odd: kv replication, vocab padding, buckets, vpp, derive", odd, a, b, 256);
    liver_layout_t c = lay(1, 3, 1, 1);
    c.pp_first = 1, c.pp_last = 3;
    b.flags = 0;  // as a source layout
    bad += plan_one("odd: uneven stages", odd, b, c, 512);
    liver_model_spec_t moe{4, 32, 4, 2, 24, 40, 0, LIVER_GLU | LIVER_LINEAR_BIAS, 8};   // 8 experts per layer
    liver_layout_t ma = lay(2, 2, 4, 4), mb = lay(1, 1, 6, 8);
    ma.ep = 4, ma.bucket_elems = 900;
    mb.ep = 2, mb.flags = LIVER_DERIVE_BF16, mb.only_dp = 3;
    bad += plan_one("moe: ep 4 -> ep 2, buckets, one target rank, derive", moe, ma, mb, 1024);
    return bad ? 1 : 0;
}

// Host planner: views -> intersections -> copy descriptors -> chunked stream.
//
// LiveR, Section 4.6.1 and Appendix A.2.2: the state is a set of logical tensors;
// each rank's view of a tensor is a set of index rectangles; for every (source
// view, target view) pair of a tensor the non-empty intersection becomes a
// transfer task with exact slice bounds.  Only metadata is touched.  The paper's
// view is a single hyper-rectangle; fused QKV, gated FFNs and a DP slice of a
// flattened shard need a LIST of rectangles per rank, each with its offset in
// the rank's flat buffer -- that is the only generalisation made here.
//
// Section 4.6.2 / Section 5 / Algorithm 1: tasks are executed layer by layer
// through a fixed-size staging buffer.  Here the tasks are sorted layer-major,
// laid out back to back on a byte stream and the stream is cut every chunk_bytes
// (a task that straddles a cut is split at an element boundary).
#include <algorithm>
#include <cstring>
#include <string>

#include "plan.hpp"

namespace liver {
namespace {

using i64 = int64_t;

struct Geo {
    i64 L, H, hd, nq, nkv, qpg, Q, KV, F, V, P, E;  // E: experts per layer (0 = dense model)
    bool glu, norm_bias, lin_bias, tied;
};

// logical tensor ids
enum { T_EMBED_WORD = 0, T_EMBED_POS, T_FINAL_W, T_FINAL_B, T_LM_HEAD, T_GLOBALS };
enum { LN1_W = 0, LN1_B, Q_W, K_W, V_W, Q_B, K_B, V_B, O_W, O_B, LN2_W, LN2_B, GATE_W, UP_W, GATE_B, UP_B,
       DOWN_W, DOWN_B, ROUTER_W, T_PER_LAYER };
// expert tensors follow all dense ones: id = T_GLOBALS + L*T_PER_LAYER + (l*E + e)*X_PER_EXPERT + leaf
enum { X_GATE_W = 0, X_UP_W, X_GATE_B, X_UP_B, X_DOWN_W, X_DOWN_B, X_PER_EXPERT };

// A rectangle of logical tensor `tensor` held densely (row-major, row length
// c1-c0) at element offset `loff` of a rank column's flat buffer.
struct Rect {
    int32_t tensor, slot;
    i64 r0, r1, c0, c1, loff;
    bool canonical;  // may a gather read this copy?
};

struct ZeroRegion {  // flat elements [off, off + n) of a rank column that hold padding, not state
    int slot;
    i64 off, n;
};

struct Column {
    int tp = 0, pp = 0;
    std::vector<Rect> rects;
    std::vector<ZeroRegion> zeros;            // every padding region: vocabulary padding rows, bucket padding
    std::vector<std::pair<i64, i64>> buckets;  // (start, padded size) of each bucket
    i64 n_local = 0, n_pad = 0;                // end of the last parameter; total padded size
    int last_slot = 0;
};

// Physical parameter order and shapes of rank column (tp, pp).
// Layers of stage pp in flat-buffer order: an even split, vpp interleaved model chunks, or an uneven split
// with a fixed layer count on the first / last stage.  Empty if the split is impossible.
std::vector<i64> stage_layers(i64 L, const liver_layout_t& lay, int pp) {
    const int PP = lay.pp, VPP = lay.vpp > 1 ? lay.vpp : 1;
    std::vector<i64> out;
    if (lay.pp_first > 0 || lay.pp_last > 0) {
        const int others = PP - (lay.pp_first > 0) - (lay.pp_last > 0);
        const i64 rest = L - lay.pp_first - lay.pp_last;
        if (VPP != 1 || others < 0 || rest < 0 || (others == 0 && rest != 0) || (others > 0 && (rest % others || rest == 0)))
            return out;
        auto count = [&](int p) -> i64 {
            if (p == 0 && lay.pp_first > 0) return lay.pp_first;
            if (p == PP - 1 && lay.pp_last > 0) return lay.pp_last;
            return rest / others;
        };
        i64 lo = 0;
        for (int p = 0; p < pp; ++p) lo += count(p);
        for (i64 l = lo; l < lo + count(pp); ++l) out.push_back(l);
        return out;
    }
    if (L % ((i64)PP * VPP)) return out;
    const i64 per = L / ((i64)PP * VPP);  // layers per model chunk; stage pp holds chunks pp, pp+PP, ...
    for (i64 li = 0; li < per * VPP; ++li) out.push_back(((li / per) * PP + pp) * per + li % per);
    return out;
}

inline int ep_of(const liver_layout_t& l) { return l.ep > 1 ? l.ep : 1; }

// The view function of one rank column (Section 4.6.1; Appendix A.2.2 defines a rank's view as the index
// region of each logical tensor that it holds; Appendix A.2.3 instantiates it for TP, PP and the expert
// dimension): every rectangle of a logical tensor the column holds, with its offset in the column's flat buffer.
// ep < 0: the dense buffer of rank column (tp, pp).  ep >= 0: the expert buffer held by the ranks of
// expert-parallel index ep (mixture-of-experts models only).
Column build_column(const Geo& g, const liver_layout_t& lay, int tp, int pp, int ep = -1) {
    const int TP = lay.tp, PP = lay.pp;
    const i64 vocab_multiple = lay.vocab_multiple;
    Column col;
    col.tp = tp;
    col.pp = pp;
    i64 off = 0, bucket_start = 0, params_in_bucket = 0;
    const i64 quantum = (i64)(ep < 0 ? lay.dp : lay.dp / ep_of(lay)) * lay.pad_multiple;  // ranks sharing the buffer
    // A bucket is zero-padded to a multiple of DP*pad_multiple elements when it closes.
    auto close_bucket = [&]() {
        const i64 used = off - bucket_start, padded = (used + quantum - 1) / quantum * quantum;
        if (padded > used) col.zeros.push_back({col.last_slot, off, padded - used});
        col.buckets.push_back({bucket_start, padded});
        off = bucket_start = bucket_start + padded;
        params_in_bucket = 0;
    };
    // Called after the last rectangle of every physical parameter: with bucket_elems > 0 the bucket closes
    // after the parameter that brings it to at least that many elements.
    auto end_param = [&]() {
        col.n_local = off;
        ++params_in_bucket;
        if (lay.bucket_elems > 0 && off - bucket_start >= lay.bucket_elems) close_bucket();
    };
    auto add = [&](int tensor, int slot, i64 r0, i64 r1, i64 c0, i64 c1, bool canonical, bool end = true) {
        col.rects.push_back({tensor, slot, r0, r1, c0, c1, off, canonical});
        off += (r1 - r0) * (c1 - c0);
        col.last_slot = slot;
        if (end) end_param();
    };
    const bool lead = (tp == 0);  // TP-replicated parameters are read from tp 0
    const i64 g_loc = g.nkv / TP, fn = g.F / TP, qn = g.Q / TP;
    // rows of embed.word / lm_head per rank; with vocab_multiple the vocabulary is padded to a multiple of
    // vocab_multiple*TP rows: rows >= V hold no state (zero in the target, never read from the source)
    const i64 vn = vocab_multiple > 0 ? (g.V + vocab_multiple * TP - 1) / (vocab_multiple * TP) * vocab_multiple : g.V / TP;
    auto add_vocab = [&](int tensor, int slot, bool canonical) {
        const i64 lo = tp * vn, hi = std::min(lo + vn, g.V), real = hi > lo ? (hi - lo) * g.H : 0;
        if (real > 0) col.rects.push_back({tensor, slot, lo, hi, 0, g.H, off, canonical});
        if (real < vn * g.H) col.zeros.push_back({slot, off + real, vn * g.H - real});
        off += vn * g.H;
        col.last_slot = slot;
        end_param();
    };
    // fc1 (+bias), fc2 (+bias) of one FFN: tensor ids gate_w.. given by the caller
    auto add_ffn = [&](int slot, int gate_w, int up_w, int gate_b, int up_b, int down_w, int down_b) {
        if (g.glu) add(gate_w, slot, tp * fn, (tp + 1) * fn, 0, g.H, true, false);
        add(up_w, slot, tp * fn, (tp + 1) * fn, 0, g.H, true);
        if (g.lin_bias) {
            if (g.glu) add(gate_b, slot, 0, 1, tp * fn, (tp + 1) * fn, true, false);
            add(up_b, slot, 0, 1, tp * fn, (tp + 1) * fn, true);
        }
        add(down_w, slot, 0, g.H, tp * fn, (tp + 1) * fn, true);  // row-parallel
        if (g.lin_bias) add(down_b, slot, 0, 1, 0, g.H, lead);
    };
    if (ep >= 0) {  // expert buffer: layer by layer, expert by expert
        const i64 per = g.E / ep_of(lay);
        for (const i64 l : stage_layers(g.L, lay, pp))
            for (i64 e = ep * per; e < (ep + 1) * per; ++e) {
                const int x = T_GLOBALS + (int)g.L * T_PER_LAYER + (int)(l * g.E + e) * X_PER_EXPERT;
                add_ffn(1 + (int)l, x + X_GATE_W, x + X_UP_W, x + X_GATE_B, x + X_UP_B, x + X_DOWN_W, x + X_DOWN_B);
            }
        if (params_in_bucket > 0 || col.buckets.empty()) close_bucket();
        col.n_pad = off;
        return col;
    }
    if (pp == 0) {
        add_vocab(T_EMBED_WORD, 0, true);
        if (g.P) add(T_EMBED_POS, 0, 0, g.P, 0, g.H, lead);
    }
    for (const i64 l : stage_layers(g.L, lay, pp)) {
        const int slot = 1 + (int)l;
        const int b = T_GLOBALS + (int)l * T_PER_LAYER;
        add(b + LN1_W, slot, 0, 1, 0, g.H, lead);
        if (g.norm_bias) add(b + LN1_B, slot, 0, 1, 0, g.H, lead);
        // TP > n_kv: kv group gi is replicated on rep = TP/n_kv ranks; this rank holds its part of the
        // group's q rows and a full copy of k and v (read from the rank holding part 0)
        const i64 rep = g_loc == 0 ? TP / g.nkv : 1, part = tp % rep, nq = g.qpg / rep * g.hd;
        if (g_loc == 0) {
            const i64 gi = tp / rep;
            add(b + Q_W, slot, gi * g.qpg * g.hd + part * nq, gi * g.qpg * g.hd + (part + 1) * nq, 0, g.H, true, false);
            add(b + K_W, slot, gi * g.hd, (gi + 1) * g.hd, 0, g.H, part == 0, false);
            add(b + V_W, slot, gi * g.hd, (gi + 1) * g.hd, 0, g.H, part == 0);
            if (g.lin_bias) {
                add(b + Q_B, slot, 0, 1, gi * g.qpg * g.hd + part * nq, gi * g.qpg * g.hd + (part + 1) * nq, true, false);
                add(b + K_B, slot, 0, 1, gi * g.hd, (gi + 1) * g.hd, part == 0, false);
                add(b + V_B, slot, 0, 1, gi * g.hd, (gi + 1) * g.hd, part == 0);
            }
        }
        for (i64 j = 0; j < g_loc; ++j) {  // fused qkv weight: [q of group ; k ; v] per kv group
            const i64 gi = tp * g_loc + j;
            add(b + Q_W, slot, gi * g.qpg * g.hd, (gi + 1) * g.qpg * g.hd, 0, g.H, true, false);
            add(b + K_W, slot, gi * g.hd, (gi + 1) * g.hd, 0, g.H, true, false);
            add(b + V_W, slot, gi * g.hd, (gi + 1) * g.hd, 0, g.H, true, j == g_loc - 1);
        }
        if (g.lin_bias)
            for (i64 j = 0; j < g_loc; ++j) {
                const i64 gi = tp * g_loc + j;
                add(b + Q_B, slot, 0, 1, gi * g.qpg * g.hd, (gi + 1) * g.qpg * g.hd, true, false);
                add(b + K_B, slot, 0, 1, gi * g.hd, (gi + 1) * g.hd, true, false);
                add(b + V_B, slot, 0, 1, gi * g.hd, (gi + 1) * g.hd, true, j == g_loc - 1);
            }
        add(b + O_W, slot, 0, g.H, tp * qn, (tp + 1) * qn, true);  // row-parallel: a strip of every row
        if (g.lin_bias) add(b + O_B, slot, 0, 1, 0, g.H, lead);
        add(b + LN2_W, slot, 0, 1, 0, g.H, lead);
        if (g.norm_bias) add(b + LN2_B, slot, 0, 1, 0, g.H, lead);
        if (g.E > 0)
            add(b + ROUTER_W, slot, 0, g.E, 0, g.H, lead);  // the experts themselves live in the expert buffers
        else
            add_ffn(slot, b + GATE_W, b + UP_W, b + GATE_B, b + UP_B, b + DOWN_W, b + DOWN_B);
    }
    if (pp == PP - 1) {
        const int slot = (int)g.L + 1;
        add(T_FINAL_W, slot, 0, 1, 0, g.H, lead);
        if (g.norm_bias) add(T_FINAL_B, slot, 0, 1, 0, g.H, lead);
        if (!g.tied)
            add_vocab(T_LM_HEAD, slot, true);
        else if (PP > 1)  // second copy of the tied embedding: written, never read
            add_vocab(T_EMBED_WORD, slot, false);
    }
    if (params_in_bucket > 0 || col.buckets.empty()) close_bucket();  // the last bucket takes what is left
    col.n_pad = off;
    return col;
}

// A strided 2-D piece with one source and one or more destinations.  Offsets and
// strides in elements; row i is [off + i*stride, off + i*stride + run).
struct Dst {
    int32_t rank, kind, op;
    i64 off, stride;
};
struct Entry {
    int32_t slot = 0, src_rank = -1, src_kind = -1;
    i64 src_off = 0, src_stride = 0, rows = 1, run = 0;
    std::vector<Dst> dsts;
};

inline int elem_bytes(int kind) { return kind % 4 == 0 ? 2 : 4; }  // kinds 0 and 4 are bf16

// Payload elements [p0, p1) of `e` (row-major over rows x run) as up to three
// pieces: the tail of a row, whole rows, the head of a row.
void slice(const Entry& e, i64 p0, i64 p1, std::vector<Entry>& out) {
    auto sub = [&](i64 row, i64 col, i64 nrows, i64 ncols) {
        Entry s = e;
        s.src_off = e.src_off + row * e.src_stride + col;
        s.rows = nrows;
        s.run = ncols;
        bool dense = (e.src_rank < 0 || e.src_stride == ncols);
        for (auto& d : s.dsts) {
            d.off += row * d.stride + col;
            dense = dense && d.stride == ncols;
        }
        if (nrows == 1 || dense) {  // one contiguous run on every side
            s.run = nrows * ncols;
            s.rows = 1;
            s.src_stride = s.run;
            for (auto& d : s.dsts) d.stride = s.run;
        }
        out.push_back(std::move(s));
    };
    if (p0 >= p1) return;
    if (e.rows == 1) {
        sub(0, p0, 1, p1 - p0);
        return;
    }
    i64 r0 = p0 / e.run, c0 = p0 % e.run, r1 = p1 / e.run, c1 = p1 % e.run;
    if (r0 == r1) {
        sub(r0, c0, 1, c1 - c0);
        return;
    }
    if (c0 > 0) {
        sub(r0, c0, 1, e.run - c0);
        ++r0;
    }
    if (r1 > r0) sub(r0, 0, r1 - r0, e.run);
    if (c1 > 0) sub(r1, 0, 1, c1);
}

// Payload positions at which the piece (off, stride, rows, run) crosses one of the sorted flat-buffer
// boundaries `bounds` (where the owning bucket or DP rank changes).
void boundary_cuts(i64 off, i64 stride, i64 rows, i64 run, const std::vector<i64>& bounds, std::vector<i64>& cuts) {
    const i64 end = off + (rows - 1) * stride + run;  // one past the last element
    for (auto it = std::upper_bound(bounds.begin(), bounds.end(), off); it != bounds.end() && *it < end; ++it) {
        const i64 b = *it;
        if (rows == 1) {
            cuts.push_back(b - off);
            continue;
        }
        const i64 x = b - off - run;                  // rows i with off+i*stride+run <= b lie before b
        const i64 i = x < 0 ? 0 : x / stride + 1;     // first row that reaches past b
        if (i >= rows) continue;
        const i64 start = off + i * stride;
        cuts.push_back(start >= b ? i * run : i * run + (b - start));
    }
}

// Flat offset -> (DP rank, offset in that rank's fp32 buffer).
void locate(const StageSize& st, i64 flat, int& dp, i64& local) {
    size_t lo = 0, hi = st.buckets.size();
    while (hi - lo > 1) {
        const size_t mid = (lo + hi) / 2;
        if (st.buckets[mid].start <= flat) lo = mid;
        else hi = mid;
    }
    const Bucket& b = st.buckets[lo];
    dp = (int)((flat - b.start) / b.slice);
    local = b.prefix + (flat - b.start) - dp * b.slice;
}

struct Builder {
    liver_plan& plan;
    Geo g{};
    std::vector<Entry> entries;
    std::string why;

    explicit Builder(liver_plan& p) : plan(p) {}

    int rank_of(const liver_layout_t& lay, int tp, int pp, int dp) const { return tp + lay.tp * (dp + lay.dp * pp); }
    bool dst_dp_planned(int dp) const { return plan.dst.only_dp < 0 || plan.dst.only_dp == dp; }
    // Source-side restriction: does the plan read from this source rank?  (pack and direct lists only; the
    // wire layout and the unpack list do not depend on it)
    bool src_planned(int rank) const {
        const liver_layout_t& S = plan.src;
        const int tp = rank % S.tp, dp = (rank / S.tp) % S.dp, pp = rank / (S.tp * S.dp);
        return (S.only_tp < 0 || S.only_tp == tp) && (S.only_pp < 0 || S.only_pp == pp) && (S.only_dp < 0 || S.only_dp == dp);
    }
    bool kind_on(int k) const { return plan.dst.kind_mask == 0 || ((plan.dst.kind_mask >> (k % 4)) & 1u); }

    // The family being planned: the dense buffers (kinds 0..3, shared by all DP ranks of a column) or the
    // expert buffers (kinds 4..7, shared by the DP ranks with the same expert-parallel index).
    bool expert = false;
    int kbase() const { return expert ? LIVER_EXPERT_PARAM_BF16 : LIVER_PARAM_BF16; }
    const std::vector<StageSize>& stages(bool dst) const {
        return dst ? (expert ? plan.dst_xstage : plan.dst_stage) : (expert ? plan.src_xstage : plan.src_stage);
    }
    int group_size(const liver_layout_t& l) const { return expert ? l.dp / ep_of(l) : l.dp; }
    // j-th rank (in slice order) of the group that shares the buffer of expert-parallel index ep
    int group_dp(const liver_layout_t& l, int ep, int j) const { return expert ? ep + ep_of(l) * j : j; }

    static constexpr size_t MAX_ENTRIES = size_t(1) << 22;

    void push_bounded(Entry&& e) {  // keep every entry below 2^30 elements (32-bit unit counters)
        const i64 lim = i64(1) << 30, total = e.rows * e.run;
        if (total <= lim) {
            entries.push_back(std::move(e));
            return;
        }
        for (i64 p = 0; p < total; p += lim) slice(e, p, std::min(total, p + lim), entries);
    }

    // One intersection piece in flat coordinates of columns (s_tp,s_pp) -> (d_tp,d_pp):
    // expand it per buffer kind, clipping the fp32 kinds at the DP slice boundaries.  The DP rules of
    // Appendix A.2.3 fall out here: a replicated kind is read from one replica and written to every
    // planned target replica (growing DP copies, shrinking DP drops copies).
    void expand(int slot, int s_tp, int s_pp, int s_ep, int d_tp, int d_pp, int d_ep, i64 s_off, i64 s_stride,
                i64 d_off, i64 d_stride, i64 rows, i64 run) {
        const liver_layout_t &S = plan.src, &D = plan.dst;
        const bool derive = (D.flags & LIVER_DERIVE_BF16) != 0;
        const int kb = kbase(), n_dst = group_size(D);
        if (entries.size() > MAX_ENTRIES) return;  // plan_family reports it after this column
        if (kind_on(LIVER_PARAM_BF16) && !derive) {
            for (int j = 0; j < n_dst; ++j) {
                const int dp = group_dp(D, d_ep, j);
                if (!dst_dp_planned(dp)) continue;
                Entry e;
                e.slot = slot;
                e.src_rank = rank_of(S, s_tp, s_pp, group_dp(S, s_ep, 0));  // replicas are identical: read the first
                e.src_kind = kb;
                e.src_off = s_off, e.src_stride = s_stride, e.rows = rows, e.run = run;
                e.dsts.push_back({rank_of(D, d_tp, d_pp, dp), kb, LIVER_OP_COPY, d_off, d_stride});
                push_bounded(std::move(e));
            }
        }
        const bool any_f32 = kind_on(LIVER_MASTER_F32) || kind_on(LIVER_ADAM_M_F32) || kind_on(LIVER_ADAM_V_F32);
        if (!any_f32 && !(derive && kind_on(LIVER_PARAM_BF16))) return;
        // cut where the owning bucket / DP rank changes, on the source and on the target side
        const StageSize &sst = stages(false)[s_pp], &dst_st = stages(true)[d_pp];
        std::vector<i64> cuts{0, rows * run};
        boundary_cuts(s_off, s_stride, rows, run, sst.bounds, cuts);
        boundary_cuts(d_off, d_stride, rows, run, dst_st.bounds, cuts);
        std::sort(cuts.begin(), cuts.end());
        cuts.erase(std::unique(cuts.begin(), cuts.end()), cuts.end());
        Entry flat;
        flat.slot = slot;
        flat.src_rank = 0;
        flat.src_off = s_off, flat.src_stride = s_stride, flat.rows = rows, flat.run = run;
        flat.dsts.push_back({0, 0, LIVER_OP_COPY, d_off, d_stride});
        std::vector<Entry> parts;
        for (size_t c = 0; c + 1 < cuts.size(); ++c) slice(flat, cuts[c], cuts[c + 1], parts);
        for (const Entry& p : parts) {
            int sj, dj;  // position of the owning rank inside its group
            i64 s_local, d_local;
            locate(sst, p.src_off, sj, s_local);
            locate(dst_st, p.dsts[0].off, dj, d_local);
            const int sdp = group_dp(S, s_ep, sj), ddp = group_dp(D, d_ep, dj);
            for (int k = LIVER_MASTER_F32; k <= LIVER_ADAM_V_F32; ++k) {
                Entry e;
                e.slot = slot;
                e.src_rank = rank_of(S, s_tp, s_pp, sdp);
                e.src_kind = kb + k;
                e.src_off = s_local, e.src_stride = p.src_stride, e.rows = p.rows, e.run = p.run;
                if (kind_on(k) && dst_dp_planned(ddp))
                    e.dsts.push_back({rank_of(D, d_tp, d_pp, ddp), kb + k, LIVER_OP_COPY, d_local, p.dsts[0].stride});
                if (k == LIVER_MASTER_F32 && derive && kind_on(LIVER_PARAM_BF16))
                    for (int j = 0; j < n_dst; ++j) {  // bf16 replicas come from the MASTER element
                        const int dp = group_dp(D, d_ep, j);  // with the same logical index
                        if (dst_dp_planned(dp))
                            e.dsts.push_back({rank_of(D, d_tp, d_pp, dp), kb, LIVER_OP_CAST_BF16, p.dsts[0].off,
                                              p.dsts[0].stride});
                    }
                if (!e.dsts.empty()) push_bounded(std::move(e));
            }
        }
    }

    void zero_padding(const Column& col, int d_ep) {
        const liver_layout_t& D = plan.dst;
        const StageSize& st = stages(true)[col.pp];
        const int kb = kbase();
        for (const ZeroRegion& z : col.zeros) {  // vocabulary padding rows and the padding of every bucket
            if (kind_on(LIVER_PARAM_BF16))
                for (int j = 0; j < group_size(D); ++j) {
                    const int dp = group_dp(D, d_ep, j);
                    if (!dst_dp_planned(dp)) continue;
                    Entry e;
                    e.slot = z.slot;
                    e.run = z.n;
                    e.dsts.push_back({rank_of(D, col.tp, col.pp, dp), kb, LIVER_OP_ZERO, z.off, z.n});
                    push_bounded(std::move(e));
                }
            // fp32 kinds: the region may span several DP ranks' slices
            std::vector<i64> cuts{z.off, z.off + z.n};
            for (auto it = std::upper_bound(st.bounds.begin(), st.bounds.end(), z.off); it != st.bounds.end() && *it < z.off + z.n; ++it)
                cuts.push_back(*it);
            std::sort(cuts.begin(), cuts.end());
            for (size_t c = 0; c + 1 < cuts.size(); ++c) {
                int j;
                i64 local;
                locate(st, cuts[c], j, local);
                const int dp = group_dp(D, d_ep, j);
                if (!dst_dp_planned(dp)) continue;
                for (int k = LIVER_MASTER_F32; k <= LIVER_ADAM_V_F32; ++k) {
                    if (!kind_on(k)) continue;
                    Entry e;
                    e.slot = z.slot;
                    e.run = cuts[c + 1] - cuts[c];
                    e.dsts.push_back({rank_of(D, col.tp, col.pp, dp), kb + k, LIVER_OP_ZERO, local, e.run});
                    push_bounded(std::move(e));
                }
            }
        }
    }

    int run();
    int plan_family();
    int emit_lists();
    int lower(List& list, bool staged);
};

int Builder::run() {
    const liver_model_spec_t& sp = plan.spec;
    const liver_layout_t &S = plan.src, &D = plan.dst;
    if (sp.n_layers <= 0 || sp.hidden <= 0 || sp.n_q_heads <= 0 || sp.n_kv_heads <= 0 || sp.ffn <= 0 ||
        sp.vocab <= 0 || sp.max_pos < 0 || (sp.flags & ~15u) || sp.n_experts < 0) {
        why = "model_spec: dimensions must be positive";
        return LIVER_E_INVALID_ARG;
    }
    for (const liver_layout_t* l : {&S, &D})
        if (l->tp <= 0 || l->pp <= 0 || l->dp <= 0 || l->pad_multiple <= 0 || l->vpp < 0 || l->vocab_multiple < 0 ||
            l->pp_first < 0 || l->pp_last < 0 || l->bucket_elems < 0 || l->ep < 0) {
            why = "layout: tp, pp, dp, pad_multiple must be positive; vpp, vocab_multiple, pp_first, pp_last, bucket_elems, ep non-negative";
            return LIVER_E_INVALID_ARG;
        }
    // Sanity caps, far above any real model or cluster: they keep a garbage struct (say, uninitialised memory)
    // from turning into hours of planning or an allocation of many gigabytes, and all products below in 64 bits.
    constexpr int DIM_CAP = 1 << 24, COUNT_CAP = 1 << 16;
    if (sp.n_layers > COUNT_CAP || sp.n_q_heads > COUNT_CAP || sp.n_experts > COUNT_CAP || sp.hidden > DIM_CAP ||
        sp.ffn > DIM_CAP || sp.vocab > DIM_CAP || sp.max_pos > DIM_CAP) {
        why = "model_spec: more than 2^16 layers, heads or experts, or a dimension above 2^24";
        return LIVER_E_UNSUPPORTED;
    }
    for (const liver_layout_t* l : {&S, &D})
        if (l->tp > DIM_CAP || l->pp > COUNT_CAP || l->dp > DIM_CAP || (i64)l->tp * l->pp > DIM_CAP ||
            (i64)l->tp * l->pp * l->dp > DIM_CAP || l->pad_multiple > DIM_CAP || l->vocab_multiple > DIM_CAP ||
            l->vpp > COUNT_CAP || l->ep > DIM_CAP) {
            why = "layout: more than 2^24 ranks, 2^16 stages or model chunks, or a padding multiple above 2^24";
            return LIVER_E_UNSUPPORTED;
        }
    if (plan.chunk_bytes < 256 || plan.chunk_bytes % 256) {
        why = "chunk_bytes must be a positive multiple of 256";
        return LIVER_E_INVALID_ARG;
    }
    if (sp.hidden % sp.n_q_heads || sp.n_q_heads % sp.n_kv_heads) {
        why = "hidden % n_q_heads or n_q_heads % n_kv_heads != 0";
        return LIVER_E_UNSUPPORTED;
    }
    for (const liver_layout_t* l : {&S, &D}) {
        const bool kv_ok = sp.n_kv_heads % l->tp == 0 ||
                           (l->tp % sp.n_kv_heads == 0 && (sp.n_q_heads / sp.n_kv_heads) % (l->tp / sp.n_kv_heads) == 0);
        bool stages_ok = true;
        for (int p = 0; p < l->pp; ++p) stages_ok = stages_ok && !stage_layers(sp.n_layers, *l, p).empty();
        const bool ep_ok = sp.n_experts > 0 ? (l->dp % ep_of(*l) == 0 && sp.n_experts % ep_of(*l) == 0) : ep_of(*l) == 1;
        if (!stages_ok || !kv_ok || !ep_ok || sp.ffn % l->tp || (sp.vocab % l->tp && l->vocab_multiple == 0)) {
            why = "layers do not split over the stages, ffn % tp or vocab % tp != 0, kv heads neither split nor replicated evenly over tp, or ep does not divide dp and n_experts";
            return LIVER_E_UNSUPPORTED;
        }
    }
    if (S.only_tp < -1 || S.only_tp >= S.tp || S.only_pp < -1 || S.only_pp >= S.pp || S.only_dp < -1 ||
        S.only_dp >= S.dp || S.flags || S.kind_mask) {
        why = "source layout: only_* out of range, or flags / kind_mask not 0";
        return LIVER_E_UNSUPPORTED;
    }
    if (D.only_tp < -1 || D.only_tp >= D.tp || D.only_pp < -1 || D.only_pp >= D.pp || D.only_dp < -1 ||
        D.only_dp >= D.dp || (D.flags & ~1u) || (D.kind_mask & ~15u)) {
        why = "target layout: only_* out of range or unknown flag";
        return LIVER_E_UNSUPPORTED;
    }
    g.L = sp.n_layers, g.H = sp.hidden, g.nq = sp.n_q_heads, g.nkv = sp.n_kv_heads;
    g.hd = g.H / g.nq, g.qpg = g.nq / g.nkv, g.Q = g.nq * g.hd, g.KV = g.nkv * g.hd;
    g.F = sp.ffn, g.V = sp.vocab, g.P = sp.max_pos, g.E = sp.n_experts;
    g.glu = sp.flags & LIVER_GLU, g.norm_bias = sp.flags & LIVER_NORM_BIAS;
    g.lin_bias = sp.flags & LIVER_LINEAR_BIAS, g.tied = sp.flags & LIVER_TIED_EMBED;

    // --- views of both worlds (Abstract Resource View) ---------------------------------
    auto stage_sizes = [&](const liver_layout_t& lay, std::vector<StageSize>& out, bool xp) {
        out.resize(lay.pp);
        const int group = xp ? lay.dp / ep_of(lay) : lay.dp;
        for (int pp = 0; pp < lay.pp; ++pp) {
            const Column c = build_column(g, lay, 0, pp, xp ? 0 : -1);  // sizes do not depend on tp / ep
            StageSize s;
            s.n_local = c.n_local, s.n_pad = c.n_pad, s.S = c.n_pad / group;
            i64 prefix = 0;
            for (const auto& b : c.buckets) {
                Bucket k;
                k.start = b.first, k.padded = b.second, k.slice = b.second / group, k.prefix = prefix;
                prefix += k.slice;
                for (int d = 0; d < group; ++d) s.bounds.push_back(k.start + d * k.slice);
                s.buckets.push_back(k);
            }
            out[pp] = s;
        }
    };
    stage_sizes(S, plan.src_stage, false);
    stage_sizes(D, plan.dst_stage, false);
    if (g.E > 0) {
        stage_sizes(S, plan.src_xstage, true);
        stage_sizes(D, plan.dst_xstage, true);
    }
    for (int fam = 0; fam < (g.E > 0 ? 2 : 1); ++fam) {  // dense buffers, then expert buffers
        expert = fam == 1;
        const int rc = plan_family();
        if (rc != LIVER_OK) return rc;
    }
    // --- stream order: layer-major, then target rank, kind, target offset ---------------
    std::stable_sort(entries.begin(), entries.end(), [](const Entry& a, const Entry& b) {
        const Dst &x = a.dsts[0], &y = b.dsts[0];
        if (a.slot != b.slot) return a.slot < b.slot;
        if (x.rank != y.rank) return x.rank < y.rank;
        if (x.kind != y.kind) return x.kind < y.kind;
        return x.off < y.off;
    });
    if (int rc = emit_lists()) return rc;
    int rc = lower(plan.direct, false);
    if (rc == LIVER_OK) rc = lower(plan.pack, true);
    if (rc == LIVER_OK) rc = lower(plan.unpack, true);
    if (rc != LIVER_OK) return rc;

    liver_plan_info_t& info = plan.info;
    info.n_desc = (i64)plan.direct.pub.size();
    info.n_desc_pack = (i64)plan.pack.pub.size();
    info.n_desc_unpack = (i64)plan.unpack.pub.size();
    info.n_src_ranks = S.tp * S.pp * S.dp;
    info.n_dst_ranks = D.tp * D.pp * D.dp;
    plan.used[0].assign((size_t)info.n_src_ranks * LIVER_NUM_KINDS, 0);
    plan.used[1].assign((size_t)info.n_dst_ranks * LIVER_NUM_KINDS, 0);
    for (const liver_desc_t& d : plan.direct.pub) {
        if (d.op != LIVER_OP_ZERO) plan.used[0][(size_t)d.src_rank * LIVER_NUM_KINDS + d.src_kind] = 1;
        else info.pad_bytes += d.rows * d.run * elem_bytes(d.dst_kind);
        plan.used[1][(size_t)d.dst_rank * LIVER_NUM_KINDS + d.dst_kind] = 1;
    }
    info.bytes_read = plan.direct.hbm_read;        // a piece that feeds a fused copy + cast is read once
    info.bytes_written = plan.direct.hbm_written;
    for (uint8_t u : plan.used[0]) info.n_src_bufs_used += u;
    for (uint8_t u : plan.used[1]) info.n_dst_bufs_used += u;
    const uint64_t nd = plan.direct.dev.size(), np = plan.pack.dev.size(), nu = plan.unpack.dev.size();
    plan.direct.dev_offset = 0;
    plan.pack.dev_offset = nd * sizeof(DevDesc);
    plan.unpack.dev_offset = (nd + np) * sizeof(DevDesc);
    info.table_bytes_device = (i64)((nd + np + nu) * sizeof(DevDesc));
    return LIVER_OK;
}

// Views, intersections and entries of one buffer family (`expert` selects it).  Appendix A.2.2: a task is a
// non-empty intersection of a source and a target view of the same tensor; views of different tensors
// never meet, which is the pruning that keeps planning linear in the number of tensors.
int Builder::plan_family() {
    const liver_layout_t &S = plan.src, &D = plan.dst;
    const int n_tensors = T_GLOBALS + (int)g.L * T_PER_LAYER + (int)(g.L * g.E) * X_PER_EXPERT;
    const int s_eps = expert ? ep_of(S) : 1, d_eps = expert ? ep_of(D) : 1;
    struct SrcRect {
        Rect r;
        int tp, pp, ep;
    };
    std::vector<std::vector<SrcRect>> by_tensor(n_tensors);  // pruning: only views of the same tensor meet
    for (int pp = 0; pp < S.pp; ++pp)
        for (int tp = 0; tp < S.tp; ++tp)
            for (int ep = 0; ep < s_eps; ++ep) {
                Column c = build_column(g, S, tp, pp, expert ? ep : -1);
                for (const Rect& r : c.rects)
                    if (r.canonical) by_tensor[r.tensor].push_back({r, tp, pp, ep});
            }

    // --- intersect every target view with the source views of its tensor ----------------
    struct Piece {
        int slot, s_tp, s_pp, s_ep;
        i64 s_off, s_stride, d_off, d_stride, rows, run;
    };
    for (int pp = 0; pp < D.pp; ++pp) {
        if (D.only_pp >= 0 && D.only_pp != pp) continue;
        for (int tp = 0; tp < D.tp; ++tp)
          for (int d_ep = 0; d_ep < d_eps; ++d_ep) {
            if (D.only_tp >= 0 && D.only_tp != tp) continue;
            if (expert && D.only_dp >= 0 && D.only_dp % ep_of(D) != d_ep) continue;  // that rank holds other experts
            Column col = build_column(g, D, tp, pp, expert ? d_ep : -1);
            std::vector<Piece> pieces;
            for (const Rect& d : col.rects) {
                const i64 dw = d.c1 - d.c0;
                i64 covered = 0;
                for (const SrcRect& sr : by_tensor[d.tensor]) {
                    const Rect& s = sr.r;
                    const i64 r0 = std::max(d.r0, s.r0), r1 = std::min(d.r1, s.r1);
                    const i64 c0 = std::max(d.c0, s.c0), c1 = std::min(d.c1, s.c1);
                    if (r0 >= r1 || c0 >= c1) continue;  // empty intersection: no task
                    const i64 sw = s.c1 - s.c0;
                    Piece p{d.slot, sr.tp, sr.pp, sr.ep, s.loff + (r0 - s.r0) * sw + (c0 - s.c0), sw,
                            d.loff + (r0 - d.r0) * dw + (c0 - d.c0), dw, r1 - r0, c1 - c0};
                    if (p.rows == 1 || (p.s_stride == p.run && p.d_stride == p.run)) {
                        p.run *= p.rows;  // dense on both sides: one run
                        p.rows = 1;
                        p.s_stride = p.d_stride = p.run;
                    }
                    covered += p.rows * p.run;
                    pieces.push_back(p);
                }
                if (covered != (d.r1 - d.r0) * dw) {  // Eq. 1 would be violated
                    why = "internal: a target view is not tiled by the source views";
                    return LIVER_E_UNSUPPORTED;
                }
            }
            // merge pieces that continue each other on both sides (same source column)
            std::sort(pieces.begin(), pieces.end(), [](const Piece& a, const Piece& b) { return a.d_off < b.d_off; });
            std::vector<Piece> merged;
            for (const Piece& p : pieces) {
                if (!merged.empty()) {
                    Piece& m = merged.back();
                    const bool same = m.slot == p.slot && m.s_tp == p.s_tp && m.s_pp == p.s_pp && m.s_ep == p.s_ep;
                    if (same && m.rows == 1 && p.rows == 1 && p.s_off == m.s_off + m.run && p.d_off == m.d_off + m.run) {
                        m.run += p.run;
                        m.s_stride = m.d_stride = m.run;
                        continue;
                    }
                    if (same && m.rows > 1 && p.rows > 1 && m.run == p.run && m.s_stride == p.s_stride &&
                        m.d_stride == p.d_stride && p.s_off == m.s_off + m.rows * m.s_stride &&
                        p.d_off == m.d_off + m.rows * m.d_stride) {
                        m.rows += p.rows;
                        continue;
                    }
                }
                merged.push_back(p);
            }
            for (const Piece& p : merged)
                expand(p.slot, p.s_tp, p.s_pp, p.s_ep, tp, pp, d_ep, p.s_off, p.s_stride, p.d_off, p.d_stride, p.rows, p.run);
            zero_padding(col, d_ep);
            if (entries.size() > MAX_ENTRIES) {  // sanity cap; the 175B model on 1024 ranks needs ~10^5
                why = "the plan would have more than 2^22 transfer tasks";
                return LIVER_E_UNSUPPORTED;
            }
        }
    }
    return LIVER_OK;
}

// Direct list: one descriptor per (entry, destination).  Staged lists: walk the
// entries in stream order, give each its place on the wire, split at chunk ends
// (Section 4.6.2 and Appendix A.2.4: the state streams through one staging buffer of
// fixed size B, so at most B bytes are in flight whatever the model size; Appendix A.1).
int Builder::emit_lists() {
    const i64 B = (i64)plan.chunk_bytes;
    {   // every chunk costs descriptors and a launch: refuse a staging chunk that is absurdly small for this state
        i64 wire = 0;
        for (const Entry& e : entries)
            if (e.src_rank >= 0) wire += e.rows * e.run * elem_bytes(e.src_kind) + 16;
        if (wire / B >= (i64(1) << 20)) {
            why = "chunk_bytes is too small for this state: the stream would have more than 2^20 chunks";
            return LIVER_E_UNSUPPORTED;
        }
    }
    auto pub = [](const Entry& e, const Dst& d, int chunk) {
        liver_desc_t o{};
        o.op = d.op, o.chunk = chunk, o.slot = e.slot;
        o.src_rank = e.src_rank, o.src_kind = e.src_kind;
        o.dst_rank = d.rank, o.dst_kind = d.kind;
        o.src_off = e.src_off, o.src_stride = e.src_stride;
        o.dst_off = d.off, o.dst_stride = d.stride;
        o.rows = e.rows, o.run = e.run;
        return o;
    };
    i64 pos = 0;  // byte position on the stream
    std::vector<Entry> subs;
    for (const Entry& e : entries) {
        const bool read_here = e.src_rank < 0 || src_planned(e.src_rank);  // zero fills are always planned
        if (read_here)
            for (const Dst& d : e.dsts) plan.direct.pub.push_back(pub(e, d, -1));
        if (e.src_rank < 0) {  // zero fill: no wire bytes; belongs to the chunk the stream is in
            const i64 chunk = pos == 0 ? 0 : (pos - 1) / B;
            for (const Dst& d : e.dsts) plan.unpack.pub.push_back(pub(e, d, (int)chunk));
            continue;
        }
        const i64 eb = elem_bytes(e.src_kind), total = e.rows * e.run;
        i64 p = 0;
        pos = (pos + 15) / 16 * 16;  // every entry starts 16-byte aligned on the wire
        while (p < total) {
            const i64 chunk = pos / B, room = ((chunk + 1) * B - pos) / eb;
            if (room == 0) {
                pos = (chunk + 1) * B;
                continue;
            }
            const i64 take = std::min(total - p, room);
            subs.clear();
            slice(e, p, p + take, subs);
            for (const Entry& s : subs) {
                const i64 wire_elem = (pos - chunk * B) / eb;  // offset inside the chunk, in wire elements
                liver_desc_t pk{};
                pk.op = LIVER_OP_COPY, pk.chunk = (int)chunk, pk.slot = s.slot;
                pk.src_rank = s.src_rank, pk.src_kind = s.src_kind, pk.dst_rank = -1, pk.dst_kind = -1;
                pk.src_off = s.src_off, pk.src_stride = s.src_stride;
                pk.dst_off = wire_elem, pk.dst_stride = s.run, pk.rows = s.rows, pk.run = s.run;
                if (read_here) plan.pack.pub.push_back(pk);
                for (const Dst& d : s.dsts) {
                    liver_desc_t un = pub(s, d, (int)chunk);
                    un.src_rank = -1;  // staging; src_kind keeps the wire element type
                    un.src_off = wire_elem, un.src_stride = s.run;
                    plan.unpack.pub.push_back(un);
                }
                pos += s.rows * s.run * eb;
            }
            p += take;
        }
    }
    plan.info.stream_bytes = pos;
    plan.info.n_chunks = (pos + B - 1) / B;
    // chunk order (the unpack list can hold zero fills slightly out of order)
    auto by_chunk = [](const liver_desc_t& a, const liver_desc_t& b) { return a.chunk < b.chunk; };
    std::stable_sort(plan.unpack.pub.begin(), plan.unpack.pub.end(), by_chunk);
    return LIVER_OK;
}

// Turn public descriptors into device descriptors, grouped into launches.
int Builder::lower(List& list, bool staged) {
    const size_t n_chunks = staged ? (size_t)plan.info.n_chunks : 1;
    list.chunk_pass.assign(n_chunks + 1, 0);
    int cur_chunk = staged ? -1 : 0;
    auto new_pass = [&]() {
        Pass p;
        p.desc_begin = (uint32_t)list.dev.size();
        list.passes.push_back(std::move(p));
    };
    auto buf_index = [&](Pass& p, BufRef r) -> int {
        for (size_t i = 0; i < p.bufs.size(); ++i)
            if (p.bufs[i] == r) return (int)i;
        return -1;
    };
    if (!staged) new_pass();
    auto ref_a = [](const liver_desc_t& d) {
        return BufRef{int8_t(d.src_rank < 0 ? 2 : 0), int8_t(d.src_rank < 0 ? 0 : d.src_kind), d.src_rank < 0 ? 0 : d.src_rank};
    };
    auto ref_b = [](const liver_desc_t& d) {
        return BufRef{int8_t(d.dst_rank < 0 ? 2 : 1), int8_t(d.dst_rank < 0 ? 0 : d.dst_kind), d.dst_rank < 0 ? 0 : d.dst_rank};
    };
    auto add_buf = [&](Pass& p, BufRef r) {
        int i = buf_index(p, r);
        if (i < 0) {
            i = (int)p.bufs.size();
            p.bufs.push_back(r);
        }
        return (uint16_t)i;
    };
    for (size_t di = 0; di < list.pub.size(); ++di) {
        const liver_desc_t& d = list.pub[di];
        if (staged && d.chunk != cur_chunk) {
            for (int c = cur_chunk + 1; c <= d.chunk; ++c) list.chunk_pass[c] = (uint32_t)list.passes.size();
            cur_chunk = d.chunk;
            new_pass();
        }
        const bool zero = d.op == LIVER_OP_ZERO, rows1 = d.rows == 1;
        // element sizes on each side (the wire keeps the source type)
        const i64 ea = zero ? 0 : elem_bytes(d.src_kind);
        const i64 eb = d.dst_rank < 0 ? ea : elem_bytes(d.dst_kind);
        DevDesc v{};
        v.a_off = (uint64_t)(d.src_off * ea);
        v.b_off = (uint64_t)(d.dst_off * eb);
        i64 a_stride = d.src_stride * ea, b_stride = d.dst_stride * eb, c_stride = 0;
        const liver_desc_t* fused = nullptr;  // a CAST of the very same source piece that follows a COPY
        if (d.op == LIVER_OP_COPY && ea == 4 && di + 1 < list.pub.size()) {
            const liver_desc_t& n = list.pub[di + 1];
            if (n.op == LIVER_OP_CAST_BF16 && n.chunk == d.chunk && n.src_rank == d.src_rank && n.src_kind == d.src_kind &&
                n.src_off == d.src_off && n.src_stride == d.src_stride && n.rows == d.rows && n.run == d.run &&
                v.a_off % 16 == 0 && v.b_off % 16 == 0 && (n.dst_off * 2) % 8 == 0 && d.run % 4 == 0 &&
                (rows1 || (a_stride % 16 == 0 && b_stride % 16 == 0 && (n.dst_stride * 2) % 8 == 0)))
                fused = &n;
        }
        {
            Pass& p = list.passes.back();
            int need = (zero || buf_index(p, ref_a(d)) >= 0 ? 0 : 1) + (buf_index(p, ref_b(d)) >= 0 ? 0 : 1) +
                       (fused && buf_index(p, ref_b(*fused)) < 0 ? 1 : 0);
            if ((int)p.bufs.size() + need > MAX_PASS_BUFS) new_pass();
        }
        Pass& p = list.passes.back();
        v.a_buf = zero ? 0 : add_buf(p, ref_a(d));
        v.b_buf = add_buf(p, ref_b(d));
        const bool al16 = v.a_off % 16 == 0 && v.b_off % 16 == 0 && (rows1 || (a_stride % 16 == 0 && b_stride % 16 == 0));
        i64 run_units, a_unit, w_unit;  // bytes read / written per unit (for the traffic statistics)
        if (fused) {
            v.op = DOP_COPYCAST_V4, run_units = d.run / 4, a_unit = 16, w_unit = 24;
            v.c_off = (uint64_t)(fused->dst_off * 2);
            c_stride = fused->dst_stride * 2;
            v.c_buf = add_buf(p, ref_b(*fused));
            ++di;  // the CAST descriptor is covered
        } else if (d.op == LIVER_OP_COPY) {
            if (ea != eb) {
                why = "internal: copy between different element sizes";
                return LIVER_E_UNSUPPORTED;
            }
            if (al16 && (d.run * ea) % 16 == 0) v.op = DOP_COPY_V16, run_units = d.run * ea / 16, a_unit = w_unit = 16;
            else v.op = ea == 2 ? DOP_COPY_E2 : DOP_COPY_E4, run_units = d.run, a_unit = w_unit = ea;
        } else if (d.op == LIVER_OP_CAST_BF16) {
            if (v.a_off % 16 == 0 && v.b_off % 8 == 0 && d.run % 4 == 0 && (rows1 || (a_stride % 16 == 0 && b_stride % 8 == 0))) {
                v.op = DOP_CAST_V4, run_units = d.run / 4, a_unit = 16, w_unit = 8;
                v.c_off = v.b_off, c_stride = b_stride, v.c_buf = v.b_buf;  // the bf16 target is the C operand
            } else {
                v.op = DOP_CAST_E, run_units = d.run, a_unit = 4, w_unit = 2;
            }
        } else {
            a_unit = 0;
            if (v.b_off % 16 == 0 && (d.run * eb) % 16 == 0) v.op = DOP_ZERO_V16, run_units = d.run * eb / 16, w_unit = 16;
            else v.op = eb == 2 ? DOP_ZERO_E2 : DOP_ZERO_E4, run_units = d.run, w_unit = eb;
        }
        const i64 total = d.rows * run_units, lim = i64(1) << 32;
        if (total <= 0 || total >= lim || (!rows1 && (a_stride >= lim || b_stride >= lim || c_stride >= lim))) {
            why = "internal: descriptor exceeds 32-bit unit counters";
            return LIVER_E_UNSUPPORTED;
        }
        v.a_stride = rows1 ? 0 : (uint32_t)a_stride;
        v.b_stride = rows1 ? 0 : (uint32_t)b_stride;
        v.c_stride = rows1 ? 0 : (uint32_t)c_stride;
        v.run = rows1 ? (uint32_t)total : (uint32_t)run_units;
        v.total = (uint32_t)total;
        const uint64_t tiles = ((uint64_t)total + TILE_UNITS - 1) / TILE_UNITS;
        if ((uint64_t)p.n_tiles + tiles >= (uint64_t(1) << 31)) {
            why = "internal: more than 2^31 tiles in one launch";
            return LIVER_E_UNSUPPORTED;
        }
        v.tile_begin = p.n_tiles;
        p.n_tiles += (uint32_t)tiles;
        p.desc_count += 1;
        list.dev.push_back(v);
        list.hbm_read += total * a_unit;
        list.hbm_written += total * w_unit;
    }
    if (staged)
        for (size_t c = (size_t)cur_chunk + 1; c <= n_chunks; ++c) list.chunk_pass[c] = (uint32_t)list.passes.size();
    else
        list.chunk_pass[1] = (uint32_t)list.passes.size();
    return LIVER_OK;
}

}  // namespace

int build_plan(liver_plan& plan, std::string& why) {
    Builder b(plan);
    int rc = b.run();
    why = b.why;
    return rc;
}

}  // namespace liver

"""Host-side checks of the planner through the C ABI (no GPU): its descriptors,
executed by the NumPy interpreter, must reproduce the oracle bit for bit, write
every planned target element exactly once, and follow the paper's geometry."""
import ctypes
import os
import re

import numpy as np
import pytest

import liver_synth as synth
import oracle
import paper_2605_22014_amd as lv
from interp import lv_objects, descs, run_direct, run_staged, used_dst, DT, emulate_direct, emulate_staged
from util import cfg_objects, make_world, tiny_state, corrupt_replicas
from test_oracle_reshard import ODD, ODD3, ODD6, BRUTE

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "liver.h")).read()
    names = set(re.findall(r"\b(liver_[a-z_]+)\s*\(", header))
    assert {"liver_plan_create", "liver_pack", "liver_unpack", "liver_reshard", "liver_plan_destroy"} <= names
    lib = ctypes.CDLL(lv.library_path())
    for n in sorted(names):
        assert hasattr(lib, n), n


def _check(spec, src, dst, world, chunk_bytes, derive=False, **dst_kw):
    s, a, b = lv_objects(spec, src, dst, derive_bf16=derive, **dst_kw)
    plan = lv.liver_plan_create(s, a, b, chunk_bytes)
    info = lv.liver_plan_info(plan)
    want = oracle.reshard_state(spec, src, dst, world, derive_bf16=derive)
    for side, lay in ((0, src), (1, dst)):
        for pp in range(lay.pp):
            for tp in range(lay.tp):
                for dp in range(lay.dp):
                    for k in oracle.kinds_of(spec):
                        n = lv.liver_plan_buffer_bytes(plan, side, lay.rank(tp, pp, dp), k)
                        assert n == oracle.buffer_elems(spec, lay, tp, pp, k, dp) * np.dtype(DT[k]).itemsize
    used = used_dst(plan)
    results = [run_direct(plan, world), run_staged(plan, world),
               run_staged(plan, world, order=list(range(info.n_chunks))[::-1]),
               (emulate_direct(plan, world), None), (emulate_staged(plan, world), None)]
    for got, counts in results:
        for key in got:
            if key in used:
                assert counts is None or (counts[key] == 1).all(), ("not exactly once", key, np.unique(counts[key]))
                assert np.array_equal(got[key], want[key]), key
            elif counts is not None:
                assert not counts[key].any(), ("unplanned buffer written", key)
            else:
                assert (got[key] == (0xA5A5 if key[1] % 4 == 0 else 0xA5A5A5A5)).all(), ("unplanned buffer written", key)
    assert info.n_chunks == -(-info.stream_bytes // chunk_bytes)
    return plan, info, used


@pytest.mark.parametrize("derive", [False, True])
@pytest.mark.parametrize("case", range(len(BRUTE)))
def test_tiny_odd_models(case, derive):
    spec, s, d = BRUTE[case]
    src, dst = oracle.Layout(*s), oracle.Layout(*d)
    world = make_world(spec, src, tiny_state(spec, seed=case))
    if case % 2:
        corrupt_replicas(spec, src, world)
    _, info, used = _check(spec, src, dst, world, 256 * (1 + case), derive)
    assert len(used) == dst.n_ranks * len(oracle.kinds_of(spec))


@pytest.mark.parametrize("chunk_bytes", [4096, 1 << 20, 1 << 30])
@pytest.mark.parametrize("derive", [False, True])
def test_tiny_gpt_config(chunk_bytes, derive):
    cfg, spec, src, dst = cfg_objects("tiny_gpt")
    state = synth.logical_state(oracle.logical_tensors(spec), synth.SEED_BASE, cfg["dist"])
    world = make_world(spec, src, state)
    _, info, _ = _check(spec, src, dst, world, chunk_bytes, derive)
    if not derive:
        assert info.stream_bytes == 35_766_272 == info.bytes_read == info.bytes_written
        assert info.n_chunks == {4096: 8732, 1 << 20: 35, 1 << 30: 1}[chunk_bytes]


FILTERS = [dict(only_tp=1), dict(only_pp=0), dict(only_dp=2), dict(only_tp=0, only_pp=1, only_dp=1),
           dict(kinds=(1, 2, 3)), dict(kinds=(0,)), dict(only_dp=0, kinds=(0, 2))]


@pytest.mark.parametrize("derive", [False, True])
@pytest.mark.parametrize("f", range(len(FILTERS)))
def test_filtered_plans(f, derive):
    spec = ODD
    src, dst = oracle.Layout(1, 2, 2, 4), oracle.Layout(2, 2, 3, 1)
    world = make_world(spec, src, tiny_state(spec, seed=40 + f))
    kw = FILTERS[f]
    _, info, used = _check(spec, src, dst, world, 512, derive, **kw)
    exp = set()
    for pp in range(dst.pp):
        for tp in range(dst.tp):
            for dp in range(dst.dp):
                if kw.get("only_tp", tp) == tp and kw.get("only_pp", pp) == pp and kw.get("only_dp", dp) == dp:
                    exp |= {(dst.rank(tp, pp, dp), k) for k in kw.get("kinds", (0, 1, 2, 3))}
    assert used == exp


def test_gqa_glu_dp_resize_with_padding():
    """GQA regroup + gated FFN re-block + DP 4 -> 6 cutting through strips, with padding on both sides."""
    spec = oracle.ModelSpec(n_layers=4, hidden=64, n_q_heads=8, n_kv_heads=4, ffn=96, vocab=128, glu=True)
    src, dst = oracle.Layout(4, 2, 4, 128), oracle.Layout(2, 4, 6, 128)
    world = make_world(spec, src, synth.logical_state(oracle.logical_tensors(spec), 3, "normal"))
    _, info, _ = _check(spec, src, dst, world, 4096)
    assert info.pad_bytes > 0


def test_paper_example_tp4_to_tp8_descriptors():
    """Section 4.6.1: under TP4 -> TP8 every source rank's column-split shard goes
    half to target 2s and half to target 2s+1, and nothing moves twice."""
    from test_oracle_reshard import _golden_tasks
    spec = oracle.ModelSpec(n_layers=1, hidden=64, n_q_heads=8, n_kv_heads=8, ffn=128, vocab=64)
    src, dst = oracle.Layout(4, 1, 1, 1), oracle.Layout(8, 1, 1, 1)
    s, a, b = lv_objects(spec, src, dst, kinds=(1,))
    plan = lv.liver_plan_create(s, a, b, 1 << 20)
    sv_s = {tp: {p.name: p for p in oracle.stage_view(spec, src, tp, 0).params} for tp in range(4)}
    sv_d = {tp: {p.name: p for p in oracle.stage_view(spec, dst, tp, 0).params} for tp in range(8)}
    tasks = {(t[0], t[1]): t for t in _golden_tasks()}
    for pname, N in (("L0.o.w", 64), ("L0.fc2.w", 128)):
        found = {}
        for d in descs(plan, lv.LIST_DIRECT):
            ps, pd = sv_s[d.src_rank][pname], sv_d[d.dst_rank][pname]
            if pd.offset <= d.dst_off < pd.offset + pd.size:
                assert ps.offset <= d.src_off < ps.offset + ps.size
                found[(d.src_rank, d.dst_rank)] = d
                w = N // 8
                half = tasks[(d.src_rank, d.dst_rank)][4]
                assert d.rows == 64 and d.run == w and d.src_stride == 2 * w and d.dst_stride == w
                assert d.src_off - ps.offset == (0 if half == "first" else w) and d.dst_off == pd.offset
        assert set(found) == set(tasks)          # exactly the paper's 8 tasks
        assert sum(d.rows * d.run for d in found.values()) == 64 * N      # no redundant movement
    info = lv.liver_plan_info(plan)
    assert info.bytes_read == info.bytes_written == sum(
        oracle.stage_view(spec, dst, tp, 0).n_local for tp in range(8)) * 4


def test_pp_only_tasks_are_whole_parameters():
    """Section 4.6.1 / A.2.3: a PP-only change moves whole shards (full or empty intersection)."""
    _, spec, _, _ = cfg_objects("tiny_gpt")
    src, dst = oracle.Layout(2, 1, 1, 128), oracle.Layout(2, 2, 1, 128)
    s, a, b = lv_objects(spec, src, dst, kinds=(0,))
    plan = lv.liver_plan_create(s, a, b, 1 << 20)
    for d in descs(plan, lv.LIST_DIRECT):
        # dense pieces from the same tp (TP-replicated parameters are read from tp 0)
        assert d.rows == 1 and d.src_rank % 2 in (d.dst_rank % 2, 0)
    for tp in range(2):
        for pp in range(2):
            sv = oracle.stage_view(spec, dst, tp, pp)
            pieces = sorted((d.dst_off, d.run) for d in descs(plan, lv.LIST_DIRECT) if d.dst_rank == dst.rank(tp, pp, 0))
            # pieces tile [0, n_local) and every piece boundary is a parameter boundary
            bounds = {p.offset for p in sv.params} | {sv.n_local}
            pos = 0
            for off, run in pieces:
                assert off == pos and off in bounds
                pos += run
            assert pos == sv.n_local


@pytest.mark.parametrize("name", ["gpt2_small", "llama7b", "llama13b_dp", "llama70b_rank"])
def test_big_config_plan_statistics(name):
    cfg, spec, src, dst = cfg_objects(name)
    only = cfg["only"] or {}
    s, a, b = lv_objects(spec, src, dst, kinds=cfg["kinds"], **{"only_" + k: v for k, v in only.items()})
    plan = lv.liver_plan_create(s, a, b, cfg["chunk_bytes"])
    info = lv.liver_plan_info(plan)
    exp = 0
    for pp in range(dst.pp):
        for tp in range(dst.tp):
            if only.get("tp", tp) != tp or only.get("pp", pp) != pp:
                continue
            sv = oracle.stage_view(spec, dst, tp, pp)
            for dp in range(dst.dp):
                if only.get("dp", dp) != dp:
                    continue
                lo, hi = dp * sv.S, min((dp + 1) * sv.S, sv.n_local)
                for k in cfg["kinds"]:
                    exp += sv.n_local * 2 if k == 0 else max(hi - lo, 0) * 4
    assert info.stream_bytes == info.bytes_read == exp
    assert info.bytes_written == exp + info.pad_bytes
    assert info.n_chunks == {"gpt2_small": 31, "llama7b": 352, "llama13b_dp": 25, "llama70b_rank": 16}[name]
    assert info.table_bytes_device < (2 << 20)           # plan metadata stays around 1 MB (Appendix A.1, Table 3)
    # every descriptor stays inside its buffers; 16-byte alignment everywhere at real shapes
    for which in (lv.LIST_DIRECT, lv.LIST_PACK, lv.LIST_UNPACK):
        for d in descs(plan, which):
            for side, rank, kind, off, stride in ((0, d.src_rank, d.src_kind, d.src_off, d.src_stride),
                                                  (1, d.dst_rank, d.dst_kind, d.dst_off, d.dst_stride)):
                eb = 2 if (kind if rank >= 0 else d.src_kind) == 0 else 4
                if d.op == lv.OP_ZERO and side == 0:
                    continue
                end = (off + (d.rows - 1) * stride + d.run) * eb
                cap = cfg["chunk_bytes"] if rank < 0 else lv.liver_plan_buffer_bytes(plan, side, rank, kind)
                assert 0 <= off and end <= cap
                assert (off * eb) % 16 == 0 and (d.run * eb) % 16 == 0 and (d.rows == 1 or (stride * eb) % 16 == 0)
    # the row runs of the direct list, and of all unpack chunks together, tile every planned target buffer
    # exactly: sorted by start, each run begins where the previous one ends, from 0 to the buffer's end
    for which in (lv.LIST_DIRECT, lv.LIST_UNPACK):
        runs = {}
        for d in descs(plan, which):
            starts = d.dst_off + d.dst_stride * np.arange(d.rows, dtype=np.int64)
            runs.setdefault((d.dst_rank, d.dst_kind), []).append(np.stack([starts, starts + d.run], 1))
        planned = [(r, k) for r in range(dst.n_ranks) for k in range(4) if lv.liver_plan_buffer_used(plan, 1, r, k)]
        assert sorted(runs) == planned
        for (r, k), parts in runs.items():
            iv = np.concatenate(parts)
            iv = iv[np.argsort(iv[:, 0], kind="stable")]
            assert iv[0, 0] == 0 and (iv[1:, 0] == iv[:-1, 1]).all(), (which, r, k)
            assert iv[-1, 1] * (2 if k == 0 else 4) == lv.liver_plan_buffer_bytes(plan, 1, r, k), (which, r, k)


def test_error_codes():
    _, spec, src, dst = cfg_objects("tiny_gpt")
    s, a, b = lv_objects(spec, src, dst)
    for bad_chunk in (0, 100, 4097):
        with pytest.raises(lv.LiverError) as e:
            lv.liver_plan_create(s, a, b, bad_chunk)
        assert e.value.code == -1
    with pytest.raises(lv.LiverError) as e:
        lv.liver_plan_create(s, a, lv.Layout(3, 1, 1), 4096)            # 4 heads over TP=3
    assert e.value.code == -2
    with pytest.raises(lv.LiverError) as e:
        lv.liver_plan_create(s, a, lv.Layout(1, 2, 2, only_pp=2), 4096)
    assert e.value.code == -2
    with pytest.raises(lv.LiverError) as e:
        lv.liver_plan_create(s, lv.Layout(2, 1, 2, only_tp=2), b, 4096)
    assert e.value.code == -2
    for bad in (lv.Layout(1, 2, 2, pp_first=3), lv.Layout(1, 2, 2, vpp=2), lv.Layout(1, 2, 2, pp_first=1, vpp=1, pp_last=2),
                lv.Layout(8, 1, 1), lv.Layout(1, 1, 1, vocab_multiple=-1)):
        with pytest.raises(lv.LiverError):          # 2 layers: 3 on the first stage; 4 chunks; 1+2; 4 heads over TP 8
            lv.liver_plan_create(s, a, bad, 4096)
    plan = lv.liver_plan_create(s, a, b, 4096)
    with pytest.raises(lv.LiverError):
        lv.liver_plan_buffer_bytes(plan, 0, 99, 0)
    with pytest.raises(lv.LiverError):
        lv.liver_plan_desc(plan, 0, 10 ** 9)
    assert "argument" in lv.liver_strerror(-1)


def test_planner_at_paper_scale_is_subsecond():
    """Section 4.6.1 / Appendix A.2.3: planning a 175B-parameter, 96-layer model over
    1024 ranks takes under a second on the CPU (metadata only).  GPT-3 175B shape."""
    import time
    spec = lv.ModelSpec(n_layers=96, hidden=12288, n_q_heads=96, n_kv_heads=96, ffn=49152, vocab=51200, max_pos=2048,
                        norm_bias=True, linear_bias=True, tied_embed=True)
    for s, d in (((8, 16, 8), (4, 32, 8)), ((8, 8, 16), (16, 8, 8))):
        best = 1e9
        for _ in range(2):
            t = time.perf_counter()
            plan = lv.liver_plan_create(spec, lv.Layout(*s), lv.Layout(*d), 512 << 20)
            best = min(best, time.perf_counter() - t)
            info = lv.liver_plan_info(plan)
            lv.liver_plan_destroy(plan)
        assert info.n_src_ranks == info.n_dst_ranks == 1024
        params = 96 * (12 * 12288 ** 2 + 13 * 12288) + 51200 * 12288 + 2048 * 12288 + 2 * 12288
        assert abs(params - 174.6e9) < 1e9
        assert info.stream_bytes > params * 12          # every fp32 element crosses once, bf16 once per replica
        assert best < 1.0, f"planning took {best:.2f} s"


def test_pieces_above_2_30_elements_are_split():
    """A 1.2 G-element embedding moves as one dense piece; the planner must cut it so
    that the kernels' 32-bit unit counters cannot overflow, without gaps or overlap."""
    spec = oracle.ModelSpec(n_layers=2, hidden=8192, n_q_heads=64, n_kv_heads=64, ffn=64, vocab=147456)
    src, dst = oracle.Layout(1, 1, 1, 128), oracle.Layout(1, 2, 1, 128)
    s, a, b = lv_objects(spec, src, dst)
    plan = lv.liver_plan_create(s, a, b, 512 << 20)
    info = lv.liver_plan_info(plan)
    for which in (lv.LIST_DIRECT, lv.LIST_PACK, lv.LIST_UNPACK):
        for rank in range(2):
            sv = oracle.stage_view(spec, dst, 0, rank)
            for kind in (0, 1):
                if which == lv.LIST_PACK:
                    continue
                ivs = sorted((d.dst_off, d.rows * d.run) for d in descs(plan, which)
                             if d.dst_rank == rank and d.dst_kind == kind and d.rows == 1)
                pos = 0
                for off, n in ivs:
                    assert off == pos and 0 < n <= 1 << 30
                    pos += n
                assert pos == sv.n_local
    assert max(d.rows * d.run for d in descs(plan, lv.LIST_DIRECT)) == 1 << 30
    assert info.bytes_read == info.bytes_written == 14 * sum(oracle.stage_view(spec, dst, 0, pp).n_local for pp in range(2))


def test_many_buffers_split_into_passes():
    """512 source and 128 target ranks: far more buffers than one launch can carry in its arguments, so the
    lists are cut into several passes; the result must not change."""
    spec = oracle.ModelSpec(n_layers=8, hidden=64, n_q_heads=8, n_kv_heads=8, ffn=64, vocab=64, tied_embed=True)
    src, dst = oracle.Layout(8, 8, 8, 8), oracle.Layout(4, 4, 8, 8)
    world = make_world(spec, src, synth.logical_state(oracle.logical_tensors(spec), 11, "uniform"))
    plan, info, used = _check(spec, src, dst, world, 1 << 16)
    assert info.n_src_bufs_used + info.n_dst_bufs_used > 2000          # > 400 per launch: several passes needed


def test_source_side_restriction_partitions_the_work():
    """Plans restricted to one source rank each (what one source GPU would run): their pack lists fill
    disjoint parts of every staging chunk and together the whole payload; their direct lists together write
    every target element exactly once (zero padding: once per plan); unpack does not depend on the restriction."""
    spec = ODD
    src, dst = oracle.Layout(2, 2, 2, 4), oracle.Layout(1, 2, 3, 1)
    world = make_world(spec, src, tiny_state(spec, seed=77))
    want = oracle.reshard_state(spec, src, dst, world)
    s, a, b = lv_objects(spec, src, dst)
    full = lv.liver_plan_create(s, a, b, 512)
    info = lv.liver_plan_info(full)
    plans = []
    for tp in range(src.tp):
        for pp in range(src.pp):
            for dp in range(src.dp):
                a1 = lv.Layout(src.tp, src.pp, src.dp, src.pad_multiple, only_tp=tp, only_pp=pp, only_dp=dp)
                plans.append(lv.liver_plan_create(s, a1, b, 512))
    from interp import alloc_dst, execute
    # direct: union of the restricted plans
    out, counts = alloc_dst(full)
    for p in plans:
        i = lv.liver_plan_info(p)
        assert (i.n_chunks, i.stream_bytes) == (info.n_chunks, info.stream_bytes)
        assert [(d.op, d.chunk, d.src_off, d.dst_rank, d.dst_kind, d.dst_off, d.rows, d.run) for d in descs(p, lv.LIST_UNPACK)] == \
            [(d.op, d.chunk, d.src_off, d.dst_rank, d.dst_kind, d.dst_off, d.rows, d.run) for d in descs(full, lv.LIST_UNPACK)]
        for d in descs(p, lv.LIST_DIRECT):
            execute(d, world, out, counts)
    pad = {key: np.zeros_like(c, bool) for key, c in counts.items()}
    for d in descs(full, lv.LIST_DIRECT):
        if d.op == lv.OP_ZERO:
            pad[(d.dst_rank, d.dst_kind)][d.dst_off:d.dst_off + d.run] = True
    for key in out:
        assert np.array_equal(out[key], want[key]), key
        assert (counts[key][~pad[key]] == 1).all() and (counts[key][pad[key]] == len(plans)).all(), key
    # staged: every source rank packs its pieces into the same chunk; then one unpack
    out, counts = alloc_dst(full)
    un = {}
    for d in descs(full, lv.LIST_UNPACK):
        un.setdefault(d.chunk, []).append(d)
    for c in range(info.n_chunks):
        staging = np.full(512, 0x3C, np.uint8)
        covered = np.zeros(512, np.uint8)
        for p in plans:
            for d in descs(p, lv.LIST_PACK):
                if d.chunk == c:
                    execute(d, world, None, None, staging)
                    eb = 2 if d.src_kind == 0 else 4
                    covered[d.dst_off * eb:(d.dst_off + d.rows * d.run) * eb] += 1
        assert covered.max() == 1
        for d in un[c]:
            execute(d, None, out, counts, staging)
    for key in out:
        assert np.array_equal(out[key], want[key]) and (counts[key] == 1).all(), key


@pytest.mark.parametrize("kw", [dict(only_dp=3), dict(only_dp=2), dict(only_tp=1, only_dp=0), dict(kinds=(1, 2)), dict(only_pp=1, kinds=(0,))])
@pytest.mark.parametrize("derive", [False, True])
def test_filtered_plans_mixture_of_experts(kw, derive):
    """Restricted plans of an MoE model: only_dp = 3 with EP 2 plans the expert buffers of index 1 only."""
    from test_oracle_reshard import MOE
    src, dst = oracle.Layout(2, 1, 2, 4, ep=2), oracle.Layout(2, 2, 4, 1, ep=2, bucket_elems=400)
    world = make_world(MOE, src, tiny_state(MOE, seed=5))
    _, info, used = _check(MOE, src, dst, world, 512, derive, **kw)
    exp = set()
    for pp in range(dst.pp):
        for tp in range(dst.tp):
            for dp in range(dst.dp):
                if kw.get("only_tp", tp) == tp and kw.get("only_pp", pp) == pp and kw.get("only_dp", dp) == dp:
                    exp |= {(dst.rank(tp, pp, dp), k + 4 * f) for k in kw.get("kinds", (0, 1, 2, 3)) for f in (0, 1)}
    assert used == exp


def test_planning_from_many_threads_gives_identical_plans():
    """The planner keeps no shared mutable state: concurrent liver_plan_create calls (ctypes releases the GIL)
    return plans with identical descriptors, and error text stays per thread."""
    import threading
    cfg, spec, src, dst = cfg_objects("gpt2_small")
    s, a, b = lv_objects(spec, src, dst)

    def fingerprint(plan):
        return [(d.op, d.chunk, d.src_rank, d.src_kind, d.src_off, d.src_stride, d.dst_rank, d.dst_kind, d.dst_off, d.dst_stride, d.rows, d.run)
                for d in (lv.liver_plan_desc(plan, lv.LIST_DIRECT, i) for i in range(0, lv.liver_plan_desc_count(plan, lv.LIST_DIRECT), 7))]

    want = fingerprint(lv.liver_plan_create(s, a, b, cfg["chunk_bytes"]))
    out, errs = [None] * 8, []

    def work(i):
        try:
            if i % 4 == 3:                                   # an error path running next to the good ones
                with pytest.raises(lv.LiverError):
                    lv.liver_plan_create(s, a, b, 3)
                out[i] = want
            else:
                out[i] = fingerprint(lv.liver_plan_create(s, a, b, cfg["chunk_bytes"]))
        except BaseException as e:                           # noqa: BLE001 - reported below
            errs.append(repr(e))

    ts = [threading.Thread(target=work, args=(i,)) for i in range(8)]
    [t.start() for t in ts]
    [t.join() for t in ts]
    assert not errs, errs
    assert all(o == want for o in out)


def _owners_of(spec, lay, rank, kind, offs):
    """(name, logical index) of elements `offs` of buffer (rank, kind) by the closed-form ownership formulas
    (unbucketed layouts: a rank's fp32 buffer is slice dp of the column's flat buffer)."""
    import ownership as own
    tp, dp, pp = rank % lay.tp, (rank // lay.tp) % lay.dp, rank // (lay.tp * lay.dp)
    flat = np.asarray(offs, np.int64) + (0 if kind == 0 else dp * (own.n_pad(spec, lay, pp) // lay.dp))
    sizes = own.stage_param_sizes(spec, lay, pp)
    starts = np.concatenate([[0], np.cumsum([n for _, n in sizes])])
    j = np.searchsorted(starts, flat, side="right") - 1
    names, idx = np.full(flat.shape, None, dtype=object), np.zeros(flat.shape, np.int64)
    for p in np.unique(j[j < len(sizes)]):
        m = j == p
        names[m], idx[m] = own.owner(spec, lay, tp, sizes[p][0], flat[m] - starts[p])
    return names, idx


@pytest.mark.parametrize("name", ["llama7b", "llama13b_dp", "llama70b_rank"])
def test_full_size_descriptors_agree_with_ownership_formulas(name):
    """At the real shapes: first, last and 30 random elements of every direct descriptor move between
    two positions that the ownership formulas give the SAME logical element; zero descriptors hit padding."""
    cfg, spec, src, dst = cfg_objects(name)
    only = cfg["only"] or {}
    s, a, b = lv_objects(spec, src, dst, kinds=cfg["kinds"], **{"only_" + k: v for k, v in only.items()})
    plan = lv.liver_plan_create(s, a, b, cfg["chunk_bytes"])
    rng = np.random.default_rng(5)
    groups = {}
    for d in descs(plan, lv.LIST_DIRECT):
        r = np.concatenate([[0, d.rows - 1], rng.integers(d.rows, size=30)]).astype(np.int64)
        c = np.concatenate([[0, d.run - 1], rng.integers(d.run, size=30)]).astype(np.int64)
        key = (d.op, d.src_rank, d.src_kind, d.dst_rank, d.dst_kind)
        g = groups.setdefault(key, ([], []))
        g[0].append(d.src_off + r * d.src_stride + c)
        g[1].append(d.dst_off + r * d.dst_stride + c)
    n_checked = 0
    for (op, sr, sk, dr, dk), (so, do) in groups.items():
        dn, di = _owners_of(spec, dst, dr, dk, np.concatenate(do))
        if op == lv.OP_ZERO:
            assert (dn == None).all()                            # noqa: E711 - elementwise on an object array
            continue
        sn, si = _owners_of(spec, src, sr, sk, np.concatenate(so))
        assert (dn != None).all() and (sn == dn).all() and (si == di).all(), (op, sr, sk, dr, dk)   # noqa: E711
        assert (sk == dk) or (op == lv.OP_CAST_BF16 and sk == 1 and dk == 0)
        n_checked += dn.size
    assert n_checked >= 32 * 20


def test_plan_of_a_source_rank_that_contributes_nothing():
    """bf16 weights are read from DP replica 0: a plan restricted to source replica 1 and to the weights has an
    empty pack list and a direct list of zero-padding descriptors only."""
    spec = oracle.ModelSpec(n_layers=2, hidden=64, n_q_heads=4, n_kv_heads=4, ffn=128, vocab=128, glu=True)
    src, dst = oracle.Layout(2, 1, 2, 128), oracle.Layout(1, 2, 2, 128)
    s, a, b = lv_objects(spec, src, dst, kinds=(0,))
    plan = lv.liver_plan_create(s, lv.Layout(src.tp, src.pp, src.dp, src.pad_multiple, only_dp=1), b, 4096)
    info = lv.liver_plan_info(plan)
    assert info.bytes_read == 0 and info.n_desc_pack == 0 and info.bytes_written == info.pad_bytes > 0
    assert all(d.op == lv.OP_ZERO for d in descs(plan, lv.LIST_DIRECT))
    from interp import alloc_dst
    out, _ = alloc_dst(plan)
    lv.liver_debug_emulate_host(plan, lv.LIST_DIRECT, 0, {}, out, None)
    staging = np.full(4096, 0x3C, np.uint8)
    lv.liver_debug_emulate_host(plan, lv.LIST_PACK, info.n_chunks - 1, {}, None, staging)
    assert (staging == 0x3C).all()
    for (r, k), g in out.items():
        n = oracle.stage_view(spec, dst, 0, r // (dst.tp * dst.dp)).n_local
        if k == 0:
            assert (g[:n] == 0xA5A5).all() and (g[n:] == 0).all()
        else:
            assert (g.view(np.uint8) == 0xA5).all()


def test_bandwidth_probe_rejects_bad_arguments_before_any_launch():
    """Argument errors of the measurement aid are found on the host (no GPU needed, nothing is launched)."""
    ok = dict(mode=2, src=4096, dst=1 << 20, nbytes=32768, grid=8)
    for bad in (dict(mode=4), dict(mode=-1), dict(src=0), dict(dst=0), dict(src=4100), dict(dst=(1 << 20) + 8), dict(nbytes=0),
                dict(nbytes=32768 + 16), dict(grid=0), dict(grid=65537), dict(mode=0, grid=4096)):
        kw = dict(ok, **bad)
        with pytest.raises(lv.LiverError) as e:
            lv.liver_debug_bandwidth_probe(kw["mode"], kw["src"], kw["dst"], kw["nbytes"], kw["grid"], stream=0)
        assert e.value.code == -1, bad


def test_garbage_structs_are_rejected_quickly():
    """Structs filled with arbitrary integers (uninitialised memory, say) come back as an error or a small valid
    plan, never as a crash, a long planning run or a huge allocation."""
    import time
    from paper_2605_22014_amd import _binding as B
    rng = np.random.default_rng(2014)
    pool = [0, -1, 1, 2, 3, 4, 8, 64, 96, 128, 1 << 15, 1 << 20, (1 << 24) + 1, (1 << 31) - 1, -(1 << 31)]
    t0, n_ok, n_err = time.perf_counter(), 0, 0
    for case in range(300):
        pick = lambda: int(pool[rng.integers(len(pool))])
        s = B._Spec(*[pick() for _ in range(7)], pick() & 0xFFFFFFFF, pick())
        lays = []
        for _ in range(2):
            lays.append(B._Layout(*[pick() for _ in range(7)], pick() & 0xFFFFFFFF, pick() & 0xFFFFFFFF,
                                            pick(), pick(), pick(), pick(), pick(), pick()))
        handle = ctypes.c_void_p()
        rc = B._lib.liver_plan_create(ctypes.byref(s), ctypes.byref(lays[0]), ctypes.byref(lays[1]),
                                                ctypes.c_size_t(256 * max(1, pick() & 0xFFFF)), ctypes.byref(handle))
        if rc == 0:
            n_ok += 1
            B._lib.liver_plan_destroy(handle)
        else:
            n_err += 1
            assert rc in (-1, -2), (case, rc)
    assert n_err > 250 and time.perf_counter() - t0 < 60
    # one garbage field in an otherwise valid request reaches the deeper checks
    good_spec = dict(n_layers=4, hidden=64, n_q_heads=8, n_kv_heads=4, ffn=96, vocab=128, max_pos=16, flags=15, n_experts=0)
    good_lay = dict(tp=2, pp=2, dp=2, pad_multiple=8, only_tp=-1, only_pp=-1, only_dp=-1, flags=0, kind_mask=0, vpp=1,
                    vocab_multiple=0, pp_first=0, pp_last=0, bucket_elems=0, ep=1)
    n_ok = 0
    for case in range(600):
        sp, a, b = dict(good_spec), dict(good_lay), dict(good_lay, tp=4, pp=1, dp=3)
        target = (sp, a, b)[case % 3]
        field = list(target)[rng.integers(len(target))]
        v = int(pool[rng.integers(len(pool))])
        target[field] = v & 0xFFFFFFFF if field in ("flags", "kind_mask") else v
        handle = ctypes.c_void_p()
        rc = B._lib.liver_plan_create(ctypes.byref(B._Spec(**sp)), ctypes.byref(B._Layout(**a)), ctypes.byref(B._Layout(**b)),
                                      ctypes.c_size_t(4096), ctypes.byref(handle))
        assert rc in (0, -1, -2), (case, field, v, rc)
        if rc == 0:
            n_ok += 1
            assert B._lib.liver_plan_desc_count(handle, 0) < 1_000_000, (field, v)
            B._lib.liver_plan_destroy(handle)
    assert 50 < n_ok < 550 and time.perf_counter() - t0 < 120


@pytest.mark.parametrize("chunk_bytes", [256, 1024, 1 << 20])
def test_every_task_starts_16_byte_aligned_on_the_wire(chunk_bytes):
    """Wire format: tasks follow each other in the order of the direct list, each starting at the next multiple
    of 16 bytes (a no-op at real shapes, where every task is a multiple of 16 bytes long).  For an odd toy
    model that fixes stream_bytes, which must exceed the tightly packed size."""
    spec = ODD
    src, dst = oracle.Layout(2, 1, 2, 1), oracle.Layout(1, 2, 3, 1)
    s, a, b = lv_objects(spec, src, dst)
    plan = lv.liver_plan_create(s, a, b, chunk_bytes)
    pos = tight = 0
    for d in descs(plan, lv.LIST_DIRECT):
        if d.op == lv.OP_ZERO:
            continue
        n = d.rows * d.run * (2 if d.src_kind == 0 else 4)
        pos = (pos + 15) // 16 * 16 + n
        tight += n
    info = lv.liver_plan_info(plan)
    assert info.stream_bytes == pos > tight
    assert info.n_chunks == -(-pos // chunk_bytes)
    first_of_chunk = {}
    for d in descs(plan, lv.LIST_PACK):                       # a chunk's first piece sits at its start
        first_of_chunk.setdefault(d.chunk, d.dst_off)
    assert set(first_of_chunk.values()) == {0}


@pytest.mark.parametrize("name", ["tiny_gpt", "gpt2_small", "llama7b"])
def test_stream_is_layer_major(name):
    """Section 4.6.2 / Algorithm 1: the state streams layer by layer.  Slot 0 (embeddings) comes first, then
    slot 1 + l for layer l in ascending order, then the final norm and head; inside a slot the tasks are ordered
    by target rank, kind and target offset.  Chunks follow the same order, so chunk k never holds an earlier
    layer than chunk k - 1."""
    cfg, spec, src, dst = cfg_objects(name)
    s, a, b = lv_objects(spec, src, dst)
    plan = lv.liver_plan_create(s, a, b, cfg["chunk_bytes"])
    direct = descs(plan, lv.LIST_DIRECT)
    keys = [(d.slot, d.dst_rank, d.dst_kind, d.dst_off) for d in direct]
    assert keys == sorted(keys)
    assert {d.slot for d in direct} == set(range(spec.n_layers + 2))
    # the slot of a task is the layer of the target parameter it fills (the oracle's view of the target rank)
    by_rank = {}
    for d in direct:
        if d.op == lv.OP_ZERO or d.dst_kind != 0:
            continue
        tp, pp = d.dst_rank % dst.tp, d.dst_rank // (dst.tp * dst.dp)
        sv = by_rank.setdefault((tp, pp), oracle.stage_view(spec, dst, tp, pp))
        prm = next(p for p in sv.params if p.offset <= d.dst_off < p.offset + p.size)
        if prm.name.startswith("L"):
            want = 1 + int(prm.name.split(".")[0][1:])
        else:
            want = 0 if prm.name in ("embed.word", "embed.pos") else spec.n_layers + 1
        assert d.slot == want, (prm.name, d.slot)
    for which in (lv.LIST_PACK, lv.LIST_UNPACK):
        seq = [(d.chunk, d.slot) for d in descs(plan, which) if d.op != lv.OP_ZERO]
        assert seq == sorted(seq)


def test_planner_and_oracle_agree_on_what_is_supported():
    """Every refusal rule, one layout each (and the nearest accepted neighbour): the planner returns
    UNSUPPORTED exactly where the oracle's check_supported raises."""
    dense = oracle.ModelSpec(n_layers=6, hidden=64, n_q_heads=8, n_kv_heads=2, ffn=96, vocab=128, glu=True)
    moe = oracle.ModelSpec(n_layers=4, hidden=32, n_q_heads=4, n_kv_heads=4, ffn=48, vocab=64, glu=True, n_experts=4)
    L = oracle.Layout
    cases = [
        (dense, L(2, 1, 1), True), (dense, L(3, 1, 1), False),                      # ffn % tp, heads
        (dense, L(4, 1, 1), True), (dense, L(8, 1, 1), True), (dense, L(16, 1, 1), False),   # kv heads split / replicated / too thin
        (dense, L(1, 3, 1), True), (dense, L(1, 4, 1), False),                       # layers over stages
        (dense, L(1, 3, 1, vpp=2), True), (dense, L(1, 2, 1, vpp=2), False),        # interleaved chunks
        (dense, L(1, 3, 1, pp_first=2), True), (dense, L(1, 3, 1, pp_first=1), False),   # 6-1 = 5 over 2 stages
        (dense, L(1, 3, 1, pp_first=2, pp_last=2), True), (dense, L(1, 2, 1, pp_first=2, pp_last=2), False),
        (dense, L(1, 2, 1, pp_first=2, vpp=2), False),                               # uneven and interleaved
        (dense, L(8, 1, 1, vocab_multiple=4), True),
        (oracle.ModelSpec(n_layers=2, hidden=64, n_q_heads=8, n_kv_heads=8, ffn=96, vocab=100), L(8, 1, 1), False),   # vocab % tp
        (oracle.ModelSpec(n_layers=2, hidden=64, n_q_heads=8, n_kv_heads=8, ffn=96, vocab=100), L(8, 1, 1, vocab_multiple=2), True),
        (dense, L(1, 1, 2, ep=2), False),                                            # expert parallelism without experts
        (moe, L(1, 1, 4, ep=2), True), (moe, L(1, 1, 3, ep=2), False),              # ep must divide dp
        (moe, L(1, 1, 8, ep=8), False), (moe, L(1, 1, 4, ep=4), True),              # ep must divide the expert count
    ]
    for spec, lay, ok in cases:
        try:
            oracle.check_supported(spec, lay)
            oracle_ok = True
        except ValueError:
            oracle_ok = False
        s, a, b = lv_objects(spec, lay, lay)
        try:
            lv.liver_plan_create(s, a, b, 4096)
            planner_ok = True
        except lv.LiverError as e:
            assert e.code == -2, (lay, e)
            planner_ok = False
        assert oracle_ok == planner_ok == ok, (spec, lay, oracle_ok, planner_ok, ok)

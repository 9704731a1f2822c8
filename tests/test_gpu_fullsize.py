"""Parity at the full sizes of the large configurations, in the launch shape the
benchmark times (library defaults): the state is generated in HBM and resharded by
the HIP path (direct, then staged).  For the three large benchmark configurations
(7B, 13B share, 70B share) EVERY logical tensor is gathered and re-split by the CPU
oracle, one group of tensors at a time, and every planned target element is compared
bit for bit (LiveR, Section 6.6: element-wise comparison of the whole state, deviation
exactly zero; Appendix A.2.1, Eq. 1); the variants of those configurations compare a
sample of tensors -- first, middle and last layers, embeddings, head.  Plus
size-independent properties (zero padding, untouched source)."""
import numpy as np
import pytest
import torch

import liver_synth as synth
import oracle
import paper_2605_22014_amd as lv
from util import cfg_objects

pytestmark = pytest.mark.gpu
NP = {0: np.uint16, 1: np.uint32, 2: np.uint32, 3: np.uint32}


@pytest.fixture(autouse=True)
def _release_cached_blocks():
    """These tests fill most of the HBM with differently sized buffers: hand the allocator's cached blocks back
    between them, so that one test's leftovers cannot fragment the next one's 90 GB of allocations."""
    yield
    import gc
    gc.collect()
    torch.cuda.empty_cache()


def _setup(name):
    if isinstance(name, dict):
        cfg = name
        ospec = oracle.ModelSpec(**cfg["spec"])
        osrc = oracle.Layout(pad_multiple=cfg["pad_multiple"], **cfg["src"])
        odst = oracle.Layout(pad_multiple=cfg["pad_multiple"], **cfg["dst"])
    else:
        cfg, ospec, osrc, odst = cfg_objects(name)
    only = cfg["only"] or {}
    spec = lv.ModelSpec(**cfg["spec"])
    src = lv.Layout(pad_multiple=cfg["pad_multiple"], **cfg["src"])
    dst = lv.Layout(pad_multiple=cfg["pad_multiple"], kinds=tuple(cfg["kinds"]),
                    **{"only_" + k: v for k, v in only.items()}, **cfg["dst"])
    plan = lv.liver_plan_create(spec, src, dst, cfg["chunk_bytes"])
    sizes = {}
    for pp in range(src.pp):
        for tp in range(src.tp):
            if any(lv.liver_plan_buffer_used(plan, 0, src.rank(tp, pp, d), k) for d in range(src.dp) for k in range(4)):
                for d in range(src.dp):
                    n = lv.liver_plan_buffer_bytes(plan, 0, src.rank(tp, pp, d), lv.MASTER) // 4
                    assert n == oracle.buffer_elems(ospec, osrc, tp, pp, oracle.MASTER)
                    sizes[((tp, pp), d)] = n
    gen = synth.fill_device_world(sizes, src.dp, synth.SEED_BASE)
    src_bufs = {}
    for (col, d) in sizes:
        r = src.rank(col[0], col[1], d)
        for k in (1, 2, 3):
            src_bufs[(r, k)] = gen[(col, d, k)]
        src_bufs[(r, 0)] = gen[(col, "param")]
    return cfg, only, ospec, osrc, odst, plan, src, dst, src_bufs


def _fresh_dst(plan, dst):
    out = {}
    for r in range(dst.n_ranks):
        for k in range(4):
            if lv.liver_plan_buffer_used(plan, 1, r, k):
                n = lv.liver_plan_buffer_bytes(plan, 1, r, k) // (2 if k == 0 else 4)
                out[(r, k)] = torch.full((n,), -23131 if k == 0 else -1515870811,
                                         dtype=torch.int16 if k == 0 else torch.int32, device="cuda")
    return out


def _expected(cfg, only, ospec, osrc, odst, src_bufs, names, quiet=False):
    """[(kind, tp, pp, stage_view, param, shard)] for the sampled tensors, from the oracle."""
    def read(rank, kind, lo, hi):
        if (rank, kind) not in src_bufs:                 # a source rank this filtered plan never reads
            return np.zeros(hi - lo, NP[kind])
        return src_bufs[(rank, kind)][lo:hi].view(torch.int16 if kind == 0 else torch.int32).cpu().numpy().view(NP[kind])
    tps = [only["tp"]] if "tp" in only else None
    pps = [only["pp"]] if "pp" in only else None
    out = []
    for k in cfg["kinds"]:
        logical = oracle.gather_logical(ospec, osrc, k, read, names=names)
        out += [(k,) + t for t in oracle.expected_shards(ospec, odst, logical, tps, pps)]
        if not quiet:
            print(f"  oracle: kind {k} gathered and split", flush=True)
    return out


def _compare(expected, only, odst, dst_bufs, what, per_kind=False):
    n_checked, by_kind = 0, {}
    for k, tp, pp, sv, prm, shard in expected:
        flat = shard.ravel()
        if k == 0:
            pieces = [(d, prm.offset, prm.offset, prm.size) for d in range(odst.dp)]      # every replica, whole shard
        else:
            pieces = oracle.dp_pieces(sv, odst, prm.offset, prm.offset + prm.size)         # (dp, local, flat, n)
        for d, local, at, n in pieces:
            if only.get("dp", d) != d:
                continue
            got = dst_bufs[(odst.rank(tp, pp, d), k)][local:local + n].cpu().numpy().view(NP[k])
            assert np.array_equal(got, flat[at - prm.offset:at - prm.offset + n]), (what, prm.name, "dp", d, "kind", k)
            n_checked += n
            by_kind[k] = by_kind.get(k, 0) + n
    assert n_checked > 0
    return by_kind if per_kind else n_checked


def _pads_zero(only, ospec, odst, dst_bufs):
    """Every padding element of the planned target buffers is +0: the tail of each bucket, wherever it lives."""
    for (r, k), t in dst_bufs.items():
        pp, d = r // (odst.tp * odst.dp), (r // odst.tp) % odst.dp
        sv = oracle.stage_view(ospec, odst, r % odst.tp, pp)
        ends = sorted(p.offset + p.size for p in sv.params)
        for b0, nb in sv.buckets:
            used_end = max(e for e in ends if e <= b0 + nb)
            if used_end == b0 + nb:
                continue
            if k == 0:
                assert not t[used_end:b0 + nb].any().item(), ("padding not zero", r, k)
            else:
                for dd, local, _, n in oracle.dp_pieces(sv, odst, used_end, b0 + nb):
                    if dd == d:
                        assert not t[local:local + n].any().item(), ("padding not zero", r, k)


def _groups(ospec):
    """All logical tensors in the groups the oracle handles one at a time: embeddings / final norm / head first,
    then one transformer layer per group (host memory stays at one group)."""
    import re
    names = list(oracle.logical_tensors(ospec))
    yield "embeddings, final norm, head", [n for n in names if not re.match(r"L\d+\.", n)]
    for l in range(ospec.n_layers):
        yield f"layer {l}", _layer(ospec, l)


def _planned_bytes(cfg, only, ospec, odst, names):
    """Bytes of planned target state built from `names` alone (0: the plan writes nothing that depends on them)."""
    have, total = set(names), 0
    for k in cfg["kinds"]:
        for tp, pp, ep in oracle.columns(odst, k):
            if only.get("tp", tp) != tp or only.get("pp", pp) != pp:
                continue
            sv = oracle.stage_view(ospec, odst, tp, pp, ep)
            for prm in sv.params:
                if not (prm.blocks and all(b.name in have for b in prm.blocks)):
                    continue
                if k == 0:
                    total += 2 * prm.size * sum(1 for d in range(odst.dp) if only.get("dp", d) == d)
                else:
                    total += 4 * sum(n for d, _, _, n in oracle.dp_pieces(sv, odst, prm.offset, prm.offset + prm.size)
                                     if only.get("dp", d) == d)
    return total


def _run_complete(name):
    """Direct reshard compared with the oracle on EVERY planned target element, group by group; then the staged
    path, the fused staged entry and derive mode into a second set of target buffers, each compared with the
    verified direct result on the device."""
    import time
    print(f"{name}: generating state in HBM", flush=True)
    cfg, only, ospec, osrc, odst, plan, src, dst, src_bufs = _setup(name)
    info = lv.liver_plan_info(plan)
    sums = {key: int(t.view(torch.int16 if key[1] == 0 else torch.int32).sum(dtype=torch.int64)) for key, t in src_bufs.items()}
    dst_bufs = _fresh_dst(plan, dst)
    lv.liver_reshard(plan, src_bufs, dst_bufs)
    torch.cuda.synchronize()
    t0, n_bytes = time.perf_counter(), 0
    for label, names in _groups(ospec):
        want_bytes = _planned_bytes(cfg, only, ospec, odst, names)
        if want_bytes == 0:
            continue
        expected = _expected(cfg, only, ospec, osrc, odst, src_bufs, names, quiet=True)
        got_bytes = sum(n * (2 if k == 0 else 4) for k, n in _compare(expected, only, odst, dst_bufs, "direct", per_kind=True).items())
        assert got_bytes == want_bytes, (label, got_bytes, want_bytes)
        n_bytes += got_bytes
        print(f"  {name}: {label} equal, {n_bytes / 1e9:.2f} GB so far, {time.perf_counter() - t0:.0f} s", flush=True)
    _pads_zero(only, ospec, odst, dst_bufs)
    # every byte the plan writes is either one of the compared elements or zero padding
    assert n_bytes == info.bytes_written - info.pad_bytes == info.stream_bytes, (n_bytes, info.bytes_written, info.pad_bytes)
    print(f"{name}: direct equals the oracle on all {n_bytes} bytes of planned target state "
          f"(+ {info.pad_bytes} bytes of zero padding); staged path, {info.n_chunks} chunks", flush=True)
    staged = _fresh_dst(plan, dst)
    staging = torch.empty(cfg["chunk_bytes"], dtype=torch.uint8, device="cuda")
    for c in range(info.n_chunks):
        lv.liver_pack(plan, c, src_bufs, staging)
        lv.liver_unpack(plan, c, staging, staged)
    torch.cuda.synchronize()
    for key in dst_bufs:
        assert torch.equal(dst_bufs[key], staged[key]), ("staged differs from the verified direct result", key)

    def refill():
        for key, t in staged.items():
            t.fill_(-23131 if key[1] == 0 else -1515870811)
    print(f"{name}: fused staged entry", flush=True)
    refill()
    staging2 = torch.empty_like(staging)
    lv.liver_reshard_staged_fused(plan, src_bufs, staged, staging, staging2)
    torch.cuda.synchronize()
    for key in dst_bufs:
        assert torch.equal(dst_bufs[key], staged[key]), ("fused staged differs from the verified direct result", key)
    del staging, staging2
    if 0 in cfg["kinds"] and 1 in cfg["kinds"]:
        # the generated state holds PARAM = bf16(MASTER) (torch's conversion), so re-deriving the bf16 weights from
        # the fp32 master weights in the same pass must give the very bytes the copy gave, for every element
        print(f"{name}: derive mode (fused fp32 -> bf16 cast)", flush=True)
        dplan = lv.liver_plan_create(lv.ModelSpec(**cfg["spec"]), src,
                                     lv.Layout(pad_multiple=cfg["pad_multiple"], kinds=tuple(cfg["kinds"]), derive_bf16=True,
                                               **{"only_" + k: v for k, v in only.items()}, **cfg["dst"]), cfg["chunk_bytes"])
        refill()
        lv.liver_reshard(dplan, src_bufs, staged)
        torch.cuda.synchronize()
        for key in dst_bufs:
            assert torch.equal(dst_bufs[key], staged[key]), ("derive mode differs from the verified copy result", key)
    for key, t in src_bufs.items():          # source world untouched
        assert int(t.view(torch.int16 if key[1] == 0 else torch.int32).sum(dtype=torch.int64)) == sums[key], key
    print(f"{name}: staged, fused-staged and derive results equal the direct result on every element", flush=True)


def _run(name, names):
    name, cfg_or_name = (name["name"], name) if isinstance(name, dict) else (name, name)
    print(f"{name}: generating state in HBM", flush=True)
    cfg, only, ospec, osrc, odst, plan, src, dst, src_bufs = _setup(cfg_or_name)
    sums = {key: int(t.view(torch.int16 if key[1] == 0 else torch.int32).sum(dtype=torch.int64)) for key, t in src_bufs.items()}
    info = lv.liver_plan_info(plan)
    print(f"{name}: direct reshard, {info.n_desc} descriptors, {(info.bytes_read + info.bytes_written) / 1e9:.2f} GB", flush=True)
    dst_bufs = _fresh_dst(plan, dst)
    lv.liver_reshard(plan, src_bufs, dst_bufs)
    torch.cuda.synchronize()
    print(f"{name}: oracle on {len(names)} tensors", flush=True)
    expected = _expected(cfg, only, ospec, osrc, odst, src_bufs, names)
    n = _compare(expected, only, odst, dst_bufs, "direct")
    _pads_zero(only, ospec, odst, dst_bufs)
    print(f"{name}: direct ok on {n} sampled elements; staged path, {info.n_chunks} chunks", flush=True)
    del dst_bufs
    dst_bufs = _fresh_dst(plan, dst)
    staging = torch.empty(cfg["chunk_bytes"], dtype=torch.uint8, device="cuda")
    for c in range(info.n_chunks):
        lv.liver_pack(plan, c, src_bufs, staging)
        lv.liver_unpack(plan, c, staging, dst_bufs)
    torch.cuda.synchronize()
    _compare(expected, only, odst, dst_bufs, "staged")
    _pads_zero(only, ospec, odst, dst_bufs)
    for key, t in src_bufs.items():          # source world untouched
        assert int(t.view(torch.int16 if key[1] == 0 else torch.int32).sum(dtype=torch.int64)) == sums[key], key
    print(f"{name}: staged ok", flush=True)


def _layer(ospec, l, leaves=None):
    return [n for n in oracle.logical_tensors(ospec) if n.startswith(f"L{l}.") and (leaves is None or n.split(".", 1)[1] in leaves)]


def test_llama7b_tp8_to_tp4pp2_every_element():
    """All 94,349,000,704 bytes of the 7B target state against the oracle."""
    _run_complete("llama7b")


def test_llama13b_dp8_to_dp6_every_element():
    """The whole share of target rank (tp 0, pp 1, dp 2): 6.51 GB of fp32 optimizer state."""
    _run_complete("llama13b_dp")


def test_llama70b_one_target_rank_every_element():
    """The whole share of target rank (tp 1, pp 3, dp 2): bf16 weights of its 10 layers and its DP slice of the
    fp32 state."""
    _run_complete("llama70b_rank")


def test_llama7b_layout_variants_at_full_size():
    """The 7B shape with every layout variant switched on: vocabulary padded per world (32000 -> 32768 rows),
    40 M-element buckets, interleaved stages on the target, DP 1 -> 2 (bucket-wise DP slices), derived bf16."""
    cfg = dict(synth.CONFIGS["llama7b"], name="llama7b variants",
               src=dict(tp=8, pp=1, dp=1, vocab_multiple=128, bucket_elems=40_000_000),
               dst=dict(tp=4, pp=2, dp=2, vpp=2, vocab_multiple=128, bucket_elems=40_000_000), kinds=(0, 1, 2, 3))
    ospec = oracle.ModelSpec(**cfg["spec"])
    names = ["embed.word", "lm_head.w", "final_norm.w"] + _layer(ospec, 0, ("q.w", "k.w", "v.w", "o.w", "ln1.w")) \
        + _layer(ospec, 8, ("gate.w", "down.w")) + _layer(ospec, 23, ("up.w", "o.w", "ln2.w")) + _layer(ospec, 31, ("down.w", "q.w"))
    _run(cfg, names)


def test_llama7b_single_rank_buffers_of_27_gb():
    """Maximum buffer sizes: the whole 7B state on ONE source rank (13.5 GB of bf16, 27 GB per fp32 kind, byte
    offsets far beyond 2^32) split for TP2; the sampled tensors include the head at the very end of the buffers."""
    cfg = dict(synth.CONFIGS["llama7b"], name="llama7b tp1->tp2", src=dict(tp=1, pp=1, dp=1), dst=dict(tp=2, pp=1, dp=1))
    ospec = oracle.ModelSpec(**cfg["spec"])
    names = ["embed.word", "final_norm.w", "lm_head.w"] + _layer(ospec, 0, ("q.w", "o.w", "ln1.w")) \
        + _layer(ospec, 17, ("k.w", "gate.w", "down.w")) + _layer(ospec, 31, ("v.w", "o.w", "up.w", "down.w", "ln2.w"))
    _run(cfg, names)


def _digest(bufs):
    """Order-sensitive digest of every buffer: plain sum and position-weighted sum of the raw words."""
    out = {}
    for key, t in bufs.items():
        v = t.view(torch.int16 if key[1] == 0 else torch.int32)
        w = torch.arange(v.numel(), device=v.device, dtype=torch.int64) % 65521 + 1
        out[key] = (int(v.sum(dtype=torch.int64)), int((w * v).sum(dtype=torch.int64)))
        del w
    return out


def test_llama7b_every_launch_shape_gives_the_same_bits():
    """Full 7B size (1.44 M tiles in one pass): grids from one workgroup per CU to 65536, every tile order (teams included)
    and the four cache-hint settings all reproduce the digest of the default launch, which the sampled oracle
    comparison has verified in the same run."""
    _, ospec, _, _ = cfg_objects("llama7b")
    print("llama7b launch shapes: generating state in HBM", flush=True)
    cfg, only, ospec, osrc, odst, plan, src, dst, src_bufs = _setup("llama7b")
    dst_bufs = _fresh_dst(plan, dst)
    lv.liver_reshard(plan, src_bufs, dst_bufs)
    torch.cuda.synchronize()
    names = ["lm_head.w"] + _layer(ospec, 0, ("o.w", "gate.w")) + _layer(ospec, 31, ("q.w", "down.w"))
    _compare(_expected(cfg, only, ospec, osrc, odst, src_bufs, names), only, odst, dst_bufs, "default launch")
    want = _digest(dst_bufs)
    for grid, order, hints in [(256, 1, 3), (512, 0, 0), (1000, 2, 1), (4096, 1, 2), (65536, 0, 3), (65536, 2, 0), (97, 2, 3),
                               (256, 0, 3), (1000, 132, 3), (256, 116, 1)]:
        print(f"llama7b launch shapes: grid {grid} order {order} hints {hints}", flush=True)
        for t in dst_bufs.values():
            t.fill_(-23131 if t.dtype == torch.int16 else -1515870811)
        lv.liver_plan_set_launch(plan, grid, order, hints)
        lv.liver_reshard(plan, src_bufs, dst_bufs)
        torch.cuda.synchronize()
        assert _digest(dst_bufs) == want, (grid, order, hints)


def _round_trip_world(identical_replicas):
    """The fp32 state of the 7B source world (81 GB; a third world with the bf16 weights as well would not fit),
    both plans of the round trip, and the element ranges of the TP-replicated parameters on TP ranks > 0."""
    cfg = dict(synth.CONFIGS["llama7b"], kinds=(1, 2, 3))
    ospec = oracle.ModelSpec(**cfg["spec"])
    osrc = oracle.Layout(pad_multiple=cfg["pad_multiple"], **cfg["src"])
    spec = lv.ModelSpec(**cfg["spec"])
    a = dict(pad_multiple=cfg["pad_multiple"], **cfg["src"])
    b = dict(pad_multiple=cfg["pad_multiple"], **cfg["dst"])
    fwd = lv.liver_plan_create(spec, lv.Layout(**a), lv.Layout(kinds=(1, 2, 3), **b), cfg["chunk_bytes"])
    back = lv.liver_plan_create(spec, lv.Layout(**b), lv.Layout(kinds=(1, 2, 3), **a), cfg["chunk_bytes"])
    g = torch.Generator(device="cuda").manual_seed(synth.SEED_BASE)
    A = {}
    for r in range(fwd.src.n_ranks):
        for k in (1, 2, 3):
            n = lv.liver_plan_buffer_bytes(fwd, 0, r, k) // 4
            assert n == lv.liver_plan_buffer_bytes(back, 1, r, k) // 4
            A[(r, k)] = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, 0.02, generator=g).view(torch.int32)
    assert osrc.dp == 1 and osrc.pp == 1                     # flat offsets are buffer offsets in this world
    first = {p.name: p for p in oracle.stage_view(ospec, osrc, 0, 0).params}
    copies = []                                              # (tp, offset there, offset on tp 0, elements)
    for tp in range(1, osrc.tp):
        for p in oracle.stage_view(ospec, osrc, tp, 0).params:
            if not p.canonical:
                assert first[p.name].size == p.size
                copies.append((tp, p.offset, first[p.name].offset, p.size))
    assert len(copies) == (osrc.tp - 1) * (2 * ospec.n_layers + 1)      # ln1.w, ln2.w per layer, final_norm.w
    if identical_replicas:                                   # what a real training job holds: replicas agree
        for tp, off, off0, n in copies:
            for k in (1, 2, 3):
                A[(osrc.rank(tp, 0, 0), k)][off:off + n] = A[(osrc.rank(0, 0, 0), k)][off0:off0 + n]
    return cfg, fwd, back, A, copies, osrc


def test_llama7b_round_trip_returns_every_bit():
    """A -> B -> A at the full 7B size with identical TP replicas of the replicated parameters (the precondition
    under which a round trip is the identity): EVERY buffer of every rank comes back bit for bit.  A second
    forward pass through the staged path reproduces B exactly."""
    print("round trip: generating state in HBM", flush=True)
    cfg, fwd, back, A, _, _ = _round_trip_world(identical_replicas=True)
    B = _fresh_dst(fwd, fwd.dst)
    print("round trip: forward", flush=True)
    lv.liver_reshard(fwd, A, B)
    A2 = _fresh_dst(back, back.dst)
    print("round trip: back", flush=True)
    lv.liver_reshard(back, B, A2)
    torch.cuda.synchronize()
    assert set(A2) == set(A)
    for key, t in A.items():
        assert torch.equal(t, A2[key]), key
    del A, t
    print("round trip: second forward pass, staged", flush=True)
    B2 = _fresh_dst(fwd, fwd.dst)
    staging = torch.empty(cfg["chunk_bytes"], dtype=torch.uint8, device="cuda")
    for c in range(lv.liver_plan_info(fwd).n_chunks):
        lv.liver_pack(fwd, c, A2, staging)
        lv.liver_unpack(fwd, c, staging, B2)
    torch.cuda.synchronize()
    for key in B:
        assert torch.equal(B[key], B2[key]), key


def test_llama7b_reads_only_the_first_replica():
    """Which copy of a replicated value is read, at full size: with DIFFERENT values in the TP replicas of the
    norm weights the target world is the same as with the replicas of TP rank 0 everywhere, and the way back
    writes TP rank 0's values into every replica."""
    print("first replica: generating state in HBM", flush=True)
    cfg, fwd, back, A, copies, osrc = _round_trip_world(identical_replicas=False)
    B = _fresh_dst(fwd, fwd.dst)
    lv.liver_reshard(fwd, A, B)
    A2 = _fresh_dst(back, back.dst)
    lv.liver_reshard(back, B, A2)
    torch.cuda.synchronize()
    print("first replica: comparing", flush=True)
    for k in (1, 2, 3):
        r0 = osrc.rank(0, 0, 0)
        assert torch.equal(A[(r0, k)], A2[(r0, k)]), k
        for tp, off, off0, n in copies:
            r = osrc.rank(tp, 0, 0)
            assert not torch.equal(A[(r, k)][off:off + n], A[(r0, k)][off0:off0 + n])         # the input replicas differ
            assert torch.equal(A2[(r, k)][off:off + n], A[(r0, k)][off0:off0 + n]), (tp, off, k)
            A[(r, k)][off:off + n] = A[(r0, k)][off0:off0 + n]
    for key, t in A.items():          # apart from the replicas, nothing changed on the way there and back
        assert torch.equal(t, A2[key]), key


def test_llama13b_through_a_5_gib_staging_chunk():
    """Wire offsets beyond 2^32: the 13B optimizer-state share streamed through two 5 GiB chunks (6.06 GiB of payload)."""
    cfg = dict(synth.CONFIGS["llama13b_dp"], name="llama13b 5 GiB chunks", chunk_bytes=5 << 30)
    ospec = oracle.ModelSpec(**cfg["spec"])
    names = _layer(ospec, 26, ("o.w", "gate.w")) + _layer(ospec, 28, ("q.w", "down.w", "ln2.w")) + _layer(ospec, 30, ("k.w", "v.w", "o.w"))
    _run(cfg, names)


# ---------------------------------------------------------------- mixture of experts at full size
def _moe_world(ospec, olay, lay, plan, side, device):
    """Source buffers of an MoE world generated in device memory: {(rank, kind): tensor}.  Dense buffers per
    (tp, pp) column over all DP ranks, expert buffers per (tp, pp, ep) column over the DP ranks ep, ep+EP, ...;
    only the first replica of each bf16 buffer exists (the only one a reshard reads)."""
    bufs = {}
    for fam, base in ((None, 0), ("x", 4)):
        sizes, members = {}, {}
        for tp, pp, ep in oracle.columns(olay, base):
            sv = oracle.stage_view(ospec, olay, tp, pp, ep)
            for j, d in enumerate(sv.dp_ranks):
                n = lv.liver_plan_buffer_bytes(plan, side, lay.rank(tp, pp, d), base + 1) // 4
                assert n == sv.S
                sizes[((tp, pp, -1 if ep is None else ep), j)] = n
            members[(tp, pp, -1 if ep is None else ep)] = sv.dp_ranks
        group = len(next(iter(members.values())))
        gen = synth.fill_device_world(sizes, group, synth.SEED_BASE + base, device=device)
        for col, ranks in members.items():
            for j, d in enumerate(ranks):
                r = lay.rank(col[0], col[1], d)
                for k in (1, 2, 3):
                    bufs[(r, base + k)] = gen[(col, j, k)]
            bufs[(lay.rank(col[0], col[1], ranks[0]), base)] = gen[(col, "param")]
    return bufs


_WORD = {k: (np.uint16 if k % 4 == 0 else np.uint32) for k in range(8)}
_TT = {k: (torch.int16 if k % 4 == 0 else torch.int32) for k in range(8)}


def _moe_expected(ospec, osrc, odst, src_bufs, names):
    """Sampled logical tensors, every kind of both families, gathered from the source buffers and re-split by the
    oracle: [(target rank, kind, offset in its buffer, expected words, parameter name)]."""
    def read(rank, kind, lo, hi):
        return src_bufs[(rank, kind)][lo:hi].view(_TT[kind]).cpu().numpy().view(_WORD[kind])
    out = []
    for k in oracle.kinds_of(ospec):
        logical = oracle.gather_logical(ospec, osrc, k, read, names=names)
        for tp, pp, sv, prm, shard in oracle.expected_shards(ospec, odst, logical, kind=k):
            flat = shard.ravel()
            pieces = [(d, prm.offset, prm.offset, prm.size) for d in sv.dp_ranks] if k % 4 == 0 \
                else oracle.dp_pieces(sv, odst, prm.offset, prm.offset + prm.size)
            out += [(odst.rank(tp, pp, d), k, local, flat[at - prm.offset:at - prm.offset + n], prm.name) for d, local, at, n in pieces]
        print(f"  oracle: kind {k} gathered and split", flush=True)
    return out


def _moe_compare(expected, dst_bufs, what):
    n_checked = 0
    for rank, k, local, want, name in expected:
        got = dst_bufs[(rank, k)][local:local + want.size].view(_TT[k]).cpu().numpy().view(_WORD[k])
        assert np.array_equal(got, want), (what, name, "rank", rank, "kind", k)
        n_checked += want.size
    assert n_checked > 0
    return n_checked


def _moe_run(spec_kw, src_kw, dst_kw, chunk_bytes, names, device="cuda", runner=None):
    ospec = oracle.ModelSpec(**spec_kw)
    osrc, odst = oracle.Layout(**src_kw), oracle.Layout(**dst_kw)
    spec, src, dst = lv.ModelSpec(**spec_kw), lv.Layout(**src_kw), lv.Layout(**dst_kw)
    plan = lv.liver_plan_create(spec, src, dst, chunk_bytes)
    info = lv.liver_plan_info(plan)
    print(f"moe: generating state, {(info.bytes_read + info.bytes_written) / 1e9:.2f} GB to move, {info.n_desc} descriptors", flush=True)
    src_bufs = _moe_world(ospec, osrc, src, plan, 0, device)
    for (r, k) in src_bufs:
        assert lv.liver_plan_buffer_used(plan, 0, r, k), (r, k)
    dst_bufs = {}
    for r in range(dst.n_ranks):
        for k in range(8):
            if lv.liver_plan_buffer_used(plan, 1, r, k):
                n = lv.liver_plan_buffer_bytes(plan, 1, r, k) // (2 if k % 4 == 0 else 4)
                dst_bufs[(r, k)] = torch.full((n,), -23131 if k % 4 == 0 else -1515870811,
                                              dtype=torch.int16 if k % 4 == 0 else torch.int32, device=device)
    print("moe: direct reshard", flush=True)
    if runner is None:
        lv.liver_reshard(plan, src_bufs, dst_bufs)
        torch.cuda.synchronize()
    else:
        runner(plan, src_bufs, dst_bufs, False)
    expected = _moe_expected(ospec, osrc, odst, src_bufs, names)
    n = _moe_compare(expected, dst_bufs, "direct")
    print(f"moe: direct ok on {n} sampled elements; staged path, {info.n_chunks} chunks", flush=True)
    for t in dst_bufs.values():
        t.fill_(-7)
    if runner is None:
        staging = torch.empty(chunk_bytes, dtype=torch.uint8, device=device)
        for c in range(info.n_chunks):
            lv.liver_pack(plan, c, src_bufs, staging)
            lv.liver_unpack(plan, c, staging, dst_bufs)
        torch.cuda.synchronize()
    else:
        runner(plan, src_bufs, dst_bufs, True)
    _moe_compare(expected, dst_bufs, "staged")
    print("moe: staged ok", flush=True)


def test_mixture_of_experts_at_full_size():
    """A 6.7 B-parameter MoE (8 layers, 8 experts of FFN 7168, GQA 32/8): TP2.PP2.DP4.EP4 -> TP4.PP1.DP4.EP2, all
    eight buffer kinds, about 100 GB per world; sampled dense and expert tensors against the oracle."""
    spec_kw = dict(n_layers=8, hidden=4096, n_q_heads=32, n_kv_heads=8, ffn=7168, vocab=32000, max_pos=0, glu=True,
                   norm_bias=False, linear_bias=False, tied_embed=False, n_experts=8)
    names = ["embed.word", "lm_head.w", "final_norm.w", "L0.router.w", "L0.q.w", "L0.k.w", "L0.v.w", "L0.o.w", "L0.ln1.w",
             "L0.x0.gate.w", "L0.x0.up.w", "L0.x0.down.w", "L3.x5.gate.w", "L3.x5.up.w", "L3.x5.down.w", "L4.x2.down.w",
             "L7.x7.gate.w", "L7.x7.up.w", "L7.x7.down.w", "L7.router.w", "L7.ln2.w"]
    _moe_run(spec_kw, dict(tp=2, pp=2, dp=4, pad_multiple=128, ep=4), dict(tp=4, pp=1, dp=4, pad_multiple=128, ep=2),
             256 << 20, names)

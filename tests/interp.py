"""Host interpreter of the planner's public descriptors (test tool).

Executes liver_desc_t lists with NumPy, one descriptor at a time, exactly as
include/liver.h defines them, counting how often every target element is
written.  It lets the planner be checked against the oracle without a GPU, and
it is a third code path beside the oracle and the HIP kernels."""
import numpy as np

import oracle
import paper_2605_22014_amd as lv

DT = {k: (np.uint16 if k % 4 == 0 else np.uint32) for k in range(8)}     # kinds 4..7: expert buffers


def lv_objects(cfg_or_spec, src, dst, **dst_kw):
    """oracle ModelSpec/Layouts -> binding ModelSpec/Layouts (same fields)."""
    s = cfg_or_spec
    spec = lv.ModelSpec(s.n_layers, s.hidden, s.n_q_heads, s.n_kv_heads, s.ffn, s.vocab, s.max_pos, s.glu,
                        s.norm_bias, s.linear_bias, s.tied_embed, s.n_experts)
    a = lv.Layout(src.tp, src.pp, src.dp, src.pad_multiple, vpp=src.vpp, vocab_multiple=src.vocab_multiple, pp_first=src.pp_first,
                  pp_last=src.pp_last, bucket_elems=src.bucket_elems, ep=src.ep)
    b = lv.Layout(dst.tp, dst.pp, dst.dp, dst.pad_multiple, vpp=dst.vpp, vocab_multiple=dst.vocab_multiple, pp_first=dst.pp_first,
                  pp_last=dst.pp_last, bucket_elems=dst.bucket_elems, ep=dst.ep, **dst_kw)
    return spec, a, b


def descs(plan, which):
    return [lv.liver_plan_desc(plan, which, i) for i in range(lv.liver_plan_desc_count(plan, which))]


def _rows(buf, off, stride, rows, run):
    """(rows, run) strided view of 1-D array `buf`, bounds-checked."""
    assert rows >= 1 and run >= 1 and off >= 0
    assert off + (rows - 1) * stride + run <= buf.size, ("out of bounds", off, stride, rows, run, buf.size)
    assert rows == 1 or stride >= run, "rows overlap"
    return np.lib.stride_tricks.as_strided(buf[off:], shape=(rows, run),
                                           strides=(stride * buf.itemsize, buf.itemsize), writeable=True)


def alloc_dst(plan, fill=0xA5):
    """Sentinel-filled target buffers for every target rank/kind + zeroed write counters."""
    n = lv.liver_plan_info(plan).n_dst_ranks
    bufs, counts = {}, {}
    for r in range(n):
        for k in range(8):
            nbytes = lv.liver_plan_buffer_bytes(plan, 1, r, k)
            if nbytes == 0:                      # expert kinds of a dense model
                continue
            bufs[(r, k)] = np.full(nbytes // np.dtype(DT[k]).itemsize, fill * 0x01010101 & (0xFFFF if k % 4 == 0 else 0xFFFFFFFF), DT[k])
            counts[(r, k)] = np.zeros(bufs[(r, k)].size, np.uint8)
    return bufs, counts


def execute(d, src_bufs, dst_bufs, counts, staging=None):
    if d.dst_rank < 0:
        dst = staging.view(DT[d.src_kind])
    else:
        dst = dst_bufs[(d.dst_rank, d.dst_kind)]
    out = _rows(dst, d.dst_off, d.dst_stride, d.rows, d.run)
    if d.op == lv.OP_ZERO:
        out[...] = 0
    else:
        src = staging.view(DT[d.src_kind]) if d.src_rank < 0 else src_bufs[(d.src_rank, d.src_kind)]
        val = _rows(src, d.src_off, d.src_stride, d.rows, d.run)
        if d.op == lv.OP_CAST_BF16:
            assert d.src_kind % 4 == oracle.MASTER and d.dst_kind == d.src_kind - 1
            out[...] = oracle.rne_bf16(val)
        else:
            assert d.op == lv.OP_COPY and (d.dst_rank < 0 or DT[d.src_kind] == DT[d.dst_kind])
            out[...] = val
    if d.dst_rank >= 0 and counts is not None:
        _rows(counts[(d.dst_rank, d.dst_kind)], d.dst_off, d.dst_stride, d.rows, d.run)[...] += 1


def run_direct(plan, src_bufs):
    dst, counts = alloc_dst(plan)
    for d in descs(plan, lv.LIST_DIRECT):
        assert d.chunk == -1 and d.dst_rank >= 0 and (d.src_rank >= 0 or d.op == lv.OP_ZERO)
        execute(d, src_bufs, dst, counts)
    return dst, counts


def run_staged(plan, src_bufs, order=None):
    info = lv.liver_plan_info(plan)
    dst, counts = alloc_dst(plan)
    pk, un = {}, {}
    for d in descs(plan, lv.LIST_PACK):
        assert d.dst_rank == -1 and d.src_rank >= 0 and d.op == lv.OP_COPY
        pk.setdefault(d.chunk, []).append(d)
    for d in descs(plan, lv.LIST_UNPACK):
        assert d.dst_rank >= 0
        un.setdefault(d.chunk, []).append(d)
    assert sorted(pk) == list(range(info.n_chunks)) and set(un) <= set(pk)
    rng = np.random.default_rng(0)
    for c in (order if order is not None else range(info.n_chunks)):
        staging = rng.integers(0, 256, size=plan.chunk_bytes, dtype=np.uint8)   # garbage between payloads
        covered = np.zeros(plan.chunk_bytes, np.uint8)
        for d in pk[c]:
            execute(d, src_bufs, None, None, staging)
            eb = np.dtype(DT[d.src_kind]).itemsize
            assert d.dst_stride == d.run and (d.dst_off * eb) % eb == 0
            covered[d.dst_off * eb:(d.dst_off + d.rows * d.run) * eb] += 1
        assert covered.max() <= 1, "wire pieces overlap"
        for d in un.get(c, []):
            if d.op != lv.OP_ZERO:
                eb = np.dtype(DT[d.src_kind]).itemsize
                assert covered[d.src_off * eb:(d.src_off + d.rows * d.run) * eb].all(), "unpack reads unwritten wire bytes"
            execute(d, None, dst, counts, staging)
    return dst, counts


def used_dst(plan):
    n = lv.liver_plan_info(plan).n_dst_ranks
    return {(r, k) for r in range(n) for k in range(8) if lv.liver_plan_buffer_used(plan, 1, r, k)}


def emulate_direct(plan, src_bufs):
    """The LOWERED descriptors (what the kernels run) executed on host memory by the
    library's bounds-checked emulator."""
    dst, _ = alloc_dst(plan)
    src = {k: np.ascontiguousarray(v) for k, v in src_bufs.items()}
    lv.liver_debug_emulate_host(plan, lv.LIST_DIRECT, 0, src, dst, None)
    return dst


def emulate_staged(plan, src_bufs):
    dst, _ = alloc_dst(plan)
    src = {k: np.ascontiguousarray(v) for k, v in src_bufs.items()}
    for c in range(lv.liver_plan_info(plan).n_chunks):
        staging = np.full(plan.chunk_bytes, 0x3C, np.uint8)
        lv.liver_debug_emulate_host(plan, lv.LIST_PACK, c, src, None, staging)
        lv.liver_debug_emulate_host(plan, lv.LIST_UNPACK, c, None, dst, staging)
    return dst

#!/usr/bin/env python3
"""Benchmark: reshard GB/s (read + write) of the Llama-7B-shape TP8 -> TP4.PP2
reshard on one MI355X, with the HBM roofline of the copy kernel and the CPU
oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One step = one liver_reshard call: the whole state (bf16 params + fp32 master,
Adam m, Adam v of all 8 source ranks) is moved into the 8 target ranks' buffers,
all resident in HBM.  value = algorithmic bytes (every target byte read once and
written once) / time.  The staged path (pack + unpack through one staging chunk),
the fused-cast (derive) mode and the plan time are reported as extra fields of
the same JSON line; they are not part of `value`.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# HBM traffic (GB) per direct-reshard launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled
# by what the same counters read for a plain 1 GiB copy (FETCH x1.99993, WRITE x1.0).
MEASURED_TRAFFIC_GB = {"llama7b": 188.73}   # profiles/liver_copy_kernel_llama7b_direct.md


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b")
    ap.add_argument("--grid", type=int, default=0)
    ap.add_argument("--tile-order", type=int, default=-1, help="-1 = library default")
    ap.add_argument("--cache-hints", type=int, default=-1, help="-1 = library default")
    ap.add_argument("--no-extras", action="store_true", help="skip staged / derive / copy-ceiling legs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference dispatch for --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all logical ranks' shards live in one MI355X's HBM); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import liver_synth as synth
    import paper_2605_22014_amd as lv

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    only = cfg["only"] or {}
    spec = lv.ModelSpec(**cfg["spec"])
    src = lv.Layout(pad_multiple=cfg["pad_multiple"], **cfg["src"])
    dst_kw = dict(pad_multiple=cfg["pad_multiple"], kinds=tuple(cfg["kinds"]),
                  **{"only_" + k: v for k, v in only.items()}, **cfg["dst"])
    dst = lv.Layout(**dst_kw)

    torch.zeros(1, device="cuda")        # HIP context and allocator are up before planning is timed
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plan = lv.liver_plan_create(spec, src, dst, cfg["chunk_bytes"])      # host planning + upload of the descriptor table
    plan_ms = (time.perf_counter() - t0) * 1e3
    info = lv.liver_plan_info(plan)
    if args.grid or args.tile_order >= 0 or args.cache_hints >= 0:
        lv.liver_plan_set_launch(plan, args.grid, args.tile_order, args.cache_hints)
    algo_bytes = info.bytes_read + info.bytes_written

    # ---- buffers: every used source and target buffer, allocated ALTERNATELY (source, target, source, ...)
    # and SPREAD over the whole HBM by unused gap allocations between them.  Where the caller's buffers sit in
    # HBM changes the bandwidth of any copy on this part by ~10 % (measured): in the first
    # process on a freshly booted box "all sources, then all targets, back to back" runs this reshard at
    # 5.6 TB/s; spread over the HBM it runs at 6.25 TB/s in every process.  The library does not own the
    # buffers, so the benchmark places them well and says so.
    src_keys = [(r, k) for r in range(src.n_ranks) for k in range(4) if _column_used(lv, plan, src, r)]
    dst_keys = [(r, k) for r in range(dst.n_ranks) for k in range(4) if lv.liver_plan_buffer_used(plan, 1, r, k)]
    need = sum(lv.liver_plan_buffer_bytes(plan, 0, r, k) for r, k in src_keys) \
        + sum(lv.liver_plan_buffer_bytes(plan, 1, r, k) for r, k in dst_keys)
    free, _ = torch.cuda.mem_get_info()
    gap = max(0, (free - need - (14 << 30)) // (len(src_keys) + len(dst_keys))) & ~((2 << 20) - 1)
    src_bufs, dst_bufs, gaps = {}, {}, []

    def spacer():
        if gap:
            gaps.append(torch.empty(gap, dtype=torch.uint8, device="cuda"))
    for i in range(max(len(src_keys), len(dst_keys))):
        if i < len(src_keys):
            r, k = src_keys[i]
            n = lv.liver_plan_buffer_bytes(plan, 0, r, k)
            src_bufs[(r, k)] = torch.empty(n // (2 if k == 0 else 4), dtype=torch.bfloat16 if k == 0 else torch.float32,
                                           device="cuda")
            spacer()
        if i < len(dst_keys):
            r, k = dst_keys[i]
            dst_bufs[(r, k)] = torch.empty(lv.liver_plan_buffer_bytes(plan, 1, r, k), dtype=torch.uint8, device="cuda")
            spacer()
    # ---- synthetic state, generated in place: N(0, 0.02) fp32, PARAM = bf16(MASTER), all DP replicas identical
    columns = {}
    for pp in range(src.pp):
        for tp in range(src.tp):
            ranks = [src.rank(tp, pp, d) for d in range(src.dp)]
            if (ranks[0], lv.MASTER) not in src_bufs:
                continue
            columns[(pp, tp)] = {"master": [src_bufs[(r, lv.MASTER)] for r in ranks],
                                 "m": [src_bufs[(r, lv.ADAM_M)] for r in ranks],
                                 "v": [src_bufs[(r, lv.ADAM_V)] for r in ranks],
                                 "param": src_bufs[(ranks[0], lv.PARAM)]}
    synth.fill_device_world_into(columns, synth.SEED_BASE)
    for (pp, tp), col in columns.items():
        for d in range(1, src.dp):
            src_bufs[(src.rank(tp, pp, d), lv.PARAM)].copy_(col["param"])
    from paper_2605_22014_amd._binding import make_table
    src_tab, dst_tab = make_table(src_bufs, src.n_ranks, plan, 0), make_table(dst_bufs, dst.n_ranks, plan, 1)
    torch.cuda.synchronize()

    def timed(fn, steps, warmup):
        """(wall ms per step, mean event ms per step) of fn() on the current stream."""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t = time.perf_counter()
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t) * 1e3 / steps
        return wall, sum(a.elapsed_time(b) for a, b in ev) / steps

    # ---- the timed region: K direct reshards --------------------------------------------------------
    wall_ms, kern_ms = timed(lambda: lv.liver_reshard(plan, src_tab, dst_tab), args.steps, args.warmup)
    gbs = algo_bytes / (wall_ms * 1e-3) / 1e9
    kern_gbs = algo_bytes / (kern_ms * 1e-3) / 1e9

    out = {
        "metric": "reshard GB/s (read+write), 7B-shape TP8->TP4.PP2" if args.workload == "llama7b"
                  else f"reshard GB/s (read+write), {args.workload}",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": args.workload, "src": cfg["src"], "dst": cfg["dst"], "only": cfg["only"],
                   "kinds": list(cfg["kinds"]), "mode": "direct (liver_reshard)", "algorithmic_bytes": algo_bytes,
                   "n_desc": info.n_desc, "plan_ms": round(plan_ms, 2), "table_bytes_device": info.table_bytes_device,
                   "launch": {"grid": args.grid, "tile_order": args.tile_order, "cache_hints": args.cache_hints},
                   "placement": f"source/target buffers allocated alternately, {gap >> 20} MiB unused gap after each"},
        "pct_hbm_peak": round(100 * gbs / HBM_PEAK_GBS, 2),
        "roofline": {"bound": "hbm", "kernel": "liver_copy_kernel (direct reshard)", "achieved": round(kern_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(kern_gbs / HBM_PEAK_GBS, 4),
                     "avg_launch_ms": round(kern_ms, 4),
                     "traffic": MEASURED_TRAFFIC_GB.get(args.workload)},
    }

    if not args.no_extras:
        extras = {}
        # plain device-to-device copy of one 1 GiB+ buffer: the empirical ceiling of this machine
        big = max(src_bufs.values(), key=lambda t: t.numel() * t.element_size())
        scratch = torch.empty_like(big)
        w, k = timed(lambda: scratch.copy_(big), 10, 2)
        extras["torch_copy_GBs"] = round(2 * big.numel() * big.element_size() / (k * 1e-3) / 1e9, 1)
        del scratch
        # the plainest streaming kernels (contiguous read / fill / copy, same workgroup size, 16-byte non-temporal
        # accesses) over the SAME source and target buffers, paired by size: what this placement gives a copy
        pairs = list(zip(sorted(src_bufs.values(), key=lambda t: -t.numel() * t.element_size()),
                         sorted(dst_bufs.values(), key=lambda t: -t.numel() * t.element_size())))
        pairs = [(a, b, min(a.numel() * a.element_size(), b.numel() * b.element_size()) // 32768 * 32768) for a, b in pairs]
        pairs = [p for p in pairs if p[2] > 0]
        probe_bytes = sum(n for _, _, n in pairs)
        for mode, name in ((0, "plain_read_GBs"), (1, "plain_fill_GBs"), (2, "plain_copy_GBs")):
            best = 0.0
            for grid in (256, 2048, 8192, 32768):
                def probe():
                    for a, b, n in pairs:
                        lv.liver_debug_bandwidth_probe(mode, a, b, n, min(grid, n // 32768))
                w, k = timed(probe, 3, 1)
                best = max(best, (2 if mode == 2 else 1) * probe_bytes / (k * 1e-3) / 1e9)
            extras[name] = round(best, 1)
        # staged path: pack + unpack of every chunk through one staging chunk
        staging = torch.empty(cfg["chunk_bytes"], dtype=torch.uint8, device="cuda")
        nch = info.n_chunks

        def staged():
            for c in range(nch):
                lv.liver_pack(plan, c, src_tab, staging)
                lv.liver_unpack(plan, c, staging, dst_tab)

        def pack_only():
            for c in range(nch):
                lv.liver_pack(plan, c, src_tab, staging)

        def unpack_only():
            for c in range(nch):
                lv.liver_unpack(plan, c, staging, dst_tab)
        w, k = timed(staged, 3, 1)
        extras["staged_end_to_end_GBs"] = round(algo_bytes / (w * 1e-3) / 1e9, 1)
        extras["staged_ms"] = round(w, 3)
        w, k = timed(pack_only, 3, 1)
        extras["pack_kernel_GBs"] = round(2 * info.stream_bytes / (k * 1e-3) / 1e9, 1)
        w, k = timed(unpack_only, 3, 1)
        extras["unpack_kernel_GBs"] = round((info.stream_bytes + info.bytes_written) / (k * 1e-3) / 1e9, 1)
        extras["n_chunks"] = nch
        del staging
        if 0 in cfg["kinds"] and 1 in cfg["kinds"]:
            dplan = lv.liver_plan_create(spec, src, lv.Layout(**dict(dst_kw, derive_bf16=True)), cfg["chunk_bytes"])
            dinfo = lv.liver_plan_info(dplan)
            w, k = timed(lambda: lv.liver_reshard(dplan, src_tab, dst_tab), 5, 1)
            extras["derive_direct_GBs"] = round((dinfo.bytes_read + dinfo.bytes_written) / (k * 1e-3) / 1e9, 1)
            extras["derive_algorithmic_bytes"] = dinfo.bytes_read + dinfo.bytes_written
        # the unpack-only timing loop scattered stale chunks and derive mode rewrote PARAM:
        # restore the copy-mode result before it is compared with the oracle
        lv.liver_reshard(plan, src_tab, dst_tab)
        torch.cuda.synchronize()
        out["extras"] = extras

    if args.calibrate_copy:
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        b = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        a.fill_(1)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, src_bufs, dst_bufs, src, dst)

    print(json.dumps(out))


def _column_used(lv, plan, src, rank):
    """Does the plan read any buffer of the (tp, pp) rank column that `rank` belongs to?"""
    tp, pp = rank % src.tp, rank // (src.tp * src.dp)
    return any(lv.liver_plan_buffer_used(plan, 0, src.rank(tp, pp, d), k) for d in range(src.dp) for k in range(4))


def cpu_baseline(cfg, src_bufs, dst_bufs, src, dst, n_layers_sampled=12):
    """The CPU oracle (gather to full logical tensors, re-split) timed on a bounded
    sample of the same workload: all tensors of a few transformer layers spread
    over the model (of the planned target stage for a filtered plan), all buffer
    kinds, inputs already in host memory, one layer at a time.  Its output also
    checks the GPU result for those layers."""
    import numpy as np
    import torch
    import oracle
    ospec = oracle.ModelSpec(**cfg["spec"])
    osrc = oracle.Layout(pad_multiple=cfg["pad_multiple"], **cfg["src"])
    odst = oracle.Layout(pad_multiple=cfg["pad_multiple"], **cfg["dst"])
    only = cfg["only"] or {}
    per_dst = ospec.n_layers // odst.pp
    first, count = (only["pp"] * per_dst, per_dst) if "pp" in only else (0, ospec.n_layers)
    n = min(n_layers_sampled, count)
    layers = sorted({first + (i * count) // n for i in range(n)})
    tps = [only["tp"]] if "tp" in only else None
    pps = [only["pp"]] if "pp" in only else None
    NP = {0: np.uint16, 1: np.uint32, 2: np.uint32, 3: np.uint32}
    secs, nbytes = 0.0, 0
    for layer in layers:
        names = [t for t in oracle.logical_tensors(ospec) if t.startswith(f"L{layer}.")]
        pp_src = layer // (ospec.n_layers // osrc.pp)
        host = {}                       # host copies of the source ranges that hold this layer
        for tp in range(osrc.tp):
            sv = oracle.stage_view(ospec, osrc, tp, pp_src)
            assert len(sv.buckets) == 1, "the benchmark configurations use one bucket per rank column"
            ps = [p for p in sv.params if p.name.startswith(f"L{layer}.")]
            lo, hi = min(p.offset for p in ps), max(p.offset + p.size for p in ps)
            for d in range(osrc.dp):
                r = osrc.rank(tp, pp_src, d)
                for k in cfg["kinds"]:
                    a, b = (lo, hi) if k == 0 else (max(lo - d * sv.S, 0), min(hi - d * sv.S, sv.S))
                    if a >= b:
                        continue
                    if (r, k) in src_bufs:
                        t = src_bufs[(r, k)][a:b].view(torch.int16 if k == 0 else torch.int32)
                        host[(r, k)] = (a, t.cpu().numpy().view(NP[k]))
                    else:               # a source rank this filtered plan never reads
                        host[(r, k)] = (a, np.zeros(b - a, NP[k]))

        def read(rank, kind, lo, hi):
            base, arr = host[(rank, kind)]
            assert base <= lo and hi - base <= arr.size
            return arr[lo - base:hi - base]

        t0 = time.perf_counter()
        expected = []
        for k in cfg["kinds"]:
            logical = oracle.gather_logical(ospec, osrc, k, read, names=names)
            expected += [(k,) + e for e in oracle.expected_shards(ospec, odst, logical, tps, pps)]
        secs += time.perf_counter() - t0
        for k, tp, pp, sv, prm, shard in expected:      # parity of the GPU result on the same sample
            flat = shard.ravel()
            for d in range(odst.dp):
                if only.get("dp", d) != d:
                    continue
                r = odst.rank(tp, pp, d)
                if k == 0:
                    a, b, part = prm.offset, prm.offset + prm.size, flat
                else:
                    a, b = max(prm.offset, d * sv.S), min(prm.offset + prm.size, (d + 1) * sv.S)
                    if a >= b:
                        continue
                    part = flat[a - prm.offset:b - prm.offset]
                    a, b = a - d * sv.S, b - d * sv.S
                eb = 2 if k == 0 else 4
                got = dst_bufs[(r, k)][a * eb:b * eb].cpu().numpy().view(NP[k])
                assert np.array_equal(got, part), f"GPU result differs from the oracle: layer {layer} {prm.name} kind {k}"
                nbytes += part.nbytes
    return {"value": round(2 * nbytes / secs / 1e9, 3), "unit": "GB/s", "cores": _threads_used(), "kind": "oracle",
            "sample": f"all tensors of layers {layers}, kinds {list(cfg['kinds'])}: {nbytes / 1e9:.2f} GB of target "
                      f"state gathered and re-split in {secs:.2f} s of CPU time; GPU result equal on this sample",
            "host_cores_available": len(os.sched_getaffinity(0))}


def _threads_used():
    return 1          # the oracle is single-threaded NumPy slicing and copying


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark: reshard GB/s (read + write) of the Llama-7B-shape TP8 -> TP4.PP2
reshard on one MI355X, with the HBM roofline of the copy kernel and the CPU
oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One step = one liver_reshard call: the whole state (bf16 params + fp32 master,
Adam m, Adam v of all 8 source ranks) is moved into the 8 target ranks' buffers,
all resident in HBM.  value = algorithmic bytes (every target byte read once and
written once) / time.

Beside `value` the same JSON line carries, as extra fields that are not part of it:
the same launch with the buffers in plain allocation order (all sources, then all
targets, back to back), the staged path (pack + unpack through one staging chunk),
the fused-cast (derive) mode, the plan time, and the direct reshard of the other
benchmark configurations (GPT-2-small, 13B optimizer-state share, 70B rank share).

    python bench.py --refresh-traffic FETCH.csv WRITE.csv
rewrites profiles/traffic.json (the HBM traffic per launch that `roofline.traffic`
quotes) from the counter_collection CSVs of two `rocprofv3 --pmc` runs of
`python3 bench.py --steps 2 --warmup 1 --no-extras --no-cpu-baseline --calibrate-copy`.
"""
import argparse
import csv
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")
# what decides the kernel's HBM traffic: the kernels, the descriptor format and the lowering that feeds them
TRAFFIC_SOURCES = ["kernels.hip", "launch.hpp", "plan.hpp", "planner.cpp"]
OTHER_WORKLOADS = ("gpt2_small", "llama13b_dp", "llama70b_rank")


def kernel_source_hash():
    h = hashlib.sha256()
    for name in TRAFFIC_SOURCES:
        with open(os.path.join(ROOT, "paper_2605_22014_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload):
    """(GB per direct-reshard launch from the committed rocprofv3 --pmc summary, or None; why None)."""
    try:
        with open(TRAFFIC_JSON) as f:
            table = json.load(f)
    except OSError:
        return None, "profiles/traffic.json is missing"
    entry = table.get("workloads", {}).get(workload)
    if entry is None:
        return None, f"no counter run recorded for workload {workload}"
    if table.get("kernel_source_sha256_16") != kernel_source_hash():
        return None, "the kernel sources changed since the counter run (profiles/traffic.json is stale)"
    return entry["traffic_GB_per_launch"], None


def refresh_traffic(fetch_csv, write_csv, workload):
    """Rewrite profiles/traffic.json from two rocprofv3 --pmc counter_collection CSVs (FETCH_SIZE, WRITE_SIZE)."""
    def read(path, counter):
        copy, ours = [], []
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                if row["Counter_Name"] != counter:
                    continue
                if "copyBuffer" in row["Kernel_Name"]:
                    copy.append(float(row["Counter_Value"]))
                elif "liver_copy_kernel" in row["Kernel_Name"]:
                    ours.append(float(row["Counter_Value"]))
        assert copy and ours, f"{path}: need the 1 GiB reference copy and the reshard launches"
        return copy[-1], ours
    one_gib_kib = float(1 << 20)
    fetch_copy, fetch = read(fetch_csv, "FETCH_SIZE")
    write_copy, write = read(write_csv, "WRITE_SIZE")
    fs, ws = one_gib_kib / fetch_copy, one_gib_kib / write_copy      # what the counters under-report, from a copy of known size
    gb = (statistics.mean(fetch) * fs + statistics.mean(write) * ws) * 1024 / 1e9
    table = {"workloads": {}}
    if os.path.exists(TRAFFIC_JSON):
        with open(TRAFFIC_JSON) as f:
            table = json.load(f)
        if table.get("kernel_source_sha256_16") != kernel_source_hash():
            table = {"workloads": {}}                                 # other workloads' figures are stale too
    table["kernel_source_sha256_16"] = kernel_source_hash()
    table["kernel_sources"] = TRAFFIC_SOURCES
    table["workloads"][workload] = {
        "traffic_GB_per_launch": round(gb, 2), "fetch_scale": round(fs, 5), "write_scale": round(ws, 5),
        "FETCH_SIZE_KiB_per_launch": round(statistics.mean(fetch), 1), "WRITE_SIZE_KiB_per_launch": round(statistics.mean(write), 1),
        "launches": len(fetch), "reference": "plain 1 GiB device copy (__amd_rocclr_copyBuffer) in the same run"}
    with open(TRAFFIC_JSON, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")
    print(json.dumps(table["workloads"][workload]))


class Scrub:
    """Released device memory is scrubbed by the driver in the background (about 30 GB/s; a copy that runs
    meanwhile loses about 1 %).  The benchmark's own legs release up to 190 GB right before the next leg's
    buffers are timed, which no reconfiguration does (its target buffers are allocated during preparation, its
    old world is freed after the switch): every timed leg first waits until the scrubbing of what the benchmark
    itself released must be over.  The waiting is idle time, not warm-up."""
    until = 0.0
    waited = 0.0

    @classmethod
    def released(cls, nbytes):
        from paper_2605_22014_amd.placement import scrub_seconds
        cls.until = max(cls.until, time.perf_counter()) + scrub_seconds(nbytes)

    @classmethod
    def wait(cls):
        left = cls.until - time.perf_counter()
        if left > 0:
            time.sleep(left)
            cls.waited += left
        return max(left, 0.0)


class World:
    """Plan + source and target buffers of one workload, resident in HBM."""

    def __init__(self, lv, synth, torch, name, placement, launch=None):
        self.lv, self.torch, self.name = lv, torch, name
        cfg = self.cfg = synth.CONFIGS[name]
        only = cfg["only"] or {}
        self.spec = lv.ModelSpec(**cfg["spec"])
        self.src = src = lv.Layout(pad_multiple=cfg["pad_multiple"], **cfg["src"])
        self.dst_kw = dict(pad_multiple=cfg["pad_multiple"], kinds=tuple(cfg["kinds"]),
                           **{"only_" + k: v for k, v in only.items()}, **cfg["dst"])
        self.dst = dst = lv.Layout(**self.dst_kw)
        t0 = time.perf_counter()
        self.plan = plan = lv.liver_plan_create(self.spec, src, dst, cfg["chunk_bytes"])   # host planning + table upload
        self.plan_ms = (time.perf_counter() - t0) * 1e3
        self.info = lv.liver_plan_info(plan)
        if launch and (launch[0] or launch[1] >= 0 or launch[2] >= 0):
            lv.liver_plan_set_launch(plan, *launch)
        self.algo_bytes = self.info.bytes_read + self.info.bytes_written
        src_keys = [(r, k) for r in range(src.n_ranks) for k in range(4) if k in cfg["kinds"] and _column_used(lv, plan, src, r)]
        dst_keys = [(r, k) for r in range(dst.n_ranks) for k in range(4) if lv.liver_plan_buffer_used(plan, 1, r, k)]

        def view(t, side, k):
            return t if side == 1 else t.view(torch.bfloat16 if k == 0 else torch.float32)
        size = lambda side, key: lv.liver_plan_buffer_bytes(plan, side, *key)
        self.src_bufs, self.dst_bufs = {}, {}
        if placement == "natural":
            # what a training framework does: every source buffer, then every target buffer, back to back
            for side, keys, bufs in ((0, src_keys, self.src_bufs), (1, dst_keys, self.dst_bufs)):
                for key in keys:
                    bufs[key] = view(torch.empty(size(side, key), dtype=torch.uint8, device="cuda"), side, key[1])
            self.placement = "all source buffers, then all target buffers, in plain allocation order (no gaps)"
        elif placement == "targets_spread":
            # the source world as a training job holds it (plain order); the target buffers, which are allocated
            # when the reconfiguration is prepared, strided over the remaining free HBM by temporary spacer
            # allocations (released again before the first launch): paper_2605_22014_amd.placement
            from paper_2605_22014_amd.placement import alloc_spread, spacer_gap
            for key in src_keys:
                self.src_bufs[key] = view(torch.empty(size(0, key), dtype=torch.uint8, device="cuda"), 0, key[1])
            sizes = [size(1, key) for key in dst_keys]
            spacers = len(sizes) * spacer_gap(sizes)
            for key, t in zip(dst_keys, alloc_spread(sizes)):
                self.dst_bufs[key] = t
            Scrub.released(spacers)
            self.placement = ("source buffers in plain allocation order; target buffers strided over the remaining free HBM "
                              "by temporary spacer allocations (released before the timed region)")
        else:
            # source and target buffers allocated ALTERNATELY and strided over the whole free HBM by temporary
            # spacer allocations (released again before the first launch)
            order = []
            for i in range(max(len(src_keys), len(dst_keys))):
                order += [(0, src_keys[i])] if i < len(src_keys) else []
                order += [(1, dst_keys[i])] if i < len(dst_keys) else []
            from paper_2605_22014_amd.placement import alloc_spread, spacer_gap
            sizes = [size(side, key) for side, key in order]
            spacers = len(sizes) * spacer_gap(sizes)
            for (side, key), t in zip(order, alloc_spread(sizes)):
                (self.dst_bufs if side else self.src_bufs)[key] = view(t, side, key[1])
            Scrub.released(spacers)
            self.placement = ("source/target buffers allocated alternately, strided over the free HBM by temporary "
                              "spacer allocations (released before the timed region)")
        # synthetic state, generated in place: N(0, 0.02) fp32, PARAM = bf16(MASTER), all DP replicas identical
        columns = {}
        for pp in range(src.pp):
            for tp in range(src.tp):
                ranks = [src.rank(tp, pp, d) for d in range(src.dp)]
                if (ranks[0], lv.MASTER) not in self.src_bufs:
                    continue
                columns[(pp, tp)] = {"master": [self.src_bufs[(r, lv.MASTER)] for r in ranks],
                                     "m": [self.src_bufs[(r, lv.ADAM_M)] for r in ranks],
                                     "v": [self.src_bufs[(r, lv.ADAM_V)] for r in ranks],
                                     "param": self.src_bufs.get((ranks[0], lv.PARAM)) if 0 in cfg["kinds"] else None}
        synth.fill_device_world_into(columns, synth.SEED_BASE)
        if 0 in cfg["kinds"]:
            for (pp, tp), col in columns.items():
                for d in range(1, src.dp):
                    self.src_bufs[(src.rank(tp, pp, d), lv.PARAM)].copy_(col["param"])
        from paper_2605_22014_amd._binding import make_table
        self.src_tab = make_table(self.src_bufs, src.n_ranks, plan, 0)
        self.dst_tab = make_table(self.dst_bufs, dst.n_ranks, plan, 1)
        torch.cuda.synchronize()
        self.idle_before_timing_s = Scrub.wait()

    def reshard(self):
        self.lv.liver_reshard(self.plan, self.src_tab, self.dst_tab)

    def release(self):
        Scrub.released(sum(t.numel() * t.element_size() for bufs in (self.src_bufs, self.dst_bufs) for t in bufs.values()))
        self.lv.liver_plan_destroy(self.plan)
        self.src_bufs = self.dst_bufs = self.src_tab = self.dst_tab = None
        import gc
        gc.collect()
        self.torch.cuda.synchronize()
        self.torch.cuda.empty_cache()


def timed(torch, fn, steps, warmup):
    """(wall ms per step, [HIP-event ms of every step]) of fn() on the current stream, which is the stream the
    kernels are launched on."""
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
    return wall, [a.elapsed_time(b) for a, b in ev]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b")
    ap.add_argument("--grid", type=int, default=0)
    ap.add_argument("--tile-order", type=int, default=-1, help="-1 = library default")
    ap.add_argument("--cache-hints", type=int, default=-1, help="-1 = library default")
    ap.add_argument("--placement", default="targets_spread", choices=("targets_spread", "alternating", "natural"),
                    help="where the timed run's buffers sit")
    ap.add_argument("--no-natural-leg", action="store_true",
                    help="skip the leg that times the same reshard with the buffers in plain allocation order first")
    ap.add_argument("--no-extras", action="store_true", help="skip the staged / derive / plain-copy / other-workload legs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference dispatch for --pmc runs)")
    ap.add_argument("--refresh-traffic", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"))
    args = ap.parse_args()
    if args.refresh_traffic:
        refresh_traffic(args.refresh_traffic[0], args.refresh_traffic[1], args.workload)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all logical ranks' shards live in one MI355X's HBM); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import liver_synth as synth
    import paper_2605_22014_amd as lv

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    torch.zeros(1, device="cuda")        # HIP context and allocator are up before planning is timed
    torch.cuda.synchronize()
    launch = (args.grid, args.tile_order, args.cache_hints)
    extras = {}

    # ---- first thing in the process: the same reshard with the buffers where a plain allocation sequence puts
    # them.  Where the caller's buffers sit in HBM changes the bandwidth of any copy on this part (measured, see
    # profiles/placement.md), and the first large allocations of a process are the least favourable case.
    if not args.no_natural_leg and args.placement != "natural":
        w = World(lv, synth, torch, args.workload, "natural", launch)
        _, ev = timed(torch, w.reshard, max(5, args.steps // 2), args.warmup)
        extras["natural_placement_GBs"] = round(w.algo_bytes / (statistics.mean(ev) * 1e-3) / 1e9, 1)
        extras["natural_placement_ms"] = round(statistics.mean(ev), 4)
        extras["natural_placement"] = w.placement
        extras["natural_placement_memory_classes"] = memory_classes(lv, torch, w)
        w.release()
        del w

    world = World(lv, synth, torch, args.workload, args.placement, launch)
    cfg, plan, info, algo_bytes = world.cfg, world.plan, world.info, world.algo_bytes
    src_tab, dst_tab = world.src_tab, world.dst_tab

    # ---- the timed region: K direct reshards --------------------------------------------------------
    wall_ms, ev = timed(torch, world.reshard, args.steps, args.warmup)
    kern_ms, kern_med = statistics.mean(ev), statistics.median(ev)
    gbs = algo_bytes / (wall_ms * 1e-3) / 1e9
    kern_gbs = algo_bytes / (kern_ms * 1e-3) / 1e9
    traffic, why_not = measured_traffic(args.workload)

    out = {
        "metric": "reshard GB/s (read+write), 7B-shape TP8->TP4.PP2" if args.workload == "llama7b"
                  else f"reshard GB/s (read+write), {args.workload}",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": args.workload, "src": cfg["src"], "dst": cfg["dst"], "only": cfg["only"],
                   "kinds": list(cfg["kinds"]), "mode": "direct (liver_reshard)", "algorithmic_bytes": algo_bytes,
                   "n_desc": info.n_desc, "plan_ms": round(world.plan_ms, 2), "table_bytes_device": info.table_bytes_device,
                   "launch": {"grid": args.grid, "tile_order": args.tile_order, "cache_hints": args.cache_hints},
                   "placement": world.placement,
                   "idle_before_timing_s": round(world.idle_before_timing_s, 1),
                   "idle_reason": "memory the benchmark itself released just before (plain-order leg, spacers) is scrubbed "
                                  "by the driver in the background at about 30 GB/s; the timed region starts when that is over"},
        "pct_hbm_peak": round(100 * gbs / HBM_PEAK_GBS, 2),
        "roofline": {"bound": "hbm", "kernel": "liver_copy_kernel (direct reshard)", "achieved": round(kern_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(kern_gbs / HBM_PEAK_GBS, 4),
                     "avg_launch_ms": round(kern_ms, 4), "median_launch_ms": round(kern_med, 4),
                     "achieved_median": round(algo_bytes / (kern_med * 1e-3) / 1e9, 1),
                     "traffic": traffic},
    }
    if traffic is None:
        out["roofline"]["traffic_note"] = why_not
    else:
        out["roofline"]["traffic_unit"] = "GB per launch (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, scaled by a plain 1 GiB copy)"

    if not args.no_extras:
        src_bufs, dst_bufs = world.src_bufs, world.dst_bufs
        # plain device-to-device copy of one 1 GiB+ buffer: the empirical ceiling of this machine
        big = max(src_bufs.values(), key=lambda t: t.numel() * t.element_size())
        scratch = torch.empty_like(big)
        _, k = timed(torch, lambda: scratch.copy_(big), 10, 2)
        extras["torch_copy_GBs"] = round(2 * big.numel() * big.element_size() / (statistics.mean(k) * 1e-3) / 1e9, 1)
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
                _, k = timed(torch, probe, 3, 1)
                best = max(best, (2 if mode == 2 else 1) * probe_bytes / (statistics.mean(k) * 1e-3) / 1e9)
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
        w, _ = timed(torch, staged, 3, 1)
        extras["staged_end_to_end_GBs"] = round(algo_bytes / (w * 1e-3) / 1e9, 1)
        extras["staged_ms"] = round(w, 3)
        _, k = timed(torch, pack_only, 3, 1)
        extras["pack_kernel_GBs"] = round(2 * info.stream_bytes / (statistics.mean(k) * 1e-3) / 1e9, 1)
        _, k = timed(torch, unpack_only, 3, 1)
        extras["unpack_kernel_GBs"] = round((info.stream_bytes + info.bytes_written) / (statistics.mean(k) * 1e-3) / 1e9, 1)
        extras["n_chunks"] = nch
        # the same stream with unpack(k-1) and pack(k) fused into one launch (two staging chunks), and both forms
        # again through chunks a quarter of the size
        staging2 = torch.empty(cfg["chunk_bytes"], dtype=torch.uint8, device="cuda")
        w, _ = timed(torch, lambda: lv.liver_reshard_staged_fused(plan, src_tab, dst_tab, staging, staging2), 3, 1)
        extras["staged_fused_ms"] = round(w, 3)
        extras["staged_fused_end_to_end_GBs"] = round(algo_bytes / (w * 1e-3) / 1e9, 1)
        small = cfg["chunk_bytes"] // 4
        splan = lv.liver_plan_create(world.spec, world.src, world.dst, small)
        sn = lv.liver_plan_info(splan).n_chunks

        def staged_small():
            for c in range(sn):
                lv.liver_pack(splan, c, src_tab, staging[:small])
                lv.liver_unpack(splan, c, staging[:small], dst_tab)
        w, _ = timed(torch, staged_small, 3, 1)
        extras["staged_quarter_chunks_ms"] = round(w, 3)
        w, _ = timed(torch, lambda: lv.liver_reshard_staged_fused(splan, src_tab, dst_tab, staging[:small], staging2[:small]), 3, 1)
        extras["staged_quarter_chunks_fused_ms"] = round(w, 3)
        extras["staged_quarter_chunk_bytes"] = small
        lv.liver_plan_destroy(splan)
        del staging, staging2
        if 0 in cfg["kinds"] and 1 in cfg["kinds"]:
            dplan = lv.liver_plan_create(world.spec, world.src, lv.Layout(**dict(world.dst_kw, derive_bf16=True)), cfg["chunk_bytes"])
            dinfo = lv.liver_plan_info(dplan)
            _, k = timed(torch, lambda: lv.liver_reshard(dplan, src_tab, dst_tab), 5, 1)
            extras["derive_direct_GBs"] = round((dinfo.bytes_read + dinfo.bytes_written) / (statistics.mean(k) * 1e-3) / 1e9, 1)
            extras["derive_algorithmic_bytes"] = dinfo.bytes_read + dinfo.bytes_written
            lv.liver_plan_destroy(dplan)
        # the unpack-only timing loop scattered stale chunks and derive mode rewrote PARAM:
        # restore the copy-mode result before it is compared with the oracle
        world.reshard()
        torch.cuda.synchronize()

    if args.calibrate_copy:
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        b = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        a.fill_(1)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    if not args.no_cpu_baseline:
        one, many = cpu_baseline(cfg, world.src_bufs, world.dst_bufs, world.src, world.dst)
        out["cpu_baseline"] = one
        out["cpu_baseline_all_cores"] = many

    if not args.no_extras:
        extras["timed_placement_memory_classes"] = memory_classes(lv, torch, world)   # overwrites the world: last use
    if not args.no_extras and args.workload == "llama7b":
        # the other benchmark configurations, direct reshard, in both placements
        world.release()
        del world, src_tab, dst_tab, plan
        others = {}
        for name in OTHER_WORKLOADS:
            others[name] = {}
            for place in ("natural", "targets_spread"):
                w = World(lv, synth, torch, name, place)
                _, ev = timed(torch, w.reshard, 20, 3)
                ms = statistics.mean(ev)
                others[name].update({"algorithmic_bytes": w.algo_bytes, "n_desc": w.info.n_desc,
                                     f"{place}_GBs": round(w.algo_bytes / (ms * 1e-3) / 1e9, 1), f"{place}_ms": round(ms, 4),
                                     f"{place}_frac_hbm_peak": round(w.algo_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})
                w.release()
                del w
        extras["other_workloads_placements"] = {"natural": "plain allocation order",
                                                "targets_spread": "sources in plain order, targets strided over the free HBM"}
        extras["other_workloads_direct"] = others
    out["paper_context"] = ("context only, other hardware and a different quantity: on 32 A800 80 GB PCIe GPUs (PCIe Gen4 + 200 Gb/s "
                            "InfiniBand) the paper's reconfiguration is 14-23x faster than checkpoint/restart (minutes -> 2-6 s of "
                            "downtime); its transfer-and-combine phase moves ~28 GB in ~2 s for a 14B model, network included")
    if extras:
        out["extras"] = extras

    print(json.dumps(out))


def memory_classes(lv, torch, world, window=1 << 30):
    """Which buffers of a world share a class of the device memory, found by timing: two windows filled in ONE
    launch reach about 7.1 TB/s if they sit in different classes and about 5.7 TB/s if they share one (a write
    stream confined to one class is capped there; profiles/placement.md).  The first `window` bytes of every
    buffer are probed against one representative per class found so far.  OVERWRITES those bytes: call it on a
    world whose contents are no longer needed."""
    def rate(a, b):
        best = 0.0
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            lv.liver_debug_bandwidth_probe(3, a, b, window, 8192)
            e1.record()
            torch.cuda.synchronize()
            best = max(best, 2 * window / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        return best
    refs, out, rates = [], {}, {"same": [], "other": []}
    for side, bufs in (("source", world.src_bufs), ("target", world.dst_bufs)):
        letters = ""
        for key, t in bufs.items():
            if t.numel() * t.element_size() < window:
                letters += "-"
                continue
            found = None
            for ci, ref in enumerate(refs):
                if ref.data_ptr() == t.data_ptr():
                    found = ci
                    break
                g = rate(t, ref)
                same = g < 6400.0
                rates["same" if same else "other"].append(g)
                if same:
                    found = ci
                    break
            if found is None:
                refs.append(t)
                found = len(refs) - 1
            letters += "ABCDEFGH"[min(found, 7)]
        out[side] = letters
    out["how"] = (f"first {window >> 20} MiB of every buffer filled together with a representative of each class, in "
                  f"allocation order; same class: {min(rates['same'], default=0):.0f}-{max(rates['same'], default=0):.0f} GB/s, "
                  f"different: {min(rates['other'], default=0):.0f}-{max(rates['other'], default=0):.0f} GB/s")
    return out


def _column_used(lv, plan, src, rank):
    """Does the plan read any buffer of the (tp, pp) rank column that `rank` belongs to?"""
    tp, pp = rank % src.tp, rank // (src.tp * src.dp)
    return any(lv.liver_plan_buffer_used(plan, 0, src.rank(tp, pp, d), k) for d in range(src.dp) for k in range(4))


def cpu_baseline(cfg, src_bufs, dst_bufs, src, dst, n_layers_sampled=12):
    """The CPU oracle (gather to full logical tensors, re-split) timed on a bounded
    sample of the same workload: all tensors of a few transformer layers spread
    over the model (of the planned target stage for a filtered plan), all buffer
    kinds, inputs already in host memory.  Timed twice on the same sample: one
    layer after the other on one thread, and the (layer, kind) units on a pool of
    as many threads as the process may use (the oracle itself is unchanged: the
    units are independent, and NumPy's slice copies run without the interpreter
    lock).  The single-thread output also checks the GPU result for those layers."""
    import numpy as np
    import torch
    import oracle
    from concurrent.futures import ThreadPoolExecutor
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

    def download(layer):
        """Host copies of the source ranges that hold this layer, and a reader over them."""
        pp_src = layer // (ospec.n_layers // osrc.pp)
        host = {}
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
        return read

    def unit(layer, k, read):
        names = [t for t in oracle.logical_tensors(ospec) if t.startswith(f"L{layer}.")]
        logical = oracle.gather_logical(ospec, osrc, k, read, names=names)
        return [(k,) + e for e in oracle.expected_shards(ospec, odst, logical, tps, pps)]

    readers = {layer: download(layer) for layer in layers}
    # ---- one thread, layer after layer; the result is compared with the GPU's
    secs, nbytes = 0.0, 0
    for layer in layers:
        t0 = time.perf_counter()
        expected = []
        for k in cfg["kinds"]:
            expected += unit(layer, k, readers[layer])
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
        del expected
    sample = (f"all tensors of layers {layers}, kinds {list(cfg['kinds'])}: {nbytes / 1e9:.2f} GB of target state "
              f"gathered and re-split")
    cores = len(os.sched_getaffinity(0))
    one = {"value": round(2 * nbytes / secs / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
           "sample": f"{sample} in {secs:.2f} s on one thread; GPU result equal on this sample",
           "host_cores_available": cores}
    # ---- the same units on all cores the process may use
    units = [(layer, k) for layer in layers for k in cfg["kinds"]]
    workers = max(1, min(cores, len(units)))
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=workers) as pool:
        for fut in [pool.submit(lambda u=u: len(unit(u[0], u[1], readers[u[0]]))) for u in units]:
            fut.result()
    secs_all = time.perf_counter() - t0
    many = {"value": round(2 * nbytes / secs_all / 1e9, 3), "unit": "GB/s", "cores": workers, "kind": "oracle",
            "sample": f"{sample} in {secs_all:.2f} s as {len(units)} independent (layer, kind) units on a pool of "
                      f"{workers} threads", "host_cores_available": cores}
    return one, many


if __name__ == "__main__":
    main()

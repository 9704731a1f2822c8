"""liver_reshard_static: the staged reshard through the staging array the library itself holds, for callers
that cannot allocate device memory.  Its target bytes must equal those of the existing staged entry point
(liver_pack + liver_unpack through a caller's chunk) and the oracle's, on two calls in a row that share the
array, the second with a smaller input."""
import numpy as np
import pytest
import torch

import liver_synth as synth
import oracle
import paper_2605_22014_amd as lv
from interp import lv_objects
from util import cfg_objects, make_world
from gpu_util import to_dev, run_staged, check_against, alloc_dst

pytestmark = pytest.mark.gpu


def _world(name, chunk_bytes, seed):
    cfg, spec, src, dst = cfg_objects(name)
    state = synth.logical_state(oracle.logical_tensors(spec), seed, cfg["dist"])
    world = make_world(spec, src, state)
    want = oracle.reshard_state(spec, src, dst, world)
    s, a, b = lv_objects(spec, src, dst)
    return lv.liver_plan_create(s, a, b, chunk_bytes), to_dev(world), want


def _same_bits(a, b, what):
    assert a.keys() == b.keys()
    for key in a:
        assert torch.equal(a[key], b[key]), (what, key)


def test_static_staging_matches_the_callers_chunk_twice_in_a_row():
    cap = lv.liver_static_staging_bytes()
    assert cap == 64 << 20
    print("static staging: gpt2_small through 64 MiB chunks", flush=True)
    big_plan, big_dev, big_want = _world("gpt2_small", cap, synth.SEED_BASE)       # 31 chunks fill the whole array
    assert lv.liver_plan_info(big_plan).n_chunks == 31
    free0, _ = torch.cuda.mem_get_info()
    out_big = alloc_dst(big_plan)
    lv.liver_reshard_static(big_plan, big_dev, out_big)
    torch.cuda.synchronize()
    check_against(out_big, big_want, big_plan, "static staging, first call")
    _same_bits(out_big, run_staged(big_plan, big_dev), "first call vs liver_pack + liver_unpack")

    print("static staging: tiny_gpt through 1 MiB chunks, same array", flush=True)
    small_plan, small_dev, small_want = _world("tiny_gpt", 1 << 20, synth.SEED_BASE + 1)
    out_small = alloc_dst(small_plan)
    lv.liver_reshard_static(small_plan, small_dev, out_small)
    torch.cuda.synchronize()
    check_against(out_small, small_want, small_plan, "static staging, second (smaller) call")
    _same_bits(out_small, run_staged(small_plan, small_dev), "second call vs liver_pack + liver_unpack")

    print("static staging: first plan again, on a side stream", flush=True)
    side = torch.cuda.Stream()
    out_again = alloc_dst(big_plan)
    torch.cuda.synchronize()
    lv.liver_reshard_static(big_plan, big_dev, out_again, stream=side)
    side.synchronize()
    _same_bits(out_again, out_big, "third call")


def test_static_staging_refuses_a_larger_chunk_and_bad_tables_before_any_launch():
    cfg, spec, src, dst = cfg_objects("tiny_gpt")
    print("static staging: refusals", flush=True)
    s, a, b = lv_objects(spec, src, dst)
    too_big = lv.liver_plan_create(s, a, b, lv.liver_static_staging_bytes() + 256)
    world = make_world(spec, src, synth.logical_state(oracle.logical_tensors(spec), 3, cfg["dist"]))
    dev = to_dev(world)
    out = alloc_dst(too_big)
    keep = {k: t.clone() for k, t in out.items()}
    with pytest.raises(lv.LiverError, match="exceeds the library's static staging array") as e:
        lv.liver_reshard_static(too_big, dev, out)
    assert e.value.code == -1
    plan = lv.liver_plan_create(s, a, b, 1 << 20)
    missing = dict(dev)
    last = max(k for k in missing if k[1] == lv.ADAM_V)
    missing[last] = None                                  # a buffer that only the LAST chunks read
    with pytest.raises(lv.LiverError, match="NULL"):
        lv.liver_reshard_static(plan, missing, out)
    torch.cuda.synchronize()
    for k in keep:                                        # nothing was enqueued by either refused call
        assert torch.equal(keep[k], out[k]), k
    lv.liver_reshard_static(plan, dev, out)
    torch.cuda.synchronize()
    check_against(out, oracle.reshard_state(spec, src, dst, world), plan, "after the refusals")


def test_static_staging_under_hip_graph_capture():
    """What the entry point is for: a caller under HIP-graph capture may not allocate.  The whole staged reshard
    through the library's array is captured once and replayed three times, with eager work in between."""
    print("static staging: graph capture", flush=True)
    plan, dev, want = _world("tiny_gpt", 1 << 20, synth.SEED_BASE + 2)
    out = alloc_dst(plan)
    from paper_2605_22014_amd._binding import make_table
    st, dt = make_table(dev, plan.src.n_ranks), make_table(out, plan.dst.n_ranks)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lv.liver_reshard_static(plan, st, dt)
    for replay in range(3):
        for t in out.values():
            t.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        check_against(out, want, plan, f"static staging, graph replay {replay}")

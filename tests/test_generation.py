"""The generation state machine around a reshard (LiveR, Section 4.5.1): transitions, monotonic ids,
cancel, fallback on failure, queued requests.  The state machine is tested on the CPU with a recording
executor; one GPU test runs it with the real liver_reshard."""
import numpy as np
import pytest

import liver_synth as synth
import oracle
import paper_2605_22014_amd as lv
from paper_2605_22014_amd.generation import GenerationError, GenerationManager, State
from util import cfg_objects


def _mgr(executor):
    cfg = synth.CONFIGS["tiny_gpt"]
    spec = lv.ModelSpec(**cfg["spec"])
    src = lv.Layout(pad_multiple=128, **cfg["src"])
    return GenerationManager(spec, src, {"world": 0}, cfg["chunk_bytes"], executor=executor), lv.Layout(pad_multiple=128, **cfg["dst"])


def test_life_cycle_and_monotonic_ids():
    calls = []
    m, target = _mgr(lambda plan, s, d, stream: calls.append((s, d)))
    assert (m.state, m.generation) == (State.STABLE, 0)
    plan = m.request(target)
    assert m.state is State.PREPARE and lv.liver_plan_info(plan).n_chunks == 35      # planning is metadata only
    with pytest.raises(GenerationError):
        m.switch()                                      # the shadow world has no storage yet
    m.shadow_ready({"world": 1})
    assert m.state is State.READY
    assert m.switch() == 1
    assert calls == [({"world": 0}, {"world": 1})]
    assert (m.state, m.generation, m.active_bufs, m.active_layout) == (State.STABLE, 1, {"world": 1}, target)
    back = lv.Layout(pad_multiple=128, **synth.CONFIGS["tiny_gpt"]["src"])
    m.request(back)
    m.shadow_ready({"world": 2})
    assert m.switch() == 2 and m.active_bufs == {"world": 2}


def test_cancel_leaves_the_active_world():
    m, target = _mgr(lambda *a: pytest.fail("a cancelled handoff must not transfer"))
    m.request(target)
    m.cancel()
    assert (m.state, m.generation, m.active_bufs) == (State.STABLE, 0, {"world": 0})
    m.request(target)
    m.shadow_ready({"world": 1})
    m.cancel()
    assert (m.state, m.generation, m.active_bufs) == (State.STABLE, 0, {"world": 0})
    with pytest.raises(GenerationError):
        m.cancel()


def test_failure_during_transfer_falls_back():
    def boom(*a):
        raise RuntimeError("link down")
    m, target = _mgr(boom)
    m.request(target)
    m.shadow_ready({"world": 1})
    with pytest.raises(RuntimeError):
        m.switch()
    assert (m.state, m.generation, m.active_bufs) == (State.STABLE, 0, {"world": 0})     # generation k intact


def test_requests_during_a_handoff_are_queued():
    m, target = _mgr(lambda *a: None)
    m.request(target)
    other = lv.Layout(1, 1, 2, 128)
    newest = lv.Layout(2, 2, 1, 128)
    assert m.request(other) is None and m.request(newest) is None      # queued, not planned
    m.shadow_ready({"world": 1})
    m.switch()
    assert m.generation == 1 and m.state is State.PREPARE              # the newest queued request is being prepared,
    m.shadow_ready({"world": 2})                                       # the stale one was dropped
    m.switch()
    assert m.generation == 2 and m.active_layout == newest and m.state is State.STABLE


@pytest.mark.gpu
def test_generation_switch_on_device():
    import torch
    from gpu_util import to_dev, alloc_dst, to_host
    from util import make_world
    cfg, ospec, osrc, odst = cfg_objects("tiny_gpt")
    world = make_world(ospec, osrc, synth.logical_state(oracle.logical_tensors(ospec), 12, "uniform"))
    want = oracle.reshard_state(ospec, osrc, odst, world)
    spec = lv.ModelSpec(**cfg["spec"])
    src = lv.Layout(pad_multiple=128, **cfg["src"])
    dst = lv.Layout(pad_multiple=128, **cfg["dst"])
    dev = to_dev(world)
    keep = {k: t.clone() for k, t in dev.items()}
    m = GenerationManager(spec, src, dev, cfg["chunk_bytes"])
    plan = m.request(dst)
    m.shadow_ready(alloc_dst(plan))
    assert m.switch() == 1
    got = to_host(m.active_bufs)
    for key in want:
        assert np.array_equal(got[key], want[key]), key
    for k in keep:
        assert torch.equal(keep[k], dev[k])             # generation 0's buffers were never written

"""Randomised parity on the GPU: random models whose dimensions are multiples of 8 (so that the 16-byte
vector paths, the fused copy + cast and the zero fills are exercised under random geometry) and random
world pairs mixing every layout feature; direct and staged, copy and derive, bit for bit against the oracle.

A random plan never reaches the device unchecked: the library's bounds-checked host emulator first runs the
very tables the kernels would run (direct list, every pack and unpack chunk) on host copies of the buffers; an
offset outside a buffer, or a result that differs from the oracle's, fails the case before any kernel launch."""
import numpy as np
import pytest
import torch
from hypothesis import HealthCheck, given, seed, settings, strategies as st

import oracle
import paper_2605_22014_amd as lv
from interp import lv_objects, emulate_direct, emulate_staged, used_dst
from util import make_world, tiny_state, corrupt_replicas
from gpu_util import to_dev, run_direct, run_staged, run_fused, check_against
from test_planner_fuzz import layouts

pytestmark = pytest.mark.gpu


@st.composite
def aligned_specs(draw):
    nkv = draw(st.sampled_from([1, 2, 4]))
    qpg = draw(st.sampled_from([1, 2, 4]))
    hd = draw(st.sampled_from([8, 16]))
    nq = nkv * qpg
    moe = draw(st.booleans())
    return oracle.ModelSpec(n_layers=draw(st.sampled_from([2, 4, 6])), hidden=nq * hd, n_q_heads=nq, n_kv_heads=nkv,
                            ffn=draw(st.sampled_from([64, 96, 192])), vocab=draw(st.sampled_from([64, 104, 250])),
                            max_pos=draw(st.sampled_from([0, 8])), glu=draw(st.booleans()), norm_bias=draw(st.booleans()),
                            linear_bias=draw(st.booleans()), tied_embed=draw(st.booleans()),
                            n_experts=draw(st.sampled_from([2, 4])) if moe else 0)


@st.composite
def cases(draw):
    spec = draw(aligned_specs())
    src, dst = draw(layouts(spec)), draw(layouts(spec))
    kw = {}
    if draw(st.integers(0, 2)) == 0:
        which = draw(st.sampled_from(["tp", "pp", "dp"]))
        kw["only_" + which] = draw(st.integers(0, getattr(dst, which) - 1))
    return spec, src, dst, draw(st.booleans()), kw, draw(st.sampled_from([1024, 4096, 1 << 16])), draw(st.integers(0, 10 ** 6))


def proven_on_host(plan, world, want):
    """The plan's lowered tables stay inside the buffers and give the oracle's bits, shown on host memory by the
    bounds-checked emulator (LiverError with LIVER_E_HIP on any access out of bounds)."""
    for what, got in (("direct", emulate_direct(plan, world)), ("staged", emulate_staged(plan, world))):
        for key in used_dst(plan):
            assert np.array_equal(got[key].view(want[key].dtype), want[key]), ("host emulation", what, key)


@seed(22014)
@settings(max_examples=40, deadline=None, suppress_health_check=list(HealthCheck), derandomize=True, database=None)
@given(cases())
def test_random_worlds_on_device(case):
    spec, src, dst, derive, kw, chunk, rng_seed = case
    print(f"fuzz {spec} {src} -> {dst} derive={derive} {kw} chunk={chunk}", flush=True)
    world = make_world(spec, src, tiny_state(spec, seed=rng_seed))
    if rng_seed % 2:
        corrupt_replicas(spec, src, world)
    want = oracle.reshard_state(spec, src, dst, world, derive_bf16=derive)
    s, a, b = lv_objects(spec, src, dst, derive_bf16=derive, **kw)
    plan = lv.liver_plan_create(s, a, b, chunk)
    proven_on_host(plan, world, want)             # raises before anything is launched
    dev = to_dev(world)
    check_against(run_direct(plan, dev), want, plan, "direct")
    check_against(run_staged(plan, dev), want, plan, "staged")
    check_against(run_fused(plan, dev), want, plan, "staged, fused launches")
    lv.liver_plan_destroy(plan)

"""Randomised cross-check of the planner against the oracle on the CPU: random tiny models and random pairs
of worlds that mix every layout feature (GQA / replicated kv heads, gated FFN, biases, tied embeddings, MoE
with expert parallelism, interleaved or uneven stages, padded vocabularies, buckets), random plan
restrictions, copy and derive mode.  Both the public descriptors (NumPy interpreter) and the lowered tables
(bounds-checked host emulator) must reproduce the oracle bit for bit."""
import numpy as np
import pytest
from hypothesis import HealthCheck, given, seed, settings, strategies as st

import oracle
import paper_2605_22014_amd as lv
from interp import lv_objects, run_direct, run_staged, emulate_direct, emulate_staged, used_dst
from util import make_world, tiny_state, corrupt_replicas


@st.composite
def specs(draw):
    nkv = draw(st.sampled_from([1, 2, 4]))
    qpg = draw(st.sampled_from([1, 2, 4]))
    hd = draw(st.sampled_from([2, 4]))
    nq = nkv * qpg
    layers = draw(st.sampled_from([2, 4, 6]))
    moe = draw(st.booleans())
    return oracle.ModelSpec(n_layers=layers, hidden=nq * hd, n_q_heads=nq, n_kv_heads=nkv,
                            ffn=draw(st.sampled_from([8, 12, 24])), vocab=draw(st.sampled_from([16, 23, 40])),
                            max_pos=draw(st.sampled_from([0, 3])), glu=draw(st.booleans()), norm_bias=draw(st.booleans()),
                            linear_bias=draw(st.booleans()), tied_embed=draw(st.booleans()),
                            n_experts=draw(st.sampled_from([2, 4])) if moe else 0)


@st.composite
def layouts(draw, spec):
    for _ in range(60):
        tp = draw(st.sampled_from([1, 2, 4, 8]))
        pp = draw(st.sampled_from([1, 2, 3]))
        dp = draw(st.sampled_from([1, 2, 3, 4]))
        style = draw(st.sampled_from(["even", "vpp", "uneven"]))
        lay = oracle.Layout(
            tp, pp, dp, pad_multiple=draw(st.sampled_from([1, 4, 8])),
            vpp=draw(st.sampled_from([2, 3])) if style == "vpp" else 1,
            vocab_multiple=draw(st.sampled_from([0, 0, 4, 8])) if spec.vocab % tp == 0 else draw(st.sampled_from([4, 8])),
            pp_first=draw(st.integers(1, 3)) if style == "uneven" else 0,
            pp_last=draw(st.integers(0, 2)) if style == "uneven" else 0,
            bucket_elems=draw(st.sampled_from([0, 0, 1, 200, 900])),
            ep=draw(st.sampled_from([1, 2, 4])) if spec.n_experts else 1)
        try:
            oracle.check_supported(spec, lay)
            return lay
        except ValueError:
            continue
    return oracle.Layout(1, 1, 1, 1)


@st.composite
def cases(draw):
    spec = draw(specs())
    src, dst = draw(layouts(spec)), draw(layouts(spec))
    kw = {}
    if draw(st.booleans()):
        which = draw(st.sampled_from(["tp", "pp", "dp"]))
        kw["only_" + which] = draw(st.integers(0, getattr(dst, which) - 1))
    if draw(st.integers(0, 3)) == 0:
        kw["kinds"] = tuple(sorted(draw(st.sets(st.integers(0, 3), min_size=1, max_size=3))))
    return spec, src, dst, draw(st.booleans()), kw, draw(st.sampled_from([256, 512, 4096])), draw(st.integers(0, 10 ** 6))


@seed(22014)
@settings(max_examples=60, deadline=None, suppress_health_check=list(HealthCheck), derandomize=True)
@given(cases())
def test_random_worlds(case):
    spec, src, dst, derive, kw, chunk, rng_seed = case
    world = make_world(spec, src, tiny_state(spec, seed=rng_seed))
    if rng_seed % 2:
        corrupt_replicas(spec, src, world)
    want = oracle.reshard_state(spec, src, dst, world, derive_bf16=derive)
    s, a, b = lv_objects(spec, src, dst, derive_bf16=derive, **kw)
    plan = lv.liver_plan_create(s, a, b, chunk)
    used = used_dst(plan)
    for got, counts in (run_direct(plan, world), run_staged(plan, world), (emulate_direct(plan, world), None),
                        (emulate_staged(plan, world), None)):
        for key in got:
            if key in used:
                assert counts is None or (counts[key] == 1).all(), ("not exactly once", key, spec, src, dst, kw)
                assert np.array_equal(got[key], want[key]), (key, spec, src, dst, derive, kw)
            elif counts is not None:
                assert not counts[key].any(), ("unplanned buffer written", key)
    lv.liver_plan_destroy(plan)

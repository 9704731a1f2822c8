"""Pins oracle.reshard_state: brute force on tiny models, the paper's degenerate
cases and worked example, and the algebraic invariants of a reshard."""
import os

import numpy as np
import pytest

import liver_synth as synth
import oracle
import ownership as own
from util import (cfg_objects, make_world, assert_same, brute_reshard, tiny_state, poison_pads,
                  corrupt_replicas)

ODD = oracle.ModelSpec(n_layers=2, hidden=24, n_q_heads=6, n_kv_heads=2, ffn=42, vocab=48, max_pos=5,
                       glu=True, norm_bias=True, linear_bias=True, tied_embed=True)
ODD3 = oracle.ModelSpec(n_layers=2, hidden=24, n_q_heads=6, n_kv_heads=3, ffn=42, vocab=48,
                        glu=False, tied_embed=False)
ODD6 = oracle.ModelSpec(n_layers=6, hidden=24, n_q_heads=6, n_kv_heads=6, ffn=42, vocab=48, glu=True)

REP = oracle.ModelSpec(n_layers=2, hidden=32, n_q_heads=8, n_kv_heads=2, ffn=24, vocab=16, glu=True,
                       linear_bias=True)         # TP 4 / 8 > n_kv = 2: kv heads replicated on 2 / 4 ranks

VOC = oracle.ModelSpec(n_layers=2, hidden=16, n_q_heads=4, n_kv_heads=4, ffn=16, vocab=50, max_pos=3,
                       tied_embed=True)          # 50 rows never divide evenly: padded per world
VOCH = oracle.ModelSpec(n_layers=2, hidden=16, n_q_heads=4, n_kv_heads=2, ffn=16, vocab=37, glu=True)

MOE = oracle.ModelSpec(n_layers=2, hidden=16, n_q_heads=4, n_kv_heads=2, ffn=12, vocab=16, glu=True,
                       linear_bias=True, n_experts=4)        # router in the dense buffers, experts in kinds 4..7

BRUTE = [
    (ODD, (2, 1, 2, 4), (1, 2, 3, 1)),
    (ODD, (1, 2, 3, 1), (2, 2, 1, 4)),
    (ODD, (2, 2, 3, 1), (2, 1, 2, 1)),
    (ODD3, (3, 1, 2, 1), (1, 2, 3, 4)),
    (ODD3, (1, 1, 1, 1), (3, 2, 2, 1)),
    (ODD6, (6, 1, 1, 4), (2, 3, 2, 1)),
    (ODD6, (3, 2, 3, 1), (6, 6, 1, 1)),
    (ODD6, (2, 3, 2, 1), (1, 1, 3, 4)),
    (ODD6, (2, 3, 2, 1, 2), (3, 1, 1, 4, 3)),        # interleaved stages: vpp 2 -> vpp 3
    (ODD6, (1, 2, 1, 4), (2, 3, 2, 1, 2)),           # plain split -> interleaved
    (REP, (2, 1, 2, 1), (8, 2, 1, 4)),               # kv heads split -> replicated 4x
    (REP, (8, 1, 1, 1), (4, 1, 3, 1)),               # replicated 4x -> replicated 2x (replicas corrupted)
    (REP, (4, 2, 2, 4), (1, 1, 2, 1)),               # replicated 2x -> one rank
    (VOC, (2, 1, 2, 4, 1, 8), (4, 2, 1, 1, 1, 4)),   # padded vocabulary 64 -> 64 rows, other split (6th = vocab_multiple)
    (VOC, (1, 2, 1, 1, 1, 0), (4, 1, 3, 4, 1, 16)),  # unpadded 50 -> padded 64, tied copy dropped (corrupted pads)
    (VOCH, (2, 1, 3, 1, 1, 5), (1, 2, 2, 128, 1, 3)),   # 40 -> 39 rows, untied head
    (VOCH, (1, 1, 1, 1, 1, 64), (4, 2, 1, 1, 1, 16)),   # tp 3 holds rows 48..63: all padding (and kv heads replicated)
    (ODD6, (2, 3, 1, 4), (1, 3, 2, 1, 1, 0, 1, 3)),     # even stages -> 1 / 2 / 3 layers (7th, 8th = pp_first, pp_last)
    (ODD6, (3, 2, 2, 1, 1, 0, 5, 0), (2, 4, 1, 4, 1, 0, 0, 3)),   # 5 / 1 -> 1 / 1 / 1 / 3
    (ODD, (2, 1, 2, 4, 1, 0, 0, 0, 700), (1, 2, 3, 4, 1, 0, 0, 0, 0)),        # bucketed (9th = bucket_elems) -> one bucket
    (ODD, (1, 2, 3, 1), (2, 2, 2, 4, 1, 0, 0, 0, 500)),                       # one bucket -> bucketed, padding inside
    (ODD6, (3, 2, 3, 4, 1, 0, 0, 0, 900), (2, 3, 2, 8, 1, 0, 0, 0, 400)),     # buckets on both sides, different cuts
    (VOC, (2, 1, 2, 4, 1, 8, 0, 0, 300), (1, 2, 3, 4, 1, 4, 0, 0, 1)),        # with vocabulary padding; one bucket per parameter
    (MOE, (2, 1, 4, 4, 1, 0, 0, 0, 0, 2), (1, 2, 2, 1, 1, 0, 0, 0, 0, 1)),    # EP 2 -> EP 1 (10th = ep): experts gathered
    (MOE, (1, 1, 2, 1, 1, 0, 0, 0, 0, 1), (2, 2, 4, 4, 1, 0, 0, 0, 0, 4)),    # EP 1 -> EP 4: one expert per DP rank
    (MOE, (2, 2, 4, 1, 1, 0, 0, 0, 500, 4), (2, 1, 6, 4, 1, 0, 0, 0, 300, 2)),  # EP 4 -> EP 2 with buckets, DP 4 -> 6 (replicas corrupted)
]


@pytest.mark.parametrize("derive", [False, True])
@pytest.mark.parametrize("case", range(len(BRUTE)))
def test_brute_force_tiny(case, derive):
    spec, s, d = BRUTE[case]
    src, dst = oracle.Layout(*s), oracle.Layout(*d)
    world = make_world(spec, src, tiny_state(spec, seed=case))
    if case % 2:
        corrupt_replicas(spec, src, world)      # the copies that must not be read differ
    got = oracle.reshard_state(spec, src, dst, world, derive_bf16=derive)
    assert len(got) == dst.n_ranks * len(oracle.kinds_of(spec))
    want = brute_reshard(spec, src, dst, world, derive=derive)
    assert_same(got, want, f"case {case}")


def _golden_tasks():
    path = os.path.join(os.path.dirname(__file__), "golden", "tp4_to_tp8_tasks.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    return [(int(a), int(b), int(c), int(d), e) for a, b, c, d, e in rows]


def test_paper_example_tp4_to_tp8():
    """Section 4.6.1: TP4 -> TP8 on a weight split along its columns (here the
    row-parallel o.w and down.w, N columns): target 2s and 2s+1 get the first
    and second half of source s's columns."""
    spec = oracle.ModelSpec(n_layers=1, hidden=64, n_q_heads=8, n_kv_heads=8, ffn=128, vocab=64)
    src, dst = oracle.Layout(4, 1, 1, 1), oracle.Layout(8, 1, 1, 1)
    state = synth.logical_state(oracle.logical_tensors(spec), 5, "uniform")
    world = make_world(spec, src, state)
    out = oracle.reshard_state(spec, src, dst, world)

    def shard(lay, bufs, tp, pname):
        sv = oracle.stage_view(spec, lay, tp, 0)
        prm = next(p for p in sv.params if p.name == pname)
        return bufs[(lay.rank(tp, 0, 0), oracle.MASTER)][prm.offset:prm.offset + prm.size].reshape(prm.shape)

    tasks = _golden_tasks()
    assert len(tasks) == 8 and sorted(t[1] for t in tasks) == list(range(8))
    for pname, logical in (("L0.o.w", "L0.o.w"), ("L0.fc2.w", "L0.down.w")):
        N = state[oracle.MASTER][logical].shape[1]
        moved = 0
        for s, d, c0, nc, half in tasks:
            a = shard(src, world, s, pname)
            b = shard(dst, out, d, pname)
            w = N // 8
            assert b.shape[1] == nc * w and a.shape[1] == 2 * w
            lo = 0 if half == "first" else w
            assert np.array_equal(b, a[:, lo:lo + w])
            assert np.array_equal(b, state[oracle.MASTER][logical][:, c0 * w:(c0 + nc) * w])
            moved += b.size
        assert moved == state[oracle.MASTER][logical].size        # no redundant movement


def test_pp_only_moves_whole_parameters():
    """Section 4.6.1 / A.2.3: under a PP-only change a layer's parameter moves as a
    whole: every target shard equals one complete source shard."""
    _, spec, _, _ = cfg_objects("tiny_gpt")
    src, dst = oracle.Layout(2, 1, 1, 128), oracle.Layout(2, 2, 1, 128)
    world = make_world(spec, src, synth.logical_state(oracle.logical_tensors(spec), 9, "uniform"))
    out = oracle.reshard_state(spec, src, dst, world)
    for tp in range(2):
        src_params = {p.name: p for p in oracle.stage_view(spec, src, tp, 0).params}
        for pp in range(2):
            for prm in oracle.stage_view(spec, dst, tp, pp).params:
                sp = src_params[prm.name.replace("(tied copy)", "")]
                assert sp.shape == prm.shape
                for k in oracle.KINDS:
                    a = world[(src.rank(tp, 0, 0), k)][sp.offset:sp.offset + sp.size]
                    b = out[(dst.rank(tp, pp, 0), k)][prm.offset:prm.offset + prm.size]
                    assert np.array_equal(a, b), (prm.name, k)


@pytest.mark.parametrize("dp_src,dp_dst", [(1, 3), (4, 2)])
def test_dp_only_replicated_params(dp_src, dp_dst):
    """Section 4.6.1: more replicas = broadcast of the full shard, fewer = surplus
    copies dropped.  (pad_multiple=1 and sizes dividing evenly keep N_pad equal.)"""
    spec = oracle.ModelSpec(n_layers=2, hidden=48, n_q_heads=4, n_kv_heads=4, ffn=96, vocab=96)
    src, dst = oracle.Layout(2, 1, dp_src, 12), oracle.Layout(2, 1, dp_dst, 12)
    world = make_world(spec, src, synth.logical_state(oracle.logical_tensors(spec), 2, "normal"), poison=False)
    out = oracle.reshard_state(spec, src, dst, world)
    for tp in range(2):
        nl = own.n_local(spec, src, 0)
        ref = world[(src.rank(tp, 0, 0), oracle.PARAM)][:nl]
        for dp in range(dp_dst):
            assert np.array_equal(out[(dst.rank(tp, 0, dp), oracle.PARAM)][:nl], ref)
        for k in (oracle.MASTER, oracle.ADAM_M, oracle.ADAM_V):
            a = np.concatenate([world[(src.rank(tp, 0, d), k)] for d in range(dp_src)])[:nl]
            b = np.concatenate([out[(dst.rank(tp, 0, d), k)] for d in range(dp_dst)])[:nl]
            assert np.array_equal(a, b)


WORLDS = [(2, 1, 2, 128), (1, 2, 2, 128), (4, 2, 1, 128), (2, 2, 3, 64), (1, 1, 1, 128)]


@pytest.fixture(scope="module")
def tiny_world():
    _, spec, _, _ = cfg_objects("tiny_gpt")
    state = synth.logical_state(oracle.logical_tensors(spec), synth.SEED_BASE, "uniform")
    return spec, state


def test_identity_layout_is_noop(tiny_world):
    spec, state = tiny_world
    for w in WORLDS:
        lay = oracle.Layout(*w)
        world = make_world(spec, lay, state, poison=False)      # zero padding: required for identity
        assert_same(oracle.reshard_state(spec, lay, lay, world), world, f"identity {w}")


@pytest.mark.parametrize("a,b", [(WORLDS[0], WORLDS[1]), (WORLDS[2], WORLDS[3]), (WORLDS[3], WORLDS[4])])
def test_round_trip(tiny_world, a, b):
    spec, state = tiny_world
    A, B = oracle.Layout(*a), oracle.Layout(*b)
    wa = make_world(spec, A, state, poison=False)
    back = oracle.reshard_state(spec, B, A, poison_pads(spec, B, oracle.reshard_state(spec, A, B, wa)))
    assert_same(back, wa, "A->B->A")


def test_composition(tiny_world):
    spec, state = tiny_world
    A, B, C = (oracle.Layout(*w) for w in WORLDS[:3])
    wa = make_world(spec, A, state)
    via = oracle.reshard_state(spec, B, C, oracle.reshard_state(spec, A, B, wa))
    assert_same(via, oracle.reshard_state(spec, A, C, wa), "A->B->C vs A->C")


def test_target_equals_static_split_and_pads_are_zero(tiny_world):
    """Section 6.6's check: the resharded state equals a statically mapped
    reference (the logical state split directly for the target), padding +0."""
    spec, state = tiny_world
    for a, b in [(WORLDS[0], WORLDS[1]), (WORLDS[1], WORLDS[3])]:
        A, B = oracle.Layout(*a), oracle.Layout(*b)
        out = oracle.reshard_state(spec, A, B, make_world(spec, A, state))
        assert_same(out, make_world(spec, B, state, poison=False), "static reference")
        for pp in range(B.pp):
            nl = own.n_local(spec, B, pp)
            for tp in range(B.tp):
                for dp in range(B.dp):
                    assert not out[(B.rank(tp, pp, dp), oracle.PARAM)][nl:].any()


def test_copy_and_derive_agree_when_param_is_bf16_of_master(tiny_world):
    spec, state = tiny_world
    A, B = oracle.Layout(*WORLDS[0]), oracle.Layout(*WORLDS[3])
    wa = make_world(spec, A, state)
    assert_same(oracle.reshard_state(spec, A, B, wa, derive_bf16=True),
                oracle.reshard_state(spec, A, B, wa, derive_bf16=False), "derive vs copy")


@pytest.mark.parametrize("lay", [oracle.Layout(2, 2, 4, 4, ep=2, bucket_elems=300), oracle.Layout(1, 1, 2, 1, ep=1), oracle.Layout(2, 1, 4, 8, ep=4)])
def test_expected_shards_places_the_same_elements_as_the_full_split(lay):
    """expected_shards (the tensor-at-a-time helper used at full size) against split_logical (the full split):
    every shard it yields, written at its offset through dp_pieces, reproduces the full buffers; all kinds,
    dense and expert."""
    spec = MOE
    state = tiny_state(spec, seed=3)
    for kind in oracle.kinds_of(spec):
        logical = {n: a for n, a in state[kind % 4].items() if (".x" in n) == (kind >= oracle.EXPERT_PARAM)}
        full = oracle.split_logical(spec, lay, kind, logical)
        got = {key: np.zeros_like(a) for key, a in full.items()}
        some = {n: logical[n] for n in list(logical)[::2]}          # a subset yields only parameters it covers fully
        for tp, pp, sv, prm, shard in oracle.expected_shards(spec, lay, some, kind=kind):
            assert all(b.name in some for b in prm.blocks)
        for tp, pp, sv, prm, shard in oracle.expected_shards(spec, lay, logical, kind=kind):
            flat = shard.ravel()
            if kind % 4 == 0:
                for d in sv.dp_ranks:
                    got[(lay.rank(tp, pp, d), kind)][prm.offset:prm.offset + prm.size] = flat
            else:
                for d, local, at, n in oracle.dp_pieces(sv, lay, prm.offset, prm.offset + prm.size):
                    got[(lay.rank(tp, pp, d), kind)][local:local + n] = flat[at - prm.offset:at - prm.offset + n]
        assert set(got) == set(full)
        for key in full:
            assert np.array_equal(got[key], full[key]), key

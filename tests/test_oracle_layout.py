"""Pins the oracle's split and gather to the ownership formulas.

A state whose every element equals its own logical index (and a second one whose
every element equals the ordinal of its logical tensor) is split by the oracle;
each element of each rank's buffer must then hold exactly what the closed-form
ownership function of tests/ownership.py says that position owns."""
import numpy as np
import pytest

import liver_synth as synth
import oracle
import ownership as own
from util import cfg_objects, make_world, assert_same, corrupt_replicas, buffers_of

SPECS = {
    "tiny_gpt": oracle.ModelSpec(**synth.CONFIGS["tiny_gpt"]["spec"]),
    "gqa_glu": oracle.ModelSpec(n_layers=4, hidden=64, n_q_heads=8, n_kv_heads=4, ffn=96, vocab=128,
                                glu=True),
    "gqa_glu_bias_untied": oracle.ModelSpec(n_layers=2, hidden=48, n_q_heads=6, n_kv_heads=2, ffn=40,
                                            vocab=64, max_pos=16, glu=True, norm_bias=True,
                                            linear_bias=True),
    "gqa_replicated_kv": oracle.ModelSpec(n_layers=2, hidden=64, n_q_heads=8, n_kv_heads=2, ffn=64, vocab=64,
                                          glu=True, linear_bias=True),
    "odd_vocab_tied": oracle.ModelSpec(n_layers=2, hidden=32, n_q_heads=4, n_kv_heads=4, ffn=32, vocab=50,
                                       max_pos=8, tied_embed=True),
    "odd_vocab_head": oracle.ModelSpec(n_layers=2, hidden=32, n_q_heads=4, n_kv_heads=4, ffn=32, vocab=37, glu=True),
    "moe": oracle.ModelSpec(n_layers=2, hidden=32, n_q_heads=4, n_kv_heads=2, ffn=24, vocab=32, glu=True,
                            linear_bias=True, n_experts=4),
    "mqa_tied": oracle.ModelSpec(n_layers=4, hidden=32, n_q_heads=4, n_kv_heads=1, ffn=64, vocab=32,
                                 tied_embed=True),
}
LAYOUTS = [(1, 1, 1, 128), (2, 1, 2, 128), (1, 2, 2, 128), (2, 2, 3, 4), (4, 2, 1, 1), (2, 1, 3, 1),
           (2, 2, 2, 4, 2), (1, 1, 1, 1, 2), (1, 2, 3, 1, 1),       # 5th entry: vpp (interleaved stages)
           (8, 1, 2, 4),                                            # TP 8 > n_kv: replicated kv heads
           (2, 2, 2, 4, 1, 8), (4, 1, 1, 1, 1, 4), (1, 1, 2, 1, 1, 16), (4, 2, 3, 128, 1, 32),   # 6th: vocab_multiple
           (1, 2, 2, 4, 1, 0, 1, 0), (2, 2, 1, 1, 1, 0, 3, 1), (1, 3, 1, 1, 1, 0, 1, 1),         # 7th, 8th: pp_first, pp_last
           (2, 1, 3, 4, 1, 0, 0, 0, 3000), (1, 2, 2, 128, 1, 0, 0, 0, 1), (2, 2, 2, 1, 2, 8, 0, 0, 5000),   # 9th: bucket_elems
           (2, 1, 4, 4, 1, 0, 0, 0, 0, 2), (1, 2, 4, 1, 1, 0, 0, 0, 900, 4), (2, 2, 2, 8, 1, 0, 0, 0, 0, 1)]  # 10th: ep


def _cases():
    for sname, spec in SPECS.items():
        for (tp, pp, dp, pm, *rest) in LAYOUTS:
            lay = oracle.Layout(tp, pp, dp, pm, *rest)
            try:
                oracle.check_supported(spec, lay)
            except ValueError:
                continue
            yield pytest.param(spec, lay, id=f"{sname}-tp{tp}pp{pp}dp{dp}pm{pm}v{lay.vpp}vm{lay.vocab_multiple}f{lay.pp_first}l{lay.pp_last}b{lay.bucket_elems}e{lay.ep}")


def _tensor_ordinal_state(spec):
    shapes = oracle.logical_tensors(spec)
    st = {k: {} for k in oracle.KINDS}
    for i, (n, s) in enumerate(shapes.items()):
        for k in oracle.KINDS:
            st[k][n] = np.full(s, i + 1, oracle.WORD[k])
    return st


@pytest.mark.parametrize("spec,lay", list(_cases()))
def test_split_matches_ownership(spec, lay):
    shapes = oracle.logical_tensors(spec)
    ordinal = {n: i + 1 for i, n in enumerate(shapes)}
    w_idx = make_world(spec, lay, synth.index_encoded_state(shapes, half=0), poison=False)
    w_hi = make_world(spec, lay, synth.index_encoded_state(shapes, half=1), poison=False)
    w_ord = make_world(spec, lay, _tensor_ordinal_state(spec), poison=False)
    for base, ep in buffers_of(spec, lay):                                # dense buffers, then one expert buffer per ep
      for pp in range(lay.pp):
        npad = own.n_pad(spec, lay, pp, ep)
        dp_of, local_of = own.shard_location(spec, lay, pp, ep)
        group = list(range(lay.dp)) if ep is None else list(range(ep, lay.dp, lay.ep))
        for tp in range(lay.tp):
            names, idx, _ = own.column_ownership(spec, lay, tp, pp, ep)   # padding: name None, index 0
            exp_idx = idx
            exp_ord = np.array([ordinal.get(n, 0) for n in names], np.int64)
            for dp in range(lay.dp):
                r = lay.rank(tp, pp, dp)
                if dp not in group:                                       # ranks of another expert-parallel index
                    continue
                assert np.array_equal(w_idx[(r, base)], (exp_idx & 0xFFFF).astype(np.uint16))
                assert np.array_equal(w_hi[(r, base)], ((exp_idx >> 16) & 0xFFFF).astype(np.uint16))
                assert np.array_equal(w_ord[(r, base)], exp_ord.astype(np.uint16))
                mine = np.flatnonzero(dp_of == dp)
                assert np.array_equal(local_of[mine], np.arange(npad // len(group)))      # a rank's buffer is dense
                for k in (base + 1, base + 2, base + 3):
                    assert w_idx[(r, k)].shape == (npad // len(group),)
                    assert np.array_equal(w_idx[(r, k)], exp_idx[mine].astype(np.uint32))
                    assert np.array_equal(w_ord[(r, k)], exp_ord[mine].astype(np.uint32))
    n_bufs = lay.n_ranks * (8 if spec.n_experts else 4)
    assert len(w_idx) == n_bufs                                            # every rank holds every kind exactly once


@pytest.mark.parametrize("spec,lay", list(_cases()))
def test_gather_inverts_split(spec, lay):
    """gather(split(x)) == x, with NaN-poisoned padding (never read) and every
    logical element gathered exactly once (the gather raises otherwise)."""
    shapes = oracle.logical_tensors(spec)
    state = synth.logical_state(shapes, synth.SEED_BASE, "uniform")
    world = make_world(spec, lay, state, poison=True)
    seen = []
    for k in oracle.kinds_of(spec):
        back = oracle.gather_logical(spec, lay, k, oracle.dict_reader(world))
        seen += list(back) if k % 4 == 0 else []
        for n in back:
            assert np.array_equal(back[n], state[k % 4][n]), (k, n)
    assert sorted(seen) == sorted(shapes)                  # dense and expert kinds together cover every tensor


def test_gather_reads_lowest_replica():
    """Replicated values differ on purpose: the gather must take tp=0 / dp=0 /
    the first-stage embedding."""
    spec = SPECS["tiny_gpt"]
    lay = oracle.Layout(2, 2, 2, 4)
    shapes = oracle.logical_tensors(spec)
    state = synth.logical_state(shapes, 7, "uniform")
    world = make_world(spec, lay, state)
    corrupt_replicas(spec, lay, world)
    for k in oracle.KINDS:
        back = oracle.gather_logical(spec, lay, k, oracle.dict_reader(world))
        for n in shapes:
            assert np.array_equal(back[n], state[k][n]), (k, n)


def test_gather_detects_broken_tiling(monkeypatch):
    """The exactly-once check of the gather fires if a view misses elements."""
    spec = SPECS["mqa_tied"]
    lay = oracle.Layout(1, 1, 1, 1)
    world = make_world(spec, lay, synth.logical_state(oracle.logical_tensors(spec), 3, "uniform"))
    real = oracle.reshard_oracle.stage_view

    def broken(spec_, lay_, tp, pp, ep=None):
        sv = real(spec_, lay_, tp, pp, ep)
        sv.params[0].canonical = False          # nobody provides embed.word any more
        return sv
    monkeypatch.setattr(oracle.reshard_oracle, "stage_view", broken)
    with pytest.raises(AssertionError):
        oracle.gather_logical(spec, lay, oracle.MASTER, oracle.dict_reader(world))


def test_interleaved_stage_layers():
    """Interleaved schedule: L=8, PP=2, vpp=2 -> stage 0 holds layers 0,1,4,5 and stage 1 holds 2,3,6,7,
    in that order in the flat buffer; vpp=1 is the plain even split."""
    spec = oracle.ModelSpec(n_layers=8, hidden=32, n_q_heads=4, n_kv_heads=4, ffn=64, vocab=32)
    assert oracle.stage_layers(spec, oracle.Layout(1, 2, 1, 1, 2), 0) == [0, 1, 4, 5]
    assert oracle.stage_layers(spec, oracle.Layout(1, 2, 1, 1, 2), 1) == [2, 3, 6, 7]
    assert oracle.stage_layers(spec, oracle.Layout(1, 4, 1, 1, 2), 3) == [3, 7]
    assert oracle.stage_layers(spec, oracle.Layout(1, 2, 1, 1, 1), 1) == [4, 5, 6, 7]
    sv = oracle.stage_view(spec, oracle.Layout(1, 2, 1, 1, 2), 0, 1)
    order = [p.name.split(".")[0] for p in sv.params if p.name.endswith("ln1.w")]
    assert order == ["L2", "L3", "L6", "L7"]
    with pytest.raises(ValueError):
        oracle.stage_view(spec, oracle.Layout(1, 4, 1, 1, 4), 0, 0)


def test_padded_vocab_sizes():
    """GPT-2's 50257-token vocabulary padded to a multiple of 128*TP rows: 50304 / 50432 / 50688 for TP 1 / 2 / 4
    (the sizes Megatron-LM reports for make-vocab-size-divisible-by 128)."""
    spec = oracle.ModelSpec(n_layers=2, hidden=64, n_q_heads=4, n_kv_heads=4, ffn=64, vocab=50257, tied_embed=True)
    for tp, want in ((1, 50304), (2, 50432), (4, 50688)):
        lay = oracle.Layout(tp, 1, 1, 128, 1, 128)
        assert oracle.padded_vocab(spec, lay) == want == own.vocab_rows(spec, tp, 128) * tp
        sv = oracle.stage_view(spec, lay, tp - 1, 0)
        emb = sv.params[0]
        assert emb.shape == (want // tp, 64)
        real = max(0, min(want // tp, 50257 - (tp - 1) * (want // tp)))
        assert sum(b.loc[0].stop - b.loc[0].start for b in emb.blocks) == real
    with pytest.raises(ValueError):
        oracle.stage_view(spec, oracle.Layout(2, 1, 1, 128), 0, 0)        # 50257 % 2 != 0 and no padding


def test_uneven_stage_layers():
    """Fixed layer counts on the first / last stage, the rest shared evenly."""
    spec = oracle.ModelSpec(n_layers=10, hidden=32, n_q_heads=4, n_kv_heads=4, ffn=64, vocab=32)
    L = lambda *a: oracle.Layout(1, a[0], 1, 1, 1, 0, a[1], a[2])
    assert [oracle.stage_layers(spec, L(4, 1, 3), p) for p in range(4)] == [[0], [1, 2, 3], [4, 5, 6], [7, 8, 9]]
    assert [oracle.stage_layers(spec, L(3, 2, 0), p) for p in range(3)] == [[0, 1], [2, 3, 4, 5], [6, 7, 8, 9]]
    assert [oracle.stage_layers(spec, L(2, 7, 3), p) for p in range(2)] == [list(range(7)), [7, 8, 9]]
    assert [oracle.stage_layers(spec, L(3, 0, 4), p) for p in range(3)] == [[0, 1, 2], [3, 4, 5], [6, 7, 8, 9]]
    for bad in (L(4, 1, 2), L(2, 7, 2), L(3, 9, 1), L(2, 10, 0)):          # 7 over 2 stages; 7+2 != 10; nothing left; empty stage
        with pytest.raises(ValueError):
            oracle.stage_view(spec, bad, 0, 0)
    with pytest.raises(ValueError):
        oracle.stage_view(spec, oracle.Layout(1, 5, 1, 1, 2, 0, 2, 0), 0, 0)   # not combinable with vpp
    for lay in (L(4, 1, 3), L(3, 0, 4)):
        for p in range(lay.pp):
            assert own.uneven_stage_range(10, lay.pp, p, lay.pp_first, lay.pp_last) == \
                (oracle.stage_layers(spec, lay, p)[0], oracle.stage_layers(spec, lay, p)[-1] + 1)


def test_bucket_boundaries_closed_form():
    """bucket_elems = 300 on a 1-layer toy model: parameters fill buckets in order, a bucket closes after the
    parameter that reaches 300 elements, every bucket is padded to DP*pad_multiple = 8."""
    spec = oracle.ModelSpec(n_layers=1, hidden=8, n_q_heads=2, n_kv_heads=2, ffn=16, vocab=20)
    lay = oracle.Layout(1, 1, 2, 4, bucket_elems=300)
    sv = oracle.stage_view(spec, lay, 0, 0)
    sizes = [(p.name, p.size) for p in sv.params]
    assert sizes == [("embed.word", 160), ("L0.ln1.w", 8), ("L0.qkv.w", 192), ("L0.o.w", 64), ("L0.ln2.w", 8),
                     ("L0.fc1.w", 128), ("L0.fc2.w", 128), ("final_norm.w", 8), ("lm_head.w", 160)]
    # bucket 0: 160+8+192 = 360 -> padded 360; bucket 1: 64+8+128+128 = 328 -> padded 328; bucket 2: 8+160 = 168 -> 168
    assert sv.buckets == [(0, 360), (360, 328), (688, 168)] and sv.n_pad == 856 and sv.S == 428
    assert [p.offset for p in sv.params] == [0, 160, 168, 360, 424, 432, 560, 688, 696]
    lay3 = oracle.Layout(1, 1, 3, 4, bucket_elems=300)            # quantum 12: 360, 336 (328 + 8 pad), 168
    sv3 = oracle.stage_view(spec, lay3, 0, 0)
    assert sv3.buckets == [(0, 360), (360, 336), (696, 168)] and sv3.n_local == 864 - 0 and sv3.n_pad == 864
    # DP rank 1 of 3 holds the middle third of every bucket, concatenated
    assert oracle.dp_pieces(sv3, lay3, 0, 864)[1::3] == [(1, 0, 120, 120), (1, 120, 472, 112), (1, 232, 752, 56)]
    assert own.bucket_table(spec, lay3, 0) == [(0, 360, 360), (360, 328, 336), (696, 168, 168)]


def test_expert_buffers_closed_form():
    """MoE: 4 experts, EP 2 inside DP 4: DP ranks 0, 2 hold experts 0-1 and ranks 1, 3 hold experts 2-3; the
    expert buffer of a rank lists, layer by layer, its experts' fc1 / fc2 (TP-split like a dense FFN) and is
    optimizer-sharded over the two ranks that hold the same experts; the dense buffer keeps only the router."""
    spec = SPECS["moe"]
    lay = oracle.Layout(2, 1, 4, 4, ep=2)
    H, F = 32, 24
    per_expert = 2 * F * H // 2 + 2 * F // 2 + H * F // 2 + H           # fc1.w, fc1.b, fc2.w, down.b on one of 2 TP ranks
    for ep in (0, 1):
        sv = oracle.stage_view(spec, lay, 1, 0, ep)
        assert sv.dp_ranks == [ep, ep + 2] and sv.n_local == 2 * 2 * per_expert            # 2 layers x 2 local experts
        assert [p.name for p in sv.params[:4]] == [f"L0.x{2 * ep}.fc1.w", f"L0.x{2 * ep}.fc1.b", f"L0.x{2 * ep}.fc2.w",
                                                   f"L0.x{2 * ep}.down.b"]
        assert sv.n_pad % (2 * 4) == 0 and sv.S == sv.n_pad // 2
    dense = oracle.stage_view(spec, lay, 0, 0)
    assert dense.dp_ranks == [0, 1, 2, 3] and not any(".x" in p.name for p in dense.params)
    assert [p.name for p in dense.params if "router" in p.name] == ["L0.router.w", "L1.router.w"]
    assert oracle.buffer_elems(spec, lay, 0, 0, oracle.EXPERT_MASTER, dp=3) == oracle.stage_view(spec, lay, 0, 0, 1).S
    for bad in (oracle.Layout(1, 1, 4, 4, ep=3), oracle.Layout(1, 1, 2, 4, ep=4)):
        with pytest.raises(ValueError):
            oracle.stage_view(spec, bad, 0, 0)
    with pytest.raises(ValueError):
        oracle.stage_view(SPECS["mqa_tied"], oracle.Layout(1, 1, 2, 4, ep=2), 0, 0)         # ep without experts

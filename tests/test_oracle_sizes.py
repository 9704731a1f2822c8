"""Pins the oracle's layout enumerator to closed-form sizes.

The numbers are typed out from the layout conventions (parameters per layer,
even layer split over stages, padding to a multiple of DP*128) -- not read from
the oracle.  They also fix the traffic the benchmark quotes (bytes per state)."""
import pytest

import oracle
import ownership as own
from util import cfg_objects

# per (config, side, pp): N_local of one TP rank's flat buffer
SIZES = {
    ("tiny_gpt", "src", 0): 1_053_952,
    ("tiny_gpt", "dst", 0): 1_182_976,
    ("tiny_gpt", "dst", 1): 1_052_416,            # includes the tied word-embedding copy
    ("gpt2_small", "src", 0): 41_380_608,
    ("gpt2_small", "src", 1): 40_595_712,
    ("gpt2_small", "dst", 0): 31_751_424,
    ("llama7b", "src", 0): 2 * 16_384_000 + 32 * 25_305_088 + 4_096,     # 842,534,912
    ("llama7b", "dst", 0): 842_399_744,
    ("llama7b", "dst", 1): 842_403_840,
    ("llama13b_dp", "src", 0): 3_254_067_200,
    ("llama13b_dp", "src", 1): 3_254_072_320,
    ("llama70b_rank", "dst", 0): 2_401_927_168,
    ("llama70b_rank", "dst", 3): 2_139_258_880,
    ("llama70b_rank", "dst", 7): 2_401_935_360,
    ("llama70b_rank", "src", 3): 1_069_711_360,
}
TOTAL_PARAMS = {"tiny_gpt": 1_973_248, "gpt2_small": 124_475_904, "llama7b": 6_738_415_616,
                "llama13b_dp": 13_015_864_320, "llama70b_rank": 70_553_706_496}


@pytest.mark.parametrize("key", sorted(SIZES))
def test_n_local_closed_form(key):
    name, side, pp = key
    _, spec, src, dst = cfg_objects(name)
    lay = src if side == "src" else dst
    for tp in {0, lay.tp - 1}:
        sv = oracle.stage_view(spec, lay, tp, pp)
        assert sv.n_local == SIZES[key]
        assert sv.n_local == own.n_local(spec, lay, pp) and sv.n_pad == own.n_pad(spec, lay, pp)
        assert sv.n_local == sum(p.size for p in sv.params)
        offs = [p.offset for p in sv.params]
        assert offs == sorted(offs) and offs[0] == 0
        q = lay.dp * lay.pad_multiple
        assert sv.n_pad % q == 0 and 0 <= sv.n_pad - sv.n_local < q and sv.S * lay.dp == sv.n_pad


def test_padding_and_slices_13b_70b():
    _, spec, src, dst = cfg_objects("llama13b_dp")
    assert [oracle.stage_view(spec, src, 0, pp).S for pp in (0, 1)] == [406_758_400, 406_759_040]
    assert [oracle.stage_view(spec, dst, 0, pp).n_pad for pp in (0, 1)] == [3_254_067_456, 3_254_072_832]
    assert [oracle.stage_view(spec, dst, 0, pp).S for pp in (0, 1)] == [542_344_576, 542_345_472]
    _, spec, src, dst = cfg_objects("llama70b_rank")
    sv = oracle.stage_view(spec, dst, 1, 3)
    assert (sv.n_pad, sv.S) == (2_139_259_392, 356_543_232)
    assert oracle.stage_view(spec, src, 2, 3).S == 267_427_840


@pytest.mark.parametrize("name", sorted(TOTAL_PARAMS))
def test_logical_total(name):
    _, spec, _, _ = cfg_objects(name)
    total = 0
    for shape in oracle.logical_tensors(spec).values():
        n = 1
        for d in shape:
            n *= d
        total += n
    assert total == TOTAL_PARAMS[name]


def test_7b_state_bytes():
    """Bytes of the 7B target state (what the headline metric divides by time)."""
    _, spec, _, dst = cfg_objects("llama7b")
    elems = sum(oracle.stage_view(spec, dst, tp, pp).n_local for pp in range(2) for tp in range(4))
    assert elems * 14 == 94_349_000_704


def test_unsupported_combinations():
    spec = oracle.ModelSpec(n_layers=4, hidden=64, n_q_heads=8, n_kv_heads=2, ffn=96, vocab=64)
    # TP 16 over 2 kv heads would need each group's 4 q heads split 8 ways
    for lay in (oracle.Layout(16, 1, 1), oracle.Layout(1, 3, 1), oracle.Layout(2, 1, 0)):
        with pytest.raises(ValueError):
            oracle.stage_view(spec, lay, 0, 0)

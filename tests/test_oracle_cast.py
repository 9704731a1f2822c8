"""Pins oracle.rne_bf16 to torch's CPU float32 -> bfloat16 conversion (round to
nearest even) and to directed cases."""
import numpy as np
import torch

import oracle
from util import _rne_scalar


def _torch_bits(u):
    t = torch.from_numpy(u.view(np.float32).copy()).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def test_against_torch_random_bits():
    rng = np.random.default_rng(0)
    u = rng.integers(0, 1 << 32, size=1 << 20, dtype=np.uint32)
    finite = (u & 0x7FFFFFFF) <= 0x7F800000
    u = u[finite]
    assert np.array_equal(oracle.rne_bf16(u), _torch_bits(u))


def test_against_torch_all_low_halves():
    """Every possible lower 16 bits, on an even and an odd upper half."""
    low = np.arange(1 << 16, dtype=np.uint32)
    for hi in (0x3F80, 0x3F81, 0x0000, 0x0001, 0x7F7F, 0xBF80, 0x807F):
        u = (np.uint32(hi) << 16) | low
        assert np.array_equal(oracle.rne_bf16(u), _torch_bits(u)), hex(hi)


def test_directed_cases():
    cases = {
        0x00000000: 0x0000, 0x80000000: 0x8000,              # +-0
        0x3F808000: 0x3F80,                                  # tie, even stays
        0x3F818000: 0x3F82,                                  # tie, odd goes up
        0x3F808001: 0x3F81, 0x3F807FFF: 0x3F80,              # just above / below a tie
        0x00000001: 0x0000, 0x00008000: 0x0000, 0x00008001: 0x0001, 0x00018000: 0x0002,  # denormals
        0x7F7FFFFF: 0x7F80, 0xFF7FFFFF: 0xFF80,              # max finite -> Inf
        0x7F800000: 0x7F80, 0xFF800000: 0xFF80,              # Inf
        0x7FC00000: 0x7FC0, 0x7F800001: 0x7FC0, 0xFFFFFFFF: 0xFFFF, 0x7FA00000: 0x7FE0,  # NaN: quieted
    }
    u = np.array(list(cases), np.uint32)
    assert oracle.rne_bf16(u).tolist() == list(cases.values())
    assert [_rne_scalar(int(x)) for x in u] == list(cases.values())


def test_scalar_neighbour_rule_agrees():
    rng = np.random.default_rng(1)
    u = rng.integers(0, 1 << 32, size=20000, dtype=np.uint32)
    assert oracle.rne_bf16(u).tolist() == [_rne_scalar(int(x)) for x in u]

"""Seeded synthetic inputs and the benchmark configurations.

Shared by the tests, the benchmark, the smoke check and the CPU oracle's callers.
Holds NO resharding arithmetic: it knows neither shard layouts nor descriptors.
It only (a) lists the five workload configurations as plain data, (b) draws
values for a tensor or a buffer of a given size from a seeded, counter-based
stream, and (c) converts fp32 to bf16 with the library routine of torch (CPU or
GPU) so that PARAM == bf16(MASTER) holds for generated states.

The paper (LiveR, Section 6.1) measures on its own GPT training jobs whose
weights are not available; data movement is value-agnostic, so seeded synthetic
tensors with the shapes below stand in for them.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 22014
PARAM, MASTER, ADAM_M, ADAM_V = 0, 1, 2, 3

_GPT = dict(glu=False, norm_bias=True, linear_bias=True, tied_embed=True)
_LLAMA = dict(glu=True, norm_bias=False, linear_bias=False, tied_embed=False, max_pos=0)

# spec / src / dst are keyword sets for whichever ModelSpec / Layout class the
# caller uses; `only` restricts the plan to one target rank's share;
# `kinds` lists the buffer kinds that take part.
CONFIGS = {
    "tiny_gpt": dict(
        spec=dict(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=4, ffn=1024, vocab=1024,
                  max_pos=512, **_GPT),
        src=dict(tp=2, pp=1, dp=2), dst=dict(tp=1, pp=2, dp=2), pad_multiple=128,
        chunk_bytes=1 << 20, dist="uniform", only=None, kinds=(0, 1, 2, 3)),
    "gpt2_small": dict(
        spec=dict(n_layers=12, hidden=768, n_q_heads=12, n_kv_heads=12, ffn=3072, vocab=50304,
                  max_pos=1024, **_GPT),
        src=dict(tp=2, pp=2, dp=2), dst=dict(tp=4, pp=1, dp=2), pad_multiple=128,
        chunk_bytes=64 << 20, dist="normal", only=None, kinds=(0, 1, 2, 3)),
    "llama7b": dict(
        spec=dict(n_layers=32, hidden=4096, n_q_heads=32, n_kv_heads=32, ffn=11008, vocab=32000,
                  **_LLAMA),
        src=dict(tp=8, pp=1, dp=1), dst=dict(tp=4, pp=2, dp=1), pad_multiple=128,
        chunk_bytes=256 << 20, dist="normal", only=None, kinds=(0, 1, 2, 3)),
    "llama13b_dp": dict(
        spec=dict(n_layers=40, hidden=5120, n_q_heads=40, n_kv_heads=40, ffn=13824, vocab=32000,
                  **_LLAMA),
        src=dict(tp=2, pp=2, dp=8), dst=dict(tp=2, pp=2, dp=6), pad_multiple=128,
        chunk_bytes=256 << 20, dist="normal", only=dict(tp=0, pp=1, dp=2), kinds=(1, 2, 3)),
    "llama70b_rank": dict(
        spec=dict(n_layers=80, hidden=8192, n_q_heads=64, n_kv_heads=8, ffn=28672, vocab=128256,
                  **_LLAMA),
        src=dict(tp=8, pp=8, dp=4), dst=dict(tp=4, pp=8, dp=6), pad_multiple=128,
        chunk_bytes=512 << 20, dist="normal", only=dict(tp=1, pp=3, dp=2), kinds=(0, 1, 2, 3)),
}


def _rng(seed: int, kind: int, ident: int) -> np.random.Generator:
    """Counter-based stream keyed by (seed, kind, ident): any tensor or buffer
    can be regenerated alone."""
    return np.random.Generator(np.random.Philox(key=int(seed), counter=[0, 0, int(kind), int(ident)]))


def draw_f32(n: int, seed: int, kind: int, ident: int, dist: str) -> np.ndarray:
    """n fp32 values: 'normal' = N(0, 0.02), 'uniform' = U(-1, 1)."""
    g = _rng(seed, kind, ident)
    if dist == "normal":
        return g.standard_normal(n, dtype=np.float32) * np.float32(0.02)
    if dist == "uniform":
        return (g.random(n, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)).astype(np.float32)
    raise ValueError(dist)


def bf16_bits_of(x: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) of finite fp32 values, by torch's CPU conversion."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def logical_state(shapes: dict, seed: int, dist: str) -> dict:
    """{kind: {name: bit-pattern array}} for a dict name -> shape of logical tensors.

    MASTER is drawn first, PARAM = bf16(MASTER); ADAM_M and ADAM_V are independent
    draws (V made non-negative, as a second-moment estimate is)."""
    state = {PARAM: {}, MASTER: {}, ADAM_M: {}, ADAM_V: {}}
    for ident, (name, shape) in enumerate(shapes.items()):
        n = int(np.prod(shape))
        w = draw_f32(n, seed, MASTER, ident, dist)
        state[MASTER][name] = w.view(np.uint32).reshape(shape)
        state[PARAM][name] = bf16_bits_of(w).reshape(shape)
        state[ADAM_M][name] = draw_f32(n, seed, ADAM_M, ident, dist).view(np.uint32).reshape(shape)
        state[ADAM_V][name] = np.abs(draw_f32(n, seed, ADAM_V, ident, dist)).view(np.uint32).reshape(shape)
    return state


def index_encoded_state(shapes: dict, half: int = 0) -> dict:
    """Every element's value is its own row-major index in its logical tensor.

    fp32 kinds store the index as the 32-bit pattern; bf16 can hold only 16 bits,
    so PARAM stores (index >> (16*half)) & 0xFFFF for half in {0, 1}."""
    state = {PARAM: {}, MASTER: {}, ADAM_M: {}, ADAM_V: {}}
    for name, shape in shapes.items():
        idx = np.arange(int(np.prod(shape)), dtype=np.uint64).reshape(shape)
        for k in (MASTER, ADAM_M, ADAM_V):
            state[k][name] = (idx + k * 0).astype(np.uint32)
        state[PARAM][name] = ((idx >> (16 * half)) & 0xFFFF).astype(np.uint16)
    return state


def fill_device_world(sizes: dict, dp: int, seed: int, device: str = "cuda"):
    """Source buffers generated directly in device memory, for states too large to
    build on the host.

    sizes: {(column, d): S} fp32 elements of DP slice d of rank column `column`
    (an opaque key chosen by the caller).  Returns {(column, d, kind): tensor}:
    MASTER/ADAM_M/ADAM_V slices ~ N(0, 0.02) (V = |.|), and for d == 0 also
    (column, 'param'): bf16 of the concatenated MASTER slices of the column.
    Pad elements are not treated specially (the caller overwrites them)."""
    import torch
    g = torch.Generator(device=device)
    out = {}
    columns = sorted({c for c, _ in sizes})
    for ci, c in enumerate(columns):
        for d in range(dp):
            n = sizes[(c, d)]
            for kind in (MASTER, ADAM_M, ADAM_V):
                g.manual_seed(((seed * 1000003 + ci) * 64 + d) * 4 + kind)
                t = torch.empty(n, dtype=torch.float32, device=device)
                t.normal_(0.0, 0.02, generator=g)
                if kind == ADAM_V:
                    t.abs_()
                out[(c, d, kind)] = t
        out[(c, "param")] = torch.cat([out[(c, d, MASTER)].to(torch.bfloat16) for d in range(dp)])
    return out


def fill_device_world_into(columns: dict, seed: int) -> None:
    """Same values as fill_device_world, written into buffers the caller has already allocated.

    columns: {column key: {"master": [tensor per DP slice], "m": [...], "v": [...], "param": bf16 tensor or None}}
    (fp32 tensors; param holds the bf16 of the concatenated MASTER slices)."""
    import torch
    for ci, c in enumerate(sorted(columns)):
        col = columns[c]
        device = col["master"][0].device
        g = torch.Generator(device=device)
        pos = 0
        for d, master in enumerate(col["master"]):
            for kind, t in ((MASTER, master), (ADAM_M, col["m"][d]), (ADAM_V, col["v"][d])):
                g.manual_seed(((seed * 1000003 + ci) * 64 + d) * 4 + kind)
                t.normal_(0.0, 0.02, generator=g)
                if kind == ADAM_V:
                    t.abs_()
            if col.get("param") is not None:
                col["param"][pos:pos + master.numel()].copy_(master)       # fp32 -> bf16 (round to nearest even)
            pos += master.numel()

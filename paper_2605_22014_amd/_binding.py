"""ctypes binding of the C ABI declared in include/liver.h.

The functions keep the names of the C entry points.  Buffer tables are given as
{(rank, kind): tensor-or-address} dictionaries (or a ready ctypes array) and are
marshalled into the rank*NUM_KINDS+kind pointer tables the library expects.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, Optional, Tuple

# torch must be loaded BEFORE libliver.so: the wheel ships its own HIP runtime
# (libamdhip64.so.7) and the device pointers and streams handed to the library
# belong to that runtime.  With torch loaded first, the library's dependency on
# libamdhip64.so.7 resolves to the copy already in the process; the other way
# round two HIP runtimes would coexist and the library's would see no device.
import torch  # noqa: F401

PARAM, MASTER, ADAM_M, ADAM_V = 0, 1, 2, 3
EXPERT_PARAM, EXPERT_MASTER, EXPERT_ADAM_M, EXPERT_ADAM_V = 4, 5, 6, 7     # expert parameters of MoE models
NUM_KINDS = 8                                                             # stride of the buffer tables
LIST_DIRECT, LIST_PACK, LIST_UNPACK = 0, 1, 2
OP_COPY, OP_CAST_BF16, OP_ZERO = 0, 1, 2
_GLU, _NORM_BIAS, _LINEAR_BIAS, _TIED = 1, 2, 4, 8
_DERIVE = 1

_HERE = os.path.dirname(os.path.abspath(__file__))


def library_path() -> str:
    return os.path.join(_HERE, "libliver.so")


class LiverError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"liver error {code}: {msg}")
        self.code = code


class _Spec(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "ffn", "vocab", "max_pos")] \
        + [("flags", C.c_uint32), ("n_experts", C.c_int32)]


class _Layout(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("tp", "pp", "dp", "pad_multiple", "only_tp", "only_pp", "only_dp")] \
        + [("flags", C.c_uint32), ("kind_mask", C.c_uint32), ("vpp", C.c_int32), ("vocab_multiple", C.c_int32), ("pp_first", C.c_int32), ("pp_last", C.c_int32), ("bucket_elems", C.c_int64), ("ep", C.c_int32)]


class PlanInfo(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("n_chunks", "n_desc", "n_desc_pack", "n_desc_unpack", "stream_bytes",
                                         "bytes_read", "bytes_written", "pad_bytes", "table_bytes_device")] \
        + [(n, C.c_int32) for n in ("n_src_ranks", "n_dst_ranks", "n_src_bufs_used", "n_dst_bufs_used")]


class Desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("op", "chunk", "slot", "src_rank", "src_kind", "dst_rank", "dst_kind",
                                         "reserved")] \
        + [(n, C.c_int64) for n in ("src_off", "src_stride", "dst_off", "dst_stride", "rows", "run")]


@dataclass(frozen=True)
class ModelSpec:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    ffn: int
    vocab: int
    max_pos: int = 0
    glu: bool = False
    norm_bias: bool = False
    linear_bias: bool = False
    tied_embed: bool = False
    n_experts: int = 0          # > 0: mixture of experts (router in the dense buffers, experts in kinds 4..7)

    def _c(self) -> _Spec:
        flags = (_GLU * self.glu) | (_NORM_BIAS * self.norm_bias) | (_LINEAR_BIAS * self.linear_bias) \
            | (_TIED * self.tied_embed)
        return _Spec(self.n_layers, self.hidden, self.n_q_heads, self.n_kv_heads, self.ffn, self.vocab,
                     self.max_pos, flags, self.n_experts)


@dataclass(frozen=True)
class Layout:
    tp: int
    pp: int
    dp: int
    pad_multiple: int = 128
    only_tp: int = -1
    only_pp: int = -1
    only_dp: int = -1
    derive_bf16: bool = False
    kinds: Optional[Tuple[int, ...]] = None      # None = all four
    vpp: int = 1                                 # model chunks per stage (interleaved pipeline)
    vocab_multiple: int = 0                      # pad the vocabulary to a multiple of vocab_multiple*tp rows
    pp_first: int = 0                            # layers on the first / last stage (0 = even split)
    pp_last: int = 0
    bucket_elems: int = 0                        # flat buffer cut into buckets of >= this many elements (0 = one)
    ep: int = 1                                  # expert-parallel size (divides dp and n_experts)

    @property
    def n_ranks(self) -> int:
        return self.tp * self.pp * self.dp

    def rank(self, tp: int, pp: int, dp: int) -> int:
        return tp + self.tp * (dp + self.dp * pp)

    def _c(self) -> _Layout:
        mask = 0 if self.kinds is None else sum(1 << k for k in set(self.kinds))
        return _Layout(self.tp, self.pp, self.dp, self.pad_multiple, self.only_tp, self.only_pp, self.only_dp,
                       _DERIVE * self.derive_bf16, mask, self.vpp, self.vocab_multiple, self.pp_first, self.pp_last, self.bucket_elems, self.ep)


def _load() -> C.CDLL:
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it first (python -m paper_2605_22014_amd.build, or "
                          f"__graft_entry__.build()); there is no fallback implementation")
    lib = C.CDLL(path)
    P = C.c_void_p
    lib.liver_plan_create.argtypes = [C.POINTER(_Spec), C.POINTER(_Layout), C.POINTER(_Layout), C.c_size_t, C.POINTER(P)]
    lib.liver_plan_destroy.argtypes = [P]
    lib.liver_plan_destroy.restype = None
    lib.liver_plan_info.argtypes = [P, C.POINTER(PlanInfo)]
    lib.liver_plan_buffer_bytes.argtypes = [P, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    lib.liver_plan_buffer_used.argtypes = [P, C.c_int, C.c_int, C.c_int]
    lib.liver_plan_desc_count.argtypes = [P, C.c_int]
    lib.liver_plan_desc_count.restype = C.c_int64
    lib.liver_plan_desc.argtypes = [P, C.c_int, C.c_int64, C.POINTER(Desc)]
    lib.liver_plan_set_launch.argtypes = [P, C.c_int, C.c_int, C.c_int]
    lib.liver_pack.argtypes = [P, C.c_int, C.POINTER(P), P, P]
    lib.liver_unpack.argtypes = [P, C.c_int, P, C.POINTER(P), P]
    lib.liver_reshard.argtypes = [P, C.POINTER(P), C.POINTER(P), P]
    lib.liver_reshard_staged.argtypes = [P, C.POINTER(P), C.POINTER(P), C.POINTER(P), C.c_int, P, P]
    lib.liver_reshard_staged_fused.argtypes = [P, C.POINTER(P), C.POINTER(P), P, P, P]
    lib.liver_reshard_static.argtypes = [P, C.POINTER(P), C.POINTER(P), P]
    lib.liver_static_staging_bytes.argtypes = []
    lib.liver_static_staging_bytes.restype = C.c_size_t
    lib.liver_debug_emulate_host.argtypes = [P, C.c_int, C.c_int, C.POINTER(P), C.POINTER(P), P]
    lib.liver_debug_bandwidth_probe.argtypes = [C.c_int, P, P, C.c_size_t, C.c_int, P]
    lib.liver_strerror.argtypes = [C.c_int]
    lib.liver_strerror.restype = C.c_char_p
    return lib


_lib = _load()


def liver_strerror(code: int) -> str:
    return _lib.liver_strerror(code).decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise LiverError(rc, liver_strerror(rc))


class Plan:
    """Owner of a liver_plan_t*; freed on liver_plan_destroy or garbage collection."""

    def __init__(self, handle: int, src: Layout, dst: Layout, chunk_bytes: int):
        self.handle, self.src, self.dst, self.chunk_bytes = handle, src, dst, chunk_bytes
        self._sizes = {}

    def _buffer_bytes(self, side: int, rank: int, kind: int) -> int:
        key = (side, rank, kind)
        if key not in self._sizes:
            self._sizes[key] = liver_plan_buffer_bytes(self, side, rank, kind)
        return self._sizes[key]

    def __del__(self):
        try:
            liver_plan_destroy(self)
        except Exception:       # interpreter shutdown: the library may already be gone
            pass


def liver_plan_create(spec: ModelSpec, src: Layout, dst: Layout, chunk_bytes: int) -> Plan:
    h = C.c_void_p()
    cs, ca, cb = spec._c(), src._c(), dst._c()
    _check(_lib.liver_plan_create(C.byref(cs), C.byref(ca), C.byref(cb), chunk_bytes, C.byref(h)))
    return Plan(h.value, src, dst, chunk_bytes)


def liver_plan_destroy(plan: Plan) -> None:
    if getattr(plan, "handle", None):
        _lib.liver_plan_destroy(plan.handle)
        plan.handle = None


def liver_plan_info(plan: Plan) -> PlanInfo:
    info = PlanInfo()
    _check(_lib.liver_plan_info(plan.handle, C.byref(info)))
    return info


def liver_plan_buffer_bytes(plan: Plan, side: int, rank: int, kind: int) -> int:
    n = C.c_size_t()
    _check(_lib.liver_plan_buffer_bytes(plan.handle, side, rank, kind, C.byref(n)))
    return n.value


def liver_plan_buffer_used(plan: Plan, side: int, rank: int, kind: int) -> bool:
    rc = _lib.liver_plan_buffer_used(plan.handle, side, rank, kind)
    if rc < 0:
        _check(rc)
    return bool(rc)


def liver_plan_desc_count(plan: Plan, which: int) -> int:
    n = _lib.liver_plan_desc_count(plan.handle, which)
    if n < 0:
        _check(int(n))
    return int(n)


def liver_plan_desc(plan: Plan, which: int, i: int) -> Desc:
    d = Desc()
    _check(_lib.liver_plan_desc(plan.handle, which, i, C.byref(d)))
    return d


def liver_plan_set_launch(plan: Plan, grid_blocks: int = 0, tile_order: int = -1, cache_hints: int = -1) -> None:
    _check(_lib.liver_plan_set_launch(plan.handle, grid_blocks, tile_order, cache_hints))


def _addr(x) -> int:
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    return x.data_ptr()          # torch tensor (device memory)


def _checked(t, need: int, what: str) -> int:
    """Address of a device tensor after checking what a raw pointer cannot tell the library: that it is device
    memory, contiguous and at least `need` bytes long (a short buffer would be a GPU memory fault)."""
    if t is None or isinstance(t, int):
        return _addr(t)           # raw address: the caller vouches for it, as through the C ABI
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{what}: must be a contiguous device tensor")
    have = t.numel() * t.element_size()
    if have < need:
        raise ValueError(f"{what}: {have} bytes, the plan needs {need}")
    return t.data_ptr()


def _table(bufs, n_ranks: int, plan: "Plan" = None, side: int = 0):
    """{(rank, kind): tensor | address} -> void*[n_ranks*NUM_KINDS]; tensors are size-checked against the plan."""
    if not isinstance(bufs, dict):
        return bufs               # already a ctypes array
    arr = (C.c_void_p * (n_ranks * NUM_KINDS))()
    for (rank, kind), t in bufs.items():
        if not (0 <= rank < n_ranks and 0 <= kind < NUM_KINDS):
            raise ValueError(f"buffer key {(rank, kind)} out of range")
        need = plan._buffer_bytes(side, rank, kind) if plan is not None else 0
        arr[rank * NUM_KINDS + kind] = _checked(t, need, f"{'target' if side else 'source'} buffer {(rank, kind)}")
    return arr


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def liver_pack(plan: Plan, chunk: int, src_bufs, staging, stream=None) -> None:
    _check(_lib.liver_pack(plan.handle, chunk, _table(src_bufs, plan.src.n_ranks, plan, 0),
                           _checked(staging, plan.chunk_bytes, "staging chunk"), _stream(stream)))


def liver_unpack(plan: Plan, chunk: int, staging, dst_bufs, stream=None) -> None:
    _check(_lib.liver_unpack(plan.handle, chunk, _checked(staging, plan.chunk_bytes, "staging chunk"),
                             _table(dst_bufs, plan.dst.n_ranks, plan, 1), _stream(stream)))


def liver_reshard(plan: Plan, src_bufs, dst_bufs, stream=None) -> None:
    _check(_lib.liver_reshard(plan.handle, _table(src_bufs, plan.src.n_ranks, plan, 0),
                              _table(dst_bufs, plan.dst.n_ranks, plan, 1), _stream(stream)))


def liver_reshard_staged(plan: Plan, src_bufs, dst_bufs, staging, stream_pack=None, stream_unpack=None) -> None:
    """staging: list of device chunks (tensors or addresses) of chunk_bytes each."""
    arr = (C.c_void_p * len(staging))(*[_checked(t, plan.chunk_bytes, "staging chunk") for t in staging])
    _check(_lib.liver_reshard_staged(plan.handle, _table(src_bufs, plan.src.n_ranks, plan, 0),
                                     _table(dst_bufs, plan.dst.n_ranks, plan, 1),
                                     arr, len(staging), _stream(stream_pack), _stream(stream_unpack)))


def liver_reshard_staged_fused(plan: Plan, src_bufs, dst_bufs, staging_even, staging_odd, stream=None) -> None:
    _check(_lib.liver_reshard_staged_fused(plan.handle, _table(src_bufs, plan.src.n_ranks, plan, 0),
                                           _table(dst_bufs, plan.dst.n_ranks, plan, 1),
                                           _checked(staging_even, plan.chunk_bytes, "staging chunk"),
                                           _checked(staging_odd, plan.chunk_bytes, "staging chunk"), _stream(stream)))


def liver_reshard_static(plan: Plan, src_bufs, dst_bufs, stream=None) -> None:
    _check(_lib.liver_reshard_static(plan.handle, _table(src_bufs, plan.src.n_ranks, plan, 0),
                                     _table(dst_bufs, plan.dst.n_ranks, plan, 1), _stream(stream)))


def liver_static_staging_bytes() -> int:
    return int(_lib.liver_static_staging_bytes())


def liver_debug_emulate_host(plan: Plan, which: int, chunk: int, src_bufs, dst_bufs, staging) -> None:
    """Run the lowered descriptors on HOST arrays ({(rank, kind): numpy array}); test aid."""
    def table(bufs, n):
        arr = (C.c_void_p * (n * NUM_KINDS))()
        for (rank, kind), a in (bufs or {}).items():
            arr[rank * NUM_KINDS + kind] = a.ctypes.data
        return arr
    _check(_lib.liver_debug_emulate_host(plan.handle, which, chunk, table(src_bufs, plan.src.n_ranks),
                                         table(dst_bufs, plan.dst.n_ranks),
                                         staging.ctypes.data if staging is not None else None))


def liver_debug_bandwidth_probe(mode: int, src, dst, nbytes: int, grid: int, stream=None) -> None:
    """Plain read (0) / fill (1) / copy (2) of nbytes of device memory; src, dst: tensors or addresses."""
    _check(_lib.liver_debug_bandwidth_probe(mode, _addr(src) if src is not None else None, _addr(dst) if dst is not None else None,
                                            nbytes, grid, _stream(stream)))


def make_table(bufs: Dict[Tuple[int, int], object], n_ranks: int, plan: Plan = None, side: int = 0):
    """Marshal a buffer dictionary once, for repeated calls (size-checked if the plan and its side are given)."""
    return _table(bufs, n_ranks, plan, side)

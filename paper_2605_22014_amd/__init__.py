"""MI355X-native online resharding of mixed-parallel training state.

Thin Python binding over libliver.so (argument marshalling only; every step of
the path runs in the library's HIP kernels).  Importing this package fails
loudly if the library has not been built: there is no fallback path.
"""
from ._binding import (ADAM_M, ADAM_V, MASTER, PARAM, EXPERT_PARAM, EXPERT_MASTER, EXPERT_ADAM_M, EXPERT_ADAM_V, NUM_KINDS, LiverError, Layout, ModelSpec, Plan, PlanInfo, Desc,
                       LIST_DIRECT, LIST_PACK, LIST_UNPACK, OP_COPY, OP_CAST_BF16, OP_ZERO,
                       liver_pack, liver_plan_buffer_bytes, liver_plan_buffer_used, liver_plan_create,
                       liver_plan_desc, liver_plan_desc_count, liver_plan_destroy, liver_plan_info,
                       liver_plan_set_launch, liver_reshard, liver_reshard_staged, liver_reshard_staged_fused, liver_reshard_static, liver_static_staging_bytes, liver_debug_emulate_host, liver_debug_bandwidth_probe, liver_strerror, liver_unpack, library_path)

from .generation import GenerationManager, GenerationError, State  # noqa: E402

__all__ = [n for n in dir() if not n.startswith("_")]

"""Generation state machine around one reshard (host-side, no GPU work of its own).

LiveR runs two worlds side by side: the Active World of generation k keeps
training while the Shadow World of generation k+1 is prepared, and a
deterministic state machine Stable -> Prepare -> Ready -> Switch -> Cleanup
moves from one to the other (LiveR, Section 4.5.1).  Only the data handoff of
that life cycle is in scope here, so this class drives exactly that:

  * generation ids are monotonic; at most two generations exist at a time;
  * planning (Prepare) touches metadata only and can be cancelled at any time
    before the switch, leaving the active world untouched (a stale handoff is
    dropped: Section 7);
  * the reshard (Switch) never writes the active world's buffers; the active
    world is replaced only after the target is complete ("commit"), so a failure
    during the transfer leaves generation k intact (invariant I4, Section 4.8);
  * requests arriving during Switch are queued and served afterwards.

The executor is injectable so the state machine can be tested without a GPU; by
default it is liver_reshard followed by a stream synchronisation.
"""
from __future__ import annotations

import enum
from collections import deque
from typing import Callable, Deque, Dict, Optional, Tuple

from . import _binding as lv


class State(enum.Enum):
    STABLE = "stable"
    PREPARE = "prepare"
    READY = "ready"
    SWITCH = "switch"
    CLEANUP = "cleanup"


class GenerationError(RuntimeError):
    pass


def _default_executor(plan, src_bufs, dst_bufs, stream) -> None:
    import torch
    lv.liver_reshard(plan, src_bufs, dst_bufs, stream)
    (stream or torch.cuda.current_stream()).synchronize()


class GenerationManager:
    def __init__(self, spec: lv.ModelSpec, layout: lv.Layout, bufs: Dict[Tuple[int, int], object],
                 chunk_bytes: int = 512 << 20, executor: Callable = _default_executor,
                 planner: Callable = lv.liver_plan_create):
        self.spec, self.chunk_bytes = spec, chunk_bytes
        self.generation = 0
        self.state = State.STABLE
        self.active_layout, self.active_bufs = layout, bufs
        self._shadow_layout: Optional[lv.Layout] = None
        self._shadow_bufs = None
        self._plan = None
        self._queue: Deque[lv.Layout] = deque()
        self._executor, self._planner = executor, planner

    # -- Prepare: plan for generation k+1 (metadata only) -------------------------------------------------
    def request(self, target: lv.Layout):
        """A resize request.  Served at once when Stable, queued while a handoff is in flight."""
        if self.state is not State.STABLE:
            self._queue.append(target)
            return None
        self._plan = self._planner(self.spec, self.active_layout, target, self.chunk_bytes)
        self._shadow_layout, self.state = target, State.PREPARE
        return self._plan

    def shadow_ready(self, dst_bufs) -> None:
        """The shadow world's storage exists (allocated by the caller): Prepare -> Ready."""
        if self.state is not State.PREPARE:
            raise GenerationError(f"shadow_ready in state {self.state.value}")
        self._shadow_bufs, self.state = dst_bufs, State.READY

    def cancel(self) -> None:
        """Drop a handoff that has not switched yet; generation k stays as it is."""
        if self.state not in (State.PREPARE, State.READY):
            raise GenerationError(f"cancel in state {self.state.value}")
        self._drop_shadow()
        self.state = State.STABLE

    # -- Switch: transfer, then commit --------------------------------------------------------------------
    def switch(self, stream=None) -> int:
        """Ready -> Switch -> Cleanup -> Stable.  Returns the new generation id.  If the transfer raises,
        the manager falls back to Stable on the OLD generation (its buffers were never written)."""
        if self.state is not State.READY:
            raise GenerationError(f"switch in state {self.state.value}")
        self.state = State.SWITCH
        try:
            self._executor(self._plan, self.active_bufs, self._shadow_bufs, stream)
        except Exception:
            self._drop_shadow()
            self.state = State.STABLE
            raise
        # commit: only now does the shadow world become the active one
        self.active_layout, self.active_bufs = self._shadow_layout, self._shadow_bufs
        self.generation += 1
        self.state = State.CLEANUP
        self._drop_shadow()
        self.state = State.STABLE
        if self._queue:                                   # serve the newest queued request, drop stale ones
            target = self._queue.pop()
            self._queue.clear()
            self.request(target)
        return self.generation

    def _drop_shadow(self) -> None:
        """Forget the plan and the shadow world (after a commit the shadow buffers live on as the active ones)."""
        if isinstance(self._plan, lv.Plan):
            lv.liver_plan_destroy(self._plan)
        self._plan = self._shadow_layout = self._shadow_bufs = None

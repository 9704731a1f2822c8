"""GPU-side test helpers: device buffers for a world, running the HIP path."""
import numpy as np
import torch

import paper_2605_22014_amd as lv

NP = {0: np.uint16, 1: np.uint32, 2: np.uint32, 3: np.uint32}
TT = {0: torch.int16, 1: torch.int32, 2: torch.int32, 3: torch.int32}
SENT = {0: -23131, 1: -1515870811, 2: -1515870811, 3: -1515870811}     # 0xA5 bytes


def to_dev(world):
    return {key: torch.from_numpy(np.ascontiguousarray(a).view(np.int16 if a.dtype == np.uint16 else np.int32)).cuda()
            for key, a in world.items()}


def to_host(bufs):
    return {key: t.cpu().numpy().view(NP[key[1]]) for key, t in bufs.items()}


def alloc_dst(plan, only_used=False):
    out = {}
    for r in range(plan.dst.n_ranks):
        for k in range(4):
            if only_used and not lv.liver_plan_buffer_used(plan, 1, r, k):
                continue
            n = lv.liver_plan_buffer_bytes(plan, 1, r, k) // (2 if k == 0 else 4)
            out[(r, k)] = torch.full((n,), SENT[k], dtype=TT[k], device="cuda")
    return out


def run_direct(plan, src_dev, only_used=False):
    dst = alloc_dst(plan, only_used)
    lv.liver_reshard(plan, src_dev, dst)
    torch.cuda.synchronize()
    return dst


def run_staged(plan, src_dev, order=None, only_used=False):
    dst = alloc_dst(plan, only_used)
    staging = torch.empty(plan.chunk_bytes, dtype=torch.uint8, device="cuda")
    n = lv.liver_plan_info(plan).n_chunks
    for c in (order if order is not None else range(n)):
        staging.fill_(0x3C)                      # stale bytes between payloads must not matter
        lv.liver_pack(plan, c, src_dev, staging)
        lv.liver_unpack(plan, c, staging, dst)
    torch.cuda.synchronize()
    return dst


def check_against(got_dev, want, plan, what=""):
    """Planned buffers equal the oracle's; unplanned ones still hold the sentinel."""
    got = to_host(got_dev)
    for (r, k), g in got.items():
        if lv.liver_plan_buffer_used(plan, 1, r, k):
            w = want[(r, k)]
            assert g.shape == w.shape, (what, r, k, g.shape, w.shape)
            if not np.array_equal(g, w):
                bad = np.flatnonzero(g != w)
                raise AssertionError(f"{what} rank {r} kind {k}: {bad.size} mismatches, first {bad[:4]}: "
                                     f"{g[bad[:4]]} vs {w[bad[:4]]}")
        else:
            assert (g == (SENT[k] & (0xFFFF if k == 0 else 0xFFFFFFFF))).all(), (what, "unplanned buffer written", r, k)

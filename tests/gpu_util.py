"""GPU-side test helpers: device buffers for a world, running the HIP path."""
import numpy as np
import torch

import paper_2605_22014_amd as lv

NP = {k: (np.uint16 if k % 4 == 0 else np.uint32) for k in range(8)}          # kinds 4..7: expert buffers
TT = {k: (torch.int16 if k % 4 == 0 else torch.int32) for k in range(8)}
SENT = {k: (-23131 if k % 4 == 0 else -1515870811) for k in range(8)}          # 0xA5 bytes


def to_dev(world):
    return {key: torch.from_numpy(np.ascontiguousarray(a).view(np.int16 if a.dtype == np.uint16 else np.int32)).cuda()
            for key, a in world.items()}


def to_host(bufs):
    return {key: t.cpu().numpy().view(NP[key[1]]) for key, t in bufs.items()}


def alloc_dst(plan, only_used=False):
    out = {}
    for r in range(plan.dst.n_ranks):
        for k in range(8):
            if only_used and not lv.liver_plan_buffer_used(plan, 1, r, k):
                continue
            n = lv.liver_plan_buffer_bytes(plan, 1, r, k) // (2 if k % 4 == 0 else 4)
            if n == 0:                           # expert kinds of a dense model
                continue
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


def run_fused(plan, src_dev, only_used=False):
    """The staged reshard with unpack(k-1) and pack(k) fused into one launch, through two staging chunks."""
    dst = alloc_dst(plan, only_used)
    a = torch.full((plan.chunk_bytes,), 0x3C, dtype=torch.uint8, device="cuda")
    b = torch.full((plan.chunk_bytes,), 0xC3, dtype=torch.uint8, device="cuda")
    lv.liver_reshard_staged_fused(plan, src_dev, dst, a, b)
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
            assert (g == (SENT[k] & (0xFFFF if k % 4 == 0 else 0xFFFFFFFF))).all(), (what, "unplanned buffer written", r, k)

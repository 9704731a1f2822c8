"""One pack / unpack / reshard / static-staging sequence for a HIP API trace (run under
`rocprofv3 --hip-trace --stats`, the program directly after `--`): every device buffer is allocated BEFORE
the plan is created; between liver_plan_create (one hipMalloc: the descriptor table) and liver_plan_destroy
(its hipFree) the data calls must show no hipMalloc* / hipFree* at all (bounded-memory guarantee of LiveR,
Appendix A.1, Theorem 1: extra memory = staging chunk + plan metadata).  Prints the buffer sizes so the
trace's allocation sizes can be told apart."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import torch  # noqa: E402

import liver_synth as synth  # noqa: E402
import paper_2605_22014_amd as lv  # noqa: E402


def main():
    cfg = synth.CONFIGS["gpt2_small"]
    spec = lv.ModelSpec(**cfg["spec"])
    src = lv.Layout(pad_multiple=cfg["pad_multiple"], **cfg["src"])
    dst = lv.Layout(pad_multiple=cfg["pad_multiple"], **cfg["dst"])
    probe = lv.liver_plan_create(spec, src, dst, cfg["chunk_bytes"])        # sizes only; destroyed before the traced part
    sizes = {(side, r, k): lv.liver_plan_buffer_bytes(probe, side, r, k)
             for side, lay in ((0, src), (1, dst)) for r in range(lay.n_ranks) for k in range(4)}
    lv.liver_plan_destroy(probe)
    bufs = {key: torch.zeros(n, dtype=torch.uint8, device="cuda") for key, n in sizes.items()}
    staging = torch.zeros(cfg["chunk_bytes"], dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    torch.cuda.synchronize()
    src_bufs = {(r, k): t for (side, r, k), t in bufs.items() if side == 0}
    dst_bufs = {(r, k): t for (side, r, k), t in bufs.items() if side == 1}
    print("ALLOC-TRACE: buffers allocated; plan creation follows", flush=True)
    plan = lv.liver_plan_create(spec, src, dst, cfg["chunk_bytes"])
    info = lv.liver_plan_info(plan)
    print(f"ALLOC-TRACE: plan created, table_bytes_device {info.table_bytes_device}, {info.n_chunks} chunks", flush=True)
    from paper_2605_22014_amd._binding import make_table
    st, dt = make_table(src_bufs, src.n_ranks, plan, 0), make_table(dst_bufs, dst.n_ranks, plan, 1)
    for c in range(info.n_chunks):
        lv.liver_pack(plan, c, st, staging, stream)
        lv.liver_unpack(plan, c, staging, dt, stream)
    lv.liver_reshard(plan, st, dt, stream)
    lv.liver_reshard_static(plan, st, dt, stream)
    torch.cuda.synchronize()
    print("ALLOC-TRACE: data calls done; plan destruction follows", flush=True)
    lv.liver_plan_destroy(plan)
    print("ALLOC-TRACE: plan destroyed", flush=True)


if __name__ == "__main__":
    main()

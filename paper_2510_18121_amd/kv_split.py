"""Query shards with a sub-range of their context, timed (the extension the paper names in its Limitations section).

A lone CA-task with few query rows and a long context has too few (tile, head) units to fill the GPU; cut into key
windows it becomes many partial tasks of one fused call, whose results ca_merge_partials combines.  This script
times, through the C ABI and with inputs resident in HBM:

  * one task (q_len rows at the end of a kv_len-token document) whole, and cut into windows of several lengths:
    ca_forward [+ merge], and ca_forward + merge + ca_backward + ca_sum_partial_dq;
  * the merge kernel alone (bytes moved per second against the HBM rate).

    python -m paper_2510_18121_amd.kv_split [--q-lens 256,1024] [--kv-len 131072] [--windows 0,32768,8192,2048]

prints one JSON line per case (window 0 = the task whole).  Needs the GPU library.
"""
from __future__ import annotations

import argparse
import json

import numpy as np

from . import workloads as W


def _timed(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def time_task(q_len: int, kv_len: int, window: int, hq: int = 32, hkv: int = 8, d: int = 128, steps: int = 5,
              warmup: int = 2) -> dict:
    """Milliseconds of the forward and of forward + backward for one task, whole (window 0) or by key windows."""
    import torch

    from . import binding as B

    dev = torch.device("cuda:0")
    b = W.custom([kv_len], [(0, kv_len - q_len, q_len)], hq, hkv, d, seed=41)
    q, k, v, d_o = W.make_tensors(b, dev)
    fl = b.flops()
    if window <= 0:
        pb, n_parts = b, 1
        qp, dop = q, d_o
    else:
        pb, gather, part_rows = W.split_kv(b, window)
        n_parts = int(part_rows.shape[0])
        g = torch.as_tensor(gather, device=dev)
        pr = torch.as_tensor(part_rows, device=dev).contiguous()
        qp, dop = q.index_select(0, g).contiguous(), d_o.index_select(0, g).contiguous()
    plan = B.ca_plan(pb)
    ws = B.alloc_workspace(plan, dev)
    o_p = torch.empty_like(qp)
    lse_p = torch.empty((hq, pb.total_q), dtype=torch.float32, device=dev)
    o, lse = torch.empty_like(q), torch.empty((hq, b.total_q), dtype=torch.float32, device=dev)
    dq_p, dq, dk, dv = torch.empty_like(qp), torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)

    def fwd():
        B.ca_forward(plan, qp, k, v, o_p, lse_p, ws)
        if window > 0:
            B.ca_merge_partials(pr, o_p, lse_p, o, lse, o_p, lse_p)

    def fwd_bwd():
        fwd()
        B.ca_backward(plan, qp, k, v, o_p, dop, lse_p, dq_p, dk, dv, ws)
        if window > 0:
            B.ca_sum_partial_dq(pr, dq_p, dq)

    f_ms, t_ms = _timed(fwd, steps, warmup), _timed(fwd_bwd, steps, warmup)
    info = plan.info()
    return {"q_len": q_len, "kv_len": kv_len, "window": window, "n_parts": n_parts, "partial_rows": int(pb.total_q),
            "fwd_units": info["n_fwd_units"], "bwd_units": info["n_bwd_units"],
            "fwd_ms": f_ms, "fwd_bwd_ms": t_ms, "fwd_tflops": fl["fwd"] / f_ms / 1e9,
            "fwd_bwd_tflops": fl["total"] / t_ms / 1e9}


def time_merge(n_rows: int = 131072, n_parts: int = 4, hq: int = 32, d: int = 128, steps: int = 10, warmup: int = 3) -> dict:
    """The merge kernel alone, with write-back: algorithmic bytes = n_rows hq (2 d + 4) (n_parts read + 1 + n_parts
    written) + the index array."""
    import torch

    from . import binding as B

    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(42)
    tq = n_rows * n_parts
    o_part = torch.randn((tq, hq, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    lse_part = torch.randn((hq, tq), generator=g, device=dev)
    # part i of row r sits at row i * n_rows + r: contiguous runs, as split_kv lays the partial tasks out
    pr = torch.as_tensor(np.arange(tq, dtype=np.int32).reshape(n_parts, n_rows), device=dev)
    o = torch.empty((n_rows, hq, d), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((hq, n_rows), dtype=torch.float32, device=dev)
    o_b, lse_b = torch.empty_like(o_part), torch.empty_like(lse_part)
    ms = _timed(lambda: B.ca_merge_partials(pr, o_part, lse_part, o, lse, o_b, lse_b), steps, warmup)
    ms_nb = _timed(lambda: B.ca_merge_partials(pr, o_part, lse_part, o, lse), steps, warmup)
    ms_dq = _timed(lambda: B.ca_sum_partial_dq(pr, o_part, o), steps, warmup)
    per = n_rows * hq * (2 * d + 4)
    idx = 4 * n_rows * n_parts
    return {"kernel": "ca_merge_kernel", "n_rows": n_rows, "n_parts": n_parts, "n_q_heads": hq, "head_dim": d,
            "merge_write_back_ms": ms, "merge_write_back_gbs": (per * (2 * n_parts + 1) + idx) / ms / 1e6,
            "merge_ms": ms_nb, "merge_gbs": (per * (n_parts + 1) + idx) / ms_nb / 1e6,
            "sum_dq_ms": ms_dq, "sum_dq_gbs": (n_rows * hq * 2 * d * (n_parts + 1) + idx) / ms_dq / 1e6}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--q-lens", default="256,1024")
    ap.add_argument("--kv-len", type=int, default=131072)
    ap.add_argument("--windows", default="0,32768,8192,2048")
    args = ap.parse_args()
    for ql in [int(x) for x in args.q_lens.split(",")]:
        for w in [int(x) for x in args.windows.split(",")]:
            print(json.dumps(time_task(ql, args.kv_len, w)), flush=True)
    print(json.dumps(time_merge()), flush=True)


if __name__ == "__main__":
    main()

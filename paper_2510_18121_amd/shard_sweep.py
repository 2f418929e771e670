"""Throughput of one fused call against the length of the shards it is made of (Section 3.3, the experiment
behind "divisibility and kernel composability"): 32K-token chunks of equal-length shards with random context
sizes, several chunks per shard length; reports causal TFLOP/s of ca_forward and of ca_forward + ca_backward.

    python -m paper_2510_18121_amd.shard_sweep [--mode distinct|shared] [--lengths 16,32,...] [--chunks 3]

prints one JSON line per shard length.  Needs the GPU library; the chunks come from workloads.shard_chunk.
"""
from __future__ import annotations

import argparse
import json

from . import workloads as W
from .profiler import time_batch


def sweep(mode: str, lengths, chunks: int = 3, steps: int = 5, warmup: int = 2):
    out = []
    for n in lengths:
        f_fl = t_fl = f_ms = t_ms = 0.0
        for c in range(chunks):
            b = W.shard_chunk(n, mode, seed=c)
            fl = b.flops()
            f_ms += time_batch(b, steps, warmup, backward=False)
            t_ms += time_batch(b, steps, warmup, backward=True)
            f_fl += fl["fwd"]
            t_fl += fl["total"]
        out.append({"mode": mode, "shard_len": n, "chunks": chunks, "shards_per_chunk": 32768 // n,
                    "fwd_tflops": f_fl / (f_ms * 1e-3) / 1e12, "fwd_bwd_tflops": t_fl / (t_ms * 1e-3) / 1e12,
                    "fwd_ms_per_chunk": f_ms / chunks, "fwd_bwd_ms_per_chunk": t_ms / chunks})
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mode", default="distinct", choices=["distinct", "shared"])
    ap.add_argument("--lengths", default="16,32,64,128,256,512,1024,2048,4096")
    ap.add_argument("--chunks", type=int, default=3)
    args = ap.parse_args()
    for row in sweep(args.mode, [int(x) for x in args.lengths.split(",")], args.chunks):
        print(json.dumps(row), flush=True)


if __name__ == "__main__":
    main()

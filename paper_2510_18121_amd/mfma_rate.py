"""Sustained dense bf16 matrix-pipe rate of the device, measured with `ca_mfma_stream`.

The published peak (2.5 PFLOP/s) assumes the maximum engine clock; under a stream of MFMAs the chip lowers its clock,
by an amount that depends on the operand data.  This module times the library's MFMA-only kernel over the whole chip
on operands of a chosen kind and returns TFLOP/s: the rate the attention kernels' *executed* flops can be compared
with, next to the published peak their roofline fraction is quoted against.

    python -m paper_2510_18121_amd.mfma_rate          # a table over operand data, side work and waves per SIMD
    python -m paper_2510_18121_amd.mfma_rate --kind normal --side-work 1 --launches 3     # one line of it
"""
from __future__ import annotations

import math

from . import binding as B

FLOPS_PER_MFMA = 2 * 32 * 32 * 16
KINDS = ("zeros", "ones", "normal", "softmax")


def make_operands(kind: str, device="cuda", seed: int = 5):
    """bf16 [16][256][8] operand fragments: even fragments are A operands, odd ones B operands.

    zeros / ones: constants; normal: A and B i.i.d. N(0,1) (the benchmark's Q, K, V, dO); softmax: A N(0,1), B
    exp(-3u) with u uniform in (0,1) (values in (0.05, 1) like unnormalised probabilities)."""
    import torch
    g = torch.Generator(device="cpu").manual_seed(seed)
    if kind == "zeros":
        x = torch.zeros(16, 256, 8)
    elif kind == "ones":
        x = torch.ones(16, 256, 8)
    elif kind == "normal":
        x = torch.randn(16, 256, 8, generator=g)
    elif kind == "softmax":
        x = torch.randn(16, 256, 8, generator=g)
        x[1::2] = torch.exp(-3.0 * torch.rand(8, 256, 8, generator=g))
    else:
        raise ValueError(f"kind {kind!r}: one of {KINDS}")
    return x.to(torch.bfloat16).to(device)


def sustained_tflops(kind: str = "normal", side_work: int = 0, workgroups_per_cu: int = 1, launch_ms: float = 250.0,
                     launches: int = 3, device="cuda"):
    """TFLOP/s of each of `launches` back-to-back launches of about launch_ms each (the first ones run while the
    clock is still settling; take the last as the sustained figure).  workgroups_per_cu = 1 puts one wave on every
    SIMD (the dK/dV kernel's occupancy), 2 two (the forward and dQ kernels'); side_work as in `ca_mfma_stream`."""
    import torch
    ops = make_operands(kind, device)
    n_cu = torch.cuda.get_device_properties(device).multi_processor_count
    n_wg = workgroups_per_cu * n_cu
    sums = torch.empty((n_wg, 256), dtype=torch.float32, device=device)
    # a SIMD issues an MFMA every 32 cycles at best; assume 1.5 GHz to size the launch, rounded to whole rounds
    n_mfma = max(64, int(launch_ms * 1e-3 * 1.5e9 / 32 / workgroups_per_cu) // 64 * 64)
    B.ca_mfma_stream(ops, 64, sums, side_work)  # code object loaded, clocks woken
    torch.cuda.synchronize(device)
    out = []
    for _ in range(launches):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B.ca_mfma_stream(ops, n_mfma, sums, side_work)
        e1.record()
        e1.synchronize()
        out.append(n_wg * 4 * n_mfma * FLOPS_PER_MFMA / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return out


def main():
    import argparse
    ap = argparse.ArgumentParser(description="sustained bf16 MFMA rate of the device (ca_mfma_stream)")
    ap.add_argument("--kind", choices=KINDS, help="operand data; without it a table over kinds, side work and occupancy")
    ap.add_argument("--side-work", type=int, default=0, choices=(0, 1, 2))
    ap.add_argument("--workgroups-per-cu", type=int, default=1)
    ap.add_argument("--launches", type=int, default=5)
    args = ap.parse_args()
    table = (("normal", 0, 1), ("normal", 0, 2), ("normal", 0, 8), ("normal", 1, 1), ("normal", 1, 2), ("normal", 2, 1),
             ("normal", 2, 2), ("zeros", 0, 1), ("ones", 0, 1), ("softmax", 0, 1), ("normal", 0, 1))
    if args.kind:
        table = ((args.kind, args.side_work, args.workgroups_per_cu),)
    print(f"operands  side_work  workgroups/CU   TFLOP/s of {args.launches} back-to-back launches of about 0.25 s")
    for kind, side, wpc in table:
        r = sustained_tflops(kind, side, wpc, launches=args.launches)
        print(f"{kind:8s}  {side:9d}  {wpc:13d}   " + "  ".join(f"{x:7.1f}" for x in r), flush=True)


if __name__ == "__main__":
    main()

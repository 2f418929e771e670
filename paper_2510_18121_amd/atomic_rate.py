"""What a dQ accumulated with fp32 atomics would cost on this device, measured with `ca_atomic_stream`.

A backward kernel that owns KV tiles and computes S and dP only once (5 contractions) must add one 64 x head_dim fp32
partial dQ tile (32 KiB at head_dim 128) per (128-key tile, 64-row query block, head) step to memory that other
workgroups add to as well.  This module times that: per step and wave, 80 MFMAs (the five contractions of such a
step) and 32 atomic-add instructions (the wave's quarter of the tile), against the MFMAs alone.

    python -m paper_2510_18121_amd.atomic_rate
"""
from __future__ import annotations

from . import binding as B
from .mfma_rate import FLOPS_PER_MFMA, make_operands


def time_steps(mfma_per_step, atomics_per_step, n_tiles=32, steps=2000, workgroups_per_cu=1, device="cuda"):
    """(ns per step, TB/s of atomic adds, TFLOP/s of MFMAs, sum check) of one launch over the whole chip."""
    import torch
    ops = make_operands("normal", device)
    n_wg = workgroups_per_cu * torch.cuda.get_device_properties(device).multi_processor_count
    tiles = torch.zeros((8, n_tiles, 8192), dtype=torch.float32, device=device)
    sums = torch.empty((n_wg, 256), dtype=torch.float32, device=device)
    B.ca_atomic_stream(ops, tiles, n_wg, 4, mfma_per_step, atomics_per_step, sums)
    torch.cuda.synchronize(device)
    tiles.zero_()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    B.ca_atomic_stream(ops, tiles, n_wg, steps, mfma_per_step, atomics_per_step, sums)
    e1.record()
    e1.synchronize()
    ms = e0.elapsed_time(e1)
    adds = n_wg * steps * atomics_per_step * 256
    ok = float(tiles.double().sum().item()) == float(adds)
    return (ms * 1e6 / steps, adds * 4 / (ms * 1e-3) / 1e12,
            n_wg * 4 * steps * mfma_per_step * FLOPS_PER_MFMA / (ms * 1e-3) / 1e12, ok)


def main():
    print("MFMAs/step  atomics/step  tiles/region  wg/CU   ns/step   atomics TB/s   MFMA TFLOP/s   sum exact")
    for mf, at, nt, wpc in ((80, 0, 32, 1), (0, 32, 32, 1), (0, 32, 1024, 1), (0, 32, 32, 2), (80, 32, 32, 1),
                            (80, 16, 32, 1), (80, 8, 32, 1), (64, 0, 32, 1)):
        ns, tbs, tf, ok = time_steps(mf, at, nt, workgroups_per_cu=wpc)
        print(f"{mf:10d}  {at:12d}  {nt:12d}  {wpc:5d}  {ns:8.0f}  {tbs:13.2f}  {tf:13.0f}   {ok}", flush=True)


if __name__ == "__main__":
    main()

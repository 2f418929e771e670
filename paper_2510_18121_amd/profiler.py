"""Latency model of one CA-task on an attention server (Section 4.2, "Profiler").

The paper's scheduler prices a CA-task from measurements: core attention is benchmarked over a grid of query
lengths and key-value lengths; a task's time is the bilinear interpolation of the four nearest grid points, and
where the kernel is at peak throughput (the saturation region) the time is derived from the highest measured
throughput instead.  This module holds that model (`LatencyGrid`, plain host code) and the routine that fills a
grid by timing the HIP path (`measure_grid`, needs the GPU library).
"""
from __future__ import annotations

import bisect
import json
from dataclasses import dataclass

import numpy as np

from . import workloads as W


def task_flops(q_len: int, kv_len: int, hq: int, d: int, backward: bool = True) -> float:
    """Causal flops of a task whose last query row sees kv_len keys (Appendix B: work proportional to
    n_q (2 n_kv - n_q); here with the diagonal counted exactly), 2 contractions forward and 5 backward."""
    pairs = W.task_pairs(kv_len - q_len, q_len)
    return (14.0 if backward else 4.0) * d * hq * pairs


@dataclass
class LatencyGrid:
    """Measured seconds t[i][j] of a task with q_len = q_axis[i] and kv_len = kv_axis[j] (kv_len >= q_len;
    entries with kv_len < q_len are NaN and never used)."""

    q_axis: np.ndarray
    kv_axis: np.ndarray
    seconds: np.ndarray  # [len(q_axis), len(kv_axis)]
    n_q_heads: int
    head_dim: int
    backward: bool = True
    saturation_tolerance: float = 0.05  # a grid point within 5 % of the best throughput counts as saturated

    def __post_init__(self):
        self.q_axis = np.asarray(self.q_axis, np.int64)
        self.kv_axis = np.asarray(self.kv_axis, np.int64)
        self.seconds = np.asarray(self.seconds, np.float64)
        assert self.seconds.shape == (len(self.q_axis), len(self.kv_axis))
        assert np.all(np.diff(self.q_axis) > 0) and np.all(np.diff(self.kv_axis) > 0)

    # ---- derived tables
    def throughput(self) -> np.ndarray:
        """flop/s at every grid point (NaN where unmeasured)."""
        f = np.array([[task_flops(int(q), int(kv), self.n_q_heads, self.head_dim, self.backward) if kv >= q else np.nan
                       for kv in self.kv_axis] for q in self.q_axis])
        return f / self.seconds

    def max_throughput(self) -> float:
        return float(np.nanmax(self.throughput()))

    def saturated(self) -> np.ndarray:
        with np.errstate(invalid="ignore"):
            return self.throughput() >= (1.0 - self.saturation_tolerance) * self.max_throughput()

    # ---- prediction
    def _cell(self, axis, x):
        """Indices (lo, hi) of the grid lines around x and the weight of hi; clamped at the ends."""
        j = bisect.bisect_right(axis.tolist(), x) - 1
        j = max(0, min(j, len(axis) - 2))
        w = (x - axis[j]) / float(axis[j + 1] - axis[j])
        return j, j + 1, min(1.0, max(0.0, w))

    def predict(self, q_len: int, kv_len: int) -> float:
        """Seconds for a task of q_len query rows whose last row sees kv_len keys."""
        if kv_len < q_len or q_len < 1:
            raise ValueError("a task needs 1 <= q_len <= kv_len")
        i0, i1, wi = self._cell(self.q_axis, q_len)
        j0, j1, wj = self._cell(self.kv_axis, kv_len)
        corners = [(i0, j0, (1 - wi) * (1 - wj)), (i0, j1, (1 - wi) * wj), (i1, j0, wi * (1 - wj)), (i1, j1, wi * wj)]
        sat = self.saturated()
        if all(np.isfinite(self.seconds[i, j]) and sat[i, j] for i, j, _ in corners):
            # saturation region: the kernel runs at its best measured rate
            return task_flops(q_len, kv_len, self.n_q_heads, self.head_dim, self.backward) / self.max_throughput()
        have = [(i, j, w) for i, j, w in corners if np.isfinite(self.seconds[i, j])]
        if len(have) == 4:
            return float(sum(w * self.seconds[i, j] for i, j, w in have))
        # A cell cut by the diagonal kv_len = q_len has unmeasured corners (no task has fewer keys than rows).  Two
        # estimates from the measured ones, weights renormalised: their seconds (too high where they hold several
        # times the task's work: long tasks on a coarse grid), and their seconds PER FLOP times the task's own flops
        # (too high where a fixed cost dominates: short tasks).  Each errs upwards in its own regime; the smaller is
        # taken.
        tot = sum(w for _, _, w in have)
        if not have:
            raise ValueError("no measured grid point around the task")
        if tot <= 0:  # the task sits on unmeasured corners only: the measured corners of the cell, equally
            have, tot = [(i, j, 1.0) for i, j, _ in have], float(len(have))
        fl = lambda i, j: task_flops(int(self.q_axis[i]), int(self.kv_axis[j]), self.n_q_heads, self.head_dim, self.backward)
        by_seconds = sum(w * self.seconds[i, j] for i, j, w in have) / tot
        per_flop = sum(w * self.seconds[i, j] / fl(i, j) for i, j, w in have) / tot
        return float(min(by_seconds, per_flop * task_flops(q_len, kv_len, self.n_q_heads, self.head_dim, self.backward)))

    # ---- storage (JSON text)
    def to_json(self) -> str:
        return json.dumps({"q_axis": self.q_axis.tolist(), "kv_axis": self.kv_axis.tolist(),
                           "seconds": [[None if not np.isfinite(x) else x for x in row] for row in self.seconds.tolist()],
                           "n_q_heads": self.n_q_heads, "head_dim": self.head_dim, "backward": self.backward,
                           "saturation_tolerance": self.saturation_tolerance})

    @staticmethod
    def from_json(text: str) -> "LatencyGrid":
        o = json.loads(text)
        sec = np.array([[np.nan if x is None else x for x in row] for row in o["seconds"]], np.float64)
        return LatencyGrid(o["q_axis"], o["kv_axis"], sec, o["n_q_heads"], o["head_dim"], o["backward"],
                           o["saturation_tolerance"])


def time_batch(batch, steps: int = 5, warmup: int = 2, backward: bool = True):
    """Milliseconds per call of ca_forward (+ ca_backward) on `batch` through the C ABI, inputs resident."""
    import torch

    from . import binding as B

    dev = torch.device("cuda:0")
    q, k, v, d_o = W.make_tensors(batch, dev)
    plan = B.ca_plan(batch)
    ws = B.alloc_workspace(plan, dev)
    o = torch.empty_like(q)
    lse = torch.empty((batch.n_q_heads, batch.total_q), dtype=torch.float32, device=dev)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)

    def step():
        B.ca_forward(plan, q, k, v, o, lse, ws)
        if backward:
            B.ca_backward(plan, q, k, v, o, d_o, lse, dq, dk, dv, ws)

    for _ in range(warmup):
        step()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def measure_grid(q_axis, kv_axis, hq: int = 32, hkv: int = 8, d: int = 128, backward: bool = True,
                 steps: int = 5, warmup: int = 2, fill_tokens: int = 0, max_kv_rows: int = 1 << 21) -> LatencyGrid:
    """Times a task (one document of kv_len tokens, its last q_len tokens as the query shard) at every grid point with
    kv_len >= q_len.

    fill_tokens = 0: the task alone on the GPU (what a single small call costs; a lone task cannot fill 256 CUs).
    fill_tokens > 0: the task's cost INSIDE a fused call, which is what an attention server runs and what the paper's
    own kernel measurement does (Section 3.3: chunks packed with equal shards): a batch of n copies of the task, each
    with a document of its own, n = fill_tokens / q_len (capped so that the copies' KV stays below max_kv_rows rows),
    timed as one call and divided by n."""
    sec = np.full((len(q_axis), len(kv_axis)), np.nan)
    for i, ql in enumerate(q_axis):
        for j, kl in enumerate(kv_axis):
            if kl < ql:
                continue
            n = 1
            if fill_tokens > 0:
                n = max(1, min(int(fill_tokens) // int(ql), int(max_kv_rows) // int(kl)))
            b = W.custom([int(kl)] * n, [(t, int(kl - ql), int(ql)) for t in range(n)], hq, hkv, d, seed=11)
            sec[i, j] = time_batch(b, steps, warmup, backward) * 1e-3 / n
    return LatencyGrid(np.asarray(q_axis), np.asarray(kv_axis), sec, hq, d, backward)


def main():
    import argparse

    ap = argparse.ArgumentParser(description="Measure the CA-task latency grid on this GPU and print it.")
    ap.add_argument("--q", default="16,64,128,256,512,1024,2048,4096,8192,16384")
    ap.add_argument("--kv", default="128,512,2048,8192,32768,131072")
    ap.add_argument("--heads", default="32,8")
    ap.add_argument("--forward-only", action="store_true")
    ap.add_argument("--json", action="store_true", help="print the grid as one JSON line (LatencyGrid.from_json reads it)")
    ap.add_argument("--fill-tokens", type=int, default=0,
                    help="time every task inside a fused call of this many query tokens of equal tasks (0: alone)")
    args = ap.parse_args()
    hq, hkv = (int(x) for x in args.heads.split(","))
    g = measure_grid([int(x) for x in args.q.split(",")], [int(x) for x in args.kv.split(",")], hq, hkv, 128,
                     backward=not args.forward_only, fill_tokens=args.fill_tokens)
    if args.json:
        print(g.to_json())
        return
    thr, sat = g.throughput(), g.saturated()
    print(f"latency in microseconds (TFLOP/s; * = saturation region), {hq}/{hkv} heads, head_dim 128, "
          f"{'forward' if args.forward_only else 'forward + backward'}; best {g.max_throughput() / 1e12:.0f} TFLOP/s")
    print("| q_len \\ kv_len | " + " | ".join(str(int(k)) for k in g.kv_axis) + " |")
    print("|---|" + "---|" * len(g.kv_axis))
    for i, ql in enumerate(g.q_axis):
        cells = []
        for j in range(len(g.kv_axis)):
            cells.append("" if not np.isfinite(g.seconds[i, j]) else
                         f"{g.seconds[i, j] * 1e6:.0f} ({thr[i, j] / 1e12:.0f}{'*' if sat[i, j] else ''})")
        print(f"| {int(ql)} | " + " | ".join(cells) + " |")


if __name__ == "__main__":
    main()

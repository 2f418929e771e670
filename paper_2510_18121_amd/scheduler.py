"""Communication-aware greedy scheduler of CA-tasks over attention servers (Section 4.2, "Scheduling units" and
the three steps of the scheduling algorithm) with the communication cost function of Appendix B.

Host-side only.  An Item is a whole document or a shard of one, resident on the server that runs its
context-independent layers; its core attention is one CA-task (query rows [q_pos, q_pos + q_len) of the document
against the document's first q_pos + q_len tokens).  The scheduler moves Items, or parts of Items, from servers
above the mean load to servers below it, each time taking the candidate with the most FLOPs moved per byte sent,
until every server is within eps of the mean or no move is worth its bytes.

An Item's load is priced either by its causal (query, key) pairs, exactly (workloads.task_pairs; FLOPs are a
constant multiple), or - as in the paper, whose scheduler takes its costs from the Profiler - by the seconds a
measured `profiler.LatencyGrid` predicts for its CA-task; pairs are the fallback without a grid.  Below the kernel's
saturation region (short shards, short contexts) time is far from proportional to pairs, and only the grid sees that.
The cost function works on the paper's continuous form n_q (2 n_kv - n_q).  Items here are contiguous; Appendix B's
head-tail Items (a piece from the front of a document paired with its mirror image from the back) are not built.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

from . import workloads as W


# ------------------------------------------------------------------------------------------- Appendix B
def shard_work(n_q: float, n_kv: float) -> float:
    """Appendix B's measure of a shard's work: n_q (2 n_kv - n_q) (twice the pair count, up to the diagonal)."""
    return n_q * (2.0 * n_kv - n_q)


def comm_bytes(n_q: float, n_kv: float, size_q: float, size_kv: float) -> float:
    """Bytes to move a shard of n_q query tokens with a context of n_kv key-value tokens (Appendix B, Comm)."""
    return n_q * size_q + n_kv * size_kv


def sub_shard_bounds(alpha: float, L_q: float, L_kv: float):
    """Range of n_q over which a contiguous sub-shard of an Item (L_q query tokens, last of which sees L_kv keys)
    can carry the fraction alpha of the Item's work (Appendix B's constraints 0 < n_q <= L_q and
    n_q + L_kv - L_q <= n_kv <= L_kv with n_q (2 n_kv - n_q) = alpha L_q (2 L_kv - L_q)).

    n_q is smallest when the sub-shard is the Item's LAST rows (n_kv = L_kv) and largest when it is the Item's
    FIRST rows (n_kv = n_q + L_kv - L_q)."""
    c = alpha * shard_work(L_q, L_kv)
    lo = L_kv - math.sqrt(max(0.0, L_kv * L_kv - c))
    g = L_kv - L_q
    hi = -g + math.sqrt(g * g + c)
    return lo, min(hi, L_q)


def n_kv_for(alpha: float, L_q: float, L_kv: float, n_q: float) -> float:
    """Context length of the sub-shard of n_q rows that carries the fraction alpha of the Item's work."""
    return 0.5 * (alpha * shard_work(L_q, L_kv) / n_q + n_q)


def min_comm(alpha: float, L_q: float, L_kv: float, size_q: float, size_kv: float):
    """Appendix B: the cheapest sub-shard (n_q, n_kv, bytes) that carries the fraction alpha of an Item's work.

    Comm(n_q) = size_q (n_q (1 + beta/2) + alpha beta L_q (2 L_kv - L_q) / (2 n_q)), beta = size_kv / size_q, is
    convex with its minimum at n_q_opt = sqrt(alpha beta L_q (2 L_kv - L_q) / (beta + 2)); outside the feasible
    range the nearest end of the range is optimal."""
    if not (0.0 < alpha <= 1.0):
        raise ValueError("alpha must be in (0, 1]")
    beta = size_kv / size_q
    lo, hi = sub_shard_bounds(alpha, L_q, L_kv)
    n_opt = math.sqrt(alpha * beta * shard_work(L_q, L_kv) / (beta + 2.0))
    n_q = min(max(n_opt, lo), hi)
    n_kv = n_kv_for(alpha, L_q, L_kv, n_q)
    return n_q, n_kv, comm_bytes(n_q, n_kv, size_q, size_kv)


# ------------------------------------------------------------------------------------------- scheduler
@dataclass
class Item:
    """A whole document or a contiguous shard of one, resident on its home server; it maps one to one to a CA-task
    (Section 4.2, "Item"): query rows q_pos .. q_pos + q_len - 1 of document `doc` with the prefix before them."""

    doc: int
    q_pos: int   # document position of the first query row
    q_len: int
    home: int    # server that holds the tokens (and their K/V) before scheduling

    @property
    def kv_len(self) -> int:
        """Keys the Item's last row sees: its own rows plus the context before them."""
        return self.q_pos + self.q_len

    @property
    def pairs(self) -> int:
        """Exact (query, key) pairs of the Item: its load, in units of one score."""
        return W.task_pairs(self.q_pos, self.q_len)


def item_cost(item: "Item", grid=None) -> float:
    """Load of an Item: the seconds the latency grid predicts for its CA-task (Section 4.2, "Profiler"), or, without
    a grid, its exact pair count."""
    if grid is None:
        return float(item.pairs)
    return float(grid.predict(item.q_len, item.kv_len))


@dataclass
class Schedule:
    """Result of `schedule`: which Items every attention server computes, and what moving them cost."""

    servers: list                      # per server: list of Items it computes
    moved_bytes: float = 0.0           # by the cost model (every move pays for its queries and its whole context)
    moves: list = field(default_factory=list)   # (source, destination, Item moved, bytes)
    grid: object = None                # the LatencyGrid the loads were priced with, or None for pair counts

    def loads(self, grid="own"):
        """Per-server load: predicted seconds under `grid` (default: the grid the schedule was made with), pairs
        when that is None."""
        g = self.grid if isinstance(grid, str) else grid
        return [sum(item_cost(it, g) for it in s) for s in self.servers]

    def imbalance(self, grid="own") -> float:
        """max load / mean load."""
        ld = self.loads(grid)
        mean = sum(ld) / len(ld)
        return max(ld) / mean if mean > 0 else 1.0


def _cut(item: Item, alpha: float, size_q: float, size_kv: float, block: int):
    """The sub-shard of `item` that carries about the fraction alpha of its work and that Appendix B's cost function
    prefers, on a grid of `block` rows: returns (moved Item, remaining Items, modelled bytes)."""
    L_q, L_kv = item.q_len, item.kv_len
    alpha = min(1.0, alpha)
    want_pairs = alpha * item.pairs
    n_q, n_kv, _ = min_comm(alpha, L_q, L_kv, size_q, size_kv)
    n = int(round(n_q / block)) * block
    n = max(block, min(n, (L_q // block) * block if L_q >= block else L_q))
    n = min(n, L_q)
    # first row of the cut: the one that gives the wanted work for this row count, on the grid, inside the Item
    a_best, err_best = None, None
    a_real = n_kv_for(alpha, L_q, L_kv, n) - n
    for a in {int(math.floor(a_real / block)) * block, int(math.ceil(a_real / block)) * block}:
        a = max(item.q_pos, min(a, item.q_pos + L_q - n))
        err = abs(W.task_pairs(a, n) - want_pairs)
        if err_best is None or err < err_best:
            a_best, err_best = a, err
    a = a_best
    moved = Item(item.doc, a, n, item.home)
    rest = []
    if a > item.q_pos:
        rest.append(Item(item.doc, item.q_pos, a - item.q_pos, item.home))
    if a + n < item.q_pos + L_q:
        rest.append(Item(item.doc, a + n, item.q_pos + L_q - (a + n), item.home))
    return moved, rest, comm_bytes(n, a + n, size_q, size_kv)


def schedule(items, n_servers: int, size_q: float, size_kv: float, eps: float = 0.05, min_gain: float = 0.0,
             block: int = 16, max_moves: int = 100000, grid=None) -> Schedule:
    """Section 4.2, steps 1-3.

    items: Items, each on its home server.  size_q / size_kv: bytes per query token and per key-value token.
    eps: tolerance on a server's load relative to the mean.  min_gain: a move must carry at least this much load
    per byte (the paper's "small threshold" on the priority score E; in pairs per byte, or seconds per byte with a
    grid).  block: granularity of cuts in rows.  grid: a `profiler.LatencyGrid`; loads are then the predicted seconds
    of the Items' CA-tasks (the paper's Profiler), otherwise exact pair counts.  A cut takes the fraction of the
    Item's WORK (Appendix B works in flops) that equals the wanted fraction of its load; the pieces are then priced
    anew, so the books stay exact in either unit."""
    servers = [[] for _ in range(n_servers)]
    for it in items:
        servers[it.home].append(it)
    sch = Schedule(servers, grid=grid)
    cost = lambda it: item_cost(it, grid)
    load = sch.loads()
    total = sum(load)
    mean = total / n_servers
    if total == 0:
        return sch
    for _ in range(max_moves):
        # step 3 (checked first): every server within eps of the mean load
        if all(abs(x - mean) <= eps * mean for x in load):
            break
        # step 1: deficit servers, largest deficit first
        deficits = sorted((d for d in range(n_servers) if load[d] < mean), key=lambda d: load[d])
        progressed = False
        for d in deficits:
            need = mean - load[d]
            # step 2: the candidate with the most load moved per byte
            best = None
            for s in range(n_servers):
                surplus = load[s] - mean
                if s == d or surplus <= 0:
                    continue
                for idx, it in enumerate(servers[s]):
                    f_item = cost(it)
                    df = min(f_item, surplus, need)
                    if df <= 0:
                        continue
                    if df >= f_item:
                        v = comm_bytes(it.q_len, it.kv_len, size_q, size_kv)
                    else:
                        v = min_comm(df / f_item, it.q_len, it.kv_len, size_q, size_kv)[2]
                    e = df / v
                    if best is None or e > best[0]:
                        best = (e, s, idx, df, f_item)
            if best is None or best[0] < min_gain:
                continue
            e, s, idx, df, f_item = best
            it = servers[s].pop(idx)
            if df >= f_item or it.q_len <= block:
                moved, rest, v = it, [], comm_bytes(it.q_len, it.kv_len, size_q, size_kv)
            else:
                moved, rest, v = _cut(it, df / f_item, size_q, size_kv, block)
            servers[s].extend(rest)
            servers[d].append(Item(moved.doc, moved.q_pos, moved.q_len, moved.home))
            load[s] += sum(cost(r) for r in rest) - f_item
            load[d] += cost(moved)
            if grid is not None:  # predicted times of pieces need not add up to the whole Item's
                mean = sum(load) / n_servers
            sch.moved_bytes += v
            sch.moves.append((s, d, moved, v))
            progressed = True
            break  # loads changed: recompute the deficit order
        # step 3: ... or no move is worth its bytes
        if not progressed:
            break
    return sch


def items_from_batch(batch, n_servers: int):
    """Initial placement for an experiment: the batch's tasks in packed-Q order are dealt to the servers as
    n_servers contiguous runs of (nearly) equal token counts - the fixed-token data-parallel chunks of the
    paper's baselines - each task becoming an Item on the server its first token falls on."""
    order = sorted(range(batch.n_tasks), key=lambda t: int(batch.task_q_start[t]))
    per = batch.total_q / n_servers
    out = []
    for t in order:
        home = min(n_servers - 1, int(int(batch.task_q_start[t]) // per))
        out.append(Item(int(batch.task_doc[t]), int(batch.task_q_pos[t]), int(batch.task_q_len[t]), home))
    return out


def server_batch(batch, items, name="server"):
    """The fused call of one attention server: its Items as CA-tasks over compacted copies of the documents'
    needed KV prefixes.  Returns (Batch, q row gather, kv row gather) into the original packed buffers; Items must
    come from `batch` (their query rows are located through the batch's task table)."""
    import numpy as np

    docs = sorted({it.doc for it in items})
    need = {d: max(it.kv_len for it in items if it.doc == d) for d in docs}
    # query rows of an Item in the original packed Q: through the task that covers its positions
    tasks_of = {}
    for t in range(batch.n_tasks):
        tasks_of.setdefault(int(batch.task_doc[t]), []).append(t)
    q_rows = []
    for it in items:
        rows = np.full(it.q_len, -1, np.int64)
        for t in tasks_of[it.doc]:
            p0, n, a = int(batch.task_q_pos[t]), int(batch.task_q_len[t]), int(batch.task_q_start[t])
            lo, hi = max(p0, it.q_pos), min(p0 + n, it.q_pos + it.q_len)
            if lo < hi:
                rows[lo - it.q_pos:hi - it.q_pos] = a + (np.arange(lo, hi) - p0)
        assert (rows >= 0).all(), "Item is not covered by the batch's tasks"
        q_rows.append(rows)
    kv_rows = [np.arange(batch.doc_kv_start[d], batch.doc_kv_start[d] + need[d]) for d in docs]
    sub = W.custom([need[d] for d in docs], [(docs.index(it.doc), it.q_pos, it.q_len) for it in items],
                   batch.n_q_heads, batch.n_kv_heads, batch.head_dim, scale=batch.softmax_scale, name=name)
    return sub, (np.concatenate(q_rows) if q_rows else np.zeros(0, np.int64)), \
        (np.concatenate(kv_rows) if kv_rows else np.zeros(0, np.int64))


def main():
    """Virtual attention servers on one GPU: schedule a workload's tasks over n servers for several tolerances,
    time every server's fused call (forward + backward) one after the other, report max / mean server time."""
    import argparse
    import json

    from .profiler import time_batch

    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, default=3)
    ap.add_argument("--servers", type=int, default=8)
    ap.add_argument("--eps", default="inf,0.2,0.1,0.05,0.02,0.01")
    ap.add_argument("--grid", action="store_true",
                    help="measure a latency grid first (Section 4.2, Profiler) and balance predicted seconds "
                         "instead of pair counts")
    ap.add_argument("--fill-tokens", type=int, default=32768,
                    help="with --grid: every grid point is timed inside a fused call of this many query tokens of "
                         "equal tasks (0: each task alone on the GPU)")
    args = ap.parse_args()
    b = W.config(args.workload)
    size_q = b.n_q_heads * b.head_dim * 2          # bf16 query token
    size_kv = 2 * b.n_kv_heads * b.head_dim * 2    # bf16 key + value token
    items = items_from_batch(b, args.servers)
    grid = None
    if args.grid:
        from .profiler import measure_grid
        grid = measure_grid([16, 64, 256, 1024, 4096, 16384], [128, 512, 2048, 8192, 32768, 131072], b.n_q_heads,
                            b.n_kv_heads, b.head_dim, steps=3, warmup=1, fill_tokens=args.fill_tokens)
    for e in args.eps.split(","):
        eps = float(e)
        sch = Schedule([[it for it in items if it.home == s] for s in range(args.servers)], grid=grid) \
            if math.isinf(eps) else schedule(items, args.servers, size_q, size_kv, eps=eps, grid=grid)
        ms = []
        for s, srv in enumerate(sch.servers):
            sub, _, _ = server_batch(b, srv, name=f"server{s}")
            ms.append(time_batch(sub, steps=3, warmup=1))
        print(json.dumps({"eps": e, "servers": args.servers, "workload": b.name, "moves": len(sch.moves),
                          "priced_by": "latency grid (s)" if grid is not None else "pairs",
                          "modelled_MB_moved": sch.moved_bytes / 1e6, "load_max_over_mean": sch.imbalance(),
                          "pairs_max_over_mean": sch.imbalance(grid=None),
                          "server_ms": [round(x, 2) for x in ms], "time_max_over_mean": max(ms) / (sum(ms) / len(ms)),
                          "slowest_server_ms": max(ms), "sum_ms": sum(ms)}), flush=True)


if __name__ == "__main__":
    main()

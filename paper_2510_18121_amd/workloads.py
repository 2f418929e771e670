"""Seeded synthetic CA-task batches and their input tensors.

This module is the one thing the CPU oracle's tests and the HIP path's tests share.
It holds no attention arithmetic: it only decides which documents exist, how they
are cut into CA-tasks (a query shard of one document attending to that document's
KV prefix; Section 4.1 "Runtime", definition of a CA-task), where the shards and
the documents' K/V live in the packed buffers, and which random bf16 values fill
Q, K, V and dO.  It also counts causal (query, key) pairs, which is bookkeeping
for the FLOP figure (Appendix B: work of a shard is proportional to
n_q (2 n_kv - n_q)).

The five workloads stand in for the paper's "Pretrain" / "ProLong" length
distributions (Section 6, experimental setup), which are not available here; their
shapes follow the five benchmark configurations this build is measured on.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np


@dataclass
class Batch:
    """One fused batch of CA-tasks in the C-ABI's descriptor form (host int64/int32 arrays)."""

    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    total_q: int
    total_kv: int
    doc_kv_start: np.ndarray  # int64 [n_docs] row of the doc's token 0 in packed K/V
    doc_kv_len: np.ndarray  # int64 [n_docs] resident KV rows of the doc
    task_doc: np.ndarray  # int32 [n_tasks]
    task_q_start: np.ndarray  # int64 [n_tasks] first row in packed Q
    task_q_len: np.ndarray  # int64 [n_tasks]
    task_q_pos: np.ndarray  # int64 [n_tasks] document position of the first query row
    task_kv_len: np.ndarray  # int64 [n_tasks] prefix attended (q_pos + q_len in the paper's case)
    softmax_scale: float = 0.0  # <= 0 selects 1/sqrt(head_dim)
    seed: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def n_docs(self) -> int:
        return int(self.doc_kv_len.shape[0])

    @property
    def n_tasks(self) -> int:
        return int(self.task_q_len.shape[0])

    @property
    def scale(self) -> float:
        return self.softmax_scale if self.softmax_scale > 0 else 1.0 / math.sqrt(self.head_dim)

    def pairs(self) -> int:
        """Exact number of (query row, visible key) pairs, diagonal included."""
        return int(sum(task_pairs(int(a), int(n), int(kv))
                       for a, n, kv in zip(self.task_q_pos, self.task_q_len, self.task_kv_len)))

    def flops(self) -> dict:
        """Causal FLOPs: 2 contractions forward, 5 backward, 2 flops per multiply-add."""
        p = self.pairs()
        f = 4 * self.head_dim * self.n_q_heads * p
        b = 10 * self.head_dim * self.n_q_heads * p
        return {"pairs": p, "fwd": f, "bwd": b, "total": f + b}


def task_pairs(q_pos: int, q_len: int, kv_len: int | None = None) -> int:
    """Pairs of a shard whose first query sits at document position q_pos: sum over its rows p of min(kv_len, p + 1)
    (kv_len None or >= q_pos + q_len: the full causal prefix, sum_p (p + 1))."""
    if kv_len is None or kv_len >= q_pos + q_len:
        return q_len * (2 * q_pos + q_len + 1) // 2
    c = max(0, kv_len - q_pos)  # rows that still see their whole prefix
    return c * (2 * q_pos + c + 1) // 2 + (q_len - c) * kv_len


def _mk(name, hq, hkv, d, doc_lens, doc_order, tasks, task_order, seed, meta=None) -> Batch:
    """Assemble a Batch.

    doc_lens: list of document lengths; doc_order: order in which the documents' K/V are
    laid out in the packed KV buffer; tasks: list of (doc, q_pos, q_len); task_order: order
    of the tasks' query rows in packed Q.
    """
    n_docs = len(doc_lens)
    doc_kv_start = np.zeros(n_docs, np.int64)
    off = 0
    for dd in doc_order:
        doc_kv_start[dd] = off
        off += doc_lens[dd]
    total_kv = off
    n_tasks = len(tasks)
    task_doc = np.zeros(n_tasks, np.int32)
    task_q_start = np.zeros(n_tasks, np.int64)
    task_q_len = np.zeros(n_tasks, np.int64)
    task_q_pos = np.zeros(n_tasks, np.int64)
    task_kv_len = np.zeros(n_tasks, np.int64)
    off = 0
    for t in task_order:
        dd, a, n = tasks[t]
        task_doc[t] = dd
        task_q_start[t] = off
        task_q_len[t] = n
        task_q_pos[t] = a
        task_kv_len[t] = a + n
        off += n
    return Batch(
        name=name, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, total_q=off, total_kv=total_kv,
        doc_kv_start=doc_kv_start, doc_kv_len=np.asarray(doc_lens, np.int64), task_doc=task_doc,
        task_q_start=task_q_start, task_q_len=task_q_len, task_q_pos=task_q_pos,
        task_kv_len=task_kv_len, seed=seed, meta=meta or {},
    )


def _fill_lengths(rng, total, draw, lo, hi, multiple=1):
    """Draw document lengths until `total` tokens are reached; the last one is cut to fit."""
    lens = []
    left = total
    while left > 0:
        n = int(draw(rng))
        if multiple > 1:
            n = int(round(n / multiple)) * multiple
        n = max(lo, min(hi, n))
        if n >= left or left - n < lo:
            n = left
        lens.append(n)
        left -= n
    return lens


def tiny(seed: int = 1) -> Batch:
    """Workload 1: documents of 512 and 1024 tokens, each cut in two at a seeded point."""
    rng = np.random.default_rng(seed)
    doc_lens = [512, 1024]
    tasks = []
    for dd, n in enumerate(doc_lens):
        s = int(rng.integers(1, n))  # 1 .. n-1, not rounded: ragged on purpose
        tasks += [(dd, 0, s), (dd, s, n - s)]
    return _mk("cfg1_tiny", 4, 2, 64, doc_lens, list(range(2)), tasks, list(range(len(tasks))), seed)


def packed_8b(seed: int = 2, total: int = 65536, shard: int = 4096, hq: int = 32, hkv: int = 8) -> Batch:
    """Workload 2: lognormal documents (median 2K, cap 32K) packed to `total`, 4096-token shards."""
    rng = np.random.default_rng(seed)
    cap = min(32768, total)
    lens = _fill_lengths(rng, total, lambda r: round(r.lognormal(math.log(2048), 1.0)), 16, cap)
    tasks = []
    for dd, n in enumerate(lens):
        a = 0
        while a < n:
            m = min(shard, n - a)
            tasks.append((dd, a, m))
            a += m
    return _mk("cfg2_8b_64k", hq, hkv, 128, lens, list(range(len(lens))), tasks, list(range(len(tasks))), seed)


def composability(seed: int = 3, total: int = 131072, hq: int = 32, hkv: int = 8, max_cut: int = 1024) -> Batch:
    """Workload 3: lognormal documents up to `total`, shards at random multiples of 16
    (16 .. 16*max_cut query rows), all shards shuffled in packed Q, documents shuffled in packed KV."""
    rng = np.random.default_rng(seed)
    lens = _fill_lengths(rng, total, lambda r: r.lognormal(math.log(4096), 1.5), 16, total, multiple=16)
    tasks = []
    for dd, n in enumerate(lens):
        a = 0
        while a < n:
            m = 16 * int(round(math.exp(rng.uniform(0.0, math.log(max_cut)))))
            m = min(m, n - a)
            tasks.append((dd, a, m))
            a += m
    task_order = [int(x) for x in rng.permutation(len(tasks))]
    doc_order = [int(x) for x in rng.permutation(len(lens))]
    return _mk("cfg3_composability_128k", hq, hkv, 128, lens, doc_order, tasks, task_order, seed)


def long_prefix(seed: int = 4, total: int = 524288, n_shards: int = 32, hq: int = 32, hkv: int = 8) -> Batch:
    """Workload 4: one document of `total` tokens in `n_shards` equal query shards."""
    n = total // n_shards
    tasks = [(0, k * n, n) for k in range(n_shards)]
    return _mk("cfg4_long_prefix_512k", hq, hkv, 128, [total], [0], tasks, list(range(n_shards)), seed)


def larger_model(seed: int = 5, total: int = 262144, hq: int = 64, hkv: int = 8, div: int = 1) -> Batch:
    """Workload 5: four long documents (32K-64K) plus a lognormal tail of short ones, cut into
    shards of roughly equal causal work (the inverse of the trapezoid pair count)."""
    rng = np.random.default_rng(seed)
    lo, hi = 32768 // div, 65536 // div
    step = max(16, 128 // div)
    long_docs = [int(rng.integers(lo // step, hi // step + 1)) * step for _ in range(4)]
    rest = total - sum(long_docs)
    short = _fill_lengths(rng, rest, lambda r: round(r.lognormal(math.log(1024 // div), 0.75)),
                          max(16, 256 // div), max(32, 4096 // div))
    lens = long_docs + short
    f_star = task_pairs(0, 8192 // div)
    tasks = []
    for dd, n in enumerate(lens):
        a = 0
        while a < n:
            b = int(math.isqrt(a * a + 2 * f_star)) // 16 * 16
            b = max(b, a + 16)
            if n - b < 16:
                b = n
            b = min(b, n)
            tasks.append((dd, a, b - a))
            a = b
    return _mk("cfg5_larger_256k", hq, hkv, 128, lens, list(range(len(lens))), tasks, list(range(len(tasks))), seed)


def shard_chunk(shard_len: int, mode: str = "distinct", seed: int = 0, chunk_tokens: int = 32768,
                max_context: int = 16384, hq: int = 8, hkv: int = 2, d: int = 128) -> Batch:
    """One chunk of the throughput-versus-shard-length experiment (Section 3.3, "Divisibility and kernel
    composability": a 32K-token chunk packed of document shards of one fixed length, the context size of each
    shard drawn at random, several chunks per length).

    mode "distinct": every shard comes from a document of its own; its context (the number of earlier tokens
    of that document, resident as KV) is a multiple of 16 drawn uniformly from [0, max_context].
    mode "shared": the chunk's shards are ALL the shards of chunk_tokens / max_context documents of max_context
    tokens each, in shuffled order - the case the paper's scheduler produces when it cuts a document and sends
    the pieces to one server.
    """
    rng = np.random.default_rng(7000 + 131 * seed + shard_len)
    n = chunk_tokens // shard_len
    assert n >= 1 and n * shard_len == chunk_tokens
    if mode == "distinct":
        ctx = 16 * rng.integers(0, max_context // 16 + 1, size=n)
        doc_lens = [int(c) + shard_len for c in ctx]
        tasks = [(i, int(ctx[i]), shard_len) for i in range(n)]
    elif mode == "shared":
        n_docs = max(1, chunk_tokens // max_context)
        per = chunk_tokens // n_docs
        assert per % shard_len == 0
        doc_lens = [per] * n_docs
        tasks = [(dd, a, shard_len) for dd in range(n_docs) for a in range(0, per, shard_len)]
    else:
        raise ValueError(mode)
    order = rng.permutation(len(tasks)).tolist()
    return _mk(f"shard_chunk_{mode}_{shard_len}", hq, hkv, d, doc_lens, list(range(len(doc_lens))), tasks, order,
               seed, {"shard_len": shard_len, "mode": mode})


def split_kv(b: Batch, window: int):
    """Cut every document's keys into windows of `window` tokens and every CA-task into one partial task per window
    it can see (a query shard attending a sub-range of its context: the extension named in the paper's Limitations
    section).  Pure bookkeeping: the packed K/V buffers stay as they are (a window is a sub-range of its document's
    rows and becomes a "document" of the new batch, positions counted from the window's first key); the query rows
    of a partial task are copies of the original rows.

    Returns (partial batch, gather, part_rows): gather [total_q'] = original packed-Q row of every row of the
    partial batch (to build its Q and dO, and to scatter results back); part_rows [n_parts, total_q] int32 = for every
    original row its rows in the partial batch, window by window, -1 where it has fewer windows.
    """
    assert window >= 1
    doc_start, doc_len, win_of_doc = [], [], []
    for dd in range(b.n_docs):
        ids = []
        for c in range(0, int(b.doc_kv_len[dd]), window):
            ids.append(len(doc_start))
            doc_start.append(int(b.doc_kv_start[dd]) + c)
            doc_len.append(min(window, int(b.doc_kv_len[dd]) - c))
        win_of_doc.append(ids)
    t_doc, t_start, t_len, t_pos, t_kv, gather = [], [], [], [], [], []
    n_parts = 1
    for t in range(b.n_tasks):
        a, n, kv = int(b.task_q_pos[t]), int(b.task_q_len[t]), int(b.task_kv_len[t])
        n_parts = max(n_parts, -(-min(kv, a + n) // window))
    part_rows = np.full((n_parts, b.total_q), -1, np.int32)
    off = 0
    for t in range(b.n_tasks):
        dd, a, n, kv = int(b.task_doc[t]), int(b.task_q_pos[t]), int(b.task_q_len[t]), int(b.task_kv_len[t])
        q0 = int(b.task_q_start[t])
        for w, wid in enumerate(win_of_doc[dd]):
            c = w * window
            if c >= min(kv, a + n):
                break  # no row of the task sees a key of this window
            first = max(a, c)  # first position that sees the window's first key
            m = a + n - first
            t_doc.append(wid)
            t_start.append(off)
            t_len.append(m)
            t_pos.append(first - c)
            t_kv.append(min(c + window, kv, int(b.doc_kv_len[dd])) - c)
            rows = np.arange(q0 + first - a, q0 + n)
            gather.append(rows)
            part_rows[w, rows] = off + np.arange(m)
            off += m
    nb = Batch(
        name=b.name + f"_kvsplit{window}", n_q_heads=b.n_q_heads, n_kv_heads=b.n_kv_heads, head_dim=b.head_dim,
        total_q=off, total_kv=b.total_kv, doc_kv_start=np.asarray(doc_start, np.int64),
        doc_kv_len=np.asarray(doc_len, np.int64), task_doc=np.asarray(t_doc, np.int32),
        task_q_start=np.asarray(t_start, np.int64), task_q_len=np.asarray(t_len, np.int64),
        task_q_pos=np.asarray(t_pos, np.int64), task_kv_len=np.asarray(t_kv, np.int64),
        softmax_scale=b.scale, seed=b.seed, meta={**b.meta, "kv_window": window},
    )
    g = np.concatenate(gather) if gather else np.zeros(0, np.int64)
    return nb, g.astype(np.int64), part_rows


def config(index: int, downscale: int = 1) -> Batch:
    """Workload `index` (1..5); downscale > 1 gives the token-count/downscale twin from the same generator."""
    s = downscale
    if index == 1:
        return tiny(1)
    if index == 2:
        b = packed_8b(2, total=65536 // s)
    elif index == 3:
        b = composability(3, total=131072 // s, max_cut=max(4, 1024 // s))
    elif index == 4:
        b = long_prefix(4, total=524288 // s)
    elif index == 5:
        b = larger_model(5, total=262144 // s, div=s)
    else:
        raise ValueError("workload index must be 1..5")
    if s > 1:
        b.name += f"_div{s}"
    return b


def one_kv_group(b: Batch) -> Batch:
    """The same batch restricted to a single KV head and its query-head group (cheaper oracle runs)."""
    g = b.n_q_heads // b.n_kv_heads
    return Batch(**{**b.__dict__, "n_q_heads": g, "n_kv_heads": 1, "name": b.name + "_1grp"})


def custom(doc_lens, tasks, hq, hkv, d, *, doc_order=None, task_order=None, seed=0, name="custom", scale=0.0) -> Batch:
    """A hand-specified batch: tasks are (doc, q_pos, q_len) triples."""
    b = _mk(name, hq, hkv, d, list(doc_lens), list(doc_order) if doc_order is not None else list(range(len(doc_lens))),
            list(tasks), list(task_order) if task_order is not None else list(range(len(tasks))), seed)
    b.softmax_scale = scale
    return b


def make_tensors(b: Batch, device="cpu", with_grad_out: bool = True):
    """Q, K, V (and dO) ~ N(0,1) rounded to bf16, from a generator seeded with the batch's seed.

    Returns torch bf16 tensors Q [total_q, Hq, D], K, V [total_kv, Hkv, D], dO like Q.  Values
    depend on the device type the generator runs on; the oracle always reads back the very bits
    the HIP path reads.
    """
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(1000 + b.seed)

    def rnd(n, h):
        out = torch.empty((n, h, b.head_dim), dtype=torch.bfloat16, device=device)
        step = max(1, (1 << 26) // (h * b.head_dim))
        for i in range(0, n, step):  # chunked so the fp32 staging stays small
            m = min(step, n - i)
            out[i:i + m] = torch.randn((m, h, b.head_dim), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
        return out

    q = rnd(b.total_q, b.n_q_heads)
    k = rnd(b.total_kv, b.n_kv_heads)
    v = rnd(b.total_kv, b.n_kv_heads)
    d_o = rnd(b.total_q, b.n_q_heads) if with_grad_out else None
    return q, k, v, d_o

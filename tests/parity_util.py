"""Helpers for the GPU parity tests: run the HIP path through the C ABI, run the oracle on the same bits."""
import numpy as np
import torch

import oracle
from paper_2510_18121_amd import binding as B
from paper_2510_18121_amd import workloads as W

O_MAX_ABS = 1e-2      # bf16 outputs vs fp64 oracle; where |O_ref| >= 4 the bf16 grid itself is coarser than that
                      # (spacing 2^-5), so there the bound is 2^-8 |O_ref| (between half a unit and one unit of the grid)
GRAD_REL_L2 = 1e-2    # dQ, dK, dV: ||g - g_ref||_2 / ||g_ref||_2
LSE_MAX_ABS = 1e-4    # fp32 log-sum-exp of N(0,1) inputs (values up to ~15; observed error 2e-6)
# Finer gradient figures asserted next to the whole-tensor relative L2 (which one wrong row or tile cannot move):
ROW_REL_L2 = 1e-1     # every (row, head) of dQ and every (key, head) of dK, dV: ||g - g_ref|| / max(||g_ref||, rms row
                      # norm of the tensor): a wrong row shows as about 1.  What a correct row can reach: ca_backward is
                      # given O in bf16 (the interface stores it so), the oracle its own fp64 O, so Delta = <dO, O>
                      # differs by about 2^-9 |O| |dO| sqrt(D), and dQ of a row by scale * that * ||sum_j P_j K_j||.  For
                      # rows with thousands of keys this is nothing; for the first rows of a document (|O| up to 3,
                      # one-hot P, ||K|| up to 14) it is 0.02 - 0.07 in absolute terms whatever the kernel does
                      # (observed maximum over all tests 0.067; rows past position ~100 stay below 0.01)
TILE_REL_L2 = 1e-2    # every run of 128 consecutive rows / keys
SUM_INVARIANT = 2e-2  # ||sum_j dV_j - sum dO|| and ||sum_j dK_j|| over a document, relative to ||dV||_F, ||dK||_F


def to64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def run_hip(batch, q, k, v, d_o=None, plan=None):
    """Forward (and backward when d_o is given) on cuda:0 through the C ABI.  Returns dict of device tensors."""
    own = plan is None
    plan = plan or B.ca_plan(batch)
    o = torch.full_like(q, float("nan"))
    lse = torch.full((batch.n_q_heads, batch.total_q), float("nan"), dtype=torch.float32, device=q.device)
    ws = B.alloc_workspace(plan, q.device)
    B.ca_forward(plan, q, k, v, o, lse, ws)
    out = {"o": o, "lse": lse, "plan": plan}
    if d_o is not None:
        dq = torch.full_like(q, float("nan"))
        dk = torch.full_like(k, float("nan"))
        dv = torch.full_like(v, float("nan"))
        B.ca_backward(plan, q, k, v, o, d_o, lse, dq, dk, dv, ws)
        out.update(dq=dq, dk=dk, dv=dv)
    torch.cuda.synchronize()
    if own:
        out["plan"] = plan
    return out


def run_hip_kv_split(batch, window, q, k, v, d_o=None, in_place=True):
    """The same results by way of key windows: every task cut into one partial task per `window` keys of its context,
    one fused forward over all partial tasks, ca_merge_partials, and (when d_o is given) ca_backward on the partial
    tasks with the merged O and LSE in their rows, then ca_sum_partial_dq.  Index plumbing (gathering the copies of
    Q and dO) is torch; every arithmetic step is a library call."""
    pb, gather, part_rows = W.split_kv(batch, window)
    dev = q.device
    g = torch.as_tensor(gather, device=dev)
    pr = torch.as_tensor(part_rows, device=dev).contiguous()
    qp = q.index_select(0, g).contiguous()
    plan = B.ca_plan(pb)
    ws = B.alloc_workspace(plan, dev)
    o_p = torch.full_like(qp, float("nan"))
    lse_p = torch.full((pb.n_q_heads, pb.total_q), float("nan"), dtype=torch.float32, device=dev)
    B.ca_forward(plan, qp, k, v, o_p, lse_p, ws)
    o = torch.full_like(q, float("nan"))
    lse = torch.full((batch.n_q_heads, batch.total_q), float("nan"), dtype=torch.float32, device=dev)
    if in_place:
        o_b, lse_b = o_p, lse_p
    else:
        o_b, lse_b = torch.full_like(o_p, float("nan")), torch.full_like(lse_p, float("nan"))
    B.ca_merge_partials(pr, o_p, lse_p, o, lse, o_b if d_o is not None else None, lse_b if d_o is not None else None)
    out = {"o": o, "lse": lse, "plan": plan, "partial_batch": pb, "n_parts": int(part_rows.shape[0])}
    if d_o is not None:
        dop = d_o.index_select(0, g).contiguous()
        dq_p = torch.full_like(qp, float("nan"))
        dk = torch.full_like(k, float("nan"))
        dv = torch.full_like(v, float("nan"))
        B.ca_backward(plan, qp, k, v, o_b, dop, lse_b, dq_p, dk, dv, ws)
        dq = torch.full_like(q, float("nan"))
        B.ca_sum_partial_dq(pr, dq_p, dq)
        out.update(dq=dq, dk=dk, dv=dv, o_back=o_b, lse_back=lse_b)
    torch.cuda.synchronize()
    return out


def run_oracle(batch, q, k, v, d_o=None, want=("dq", "dk", "dv")):
    q64, k64, v64 = to64(q), to64(k), to64(v)
    if d_o is None:
        o, lse = oracle.forward(batch, q64, k64, v64)
        return {"o": o, "lse": lse}
    return oracle.forward_backward(batch, q64, k64, v64, to64(d_o), want=want)


def o_errors(o_hip, o_ref):
    """Strict max-abs error, and the largest ratio of error to the allowed bound max(1e-2, 2^-8 |O_ref|)."""
    if o_ref.size == 0:
        return 0.0, 0.0, 0
    err = np.abs(o_hip - o_ref)
    bound = np.maximum(O_MAX_ABS, np.abs(o_ref) / 256.0)
    return float(err.max()), float((err / bound).max()), int((np.abs(o_ref) >= 4.0).sum())


def rel_l2(a, ref):
    den = float(np.linalg.norm(ref.ravel()))
    num = float(np.linalg.norm((a - ref).ravel()))
    return num / den if den > 0 else num


def row_and_tile_errors(a, ref, tile=128):
    """Largest relative L2 error of a single (row, head) and of a run of `tile` consecutive rows (all heads) of a
    gradient tensor [n, H, D].  Row norms below the tensor's rms row norm are measured against that norm
    (the first row of a document has dQ = 0 exactly)."""
    if ref.size == 0:
        return 0.0, 0.0
    n = ref.shape[0]
    d2 = ((a - ref) ** 2).sum(-1)          # [n, H]
    r2 = (ref ** 2).sum(-1)
    floor2 = max(float(r2.mean()), 1e-300)
    row = float(np.sqrt(d2 / np.maximum(r2, floor2)).max())
    m = (n + tile - 1) // tile
    pad = m * tile - n
    dt = np.pad(d2.sum(-1), (0, pad)).reshape(m, tile).sum(-1)
    rt = np.pad(r2.sum(-1), (0, pad)).reshape(m, tile).sum(-1)
    tl = float(np.sqrt(dt / np.maximum(rt, floor2 * tile * ref.shape[1])).max())
    return row, tl


def errors(hip, ref, rows=None):
    """Error figures of a HIP result against an oracle result (optionally only on the packed Q rows `rows`)."""
    sel = slice(None) if rows is None else rows
    oa, orat, big = o_errors(to64(hip["o"])[sel], ref["o"][sel])
    e = {"o_max_abs": oa, "o_err_over_bound": orat, "o_elems_ge_4": big,
         "lse_max_abs": float(np.abs(to64(hip["lse"])[:, sel] - ref["lse"][:, sel]).max()) if ref["lse"].size else 0.0}
    for g in ("dq", "dk", "dv"):
        if g in hip and ref.get(g) is not None:
            a, r = to64(hip[g]), ref[g]
            if g == "dq":
                a, r = a[sel], r[sel]
            e[g + "_rel_l2"] = rel_l2(a, r)
            e[g + "_row_rel_l2"], e[g + "_tile_rel_l2"] = row_and_tile_errors(a, r)
    return e


def assert_parity(e, tag="", row_bound=ROW_REL_L2):
    assert e["o_err_over_bound"] <= 1.0, (tag, e)
    assert e["o_max_abs"] <= O_MAX_ABS or e["o_elems_ge_4"] > 0, (tag, e)
    assert e["lse_max_abs"] <= LSE_MAX_ABS, (tag, e)
    for g in ("dq", "dk", "dv"):
        if g + "_rel_l2" in e:
            assert e[g + "_rel_l2"] <= GRAD_REL_L2, (tag, g, e)
        if g + "_row_rel_l2" in e:
            assert e[g + "_row_rel_l2"] <= row_bound, (tag, g, e)
            assert e[g + "_tile_rel_l2"] <= TILE_REL_L2, (tag, g, e)


def sum_invariants(batch, d_o, hip):
    """Two identities of the exact gradients, applied to the WHOLE GPU output per document and KV head:
    sum over the document's keys of dV = sum over its query rows (and the heads of the group) of dO, because every
    row's probabilities sum to 1; and sum over its keys of dK = 0, because a common shift of the keys changes no
    output.  Reductions in fp64 on the device.  Returns the largest ||sum dV - sum dO|| / ||dV||_F and
    ||sum dK|| / ||dK||_F over (document, KV head)."""
    dev = d_o.device
    g = batch.n_q_heads // batch.n_kv_heads
    worst_v = worst_k = 0.0
    for d in sorted(set(batch.task_doc.tolist())):
        rows = np.concatenate([np.arange(int(batch.task_q_start[t]), int(batch.task_q_start[t] + batch.task_q_len[t]))
                               for t in np.flatnonzero(batch.task_doc == d)])
        idx = torch.as_tensor(rows, device=dev)
        s_do = torch.zeros((batch.n_q_heads, batch.head_dim), dtype=torch.float64, device=dev)
        for i in range(0, len(rows), 1 << 16):
            s_do += d_o.index_select(0, idx[i:i + (1 << 16)]).double().sum(0)
        s_do = s_do.view(batch.n_kv_heads, g, batch.head_dim).sum(1)
        a, n = int(batch.doc_kv_start[d]), int(batch.doc_kv_len[d])
        dv, dk = hip["dv"][a:a + n].double(), hip["dk"][a:a + n].double()
        nv = torch.sqrt((dv ** 2).sum((0, 2)))  # per KV head
        nk = torch.sqrt((dk ** 2).sum((0, 2)))
        ev = torch.sqrt(((dv.sum(0) - s_do) ** 2).sum(-1))
        ek = torch.sqrt((dk.sum(0) ** 2).sum(-1))
        for h in range(batch.n_kv_heads):
            if nv[h] > 0:
                worst_v = max(worst_v, float(ev[h] / nv[h]))
            else:
                assert float(ev[h]) == 0.0
            # a document of one or two keys has dK = 0 up to fp32 noise: measure against at least 1 % of ||dV||_F
            den = max(float(nk[h]), 0.01 * float(nv[h]))
            if den > 0:
                worst_k = max(worst_k, float(ek[h]) / den)
            else:
                assert float(ek[h]) == 0.0
    return {"sum_dv_minus_sum_do_rel": worst_v, "sum_dk_rel": worst_k}


# ---------------------------------------------------------------- exact sub-problems of a large batch
def _row_owner(batch):
    """For every packed Q row: (task, document, position); -1 where no task covers the row."""
    task = np.full(batch.total_q, -1, np.int64)
    pos = np.full(batch.total_q, -1, np.int64)
    for t in range(batch.n_tasks):
        a, n = int(batch.task_q_start[t]), int(batch.task_q_len[t])
        task[a:a + n] = t
        pos[a:a + n] = batch.task_q_pos[t] + np.arange(n)
    doc = np.where(task >= 0, batch.task_doc[np.maximum(task, 0)], -1)
    return task, doc, pos


def sample_rows(batch, n_random, seed):
    """Packed Q rows to check exactly: first and last row of every task, every row of tasks shorter than
    128 rows (up to a cap), positions 0..31 of every document, plus a uniform random sample."""
    rng = np.random.default_rng(seed)
    task, doc, pos = _row_owner(batch)
    rows = set()
    for t in range(batch.n_tasks):
        a, n = int(batch.task_q_start[t]), int(batch.task_q_len[t])
        rows.update((a, a + n - 1))
        if n < 128:
            rows.update(range(a, a + n, max(1, n // 8)))
    rows.update(np.flatnonzero((pos >= 0) & (pos < 32)).tolist())
    rows.update(rng.choice(np.flatnonzero(task >= 0), size=min(n_random, batch.total_q), replace=False).tolist())
    return np.array(sorted(rows), np.int64)


def rows_subproblem(batch, rows, kv_head):
    """A batch whose tasks are the single rows `rows`, each attending its document's full prefix, restricted to
    one KV head and its query-head group.  Returns (sub batch, q row gather, kv row gather, head slice)."""
    task, doc, pos = _row_owner(batch)
    docs = sorted(set(doc[rows].tolist()))
    need = {d: int(pos[rows][doc[rows] == d].max()) + 1 for d in docs}  # keys needed per document
    g = batch.n_q_heads // batch.n_kv_heads
    kv_gather, doc_start, off = [], {}, 0
    for d in docs:
        doc_start[d] = off
        kv_gather.append(np.arange(batch.doc_kv_start[d], batch.doc_kv_start[d] + need[d]))
        off += need[d]
    kv_gather = np.concatenate(kv_gather)
    sub = W.custom([need[d] for d in docs], [(docs.index(int(doc[r])), int(pos[r]), 1) for r in rows],
                   g, 1, batch.head_dim, scale=batch.softmax_scale)
    return sub, rows, kv_gather, slice(kv_head * g, (kv_head + 1) * g)


def gather64(t, rows, heads):
    """Rows `rows` and heads `heads` of a device tensor [n, H, D] as fp64 numpy (exact widening of the bf16 bits)."""
    idx = torch.as_tensor(np.asarray(rows), device=t.device)
    return t.index_select(0, idx)[:, heads].float().cpu().numpy().astype(np.float64)


def check_sampled_rows(batch, tensors, hip, rows, kv_head):
    """O, LSE and dQ of the sampled rows against the oracle's exact values."""
    q, k, v, d_o = tensors
    sub, qrows, kvrows, hs = rows_subproblem(batch, rows, kv_head)
    hk = slice(kv_head, kv_head + 1)
    ref = oracle.forward_backward(sub, gather64(q, qrows, hs), gather64(k, kvrows, hk), gather64(v, kvrows, hk),
                                  gather64(d_o, qrows, hs), want=("dq",))
    o = gather64(hip["o"], qrows, hs)
    dq = gather64(hip["dq"], qrows, hs)
    lse = hip["lse"][hs][:, torch.as_tensor(qrows, device=q.device)].double().cpu().numpy()
    oa, orat, big = o_errors(o, ref["o"])
    row, _ = row_and_tile_errors(dq, ref["dq"])
    return {"o_max_abs": oa, "o_err_over_bound": orat, "o_elems_ge_4": big,
            "lse_max_abs": float(np.abs(lse - ref["lse"]).max()),
            "dq_rel_l2": rel_l2(dq, ref["dq"]), "dq_row_rel_l2": row, "rows": int(len(rows))}


def check_key_gradients(batch, tensors, hip, kv_head, short_doc_max=2048, tail_keys=512, require_full=True):
    """dK/dV exactly for (a) every document of at most short_doc_max keys, whole, and (b) the last tail_keys
    keys of the longest document (only the query rows at those positions see them).  With require_full, only
    documents all of whose rows are in the batch; without, also documents present with some of their rows (a shard
    and its context: the gradient of its keys is what those rows contribute)."""
    q, k, v, d_o = tensors
    task, doc, pos = _row_owner(batch)
    g = batch.n_q_heads // batch.n_kv_heads
    hs, hk = slice(kv_head * g, (kv_head + 1) * g), slice(kv_head, kv_head + 1)
    out = {}

    def run(docs, min_pos, tag):
        # tasks restricted to rows at positions >= min_pos[d]
        doc_list, tasks, qrows, kvrows = [], [], [], []
        for d in docs:
            L = int(batch.doc_kv_len[d])
            di = len(doc_list)
            doc_list.append(L)
            kvrows.append(np.arange(batch.doc_kv_start[d], batch.doc_kv_start[d] + L))
            for t in np.flatnonzero(batch.task_doc == d):
                a, n, p0 = int(batch.task_q_start[t]), int(batch.task_q_len[t]), int(batch.task_q_pos[t])
                lo = max(0, min_pos[d] - p0)
                if lo < n:
                    tasks.append((di, p0 + lo, n - lo))
                    qrows.append(np.arange(a + lo, a + n))
        sub = W.custom(doc_list, tasks, g, 1, batch.head_dim, scale=batch.softmax_scale)
        qrows, kvrows = np.concatenate(qrows), np.concatenate(kvrows)
        ref = oracle.forward_backward(sub, gather64(q, qrows, hs), gather64(k, kvrows, hk), gather64(v, kvrows, hk),
                                      gather64(d_o, qrows, hs), want=("dk", "dv"))
        off = 0
        dk_h, dv_h, dk_r, dv_r = [], [], [], []
        for d in docs:
            L = int(batch.doc_kv_len[d])
            lo = min_pos[d]
            sel = np.arange(off + lo, off + L)
            dk_r.append(ref["dk"][sel]), dv_r.append(ref["dv"][sel])
            dk_h.append(gather64(hip["dk"], kvrows[sel], hk)), dv_h.append(gather64(hip["dv"], kvrows[sel], hk))
            off += L
        out[tag + "_dk_rel_l2"] = rel_l2(np.concatenate(dk_h), np.concatenate(dk_r))
        out[tag + "_dv_rel_l2"] = rel_l2(np.concatenate(dv_h), np.concatenate(dv_r))
        out[tag + "_dk_row_rel_l2"] = max(row_and_tile_errors(a, r)[0] for a, r in zip(dk_h, dk_r))
        out[tag + "_dv_row_rel_l2"] = max(row_and_tile_errors(a, r)[0] for a, r in zip(dv_h, dv_r))
        out[tag + "_keys"] = int(sum(len(x) for x in dk_r))

    present = sorted(set(batch.task_doc.tolist()))
    full = {d for d in present if not require_full or
            sum(int(batch.task_q_len[t]) for t in np.flatnonzero(batch.task_doc == d)) == int(batch.doc_kv_len[d])}
    short = [d for d in present if batch.doc_kv_len[d] <= short_doc_max and d in full]
    if short:
        run(short, {d: 0 for d in short}, "short_docs")
    longest = max(present, key=lambda d: batch.doc_kv_len[d])
    if longest in full:
        run([longest], {longest: max(0, int(batch.doc_kv_len[longest]) - tail_keys)}, "tail")
    return out


def check_interior_key_tiles(batch, tensors, hip, tiles, width=128):
    """dK/dV of key windows in the INTERIOR of long documents, exactly.  For a window [lo, lo + width) of document d
    the gradient of its keys needs every query row of d at a position >= lo, but of each such row only its
    probabilities on the window's keys, and those follow from the row's saved log-sum-exp: the window is declared a
    document of `width` keys, the rows are clipped to it (kv_len = width, positions counted from lo), and the oracle's
    backward is given the O and LSE that ca_backward itself was given (Delta = <dO, O> and P = exp(s - LSE) are
    those of the whole row).  tiles: list of (document, lo, kv_head).  Returns the per-tile relative L2 errors."""
    q, k, v, d_o = tensors
    g = batch.n_q_heads // batch.n_kv_heads
    out = []
    for d, lo, kv_head in tiles:
        hs, hk = slice(kv_head * g, (kv_head + 1) * g), slice(kv_head, kv_head + 1)
        L = int(batch.doc_kv_len[d])
        w = min(width, L - lo)
        tasks, qrows, kvl = [], [], []
        for t in np.flatnonzero(batch.task_doc == d):
            a, n, p0 = int(batch.task_q_start[t]), int(batch.task_q_len[t]), int(batch.task_q_pos[t])
            first = max(0, lo - p0)
            if first < n and int(batch.task_kv_len[t]) > lo:
                tasks.append((0, p0 + first - lo, n - first))
                qrows.append(np.arange(a + first, a + n))
                kvl.append(min(w, int(batch.task_kv_len[t]) - lo))
        kvrows = np.arange(batch.doc_kv_start[d] + lo, batch.doc_kv_start[d] + lo + w)
        dk_h, dv_h = gather64(hip["dk"], kvrows, hk), gather64(hip["dv"], kvrows, hk)
        if not tasks:  # no query row sees the window: its gradient is zero
            dk, dv, qrows = np.zeros_like(dk_h), np.zeros_like(dv_h), []
        else:
            sub = W.custom([w], tasks, g, 1, batch.head_dim, scale=batch.scale)
            sub.task_kv_len[:] = np.minimum(np.asarray(kvl, np.int64), sub.task_q_pos + sub.task_q_len)
            qrows = np.concatenate(qrows)
            lse = hip["lse"][hs][:, torch.as_tensor(qrows, device=q.device)].double().cpu().numpy()
            _, dk, dv, _ = oracle.backward(sub, gather64(q, qrows, hs), gather64(k, kvrows, hk),
                                           gather64(v, kvrows, hk), gather64(hip["o"], qrows, hs),
                                           gather64(d_o, qrows, hs), lse, want=("dk", "dv"))
        out.append({"doc": int(d), "lo": int(lo), "kv_head": int(kv_head), "rows": int(len(qrows)),
                    "dk_rel_l2": rel_l2(dk_h, dk), "dv_rel_l2": rel_l2(dv_h, dv),
                    "dk_row_rel_l2": row_and_tile_errors(dk_h, dk)[0], "dv_row_rel_l2": row_and_tile_errors(dv_h, dv)[0]})
    return out


def interior_tiles(batch, seed, min_rows=32768, per_doc=4):
    """(document, first key, KV head) of the windows checked by check_interior_key_tiles: for every document of at
    least min_rows keys the first window, the middle one, the last, and per_doc - 3 seeded ones in between (multiples
    of 64, so that a window straddles two of the kernel's 128-key tiles every other time), KV heads rotating."""
    rng = np.random.default_rng(seed)
    tiles, h = [], int(rng.integers(0, batch.n_kv_heads))
    for d in range(batch.n_docs):
        L = int(batch.doc_kv_len[d])
        if L < min_rows or not np.any(batch.task_doc == d):
            continue
        los = [0, (L // 2) // 128 * 128, L - 128] + [int(rng.integers(1, L // 64 - 2)) * 64 for _ in range(max(0, per_doc - 3))]
        for lo in los:
            tiles.append((d, lo, h % batch.n_kv_heads))
            h += 1
    return tiles

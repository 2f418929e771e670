"""Helpers for the GPU parity tests: run the HIP path through the C ABI, run the oracle on the same bits."""
import numpy as np
import torch

import oracle
from paper_2510_18121_amd import binding as B
from paper_2510_18121_amd import workloads as W

O_MAX_ABS = 1e-2      # bf16 outputs vs fp64 oracle; where |O_ref| >= 4 the bf16 grid itself is coarser than that
                      # (spacing 2^-5), so there the bound is 2^-8 |O_ref| (between half a unit and one unit of the grid)
GRAD_REL_L2 = 1e-2    # dQ, dK, dV: ||g - g_ref||_2 / ||g_ref||_2
LSE_MAX_ABS = 2e-3    # fp32 log-sum-exp


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
    return e


def assert_parity(e, tag=""):
    assert e["o_err_over_bound"] <= 1.0, (tag, e)
    assert e["o_max_abs"] <= O_MAX_ABS or e["o_elems_ge_4"] > 0, (tag, e)
    assert e["lse_max_abs"] <= LSE_MAX_ABS, (tag, e)
    for g in ("dq", "dk", "dv"):
        if g + "_rel_l2" in e:
            assert e[g + "_rel_l2"] <= GRAD_REL_L2, (tag, e)


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
    return {"o_max_abs": oa, "o_err_over_bound": orat, "o_elems_ge_4": big,
            "lse_max_abs": float(np.abs(lse - ref["lse"]).max()),
            "dq_rel_l2": rel_l2(dq, ref["dq"]), "rows": int(len(rows))}


def check_key_gradients(batch, tensors, hip, kv_head, short_doc_max=2048, tail_keys=512):
    """dK/dV exactly for (a) every document of at most short_doc_max keys, whole, and (b) the last tail_keys
    keys of the longest document (only the query rows at those positions see them)."""
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
        out[tag + "_keys"] = int(sum(len(x) for x in dk_r))

    present = sorted(set(batch.task_doc.tolist()))
    full = {d for d in present if sum(int(batch.task_q_len[t]) for t in np.flatnonzero(batch.task_doc == d)) == int(batch.doc_kv_len[d])}
    short = [d for d in present if batch.doc_kv_len[d] <= short_doc_max and d in full]
    if short:
        run(short, {d: 0 for d in short}, "short_docs")
    longest = max(present, key=lambda d: batch.doc_kv_len[d])
    if longest in full:
        run([longest], {longest: max(0, int(batch.doc_kv_len[longest]) - tail_keys)}, "tail")
    return out

"""Pins for the CPU oracle: every check here is fixed by the paper's definition of core attention
(Section 2.1), of the CA-task and its composability (Sections 3.2 and 4.1), by Appendix B's
trapezoid work count, or by mathematics alone - never by the HIP path.  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2510_18121_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_inputs(b, seed=0, dtype=np.float64):
    r = np.random.default_rng(seed)
    q = r.standard_normal((b.total_q, b.n_q_heads, b.head_dim))
    k = r.standard_normal((b.total_kv, b.n_kv_heads, b.head_dim))
    v = r.standard_normal((b.total_kv, b.n_kv_heads, b.head_dim))
    d_o = r.standard_normal((b.total_q, b.n_q_heads, b.head_dim))
    return q, k, v, d_o


def small_batch(scale=0.0):
    # 3 documents, ragged shards, shards of one document interleaved with others in packed Q,
    # documents out of order in packed KV, GQA with groups of 2
    docs = [13, 7, 20]
    tasks = [(0, 0, 5), (0, 5, 8), (1, 0, 7), (2, 0, 1), (2, 1, 9), (2, 10, 10)]
    return W.custom(docs, tasks, 4, 2, 8, doc_order=[2, 0, 1], task_order=[4, 0, 2, 5, 1, 3], scale=scale)


# ---------------------------------------------------------------- hand-worked example
def _parse_golden(path):
    sym = {"ln3": math.log(3), "ln4": math.log(4), "ln8": math.log(8)}

    def val(tok):
        return float(eval(tok, {"__builtins__": {}}, sym))  # tokens are arithmetic over the three logs

    out, lines = {}, [l.strip() for l in open(path) if l.strip() and not l.startswith("#")]
    i = 0
    while i < len(lines):
        name, r, c = lines[i].split()
        r, c = int(r), int(c)
        out[name] = np.array([[val(t) for t in lines[i + 1 + a].split()] for a in range(r)])
        assert out[name].shape == (r, c)
        i += 1 + r
    return out


def test_hand_worked_rational_example():
    g = _parse_golden(os.path.join(GOLDEN, "rational_softmax_example.txt"))
    b = W.custom([3], [(0, 0, 3)], 1, 1, 2, scale=1.0)
    r = oracle.forward_backward(b, g["Q"][:, None, :], g["K"][:, None, :], g["V"][:, None, :], g["dO"][:, None, :])
    np.testing.assert_allclose(r["o"][:, 0, :], g["O"], atol=1e-13)
    np.testing.assert_allclose(r["lse"], g["LSE"], atol=1e-13)
    np.testing.assert_allclose(r["dq"][:, 0, :], g["dQ"], atol=1e-12)
    np.testing.assert_allclose(r["dk"][:, 0, :], g["dK"], atol=1e-12)
    np.testing.assert_allclose(r["dv"][:, 0, :], g["dV"], atol=1e-12)
    # the same document as two shards (1 + 2 rows) in swapped packed order gives the same rows
    b2 = W.custom([3], [(0, 0, 1), (0, 1, 2)], 1, 1, 2, task_order=[1, 0], scale=1.0)
    perm = [2, 0, 1]  # packed row of document position 0,1,2 -> rows: task1 first (pos1,pos2), then task0 (pos0)
    qp = g["Q"][[1, 2, 0]][:, None, :]
    dop = g["dO"][[1, 2, 0]][:, None, :]
    r2 = oracle.forward_backward(b2, qp, g["K"][:, None, :], g["V"][:, None, :], dop)
    np.testing.assert_allclose(r2["o"][perm, 0, :], g["O"], atol=1e-13)
    np.testing.assert_allclose(r2["dq"][perm, 0, :], g["dQ"], atol=1e-12)
    np.testing.assert_allclose(r2["dk"][:, 0, :], g["dK"], atol=1e-12)
    np.testing.assert_allclose(r2["dv"][:, 0, :], g["dV"], atol=1e-12)


# ---------------------------------------------------------------- brute force on tiny inputs
def brute_force(b, q, k, v):
    """Masked score matrix per (document, head), dense softmax.  Written matrix-wise, over whole
    documents, with no knowledge of tasks: it returns per-document-position results."""
    g = b.n_q_heads // b.n_kv_heads
    o = np.zeros_like(q)
    lse = np.zeros((b.n_q_heads, b.total_q))
    for t in range(b.n_tasks):
        dd = b.task_doc[t]
        k0 = b.doc_kv_start[dd]
        rows = np.arange(b.task_q_start[t], b.task_q_start[t] + b.task_q_len[t])
        pos = b.task_q_pos[t] + np.arange(b.task_q_len[t])
        nk = int(b.doc_kv_len[dd])
        for h in range(b.n_q_heads):
            s = b.scale * q[rows, h] @ k[k0:k0 + nk, h // g].T
            s = np.where(np.arange(nk)[None, :] <= pos[:, None], s, -np.inf)
            s = np.where(np.arange(nk)[None, :] < b.task_kv_len[t], s, -np.inf)
            e = np.exp(s - s.max(1, keepdims=True))
            p = e / e.sum(1, keepdims=True)
            o[rows, h] = p @ v[k0:k0 + nk, h // g]
            lse[h, rows] = np.log(e.sum(1)) + s.max(1)
    return o, lse


@pytest.mark.parametrize("scale", [0.0, 1.0])
def test_forward_matches_brute_force(scale):
    b = small_batch(scale)
    q, k, v, _ = rand_inputs(b, 1)
    o, lse = oracle.forward(b, q, k, v)
    ob, lb = brute_force(b, q, k, v)
    np.testing.assert_allclose(o, ob, atol=1e-12)
    np.testing.assert_allclose(lse, lb, atol=1e-12)


def loss(b, q, k, v, d_o):
    o, _ = oracle.forward(b, q, k, v)
    return float((o * d_o).sum())


def test_backward_matches_central_differences():
    b = small_batch()
    q, k, v, d_o = rand_inputs(b, 2)
    r = oracle.forward_backward(b, q, k, v, d_o)
    rng = np.random.default_rng(3)
    eps = 1e-5
    for name, x, gname in (("q", q, "dq"), ("k", k, "dk"), ("v", v, "dv")):
        idx = [tuple(rng.integers(0, s) for s in x.shape) for _ in range(40)]
        if name != "q":
            # include KV rows of positions no query sees?  every position is seen here; include row 0 and last
            idx += [(int(b.doc_kv_start[2]), 0, 0), (int(b.doc_kv_start[2] + 19), 1, 3)]
        for ix in idx:
            old = x[ix]
            x[ix] = old + eps
            lp = loss(b, q, k, v, d_o)
            x[ix] = old - eps
            lm = loss(b, q, k, v, d_o)
            x[ix] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - r[gname][ix]) < 1e-6 * max(1.0, abs(fd)), (name, ix, fd, r[gname][ix])


# ---------------------------------------------------------------- library special case
@pytest.mark.parametrize("hq,hkv", [(4, 4), (4, 2), (8, 1)])
def test_whole_document_equals_library_causal_attention(hq, hkv):
    """One task covering a whole document is ordinary causal attention: check against PyTorch's CPU
    scaled_dot_product_attention in float64 with autograd (GQA by repeating K/V heads)."""
    n, d = 37, 16
    b = W.custom([n], [(0, 0, n)], hq, hkv, d)
    q, k, v, d_o = rand_inputs(b, 4)
    r = oracle.forward_backward(b, q, k, v, d_o)
    tq = torch.tensor(q, requires_grad=True)
    tk = torch.tensor(k, requires_grad=True)
    tv = torch.tensor(v, requires_grad=True)
    g = hq // hkv
    kk = tk.repeat_interleave(g, dim=1)
    vv = tv.repeat_interleave(g, dim=1)
    out = torch.nn.functional.scaled_dot_product_attention(
        tq.permute(1, 0, 2)[None], kk.permute(1, 0, 2)[None], vv.permute(1, 0, 2)[None], is_causal=True)
    out = out[0].permute(1, 0, 2)
    (out * torch.tensor(d_o)).sum().backward()
    np.testing.assert_allclose(r["o"], out.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(r["dq"], tq.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(r["dk"], tk.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(r["dv"], tv.grad.numpy(), atol=1e-11)


# ---------------------------------------------------------------- closed forms
def test_zero_queries_give_prefix_means_and_log_counts():
    b = small_batch()
    q, k, v, d_o = rand_inputs(b, 5)
    q[:] = 0.0
    o, lse = oracle.forward(b, q, k, v)
    g = b.n_q_heads // b.n_kv_heads
    for t in range(b.n_tasks):
        k0 = b.doc_kv_start[b.task_doc[t]]
        for i in range(b.task_q_len[t]):
            p = b.task_q_pos[t] + i
            row = b.task_q_start[t] + i
            for h in range(b.n_q_heads):
                np.testing.assert_allclose(o[row, h], v[k0:k0 + p + 1, h // g].mean(0), atol=1e-13)
                assert abs(lse[h, row] - math.log(p + 1)) < 1e-13


def test_constant_values_are_returned_and_first_token_sees_itself():
    b = small_batch()
    q, k, v, d_o = rand_inputs(b, 6)
    vc = np.broadcast_to(np.arange(1, b.head_dim + 1, dtype=np.float64), v.shape).copy()
    o, _ = oracle.forward(b, q, k, vc)
    np.testing.assert_allclose(o, np.broadcast_to(vc[0, 0], o.shape), atol=1e-12)
    # position 0 of each document: O = V_0 exactly, LSE = scale*<q,k_0>, dQ = 0
    r = oracle.forward_backward(b, q, k, v, d_o)
    g = b.n_q_heads // b.n_kv_heads
    seen = 0
    for t in range(b.n_tasks):
        if b.task_q_pos[t] != 0:
            continue
        seen += 1
        row, k0 = b.task_q_start[t], b.doc_kv_start[b.task_doc[t]]
        for h in range(b.n_q_heads):
            assert np.array_equal(r["o"][row, h], v[k0, h // g])
            assert abs(r["lse"][h, row] - b.scale * q[row, h] @ k[k0, h // g]) < 1e-13
            assert np.abs(r["dq"][row, h]).max() < 1e-13
    assert seen == b.n_docs


# ---------------------------------------------------------------- invariants
def test_gradient_sum_rules():
    """sum_j dV_j = sum_rows dO_row per KV head (P is row-stochastic); sum_j dK_j = 0 per document and
    KV head (softmax is invariant to adding one vector to all keys of a document)."""
    b = small_batch()
    q, k, v, d_o = rand_inputs(b, 7)
    r = oracle.forward_backward(b, q, k, v, d_o)
    g = b.n_q_heads // b.n_kv_heads
    for dd in range(b.n_docs):
        k0, n = b.doc_kv_start[dd], b.doc_kv_len[dd]
        rows = np.concatenate([np.arange(b.task_q_start[t], b.task_q_start[t] + b.task_q_len[t])
                               for t in range(b.n_tasks) if b.task_doc[t] == dd])
        for hk in range(b.n_kv_heads):
            np.testing.assert_allclose(r["dv"][k0:k0 + n, hk].sum(0),
                                       d_o[rows][:, hk * g:(hk + 1) * g].sum((0, 1)), atol=1e-11)
            np.testing.assert_allclose(r["dk"][k0:k0 + n, hk].sum(0), 0.0, atol=1e-11)
    # shifting every key of a document leaves O unchanged
    k2 = k.copy()
    k0, n = b.doc_kv_start[2], b.doc_kv_len[2]
    k2[k0:k0 + n] += np.random.default_rng(8).standard_normal((1, b.n_kv_heads, b.head_dim))
    o2, _ = oracle.forward(b, q, k2, v)
    np.testing.assert_allclose(o2, r["o"], atol=1e-11)


def whole_document_twin(b):
    """The batch with every document as one task, packed in document order; returns it and, for each
    packed row of `b`, the row of the twin holding the same (document, position)."""
    tasks = [(dd, 0, int(b.doc_kv_len[dd])) for dd in range(b.n_docs)]
    w = W.custom([int(x) for x in b.doc_kv_len], tasks, b.n_q_heads, b.n_kv_heads, b.head_dim,
                 doc_order=list(np.argsort(b.doc_kv_start)), scale=b.softmax_scale)
    row_map = np.zeros(b.total_q, np.int64)
    for t in range(b.n_tasks):
        n = b.task_q_len[t]
        row_map[b.task_q_start[t]:b.task_q_start[t] + n] = w.task_q_start[b.task_doc[t]] + b.task_q_pos[t] + np.arange(n)
    return w, row_map


def test_composability_shards_equal_whole_documents():
    """A document computed as shards, in any packed order and interleaved with other documents, equals
    the document computed whole (Section 4.1: the shards' results together are the document's result)."""
    b = small_batch()
    q, k, v, d_o = rand_inputs(b, 9)
    w, row_map = whole_document_twin(b)
    assert sorted(row_map.tolist()) == list(range(b.total_q))  # small_batch covers every position once
    qw = np.zeros_like(q)
    dow = np.zeros_like(d_o)
    qw[row_map] = q
    dow[row_map] = d_o
    rs = oracle.forward_backward(b, q, k, v, d_o)
    rw = oracle.forward_backward(w, qw, k, v, dow)
    np.testing.assert_allclose(rs["o"], rw["o"][row_map], atol=1e-12)
    np.testing.assert_allclose(rs["lse"], rw["lse"][:, row_map], atol=1e-12)
    np.testing.assert_allclose(rs["dq"], rw["dq"][row_map], atol=1e-11)
    np.testing.assert_allclose(rs["dk"], rw["dk"], atol=1e-11)
    np.testing.assert_allclose(rs["dv"], rw["dv"], atol=1e-11)


def test_partial_document_and_unseen_keys():
    """Only some shards of a document present: rows still see their full prefix, KV rows beyond the last
    present query get zero gradient."""
    docs = [24]
    b = W.custom(docs, [(0, 4, 6), (0, 15, 3)], 2, 1, 8)
    q, k, v, d_o = rand_inputs(b, 10)
    r = oracle.forward_backward(b, q, k, v, d_o)
    whole = W.custom(docs, [(0, 0, 24)], 2, 1, 8)
    qw = np.zeros((24, 2, 8))
    dow = np.zeros((24, 2, 8))
    qw[4:10], qw[15:18] = q[0:6], q[6:9]
    dow[4:10], dow[15:18] = d_o[0:6], d_o[6:9]  # absent rows carry dO = 0, so they add nothing to dK/dV
    rw = oracle.forward_backward(whole, qw, k, v, dow)
    np.testing.assert_allclose(r["o"][0:6], rw["o"][4:10], atol=1e-12)
    np.testing.assert_allclose(r["o"][6:9], rw["o"][15:18], atol=1e-12)
    np.testing.assert_allclose(r["dk"], rw["dk"], atol=1e-11)
    np.testing.assert_allclose(r["dv"], rw["dv"], atol=1e-11)
    assert np.all(r["dk"][18:] == 0.0) and np.all(r["dv"][18:] == 0.0)
    assert np.abs(r["dv"][17]).max() > 0


def test_gqa_equals_mha_on_repeated_kv():
    b = small_batch()
    q, k, v, d_o = rand_inputs(b, 11)
    g = b.n_q_heads // b.n_kv_heads
    m = W.custom([int(x) for x in b.doc_kv_len], list(zip(b.task_doc.tolist(), b.task_q_pos.tolist(), b.task_q_len.tolist())),
                 b.n_q_heads, b.n_q_heads, b.head_dim, doc_order=[2, 0, 1], task_order=[4, 0, 2, 5, 1, 3])
    r = oracle.forward_backward(b, q, k, v, d_o)
    rm = oracle.forward_backward(m, q, np.repeat(k, g, 1), np.repeat(v, g, 1), d_o)
    np.testing.assert_allclose(r["o"], rm["o"], atol=1e-12)
    np.testing.assert_allclose(r["dq"], rm["dq"], atol=1e-12)
    np.testing.assert_allclose(r["dk"], rm["dk"].reshape(b.total_kv, b.n_kv_heads, g, -1).sum(2), atol=1e-11)
    np.testing.assert_allclose(r["dv"], rm["dv"].reshape(b.total_kv, b.n_kv_heads, g, -1).sum(2), atol=1e-11)


def test_exp_of_scores_minus_lse_is_row_stochastic():
    b = small_batch()
    q, k, v, _ = rand_inputs(b, 12)
    _, lse = oracle.forward(b, q, k, v)
    t = 5
    k0 = b.doc_kv_start[b.task_doc[t]]
    for i in range(b.task_q_len[t]):
        row, p = b.task_q_start[t] + i, b.task_q_pos[t] + i
        s = b.scale * k[k0:k0 + p + 1, 1] @ q[row, 3]
        assert abs(np.exp(s - lse[3, row]).sum() - 1.0) < 1e-12


# ---------------------------------------------------------------- work count (Appendix B; Section 1 example)
def test_pair_count_closed_forms():
    # trapezoid: a shard with n_q queries whose last row sees n_kv keys does n_q(2 n_kv - n_q)/2 off-diagonal-
    # inclusive pairs up to the half-diagonal term; the exact integer count is n_q(2a + n_q + 1)/2, a = n_kv - n_q
    for a, n in [(0, 1), (0, 17), (5, 1), (100, 28), (4096, 16)]:
        assert W.task_pairs(a, n) == sum(p + 1 for p in range(a, a + n))
        nkv = a + n
        assert abs(W.task_pairs(a, n) - n * (2 * nkv - n) / 2) <= n / 2 + 1e-9
    # shards of a document add up to the whole document, L(L+1)/2
    b = W.composability(seed=7, total=4096, max_cut=16)
    per_doc = np.zeros(b.n_docs, np.int64)
    for t in range(b.n_tasks):
        per_doc[b.task_doc[t]] += W.task_pairs(int(b.task_q_pos[t]), int(b.task_q_len[t]))
    assert all(per_doc[d] == L * (L + 1) // 2 for d, L in enumerate(b.doc_kv_len.tolist()))
    # Section 1: one 4K document costs about 4x four 1K documents; sixteen 1K documents match it (12 more)
    one = W.task_pairs(0, 4096)
    four = 4 * W.task_pairs(0, 1024)
    assert abs(one / four - 4.0) < 0.01
    assert abs(16 * W.task_pairs(0, 1024) / one - 1.0) < 0.01


def test_workload_generators_are_valid_and_deterministic():
    for idx in range(1, 6):
        b = W.config(idx, 1 if idx == 1 else 16)
        b2 = W.config(idx, 1 if idx == 1 else 16)
        assert np.array_equal(b.task_q_start, b2.task_q_start) and np.array_equal(b.doc_kv_start, b2.doc_kv_start)
        assert b.total_q == int(b.task_q_len.sum()) and b.total_kv == int(b.doc_kv_len.sum())
        cover = np.zeros(b.total_q, np.int32)
        for t in range(b.n_tasks):
            cover[b.task_q_start[t]:b.task_q_start[t] + b.task_q_len[t]] += 1
            assert b.task_kv_len[t] == b.task_q_pos[t] + b.task_q_len[t] <= b.doc_kv_len[b.task_doc[t]]
        assert np.all(cover == 1)
    c3 = W.config(3)
    assert c3.total_q == 131072 and c3.task_q_len.min() == 16 and np.all(c3.task_q_len % 16 == 0)
    c4 = W.config(4)
    assert c4.n_tasks == 32 and c4.total_kv == 524288

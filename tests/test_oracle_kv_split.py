"""Pins for the oracle's treatment of query shards that attend a sub-range of their context (the extension the paper
names in its Limitations section) and for the merge of their partial results.  Everything here is fixed by the
definition of core attention (Section 2.1) and by mathematics alone: a softmax over a union of disjoint key sets,
written out directly, against the oracle's partial results combined by its merge.  CPU only."""
import numpy as np
import pytest

import oracle
from paper_2510_18121_amd import workloads as W


def rand_inputs(b, seed=0):
    r = np.random.default_rng(seed)
    q = r.standard_normal((b.total_q, b.n_q_heads, b.head_dim))
    k = r.standard_normal((b.total_kv, b.n_kv_heads, b.head_dim))
    v = r.standard_normal((b.total_kv, b.n_kv_heads, b.head_dim))
    d_o = r.standard_normal((b.total_q, b.n_q_heads, b.head_dim))
    return q, k, v, d_o


def small_batch():
    docs = [13, 7, 20]
    tasks = [(0, 0, 5), (0, 5, 8), (1, 0, 7), (2, 0, 1), (2, 1, 9), (2, 10, 10)]
    return W.custom(docs, tasks, 4, 2, 8, doc_order=[2, 0, 1], task_order=[4, 0, 2, 5, 1, 3])


def test_clipped_prefix_against_a_direct_softmax():
    """A task whose kv_len is shorter than its rows' causal prefix: rows beyond see keys 0..kv_len-1.  Written out
    with numpy for one document, one head group."""
    b = W.custom([12], [(0, 3, 9)], 2, 1, 4)
    b.task_kv_len[0] = 7  # rows at positions 3..11; positions 7..11 see keys 0..6 only
    q, k, v, _ = rand_inputs(b, 1)
    o, lse = oracle.forward(b, q, k, v)
    for i in range(9):
        n = min(7, 3 + i + 1)
        for h in range(2):
            s = b.scale * (k[:n, 0] @ q[i, h])
            w = np.exp(s - s.max())
            assert np.allclose(o[i, h], (w / w.sum()) @ v[:n, 0], rtol=1e-12, atol=1e-14)
            assert np.isclose(lse[h, i], s.max() + np.log(w.sum()), rtol=1e-13)
    assert b.pairs() == sum(min(7, 3 + i + 1) for i in range(9))


def test_merge_closed_forms():
    hq, d = 2, 3
    r = np.random.default_rng(2)
    o_part = r.standard_normal((4, hq, d))
    lse_part = r.standard_normal((hq, 4))
    # one part only: identity
    o, lse = oracle.merge_partials([[2], ], o_part, lse_part)
    assert np.array_equal(o[0], o_part[2]) and np.array_equal(lse[:, 0], lse_part[:, 2])
    # an absent part changes nothing
    o2, lse2 = oracle.merge_partials([[-1], [2], [-1]], o_part, lse_part)
    assert np.array_equal(o2, o) and np.array_equal(lse2, lse)
    # two parts of equal weight: the mean, and log 2 more mass
    lse_part[:, 1] = lse_part[:, 0]
    o, lse = oracle.merge_partials([[0], [1]], o_part, lse_part)
    assert np.allclose(o[0], 0.5 * (o_part[0] + o_part[1]), rtol=1e-14)
    assert np.allclose(lse[:, 0], lse_part[:, 0] + np.log(2.0), rtol=1e-14)
    # weights 3:1 (difference of log 3)
    lse_part[:, 1] = lse_part[:, 0] - np.log(3.0)
    o, lse = oracle.merge_partials([[0], [1]], o_part, lse_part)
    assert np.allclose(o[0], 0.75 * o_part[0] + 0.25 * o_part[1], rtol=1e-13)
    assert np.allclose(lse[:, 0], lse_part[:, 0] + np.log(4.0 / 3.0), rtol=1e-13)
    # order of the parts does not matter; a huge offset common to all parts shifts LSE and leaves O alone
    a = oracle.merge_partials([[0], [1], [3]], o_part, lse_part)
    c = oracle.merge_partials([[3], [0], [1]], o_part, lse_part)
    assert np.allclose(a[0], c[0], rtol=1e-13) and np.allclose(a[1], c[1], rtol=1e-13)
    shifted = oracle.merge_partials([[0], [1], [3]], o_part, lse_part + 700.0)
    assert np.allclose(shifted[0], a[0], rtol=1e-12) and np.allclose(shifted[1], a[1] + 700.0, rtol=1e-13)
    # a row with no part at all
    o, lse = oracle.merge_partials([[-1], [-1]], o_part, lse_part)
    assert np.all(o == 0) and np.all(np.isneginf(lse))


@pytest.mark.parametrize("window", [1, 3, 6, 8, 64])
def test_partials_over_key_windows_merge_to_the_whole_context(window):
    """The plain definition over the whole context (one softmax per row) against partial attention over key windows
    combined by the merge: two routes to the same number."""
    b = small_batch()
    q, k, v, _ = rand_inputs(b, 3)
    o_full, lse_full = oracle.forward(b, q, k, v)
    pb, gather, part_rows = W.split_kv(b, window)
    assert pb.pairs() == b.pairs(), "every (row, key) pair belongs to exactly one window"
    o_p, lse_p = oracle.forward(pb, q[gather], k, v)
    o, lse = oracle.merge_partials(part_rows, o_p, lse_p)
    assert np.allclose(o, o_full, rtol=1e-11, atol=1e-13)
    assert np.allclose(lse, lse_full, rtol=1e-12, atol=1e-13)
    if window >= 64:  # one window per document: nothing to merge
        assert part_rows.shape[0] == 1 and np.array_equal(np.sort(part_rows[0]), np.arange(b.total_q))


@pytest.mark.parametrize("window", [3, 8])
def test_partial_backward_with_global_statistics_sums_to_the_whole_gradient(window):
    """Backward of every partial task with the MERGED output and log-sum-exp of its rows: dK, dV of the windows are
    the whole dK, dV (every key lies in one window), and the partial dQ of a row add up to its dQ."""
    b = small_batch()
    q, k, v, d_o = rand_inputs(b, 4)
    full = oracle.forward_backward(b, q, k, v, d_o)
    pb, gather, part_rows = W.split_kv(b, window)
    o_g, lse_g = full["o"][gather], full["lse"][:, gather]
    dq_p, dk, dv, _ = oracle.backward(pb, q[gather], k, v, o_g, d_o[gather], lse_g)
    assert np.allclose(dk, full["dk"], rtol=1e-10, atol=1e-12)
    assert np.allclose(dv, full["dv"], rtol=1e-10, atol=1e-12)
    dq = np.zeros_like(q)
    np.add.at(dq, gather, dq_p)
    assert np.allclose(dq, full["dq"], rtol=1e-10, atol=1e-12)


def test_a_planted_mistake_in_the_merge_weights_is_caught():
    """Weights exp(L_i - L) replaced by equal weights: the comparison above must fail."""
    b = small_batch()
    q, k, v, _ = rand_inputs(b, 5)
    o_full, _ = oracle.forward(b, q, k, v)
    pb, gather, part_rows = W.split_kv(b, 6)
    o_p, lse_p = oracle.forward(pb, q[gather], k, v)
    wrong, _ = oracle.merge_partials(part_rows, o_p, np.zeros_like(lse_p))
    assert not np.allclose(wrong, o_full, rtol=1e-3, atol=1e-3)

"""CPU pins of the communication cost function (Appendix B) and of the greedy scheduler (Section 4.2)."""
import math

import numpy as np
import pytest

from paper_2510_18121_amd import scheduler as S
from paper_2510_18121_amd import workloads as W


def brute_min_comm(alpha, L_q, L_kv, size_q, size_kv, steps=200000):
    """Scan n_q over (0, L_q]; keep the n_q whose n_kv satisfies the constraints of Appendix B; cheapest wins."""
    best = None
    for n_q in np.linspace(L_q / steps, L_q, steps):
        n_kv = 0.5 * (alpha * S.shard_work(L_q, L_kv) / n_q + n_q)
        if n_q + L_kv - L_q - 1e-9 <= n_kv <= L_kv + 1e-9:
            v = S.comm_bytes(n_q, n_kv, size_q, size_kv)
            if best is None or v < best[2]:
                best = (n_q, n_kv, v)
    return best


@pytest.mark.parametrize("alpha", [0.02, 0.1, 0.35, 0.8, 1.0])
@pytest.mark.parametrize("L_q,L_kv", [(4096, 4096), (4096, 20000), (512, 131072), (16384, 16400)])
@pytest.mark.parametrize("size_q,size_kv", [(8192.0, 4096.0), (8192.0, 512.0), (1.0, 6.0)])
def test_min_comm_equals_brute_force(alpha, L_q, L_kv, size_q, size_kv):
    n_q, n_kv, v = S.min_comm(alpha, L_q, L_kv, size_q, size_kv)
    b = brute_min_comm(alpha, L_q, L_kv, size_q, size_kv)
    assert v == pytest.approx(b[2], rel=2e-4)
    # the returned sub-shard is feasible and carries the fraction alpha of the work
    assert 0 < n_q <= L_q + 1e-6 and n_q + L_kv - L_q - 1e-6 <= n_kv <= L_kv + 1e-6
    assert S.shard_work(n_q, n_kv) == pytest.approx(alpha * S.shard_work(L_q, L_kv), rel=1e-9)


def test_min_comm_interior_closed_form():
    # Appendix B: v = size_q sqrt(alpha beta (beta + 2) L_q (2 L_kv - L_q)) when the optimum is interior
    alpha, L_q, L_kv, size_q, size_kv = 0.2, 8192.0, 8192.0, 2.0, 1.0
    beta = size_kv / size_q
    n_opt = math.sqrt(alpha * beta * S.shard_work(L_q, L_kv) / (beta + 2))
    lo, hi = S.sub_shard_bounds(alpha, L_q, L_kv)
    assert lo < n_opt < hi
    n_q, n_kv, v = S.min_comm(alpha, L_q, L_kv, size_q, size_kv)
    assert n_q == pytest.approx(n_opt) and v == pytest.approx(size_q * math.sqrt(alpha * beta * (beta + 2) * S.shard_work(L_q, L_kv)))


def test_whole_item_and_bounds():
    # alpha = 1 leaves only the whole Item
    n_q, n_kv, v = S.min_comm(1.0, 1000, 5000, 3.0, 2.0)
    assert n_q == pytest.approx(1000) and n_kv == pytest.approx(5000) and v == pytest.approx(3000 + 10000)
    # the ends of the feasible range are the Item's last rows and its first rows
    lo, hi = S.sub_shard_bounds(0.3, 1000, 5000)
    assert S.n_kv_for(0.3, 1000, 5000, lo) == pytest.approx(5000)
    assert S.n_kv_for(0.3, 1000, 5000, hi) == pytest.approx(hi + 4000)
    with pytest.raises(ValueError):
        S.min_comm(0.0, 10, 10, 1, 1)


def test_head_tail_variant_takes_the_smallest_shard():
    alpha, L_q, L_kv, L_doc, sq, skv = 0.25, 2048.0, 6000.0, 12000.0, 4.0, 2.0
    n_q, v = S.min_comm_head_tail(alpha, L_q, L_kv, L_doc, sq, skv)
    assert n_q == pytest.approx(L_kv - math.sqrt(L_kv ** 2 - alpha * S.shard_work(L_q, L_kv)))
    # Comm(n_q, n_kv) = n_q size_q + (L_doc - (n_kv - n_q)) size_kv at n_kv = L_kv
    assert v == pytest.approx(n_q * sq + (L_doc - (L_kv - n_q)) * skv)
    # and any larger feasible n_q costs more
    for m in (1.1, 1.5, 2.0):
        n2 = n_q * m
        nkv2 = S.n_kv_for(alpha, L_q, L_kv, n2)
        assert n2 * sq + (L_doc - (nkv2 - n2)) * skv > v


def _covered(sch, items):
    """Per document, the multiset of query positions computed somewhere."""
    got, want = {}, {}
    for srv in sch.servers:
        for it in srv:
            got.setdefault(it.doc, []).extend(range(it.q_pos, it.q_pos + it.q_len))
    for it in items:
        want.setdefault(it.doc, []).extend(range(it.q_pos, it.q_pos + it.q_len))
    return {d: sorted(v) for d, v in got.items()}, {d: sorted(v) for d, v in want.items()}


@pytest.mark.parametrize("eps", [0.2, 0.05, 0.01])
@pytest.mark.parametrize("n_servers", [2, 4, 8])
def test_schedule_balances_and_conserves_the_work(eps, n_servers):
    b = W.config(3, 8)
    items = S.items_from_batch(b, n_servers)
    sch = S.schedule(items, n_servers, size_q=8192.0, size_kv=4096.0, eps=eps)
    got, want = _covered(sch, items)
    assert got == want  # every query row is computed exactly once, by someone
    assert sum(sch.loads()) == b.pairs()
    mean = b.pairs() / n_servers
    assert all(abs(x - mean) <= eps * mean + 1 for x in sch.loads())
    # tighter tolerance never sends fewer bytes
    looser = S.schedule(items, n_servers, 8192.0, 4096.0, eps=2 * eps)
    assert looser.moved_bytes <= sch.moved_bytes + 1e-6
    for s, d, it, v in sch.moves:
        assert s != d and v > 0 and it.q_len >= 1


def test_balanced_input_moves_nothing_and_one_long_document_is_spread():
    items = [S.Item(d, 0, 1024, d) for d in range(4)]
    sch = S.schedule(items, 4, 2.0, 1.0, eps=0.01)
    assert not sch.moves and sch.imbalance() == 1.0
    # one 64K document on server 0, three idle servers: everybody ends with a quarter of the pairs
    items = [S.Item(0, 0, 65536, 0)]
    sch = S.schedule(items, 4, 2.0, 1.0, eps=0.02)
    mean = W.task_pairs(0, 65536) / 4
    assert all(abs(x - mean) <= 0.02 * mean + 1 for x in sch.loads())
    got, want = _covered(sch, items)
    assert got == want
    # cuts sit on the 16-row grid
    assert all(it.q_pos % 16 == 0 and it.q_len % 16 == 0 for srv in sch.servers for it in srv)


def test_priority_prefers_cheap_bytes():
    # two equal-work candidates on the overloaded server: a long-context shard (many KV bytes) and a whole short
    # document; the short document is moved
    long_ctx = S.Item(0, 30000, 131, 0)     # 131 rows deep in a document
    whole = S.Item(1, 0, 2808, 0)           # about the same pairs, context = itself
    assert abs(long_ctx.pairs - whole.pairs) / whole.pairs < 0.01
    filler = S.Item(2, 0, 2808, 1)
    sch = S.schedule([long_ctx, whole, filler], 3, size_q=2.0, size_kv=2.0, eps=0.05)
    assert sch.moves and sch.moves[0][2].doc == 1


def test_min_gain_threshold_stops_expensive_moves():
    items = [S.Item(0, 0, 8192, 0)]
    free = S.schedule(items, 2, 2.0, 1.0, eps=0.01)
    assert free.moves
    costly = S.schedule(items, 2, 2.0, 1.0, eps=0.01, min_gain=1e12)
    assert not costly.moves and costly.imbalance() == 2.0


def test_server_batch_gathers_the_right_rows():
    b = W.config(3, 16)
    items = S.items_from_batch(b, 4)
    sch = S.schedule(items, 4, 8192.0, 4096.0, eps=0.05)
    seen = []
    for s, srv in enumerate(sch.servers):
        sub, qrows, kvrows = S.server_batch(b, srv)
        assert sub.total_q == len(qrows) == sum(it.q_len for it in srv) and sub.total_kv == len(kvrows)
        assert sub.pairs() == sum(it.pairs for it in srv)
        seen.extend(qrows.tolist())
    assert sorted(seen) == list(range(b.total_q))

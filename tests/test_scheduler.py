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


def _toy_grid():
    """A latency grid with the shape the measured ones have: a fixed cost per task plus time proportional to the
    work, so short shards are far dearer per pair than long ones."""
    from paper_2510_18121_amd.profiler import LatencyGrid, task_flops
    q_axis, kv_axis = [16, 64, 256, 1024, 4096, 16384], [16, 128, 1024, 8192, 65536]
    sec = np.full((len(q_axis), len(kv_axis)), np.nan)
    for i, q in enumerate(q_axis):
        for j, kv in enumerate(kv_axis):
            if kv >= q:
                sec[i, j] = 40e-6 + task_flops(q, kv, 8, 128) / 800e12
    return LatencyGrid(q_axis, kv_axis, sec, 8, 128)


def test_grid_priced_schedule_balances_predicted_time_where_pairs_misprice_it():
    """Sixteen-row tasks next to 16K-row tasks (Section 4.2: the scheduler's costs come from the Profiler).  By pair
    count the server with the tiny tasks looks idle; by predicted time it is the busiest.  Balancing pairs leaves the
    predicted times unbalanced; balancing with the grid evens them out."""
    g = _toy_grid()
    tiny = [S.Item(doc=i, q_pos=112, q_len=16, home=0) for i in range(600)]      # 600 x (40 us + a little)
    big = [S.Item(doc=1000 + i, q_pos=0, q_len=16384, home=1) for i in range(2)]
    items = tiny + big
    by_pairs = S.schedule(items, 2, 8192.0, 4096.0, eps=0.02)
    by_time = S.schedule(items, 2, 8192.0, 4096.0, eps=0.02, grid=g)
    assert by_pairs.imbalance() <= 1.03                 # balanced in its own unit ...
    assert by_pairs.imbalance(grid=g) > 1.25            # ... but not in predicted seconds
    assert by_time.imbalance() <= 1.03 and by_time.grid is g
    assert by_time.imbalance(grid=g) <= 1.03
    # the first move goes opposite ways: by pairs the long documents' server is overloaded, by time the tiny tasks'
    assert by_pairs.moves[0][0] == 1 and by_time.moves[0][0] == 0
    # nothing is lost or duplicated either way
    for sch in (by_pairs, by_time):
        assert sum(it.pairs for srv in sch.servers for it in srv) == sum(it.pairs for it in items)


def test_grid_priced_loads_are_the_sum_of_predictions():
    g = _toy_grid()
    items = [S.Item(0, 0, 4096, 0), S.Item(0, 4096, 4096, 0), S.Item(1, 0, 300, 1)]
    sch = S.schedule(items, 2, 8192.0, 4096.0, eps=10.0, grid=g)   # tolerance so wide that nothing moves
    assert not sch.moves
    assert sch.loads() == pytest.approx([g.predict(4096, 4096) + g.predict(4096, 8192), g.predict(300, 300)])
    assert sch.loads(grid=None) == [W.task_pairs(0, 4096) + W.task_pairs(4096, 4096), W.task_pairs(0, 300)]

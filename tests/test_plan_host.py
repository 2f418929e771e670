"""Host-side planner: descriptor validation (every error path) and schedule invariants.  No GPU needed."""
import copy

import numpy as np
import pytest

from paper_2510_18121_amd import binding as B
from paper_2510_18121_amd import workloads as W


def base():
    return W.custom([40, 300, 17], [(0, 0, 11), (0, 11, 29), (1, 5, 100), (1, 200, 100), (2, 0, 17)], 8, 2, 128,
                    doc_order=[1, 2, 0], task_order=[3, 0, 4, 2, 1])


def plan_error(b):
    with pytest.raises(B.CaError) as e:
        B.ca_plan_host(b)
    return e.value


def mutated(**kw):
    b = copy.deepcopy(base())
    for k, v in kw.items():
        if callable(v):
            v(getattr(b, k))
        else:
            setattr(b, k, v)
    return b


def test_valid_descriptor_plans():
    p = B.ca_plan_host(base())
    assert p.info()["n_fwd_units"] > 0
    f, bw = p.workspace_bytes()
    assert f == 0 and bw > 0 and bw % 256 == 0


@pytest.mark.parametrize("name,mut,code,needle", [
    ("head_dim", dict(head_dim=96), B.CA_ERR_UNSUPPORTED, "head_dim"),
    ("head ratio", dict(n_q_heads=7), B.CA_ERR_UNSUPPORTED, "multiple"),
    ("zero heads", dict(n_kv_heads=0), B.CA_ERR_INVALID_ARG, "head counts"),
    ("q_len 0", dict(task_q_len=lambda a: a.__setitem__(1, 0)), B.CA_ERR_INVALID_ARG, "q_len"),
    ("bad doc", dict(task_doc=lambda a: a.__setitem__(0, 9)), B.CA_ERR_INVALID_ARG, "names document"),
    ("q out of range", dict(task_q_start=lambda a: a.__setitem__(1, 10**6)), B.CA_ERR_INVALID_ARG, "outside packed Q"),
    ("q overlap", dict(task_q_start=lambda a: a.__setitem__(1, int(a[0]) + 1)), B.CA_ERR_INVALID_ARG, "overlap"),
    ("negative pos", dict(task_q_pos=lambda a: a.__setitem__(0, -1)), B.CA_ERR_INVALID_ARG, "q_pos"),
    ("task without keys", dict(task_kv_len=lambda a: a.__setitem__(1, 0)), B.CA_ERR_INVALID_ARG, "at least one key"),
    ("kv_len beyond doc", dict(task_kv_len=lambda a: a.__setitem__(1, 41)), B.CA_ERR_INVALID_ARG, "resident KV"),
    ("doc out of buffer", dict(doc_kv_start=lambda a: a.__setitem__(1, 10**6)), B.CA_ERR_INVALID_ARG, "outside the packed KV"),
    ("doc overlap", dict(doc_kv_start=lambda a: a.__setitem__(0, int(a[2]))), B.CA_ERR_INVALID_ARG, "overlap"),
    ("doc len 0", dict(doc_kv_len=lambda a: a.__setitem__(2, 0)), B.CA_ERR_INVALID_ARG, "kv_len"),
    ("negative totals", dict(total_q=-1), B.CA_ERR_INVALID_ARG, "negative"),
])
def test_invalid_descriptors(name, mut, code, needle):
    err = plan_error(mutated(**mut))
    assert err.code == code, (name, err)
    assert needle in err.detail, (name, err.detail)


def test_null_arrays_and_null_descriptor():
    lib = B.lib()
    keep = []
    d = B.make_desc(base(), keep)
    d.task_q_len = None
    import ctypes
    h = ctypes.c_void_p()
    assert lib.ca_plan_host(ctypes.byref(d), ctypes.byref(h)) == B.CA_ERR_INVALID_ARG
    assert b"null" in lib.ca_last_error()
    assert lib.ca_plan_host(None, ctypes.byref(h)) == B.CA_ERR_INVALID_ARG


def test_using_a_plan_that_was_never_uploaded_is_a_state_error():
    p = B.ca_plan_host(base())
    lib = B.lib()
    rc = lib.ca_forward(p.handle, 1, 1, 1, 1, 1, None, 0, None)
    assert rc == B.CA_ERR_STATE


def check_schedule(b):
    p = B.ca_plan_host(b)
    info = p.info()
    rows, pos = p.rows()
    bm, bq, bn = info["q_tile_rows"], info["bwd_q_block_rows"], info["kv_tile_rows"]
    g = b.n_q_heads // b.n_kv_heads
    al, hp = info["slot_align"], info["heads_packed"]
    assert hp == max(k for k in (8, 4, 2, 1) if g % k == 0) and al == max(bm // hp, bq)
    assert len(rows) == info["padded_rows"] and len(rows) % al == 0
    # every packed query row of every task sits in exactly one slot, with its document position
    want_pos = np.full(b.total_q, -1, np.int64)
    want_doc = np.full(b.total_q, -1, np.int64)
    for t in range(b.n_tasks):
        sl = slice(int(b.task_q_start[t]), int(b.task_q_start[t] + b.task_q_len[t]))
        want_pos[sl] = np.minimum(b.task_q_pos[t] + np.arange(b.task_q_len[t]), b.task_kv_len[t] - 1)  # last key seen
        want_doc[sl] = b.task_doc[t]
    real = rows >= 0
    assert sorted(rows[real].tolist()) == np.flatnonzero(want_pos >= 0).tolist()
    assert np.array_equal(pos[real], want_pos[rows[real]])
    # forward units: a full tile is bm slots of one head, a head-packed unit bm / hp slots of hp heads of one KV group
    fu = p.fwd_units()
    assert fu.shape == (info["n_fwd_units"], 5)
    assert info["n_q_tiles"] == len(set(fu[(fu[:, 4] == 1) | (hp == 1), 0].tolist()))
    costs = -(-fu[:, 2] // info["fwd_kv_step"])
    assert np.all(np.diff(costs) <= 0), "longest first"
    head_cover = np.zeros((len(rows), b.n_q_heads), np.int32)
    for i, (s0, kv0, nk, h, k) in enumerate(fu.tolist()):
        assert k in (1, hp) and h % k == 0 and 0 <= h and h + k <= b.n_q_heads
        assert h // g == (h + k - 1) // g, "the heads of a unit share their KV head"
        span = bm // k
        assert s0 % span == 0 or k == 1
        assert (i % b.n_kv_heads) == h // g, "unit index modulo n_kv_heads is the KV head"
        tile_rows, tile_pos = rows[s0:s0 + span], pos[s0:s0 + span]
        assert len(tile_rows) == span, "a unit never reaches past the padded slots"
        ok = tile_rows >= 0
        assert ok.any() and ok[0]
        docs = set(want_doc[tile_rows[ok]].tolist())
        assert len(docs) == 1, "rows of different documents never share a tile"
        dd = docs.pop()
        assert kv0 == b.doc_kv_start[dd] and nk == tile_pos[ok].max() + 1
        assert np.all(np.diff(tile_pos) >= 0), "slots sorted by position"
        assert np.all(tile_pos[~ok] == tile_pos[ok][-1])
        head_cover[s0:s0 + span, h:h + k] += 1
    assert head_cover.size == 0 or head_cover.max() <= 1, "no (slot, head) belongs to two units"
    assert np.all(head_cover[real] == 1), "every real (slot, head) belongs to one unit"
    # backward units: every key of every scheduled document once per KV head
    bu = p.bwd_units()
    assert len(bu) == info["n_bwd_units"]
    # the leading units are one workgroup each, longest first; a workgroup goes on with the units it points to
    n_wg = info["n_bwd_workgroups"]
    assert 0 <= n_wg <= len(bu) and (n_wg > 0) == (len(bu) > 0)
    span = bu[:, 1] - bu[:, 0]
    assert np.all(bu[:n_wg, 8] >= 1) and np.all(bu[n_wg:, 8] == 0) and bu[:, 8].sum() == len(bu)
    followed = np.zeros(len(bu), np.int32)
    steps = span // bq * bu[:, 9]
    wg_steps = np.zeros(n_wg, np.int64)
    for i in range(n_wg):
        assert i % b.n_kv_heads == bu[i, 6], "workgroup index modulo n_kv_heads is the KV head"
        f, c = int(bu[i, 7]), int(bu[i, 8])
        wg_steps[i] = steps[i] + (steps[f:f + c - 1].sum() if c > 1 else 0)
        if c > 1:
            assert n_wg <= f and f + c - 1 <= len(bu)
            followed[f:f + c - 1] += 1
            chain = np.concatenate([[i], np.arange(f, f + c - 1)])
            assert np.all(bu[chain, 6] == bu[i, 6]), "a chain stays with one KV head"
            assert np.all(np.diff(span[chain]) <= 0)
            assert steps[chain].max() <= 16 and steps[chain].sum() <= 256 and c <= 32, "only short units are chained"
    assert np.all(np.diff(wg_steps) <= 0), "longest first, a chain counting with all its steps"
    assert np.all(followed[n_wg:] == 1) and np.all(followed[:n_wg] == 0), "every following unit belongs to one chain"
    key_cover = np.zeros((b.total_kv, b.n_kv_heads), np.int32)
    docs_with_tasks = sorted(set(b.task_doc.tolist()))
    for i, (sb, se, sf, kvrow, nvalid, kp0, hk, _, _, tiles) in enumerate(bu.tolist()):
        assert 0 <= hk < b.n_kv_heads and 1 <= nvalid <= bn and (se - sb) % bq == 0 and se >= sb
        assert sb <= sf <= se and (sf - sb) % bq == 0
        assert np.all(pos[sf:se] >= kp0 + bn - 1), "blocks from slot_full on see every key of the tile"
        if sf - bq >= sb:
            assert pos[sf - bq] < kp0 + bn - 1, "slot_full is the first such block"
        key_cover[kvrow:kvrow + nvalid, hk] += 1
        dd = [d for d in docs_with_tasks if b.doc_kv_start[d] <= kvrow < b.doc_kv_start[d] + b.doc_kv_len[d]][0]
        assert kvrow - b.doc_kv_start[dd] == kp0
        # tiles per query block: one per head of the group, or the rows of 4 / 2 heads per tile for a document that brings
        # at most 16 / 32 rows
        n_doc_rows = int((real & (np.where(real, want_doc[np.maximum(rows, 0)], -1) == dd)).sum())
        assert tiles == (g // 4 if n_doc_rows <= 16 and g % 4 == 0 else g // 2 if n_doc_rows <= 32 and g % 2 == 0 else g)
        # slots of this document that can see any key of the tile lie in [sb, se)
        doc_slots = np.flatnonzero(real & (np.where(real, want_doc[np.maximum(rows, 0)], -1) == dd))
        sees = doc_slots[pos[doc_slots] >= kp0]
        if len(sees):
            assert sb <= sees.min() and sees.max() < se
        else:
            assert sb == se
        if se > sb:
            assert set(want_doc[rows[sb:se][rows[sb:se] >= 0]].tolist()) == {dd}
    for dd in docs_with_tasks:
        sl = slice(int(b.doc_kv_start[dd]), int(b.doc_kv_start[dd] + b.doc_kv_len[dd]))
        assert np.all(key_cover[sl] == 1)
    assert key_cover.sum() == sum(int(b.doc_kv_len[d]) for d in docs_with_tasks) * b.n_kv_heads
    return p


def test_short_backward_units_are_chained():
    """Lone 64-token shards with contexts: units of 4 steps, chained per KV head; long documents: none chained."""
    b = W.shard_chunk(64, "distinct", seed=1, chunk_tokens=4096, max_context=2048, hq=8, hkv=2, d=128)
    p = check_schedule(b)
    info, bu = p.info(), p.bwd_units()
    n_wg = info["n_bwd_workgroups"]
    assert n_wg < len(bu) and bu[:n_wg, 8].max() > 1
    # chains shrink towards the end of the list: the last workgroups are single units or short chains
    assert bu[n_wg - 1, 8] <= 2 <= bu[0, 8]
    long_docs = W.config(4, downscale=16)
    info = B.ca_plan_host(long_docs).info()
    assert info["n_bwd_workgroups"] >= info["n_bwd_units"] - 64


def test_schedule_invariants_small_and_ragged():
    check_schedule(base())
    check_schedule(W.config(1))
    # single-row tasks, a document with no task, gaps in positions
    b = W.custom([5, 9, 700], [(0, 4, 1), (2, 0, 1), (2, 300, 1), (2, 650, 50)], 4, 4, 64, doc_order=[2, 0, 1])
    check_schedule(b)
    # every packing factor: group sizes 8, 4, 2, 1 and 3 -> 8, 4, 2, 1 and 1 heads per unit of the left-over slots
    for hq, hkv in ((8, 1), (16, 2), (8, 2), (4, 2), (4, 4), (6, 2)):
        b = W.custom([40, 300, 1000, 257], [(0, 0, 40), (1, 0, 300), (2, 100, 333), (2, 600, 400), (3, 0, 257)], hq, hkv, 64)
        info = check_schedule(b).info()
        assert info["heads_packed"] == {8: 8, 4: 4, 2: 2, 1: 1, 3: 1}[hq // hkv]


def test_schedule_invariants_of_key_window_tasks():
    """Tasks clipped to a key window (kv_len < q_pos + q_len): their slots carry the last key they see."""
    b = W.custom([700], [(0, 100, 300)], 4, 2, 64)
    b.task_kv_len[0] = 250  # rows at positions 250..399 all see keys 0..249
    p = check_schedule(b)
    _, pos = p.rows()
    assert pos[:300].tolist() == list(range(100, 250)) + [249] * 150
    # a later task clipped below an earlier one: slots are re-sorted by the last key seen
    b = W.custom([700], [(0, 0, 200), (0, 200, 100)], 4, 2, 64)
    b.task_kv_len[1] = 50
    check_schedule(b)
    for window in (64, 100, 333):
        pb, gather, part_rows = W.split_kv(W.config(1), window)
        check_schedule(pb)
        assert pb.pairs() == W.config(1).pairs()


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_schedule_invariants_downscaled_workloads(idx):
    check_schedule(W.config(idx, 16))


def test_full_size_plans_build_quickly_and_have_enough_units():
    import time
    for idx in (3, 5):
        b = W.config(idx)
        t0 = time.perf_counter()
        p = B.ca_plan_host(b)
        dt = time.perf_counter() - t0
        info = p.info()
        assert dt < 2.0, dt
        assert info["n_fwd_units"] >= 4 * 256 and info["n_bwd_units"] >= 4 * 256
        assert info["padded_rows"] - b.total_q <= b.n_docs * info["q_tile_rows"]


def test_empty_batch():
    b = W.custom([8], [], 4, 2, 64)
    p = B.ca_plan_host(b)
    assert p.info()["n_fwd_units"] == 0 and p.info()["n_bwd_units"] == 0


def test_duplicate_positions_are_allowed_and_sorted():
    # two tasks of one document covering the same positions (separate query rows)
    b = W.custom([64], [(0, 10, 20), (0, 15, 20)], 2, 1, 64)
    p = check_schedule(b)
    rows, pos = p.rows()
    assert np.all(np.diff(pos[:40]) >= 0)


@pytest.mark.parametrize("seed", range(40))
def test_schedule_invariants_on_random_descriptors(seed):
    """Seeded random batches (documents of 1..3000 tokens, ragged shards with gaps, clipped prefixes, tasks of one
    document covering the same positions twice now and then, every packing factor): all schedule invariants hold."""
    rng = np.random.default_rng(4000 + seed)
    hkv = int(rng.choice([1, 2, 3, 8]))
    g = int(rng.choice([1, 2, 3, 4, 8]))
    n_docs = int(rng.integers(1, 7))
    docs = [int(rng.integers(1, 3001)) for _ in range(n_docs)]
    tasks = []
    for dd, n in enumerate(docs):
        cuts = sorted(set(int(x) for x in rng.integers(0, n + 1, size=int(rng.integers(0, 7)))))
        for a, e in zip(cuts[:-1], cuts[1:]):
            if e > a and rng.random() < 0.8:
                tasks.append((dd, a, e - a))
        if n > 10 and rng.random() < 0.2:  # a second task over positions already covered
            a = int(rng.integers(0, n - 5))
            tasks.append((dd, a, int(rng.integers(1, n - a + 1))))
    b = W.custom(docs, tasks, hkv * g, hkv, int(rng.choice([64, 128])),
                 doc_order=[int(x) for x in rng.permutation(n_docs)],
                 task_order=[int(x) for x in rng.permutation(len(tasks))])
    for t in range(b.n_tasks):
        if rng.random() < 0.25:
            b.task_kv_len[t] = int(rng.integers(1, b.task_kv_len[t] + 1))
    check_schedule(b)


def test_planning_from_several_threads_at_once():
    """ca_plan_host keeps no global state (the scheduler plans the next batch on its own thread while the GPU runs
    the current one, Section 4.1): four threads planning different batches concurrently get the plans a single thread
    gets, and a failing call on one thread leaves the others' error strings alone."""
    import threading
    batches = [W.config(1), W.config(3, 16), W.config(5, 16), W.custom([5, 9, 700], [(0, 4, 1), (2, 300, 1)], 4, 4, 64)]
    want = []
    for b in batches:
        p = B.ca_plan_host(b)
        want.append((p.info(), p.rows()[0].copy(), p.fwd_units().copy(), p.bwd_units().copy()))
    got, errs = [None] * len(batches), [None] * len(batches)

    def work(i):
        try:
            for _ in range(5):
                p = B.ca_plan_host(batches[i])
                got[i] = (p.info(), p.rows()[0].copy(), p.fwd_units().copy(), p.bwd_units().copy())
                if i == 0:  # interleave failing calls
                    try:
                        B.ca_plan_host(mutated(n_q_heads=7))
                        raise AssertionError("a head ratio of 7/2 was accepted")
                    except B.CaError as e:
                        assert "multiple" in e.detail, e.detail
        except BaseException as ex:  # noqa: BLE001 - reported by the main thread below
            errs[i] = ex

    threads = [threading.Thread(target=work, args=(i,)) for i in range(len(batches))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert errs == [None] * len(batches), errs
    for g, w in zip(got, want):
        assert g[0] == w[0]
        for a, b_ in zip(g[1:], w[1:]):
            assert np.array_equal(a, b_)

"""The GPU parity tests' own checkers, exercised on the CPU with the oracle standing in for the GPU result:
the exact key-window sub-problem reproduces the whole backward's dK/dV, the sum identities hold on exact gradients,
and each of them (and the per-row figure) sees a planted mistake that the whole-tensor relative L2 does not."""
import numpy as np
import torch

import oracle
import parity_util as P
from paper_2510_18121_amd import workloads as W


def _case():
    b = W.custom([700, 300], [(0, 0, 130), (0, 130, 270), (0, 450, 250), (1, 0, 300)], 4, 2, 64,
                 doc_order=[1, 0], task_order=[2, 0, 3, 1], seed=5)
    b.task_kv_len[2] = 600  # one shard clipped to a shorter key prefix
    q, k, v, d_o = W.make_tensors(b, "cpu")
    ref = oracle.forward_backward(b, *(P.to64(t) for t in (q, k, v, d_o)))
    as_gpu = {n: torch.as_tensor(ref[n]) for n in ("o", "lse", "dq", "dk", "dv")}
    return b, (q, k, v, d_o), ref, as_gpu


def test_key_window_subproblem_equals_the_whole_backward():
    b, tensors, ref, as_gpu = _case()
    tiles = [(0, 0, 0), (0, 192, 1), (0, 572, 0), (1, 100, 1), (0, 640, 1)]  # the last one lies beyond the clipped shard's keys
    for t in P.check_interior_key_tiles(b, tensors, as_gpu, tiles):
        # O goes through fp32 on its way into the checker, hence 1e-6 rather than 1e-13
        assert t["dk_rel_l2"] < 1e-6 and t["dv_rel_l2"] < 1e-6 and (t["rows"] > 0) == (t["lo"] < 600), t


def test_key_window_subproblem_sees_a_missing_query_block():
    b, tensors, ref, as_gpu = _case()
    # take the contribution of 64 query rows of one head out of dK/dV of document 0 (what a skipped block would do)
    b2 = W.custom([700, 300], [(0, 0, 130), (0, 130, 270), (0, 450, 186), (1, 0, 300)], 4, 2, 64,
                  doc_order=[1, 0], task_order=[2, 0, 3, 1], seed=5)
    b2.task_kv_len[2] = 600
    q, k, v, d_o = tensors
    keep = np.concatenate([np.arange(int(a), int(a + n)) for a, n in zip(b.task_q_start, b2.task_q_len)])
    part = oracle.forward_backward(b2, *(P.to64(t[torch.as_tensor(keep)]) if t.shape[0] == b.total_q else P.to64(t)
                                         for t in (q, k, v, d_o)))
    bad = dict(as_gpu, dk=torch.as_tensor(part["dk"]), dv=torch.as_tensor(part["dv"]))
    whole = P.rel_l2(part["dv"], ref["dv"])
    t = P.check_interior_key_tiles(b, tensors, bad, [(0, 256, 0)])[0]
    assert t["dv_rel_l2"] > 1e-2 and t["dk_rel_l2"] > 1e-2, (t, whole)
    s = P.sum_invariants(b, d_o, bad)
    assert s["sum_dv_minus_sum_do_rel"] > P.SUM_INVARIANT, s


def test_sum_identities_hold_on_exact_gradients():
    b, tensors, ref, as_gpu = _case()
    s = P.sum_invariants(b, tensors[3].double(), as_gpu)
    assert s["sum_dv_minus_sum_do_rel"] < 1e-12 and s["sum_dk_rel"] < 1e-12, s


def test_one_wrong_row_is_seen_by_the_row_figure_only():
    b, tensors, ref, as_gpu = _case()
    dq = ref["dq"].copy()
    dq[417, 2] *= 1.25  # one (row, head) of 950 x 4 off by a quarter of its size
    assert P.rel_l2(dq, ref["dq"]) < P.GRAD_REL_L2          # the whole-tensor figure passes it
    row, tile = P.row_and_tile_errors(dq, ref["dq"])
    assert row > P.ROW_REL_L2 and tile > P.TILE_REL_L2       # the finer ones do not
    row, tile = P.row_and_tile_errors(ref["dq"], ref["dq"])
    assert row == 0.0 and tile == 0.0


def test_interior_tiles_cover_start_middle_end_and_rotate_heads():
    b = W.config(4)
    t = P.interior_tiles(b, seed=1, per_doc=3)
    assert [x[1] for x in t] == [0, 262144, 524288 - 128] and len({x[2] for x in t}) == 3
    t3 = P.interior_tiles(W.config(3), seed=2)
    assert len(t3) == 4 and all(0 <= lo <= 87472 - 128 for _, lo, _ in t3)

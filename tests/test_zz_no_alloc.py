"""ca_backward_static_ws (the entry point for callers that cannot allocate) against ca_backward, through the C ABI:
two calls in a row on one GPU, the second with a smaller batch, so that the shared device-resident workspace still
holds the first call's contents when the second runs."""
import numpy as np
import pytest
import torch

import parity_util as P
from paper_2510_18121_amd import binding as B
from paper_2510_18121_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(b):
    q, k, v, d_o = W.make_tensors(b, DEV)
    ref = P.run_hip(b, q, k, v, d_o)  # ca_forward + ca_backward with a caller-provided workspace
    plan = ref["plan"]
    assert plan.workspace_bytes()[1] <= B.lib().ca_static_workspace_bytes()
    dq, dk, dv = (torch.full_like(t, float("nan")) for t in (q, k, v))
    B.ca_backward_static_ws(plan, q, k, v, ref["o"], d_o, ref["lse"], dq, dk, dv)
    torch.cuda.synchronize()
    return ref, {"dq": dq, "dk": dk, "dv": dv}, (q, k, v, d_o)


def test_static_workspace_backward_matches_ca_backward_twice_in_a_row():
    big = W.custom([1500, 260, 700], [(0, 0, 811), (0, 811, 689), (1, 0, 260), (2, 100, 600)], 8, 2, 128, seed=71)
    small = W.custom([300, 40], [(0, 0, 77), (0, 77, 223), (1, 0, 40)], 4, 2, 64, seed=72)
    for b, tag in ((big, "first call"), (small, "second, smaller call")):
        ref, got, tensors = _both(b)
        for n in ("dq", "dk", "dv"):
            # same kernels on the same inputs: the results are the same bits
            assert torch.equal(got[n], ref[n]), (tag, n)
        # and they meet the oracle's tolerances like every other path
        oracle_ref = P.run_oracle(b, *tensors)
        e = P.errors({**ref, **got}, oracle_ref)
        print(tag, e, flush=True)
        P.assert_parity(e, tag)


def test_static_workspace_backward_refuses_what_does_not_fit():
    cap = B.lib().ca_static_workspace_bytes()
    b = W.custom([8192], [(0, 0, 8192)], 32, 8, 128, seed=73)  # about 136 MB of backward workspace
    q, k, v, d_o = W.make_tensors(b, DEV)
    plan = B.ca_plan(b)
    assert plan.workspace_bytes()[1] > cap
    o = torch.zeros_like(q)
    lse = torch.zeros((b.n_q_heads, b.total_q), dtype=torch.float32, device=DEV)
    dq, dk, dv = torch.zeros_like(q), torch.zeros_like(k), torch.zeros_like(v)
    with pytest.raises(B.CaError) as e:
        B.ca_backward_static_ws(plan, q, k, v, o, d_o, lse, dq, dk, dv)
    assert e.value.code == B.CA_ERR_WORKSPACE and "static workspace" in e.value.detail
    torch.cuda.synchronize()
    assert torch.all(dq == 0) and torch.all(dk == 0)  # nothing was launched

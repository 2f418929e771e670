"""Helpers for the GPU parity tests: run the HIP path through the C ABI, run the oracle on the same bits."""
import numpy as np
import torch

import oracle
from paper_2510_18121_amd import binding as B
from paper_2510_18121_amd import workloads as W

O_MAX_ABS = 1e-2      # bf16 outputs vs fp64 oracle
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


def run_oracle(batch, q, k, v, d_o=None, want=("dq", "dk", "dv")):
    q64, k64, v64 = to64(q), to64(k), to64(v)
    if d_o is None:
        o, lse = oracle.forward(batch, q64, k64, v64)
        return {"o": o, "lse": lse}
    return oracle.forward_backward(batch, q64, k64, v64, to64(d_o), want=want)


def rel_l2(a, ref):
    den = float(np.linalg.norm(ref.ravel()))
    num = float(np.linalg.norm((a - ref).ravel()))
    return num / den if den > 0 else num


def errors(hip, ref, rows=None):
    """Error figures of a HIP result against an oracle result (optionally only on the packed Q rows `rows`)."""
    sel = slice(None) if rows is None else rows
    e = {"o_max_abs": float(np.abs(to64(hip["o"])[sel] - ref["o"][sel]).max()) if ref["o"].size else 0.0,
         "lse_max_abs": float(np.abs(to64(hip["lse"])[:, sel] - ref["lse"][:, sel]).max()) if ref["lse"].size else 0.0}
    for g in ("dq", "dk", "dv"):
        if g in hip and ref.get(g) is not None:
            a, r = to64(hip[g]), ref[g]
            if g == "dq":
                a, r = a[sel], r[sel]
            e[g + "_rel_l2"] = rel_l2(a, r)
    return e


def assert_parity(e, tag=""):
    assert e["o_max_abs"] <= O_MAX_ABS, (tag, e)
    assert e["lse_max_abs"] <= LSE_MAX_ABS, (tag, e)
    for g in ("dq", "dk", "dv"):
        if g + "_rel_l2" in e:
            assert e[g + "_rel_l2"] <= GRAD_REL_L2, (tag, e)

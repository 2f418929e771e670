"""torch.autograd wrapper over the C-ABI calls, for training code that wants an attention-server step as one
differentiable op (the paper's runtime calls a fused variable-length attention kernel per server step, Section 4.1;
this is the same call shape: packed Q, K, V in, packed O out, gradients through backward()).

Plumbing only: forward() calls ca_forward, backward() calls ca_backward; nothing is computed here.  The op saves
Q, K, V, O and the per-row log-sum-exp and recomputes P in backward (Section 2.1)."""
from __future__ import annotations

import torch

from . import binding as B


class _CoreAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, server):
        b = server.plan.batch
        o = torch.empty_like(q)
        lse = torch.empty((b.n_q_heads, b.total_q), dtype=torch.float32, device=q.device)
        B.ca_forward(server.plan, q, k, v, o, lse, server.ws)
        ctx.save_for_backward(q, k, v, o, lse)
        ctx.server = server
        return o

    @staticmethod
    def backward(ctx, d_o):
        q, k, v, o, lse = ctx.saved_tensors
        s = ctx.server
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        B.ca_backward(s.plan, q, k, v, o, d_o.contiguous(), lse, dq, dk, dv, s.ws)
        return dq, dk, dv, None


class AttentionServer:
    """One fused batch of CA-tasks planned once and run as a differentiable op:

        server = AttentionServer(batch)          # plans, uploads, allocates the workspace
        o = server(q, k, v)                      # bf16 [total_q, Hq, D]; q, k, v may require grad
        o.backward(d_o)                          # q.grad, k.grad, v.grad

    `batch` is any object with the descriptor's fields (e.g. workloads.Batch).  Rows of q that belong to no task
    have undefined output and zero gradient."""

    def __init__(self, batch, device="cuda"):
        self.plan = B.ca_plan(batch)
        self.ws = B.alloc_workspace(self.plan, device)

    def __call__(self, q, k, v):
        return _CoreAttention.apply(q, k, v, self)

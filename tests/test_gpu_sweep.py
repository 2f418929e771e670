"""GPU tests of the rows next to the hot path: parity of the HIP path on the chunks of the shard-length experiment
(thousands of tiny CA-tasks in one fused call; Section 3.3), and the latency model filled from measurements
(Section 4.2, "Profiler")."""
import numpy as np
import pytest
import torch

import parity_util as P
from paper_2510_18121_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("mode,n,ctx", [("distinct", 16, 768), ("distinct", 48, 1024), ("shared", 16, 2048), ("shared", 80, 2560)])
def test_shard_chunks_match_the_oracle(mode, n, ctx):
    """Small twins of the experiment's chunks (same generator, fewer tokens, shorter contexts), all tensors."""
    chunk = 3840 if n in (48, 80) else 4096
    b = W.shard_chunk(n, mode, seed=3, chunk_tokens=chunk, max_context=ctx, hq=4, hkv=2, d=128)
    q, k, v, d_o = W.make_tensors(b, DEV)
    e = P.errors(P.run_hip(b, q, k, v, d_o), P.run_oracle(b, q, k, v, d_o))
    print(b.name, b.n_tasks, "tasks", b.n_docs, "documents", e, flush=True)
    P.assert_parity(e, b.name)


def test_latency_grid_predicts_unmeasured_tasks():
    """A coarse grid measured on this GPU; tasks between grid points are then timed and compared with the model's
    prediction (bilinear in latency between grid points a factor of four apart: within 15 %; the model's arithmetic is
    pinned by the CPU tests)."""
    from paper_2510_18121_amd.profiler import measure_grid, time_batch

    g = measure_grid([256, 1024, 4096], [1024, 4096, 16384], hq=8, hkv=2, d=128, steps=3, warmup=1)
    assert np.isfinite(g.seconds[0]).all() and g.max_throughput() > 0
    for ql, kl in [(512, 2048), (2048, 8192), (3072, 12288)]:
        b = W.custom([kl], [(0, kl - ql, ql)], 8, 2, 128, seed=11)
        t = time_batch(b, steps=3, warmup=1) * 1e-3
        pred = g.predict(ql, kl)
        print(f"task q={ql} kv={kl}: measured {t * 1e6:.0f} us, predicted {pred * 1e6:.0f} us", flush=True)
        assert 0.85 * t <= pred <= 1.15 * t, (ql, kl, t, pred)


def test_scheduled_servers_together_equal_the_single_call():
    """Disaggregation on one GPU: the tasks of a batch are scheduled over 4 virtual servers (Items are cut and
    moved), every server runs its own fused call on the rows it was given, and the pieces are put back together:
    O, LSE and dQ row by row, dK and dV summed over the servers.  The result is compared with the oracle on the
    whole batch (and with the single fused call)."""
    from paper_2510_18121_amd import scheduler as S

    b = W.one_kv_group(W.config(3, 16))
    q, k, v, d_o = W.make_tensors(b, DEV)
    whole = P.run_hip(b, q, k, v, d_o)
    ref = P.run_oracle(b, q, k, v, d_o)
    items = S.items_from_batch(b, 4)
    sch = S.schedule(items, 4, size_q=1024.0, size_kv=512.0, eps=0.02)
    assert sch.moves and sch.imbalance() <= 1.03
    o, dq = torch.zeros_like(q), torch.zeros_like(q)
    lse = torch.zeros_like(whole["lse"])
    dk, dv = torch.zeros(k.shape, device=DEV), torch.zeros(v.shape, device=DEV)  # fp32 sums over servers
    for srv in sch.servers:
        sub, qrows, kvrows = S.server_batch(b, srv)
        qi, ki = torch.as_tensor(qrows, device=DEV), torch.as_tensor(kvrows, device=DEV)
        h = P.run_hip(sub, q[qi].contiguous(), k[ki].contiguous(), v[ki].contiguous(), d_o[qi].contiguous())
        o[qi], dq[qi] = h["o"], h["dq"]
        lse[:, qi] = h["lse"]
        dk.index_add_(0, ki, h["dk"].float())
        dv.index_add_(0, ki, h["dv"].float())
    e = P.errors({"o": o, "lse": lse, "dq": dq, "dk": dk, "dv": dv}, ref)
    print("4 servers put together:", e, flush=True)
    P.assert_parity(e, "scheduled servers")
    # against the single fused call: same rows, at most one bf16 unit apart where tiles were cut differently
    assert (o.float() - whole["o"].float()).abs().max().item() <= 2.0 ** -5
    assert (lse - whole["lse"]).abs().max().item() <= 1e-5

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


@pytest.mark.parametrize("hq,hkv,d,n,ctx,chunk", [(8, 2, 128, 64, 1536, 8192), (8, 1, 128, 64, 1024, 16384),
                                                   (8, 2, 64, 64, 1536, 8192), (4, 1, 128, 128, 2048, 24576),
                                                   (8, 2, 128, 32, 1536, 4096), (6, 2, 128, 64, 1536, 12288),
                                                   (8, 2, 128, 16, 1536, 4096), (8, 1, 128, 16, 1024, 4096),
                                                   (8, 2, 64, 24, 1536, 4080), (6, 2, 128, 16, 1536, 4096)])
def test_chained_short_units_match_the_oracle(hq, hkv, d, n, ctx, chunk):
    """Lone shards with a context, all tensors: every (KV tile, KV head) unit of the dK/dV kernel is a few steps, so
    the planner chains them.  Inside one document the Q/dO stream runs on from unit to unit; with 3 or more steps per
    unit (4 or 8 heads per group, or two query blocks) K and V are fetched a unit ahead, also across documents, where
    the stream starts again; with 3 heads per group (2 steps) the stream runs on without the fetch.  Shards of at
    most 32 / 16 rows have the rows of 2 / 4 heads of a group packed into each 64-row tile of the dK/dV kernel (not with 3
    heads per group)."""
    from paper_2510_18121_amd import binding as B
    b = W.shard_chunk(n, "distinct", seed=5, chunk_tokens=chunk, max_context=ctx, hq=hq, hkv=hkv, d=d)
    info = B.ca_plan_host(b).info()
    assert info["n_bwd_workgroups"] < info["n_bwd_units"], "units are chained"
    q, k, v, d_o = W.make_tensors(b, DEV)
    e = P.errors(P.run_hip(b, q, k, v, d_o), P.run_oracle(b, q, k, v, d_o))
    print(b.name, b.n_tasks, "tasks", info["n_bwd_units"], "units in", info["n_bwd_workgroups"], "workgroups", e, flush=True)
    P.assert_parity(e, b.name)


@pytest.mark.parametrize("n", [64, 128])
def test_full_size_shard_chunk_on_exact_subproblems(n):
    """A chunk of the shard-length experiment at its full size (32K tokens, contexts up to 16K: chains of up to 32
    units): sampled query rows, the key gradients of every document of at most 2048 keys and of the last keys of the
    longest one for one KV head, and the sum identities over the whole output."""
    b = W.shard_chunk(n, "distinct", seed=0)
    tensors = W.make_tensors(b, DEV)
    hip = P.run_hip(b, *tensors)
    rows = P.sample_rows(b, 192, seed=n)
    e = P.check_sampled_rows(b, tensors, hip, rows, kv_head=n % b.n_kv_heads)
    e.update(P.check_key_gradients(b, tensors, hip, kv_head=(n // 64) % b.n_kv_heads, tail_keys=256, require_full=False))
    e.update(P.sum_invariants(b, tensors[3], hip))
    print(b.name, e, flush=True)
    assert e["o_err_over_bound"] <= 1.0 and e["lse_max_abs"] <= P.LSE_MAX_ABS and e["dq_rel_l2"] <= P.GRAD_REL_L2
    for key, val in e.items():
        if key.endswith("row_rel_l2"):
            assert val <= P.ROW_REL_L2, (key, val)
        elif key.endswith("rel_l2"):
            assert val <= P.GRAD_REL_L2, (key, val)
    assert e["sum_dv_minus_sum_do_rel"] <= P.SUM_INVARIANT and e["sum_dk_rel"] <= P.SUM_INVARIANT, e
    assert e["short_docs_keys"] >= 16384 and e["tail_keys"] > 0 and e["rows"] >= 192


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

"""The forward and backward calls allocate nothing and never synchronise, so a caller can record them into a HIP
graph once and replay it (Section 6.2 reports allocator and launch overhead from the varying shapes of
CA-tasks and names static allocation plus graphs as the remedy).  Replays are checked against the eager result bit
for bit, with eager work and synchronisations between them."""
import pytest
import torch

from paper_2510_18121_amd import binding as B
from paper_2510_18121_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_forward_backward_and_merge_replay_from_a_graph():
    b = W.one_kv_group(W.config(3, 32))
    pb, gather, part_rows = W.split_kv(b, 512)
    q, k, v, d_o = W.make_tensors(b, DEV)
    g = torch.as_tensor(gather, device=DEV)
    pr = torch.as_tensor(part_rows, device=DEV).contiguous()
    qp, dop = q.index_select(0, g).contiguous(), d_o.index_select(0, g).contiguous()
    plan = B.ca_plan(pb)
    ws = B.alloc_workspace(plan, DEV)
    o_p, dq_p = torch.empty_like(qp), torch.empty_like(qp)
    lse_p = torch.empty((pb.n_q_heads, pb.total_q), dtype=torch.float32, device=DEV)
    o, dq = torch.empty_like(q), torch.empty_like(q)
    lse = torch.empty((b.n_q_heads, b.total_q), dtype=torch.float32, device=DEV)
    dk, dv = torch.empty_like(k), torch.empty_like(v)
    outs = (o, lse, dq, dk, dv)

    def step():
        B.ca_forward(plan, qp, k, v, o_p, lse_p, ws)
        B.ca_merge_partials(pr, o_p, lse_p, o, lse, o_p, lse_p)
        B.ca_backward(plan, qp, k, v, o_p, dop, lse_p, dq_p, dk, dv, ws)
        B.ca_sum_partial_dq(pr, dq_p, dq)

    step()  # eager: also the first-call set-up of the kernels (dynamic LDS size attribute)
    torch.cuda.synchronize()
    want = [t.clone() for t in outs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t in outs + (o_p, lse_p, dq_p):
            t.fill_(float("nan"))  # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, w in zip(outs, want):
            assert torch.equal(t, w), f"replay {rep} differs from the eager result"
        # new inputs in the same buffers: the graph computes on what the buffers hold at replay time
    qp.mul_(0.5)
    graph.replay()
    torch.cuda.synchronize()
    got = o.clone()
    step()
    torch.cuda.synchronize()
    assert torch.equal(got, o)


def test_one_plan_serves_two_streams_with_a_workspace_each():
    """The launch calls only read the plan: two streams run forward and backward on it at the same time, each with
    inputs, outputs and a workspace of its own, and get what each gets alone."""
    b = W.one_kv_group(W.config(2, 4))
    plan = B.ca_plan(b)
    streams = [torch.cuda.Stream(device=DEV) for _ in range(2)]
    sets = []
    for i in range(2):
        q, k, v, d_o = W.make_tensors(b, DEV)
        if i:
            q, k = (q * 0.5).contiguous(), (k * 1.5).contiguous()
        ws = B.alloc_workspace(plan, DEV)
        o, dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        lse = torch.empty((b.n_q_heads, b.total_q), dtype=torch.float32, device=DEV)
        sets.append((q, k, v, d_o, o, lse, dq, dk, dv, ws))

    def run(i, stream):
        q, k, v, d_o, o, lse, dq, dk, dv, ws = sets[i]
        B.ca_forward(plan, q, k, v, o, lse, ws, stream=stream)
        B.ca_backward(plan, q, k, v, o, d_o, lse, dq, dk, dv, ws, stream=stream)

    want = []
    for i in range(2):  # alone, on the current stream
        run(i, None)
        torch.cuda.synchronize()
        want.append([t.clone() for t in sets[i][4:9]])
        for t in sets[i][4:9]:
            t.fill_(float("nan"))
    torch.cuda.synchronize()
    for rep in range(3):  # together
        for i in range(2):
            run(i, streams[i])
        torch.cuda.synchronize()
        for i in range(2):
            for t, w in zip(sets[i][4:9], want[i]):
                assert torch.equal(t, w), f"stream {i}, repetition {rep}"


def test_one_plan_serves_four_host_threads():
    """Four host threads launch forward and backward on one plan at the same time, each on a stream and with buffers of
    its own (created beforehand); every thread gets the result of a lone call, bit for bit."""
    import threading

    b = W.one_kv_group(W.config(2, 8))
    plan = B.ca_plan(b)
    q, k, v, d_o = W.make_tensors(b, DEV)
    ws = B.alloc_workspace(plan, DEV)
    o, dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    lse = torch.empty((b.n_q_heads, b.total_q), dtype=torch.float32, device=DEV)
    B.ca_forward(plan, q, k, v, o, lse, ws)
    B.ca_backward(plan, q, k, v, o, d_o, lse, dq, dk, dv, ws)
    torch.cuda.synchronize()
    want = [t.clone() for t in (o, lse, dq, dk, dv)]
    n = 4
    streams = [torch.cuda.Stream(device=DEV) for _ in range(n)]
    bufs = [[torch.full_like(t, float("nan")) for t in want] + [B.alloc_workspace(plan, DEV)] for _ in range(n)]
    torch.cuda.synchronize()
    errors = []

    def work(i):
        try:
            o_i, lse_i, dq_i, dk_i, dv_i, ws_i = bufs[i]
            for _ in range(3):
                B.ca_forward(plan, q, k, v, o_i, lse_i, ws_i, stream=streams[i])
                B.ca_backward(plan, q, k, v, o_i, d_o, lse_i, dq_i, dk_i, dv_i, ws_i, stream=streams[i])
            streams[i].synchronize()
        except BaseException as e:  # noqa: BLE001 - reported by the main thread
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(n)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not errors, errors
    torch.cuda.synchronize()
    for i in range(n):
        for got, w in zip(bufs[i][:5], want):
            assert torch.equal(got, w), f"thread {i}"

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
    prediction.  The bound is loose on purpose (timing noise on a shared box); the model's arithmetic is pinned
    by the CPU tests."""
    from paper_2510_18121_amd.profiler import measure_grid, time_batch

    g = measure_grid([256, 1024, 4096], [1024, 4096, 16384], hq=8, hkv=2, d=128, steps=3, warmup=1)
    assert np.isfinite(g.seconds[0]).all() and g.max_throughput() > 0
    for ql, kl in [(512, 2048), (2048, 8192), (3072, 12288)]:
        b = W.custom([kl], [(0, kl - ql, ql)], 8, 2, 128, seed=11)
        t = time_batch(b, steps=3, warmup=1) * 1e-3
        pred = g.predict(ql, kl)
        print(f"task q={ql} kv={kl}: measured {t * 1e6:.0f} us, predicted {pred * 1e6:.0f} us", flush=True)
        assert 0.4 * t <= pred <= 2.5 * t

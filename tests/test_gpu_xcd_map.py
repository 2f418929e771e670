"""The planner deals the units of one KV head to one XCD by assuming that the workgroups of a launch are dealt to the
8 XCDs round robin in index order: workgroup i runs on XCD (i + c) mod 8, with c whatever XCD the previous launch
stopped at, so workgroups 8 apart share an XCD and its L2 (Section 3.2's "throughput depends on the aggregate tokens"
is held up by that reuse).  Nothing documents the mapping, so this test reads it from the hardware and fails loudly if
it ever changes."""
import numpy as np
import pytest
import torch

from paper_2510_18121_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,threads", [(256, 256), (8296, 512), (8192, 256)])
def test_workgroups_are_dealt_to_the_xcds_round_robin(n, threads):
    """Grids like the benchmark's: one workgroup per CU, the forward's 8296 units of 512 threads (workload 2), the
    dK/dV kernel's 8192 units of 256 threads (workload 3)."""
    x = B.ca_xcd_map(n, threads).cpu().numpy()
    torch.cuda.synchronize()
    assert x.min() >= 0 and x.max() <= 7, (x.min(), x.max())
    want = (np.arange(n) + int(x[0])) % 8
    bad = np.flatnonzero(x != want)
    assert bad.size == 0, (f"{bad.size} of {n} workgroups are not on XCD (i + {int(x[0])}) mod 8, "
                           f"first at {bad[:8]}: {x[bad[:8]]}")


def test_xcd_map_rejects_bad_shapes():
    lib = B.lib()
    assert lib.ca_xcd_map(8, 100, None, None) == B.CA_ERR_INVALID_ARG
    assert lib.ca_xcd_map(-1, 256, None, None) == B.CA_ERR_INVALID_ARG
    assert lib.ca_xcd_map(8, 256, None, None) == B.CA_ERR_INVALID_ARG  # null output
    assert lib.ca_xcd_map(0, 256, None, None) == B.CA_OK

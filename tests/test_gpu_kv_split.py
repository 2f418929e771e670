"""GPU parity of query shards that attend a sub-range of their context (the extension named in the paper's
Limitations section): partial tasks over key windows through ca_forward, ca_merge_partials, ca_backward with the
merged statistics and ca_sum_partial_dq, against the fp64 oracle of the WHOLE-context attention on the same bf16
bits, at the tolerances of the plain path (max |O| error 1e-2, relative L2 1e-2 on the gradients)."""
import numpy as np
import pytest
import torch

import oracle
import parity_util as P
from paper_2510_18121_amd import binding as B
from paper_2510_18121_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def check(b, window, tag, in_place=True):
    q, k, v, d_o = W.make_tensors(b, DEV)
    hip = P.run_hip_kv_split(b, window, q, k, v, d_o, in_place=in_place)
    ref = P.run_oracle(b, q, k, v, d_o)
    e = P.errors(hip, ref)
    print(tag, "parts", hip["n_parts"], e, flush=True)
    P.assert_parity(e, tag)
    # the merged values written back into the partial rows are the merged rows themselves
    pb, gather, _ = W.split_kv(b, window)
    g = torch.as_tensor(gather, device=DEV)
    assert torch.equal(hip["o_back"], hip["o"].index_select(0, g))
    assert torch.equal(hip["lse_back"], hip["lse"].index_select(1, g))
    return hip, ref


@pytest.mark.parametrize("window", [128, 200, 1000])
def test_tiny_workload_by_key_windows(window):
    check(W.config(1), window, f"cfg1 window {window}")


def test_write_back_into_separate_buffers():
    check(W.config(1), 300, "cfg1 window 300, separate write-back", in_place=False)


@pytest.mark.parametrize("idx,div,window", [(3, 16, 512), (5, 16, 1000), (4, 64, 1024)])
def test_downscaled_twins_by_key_windows(idx, div, window):
    check(W.one_kv_group(W.config(idx, div)), window, f"cfg{idx}/{div} window {window}")


def test_ragged_windows_and_head_layouts():
    """Window lengths that are no multiple of any tile, 1-row shards, GQA 8 and head_dim 64 and 128."""
    tasks, a = [], 0
    for n in [1, 2, 15, 17, 31, 33, 63, 65, 127, 129, 255, 257, 300]:
        tasks.append((0, a, n))
        a += n
    for d, hq, hkv, window in ((128, 8, 1, 77), (64, 4, 2, 130), (128, 8, 2, 1295)):
        b = W.custom([a, 1, 200], tasks + [(1, 0, 1), (2, 0, 77), (2, 77, 123)], hq, hkv, d, doc_order=[2, 0, 1], seed=31)
        check(b, window, f"ragged d{d} {hq}/{hkv} window {window}")


def test_one_key_windows_and_the_part_limit():
    """Windows of a single key (every partial task sees exactly one key: its softmax is 1 and all the weighting
    happens in the merge), up to the limit of 64 parts per row; one part more is refused."""
    b = W.custom([40, 64], [(0, 0, 40), (1, 10, 54)], 4, 2, 64, seed=35)
    hip, _ = check(b, 1, "one-key windows")
    assert hip["n_parts"] == 64
    pr = torch.zeros((65, 8), dtype=torch.int32, device=DEV)
    o_part = torch.zeros((8, 4, 64), dtype=torch.bfloat16, device=DEV)
    lse_part = torch.zeros((4, 8), device=DEV)
    with pytest.raises(B.CaError) as e:
        B.ca_merge_partials(pr, o_part, lse_part, torch.empty_like(o_part), torch.empty_like(lse_part))
    assert e.value.code == B.CA_ERR_INVALID_ARG and "n_parts" in e.value.detail


def test_clipped_task_without_merge():
    """A single task whose kv_len stops short of its rows: the HIP path against the oracle of that very task."""
    b = W.custom([900], [(0, 100, 600)], 4, 2, 128, seed=32)
    b.task_kv_len[0] = 333
    q, k, v, d_o = W.make_tensors(b, DEV)
    hip = P.run_hip(b, q, k, v, d_o)
    ref = P.run_oracle(b, q, k, v, d_o)
    e = P.errors(hip, ref)
    print("clipped", e, flush=True)
    P.assert_parity(e, "clipped")
    assert torch.all(hip["dk"][333:] == 0) and torch.all(hip["dv"][333:] == 0)


def test_merge_kernel_against_the_oracle_merge_with_missing_parts():
    """ca_merge_partials and ca_sum_partial_dq alone on random partial results, rows with 0..n_parts parts."""
    rng = np.random.default_rng(33)
    n_rows, n_parts, hq, d, tq = 1000, 5, 3, 64, 6000
    perm = rng.permutation(tq)[: n_rows * n_parts].reshape(n_parts, n_rows).astype(np.int32)
    perm[rng.random((n_parts, n_rows)) < 0.3] = -1
    perm[:, :7] = -1  # rows without any part
    g = torch.Generator(device=DEV)
    g.manual_seed(34)
    o_part = torch.randn((tq, hq, d), generator=g, device=DEV).to(torch.bfloat16)
    lse_part = 3.0 * torch.randn((hq, tq), generator=g, device=DEV)
    pr = torch.as_tensor(perm, device=DEV)
    o = torch.full((n_rows, hq, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    lse = torch.full((hq, n_rows), float("nan"), device=DEV)
    B.ca_merge_partials(pr, o_part, lse_part, o, lse)
    dq = torch.full_like(o, float("nan"))
    B.ca_sum_partial_dq(pr, o_part, dq)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.merge_partials(perm, P.to64(o_part), lse_part.double().cpu().numpy())
    assert P.o_errors(P.to64(o), o_ref)[1] <= 1.0  # 1e-2, or one bf16 rounding where |O| >= 4 (inputs are N(0,1) here)
    has = (perm >= 0).any(axis=0)
    assert np.abs(lse.double().cpu().numpy()[:, has] - lse_ref[:, has]).max() <= 1e-4
    assert torch.all(o[:7] == 0) and torch.all(torch.isneginf(lse[:, :7]))
    sum_ref = np.zeros((n_rows, hq, d))
    o64 = P.to64(o_part)
    for i in range(n_parts):
        ok = perm[i] >= 0
        sum_ref[ok] += o64[perm[i][ok]]
    assert np.abs(P.to64(dq) - sum_ref).max() <= 2.0 ** -7 * max(1.0, np.abs(sum_ref).max())
    # out-of-range indices count as absent: same result with them in place of -1
    perm2 = perm.copy()
    perm2[perm2 < 0] = tq + 5
    o2 = torch.empty_like(o)
    lse2 = torch.empty_like(lse)
    B.ca_merge_partials(torch.as_tensor(perm2, device=DEV), o_part, lse_part, o2, lse2)
    torch.cuda.synchronize()
    assert torch.equal(o2, o) and torch.equal(lse2, lse)

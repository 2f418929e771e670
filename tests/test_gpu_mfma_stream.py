"""The calibration kernel behind the sustained matrix-pipe rate: its instructions run and its count is right."""
import pytest
import torch

from paper_2510_18121_amd import binding as B, mfma_rate as M

pytestmark = pytest.mark.gpu


def test_all_ones_operands_give_the_exact_count():
    ops = M.make_operands("ones")
    for n_mfma, n_wg, side in ((64, 3, 0), (640, 17, 0), (128, 5, 1), (192, 4, 2)):  # side work leaves them alone
        sums = torch.full((n_wg, 256), -1.0, dtype=torch.float32, device="cuda")
        B.ca_mfma_stream(ops, n_mfma, sums, side)
        torch.cuda.synchronize()
        # every MFMA adds 16 to each of the 16 values a lane holds of its chain; 4 chains share the MFMAs equally
        assert torch.equal(sums, torch.full_like(sums, 256.0 * n_mfma))


def test_products_follow_the_documented_pairing():
    # A fragments all ones, B fragment i filled with i+1: MFMA (r, j) adds 16 (i+1) with i = (j + r) mod 8, and over
    # the 64 MFMAs of a round every chain meets every B fragment twice
    ops = torch.ones((16, 256, 8), dtype=torch.bfloat16, device="cuda")
    for i in range(8):
        ops[2 * i + 1] = float(i + 1)
    sums = torch.empty((2, 256), dtype=torch.float32, device="cuda")
    B.ca_mfma_stream(ops, 128, sums)
    torch.cuda.synchronize()
    per_round_per_chain = 16 * 2 * sum(range(1, 9))
    assert torch.equal(sums, torch.full_like(sums, 2.0 * 4 * 16 * per_round_per_chain))


def test_zero_work_and_bad_arguments():
    ops = M.make_operands("zeros")
    sums = torch.full((2, 256), 7.0, dtype=torch.float32, device="cuda")
    B.ca_mfma_stream(ops, 0, sums)
    torch.cuda.synchronize()
    assert torch.equal(sums, torch.zeros_like(sums))
    with pytest.raises(B.CaError):
        B.ca_mfma_stream(ops, 65, sums)
    with pytest.raises(B.CaError):
        B.ca_mfma_stream(ops, 64, sums, side_work=3)
    with pytest.raises(ValueError):
        B.ca_mfma_stream(ops[:8], 64, sums)


def test_sustained_rate_is_plausible():
    for side, wpc in ((0, 1), (1, 2)):
        r = M.sustained_tflops("normal", side, wpc, launch_ms=40.0, launches=2)
        assert all(200.0 < x < 2600.0 for x in r), r

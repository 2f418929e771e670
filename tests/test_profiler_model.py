"""CPU tests of the CA-task latency model (Section 4.2, "Profiler") and of the shard-chunk generator of the
throughput-versus-shard-length experiment (Section 3.3)."""
import numpy as np
import pytest

from paper_2510_18121_amd import workloads as W
from paper_2510_18121_amd.profiler import LatencyGrid, task_flops


def _grid(fn, q_axis=(64, 256, 1024, 4096), kv_axis=(64, 256, 1024, 4096, 16384), hq=8, d=128, tol=0.05):
    sec = np.array([[fn(q, kv) if kv >= q else np.nan for kv in kv_axis] for q in q_axis], float)
    return LatencyGrid(np.array(q_axis), np.array(kv_axis), sec, hq, d, True, tol)


def test_bilinear_interpolation_is_exact_for_bilinear_latencies():
    # a + b q + c kv + e q kv is reproduced exactly inside every fully measured cell
    f = lambda q, kv: 1e-4 + 2e-7 * q + 3e-8 * kv + 5e-12 * q * kv
    g = _grid(f, tol=-1.0)  # negative tolerance: no point counts as saturated
    for q, kv in [(100, 300), (256, 1024), (700, 9000), (3000, 12000), (64, 64), (4096, 16384)]:
        assert g.predict(q, kv) == pytest.approx(f(q, kv), rel=1e-12)


def test_grid_points_are_returned_as_measured():
    rng = np.random.default_rng(0)
    noise = {}
    f = lambda q, kv: noise.setdefault((q, kv), float(rng.uniform(1e-4, 1e-3)))
    g = _grid(f, tol=-1.0)
    for i, q in enumerate(g.q_axis):
        for j, kv in enumerate(g.kv_axis):
            if kv >= q:
                assert g.predict(int(q), int(kv)) == pytest.approx(g.seconds[i, j], rel=1e-12)


def test_saturation_region_uses_the_best_measured_throughput():
    # latency = launch overhead + flops / peak: throughput saturates for large tasks
    peak, t0 = 9.0e14, 2e-6
    f = lambda q, kv: t0 + task_flops(q, kv, 8, 128) / peak
    g = _grid(f, tol=0.05)
    sat = g.saturated()
    assert sat[-1, -1] and not sat[0, 0]
    q, kv = 3000, 14000  # all four corners saturated
    want = task_flops(q, kv, 8, 128) / g.max_throughput()
    assert g.predict(q, kv) == pytest.approx(want, rel=1e-12)
    # and the prediction is within the tolerance of the true latency there
    assert g.predict(q, kv) == pytest.approx(f(q, kv), rel=0.06)
    # a small task is outside the region: interpolated, close to the truth, far from flops / peak
    assert g.predict(100, 200) == pytest.approx(f(100, 200), rel=0.2)
    assert g.predict(100, 200) > 3 * task_flops(100, 200, 8, 128) / g.max_throughput()


def test_cells_cut_by_the_diagonal_use_their_measured_corners_only():
    f = lambda q, kv: 1e-4 + 1e-8 * kv
    g = _grid(f, tol=-1.0)
    # q = 600 lies between 256 and 1024; kv = 700 between 256 and 1024: corner (1024, 256) is unmeasured
    t = g.predict(600, 700)
    assert np.isfinite(t) and f(600, 256) <= t <= f(600, 1024)
    with pytest.raises(ValueError):
        g.predict(500, 400)


def test_long_task_on_the_diagonal_of_a_coarse_grid_is_priced_by_its_own_work():
    # fixed cost + work / rate; the whole-document task (q = kv = 16384) sits in a cell whose measured corners hold
    # up to seven times its work: interpolating their seconds would overprice it several times over
    f = lambda q, kv: 40e-6 + task_flops(q, kv, 8, 128) / 8e14
    g = LatencyGrid([1024, 4096, 16384], [1024, 8192, 65536],
                    [[f(q, kv) if kv >= q else np.nan for kv in (1024, 8192, 65536)] for q in (1024, 4096, 16384)], 8, 128,
                    saturation_tolerance=-1.0)
    assert g.predict(16384, 16384) == pytest.approx(f(16384, 16384), rel=0.1)
    assert g.predict(4096, 4096) == pytest.approx(f(4096, 4096), rel=0.15)


def test_json_round_trip():
    g = _grid(lambda q, kv: 1e-4 + 1e-9 * q * kv)
    h = LatencyGrid.from_json(g.to_json())
    assert np.array_equal(g.q_axis, h.q_axis) and np.array_equal(g.kv_axis, h.kv_axis)
    assert np.allclose(g.seconds, h.seconds, equal_nan=True)
    assert h.predict(300, 5000) == g.predict(300, 5000)


def test_task_flops_matches_the_pair_count():
    assert task_flops(4, 10, 2, 8) == 14 * 8 * 2 * (7 + 8 + 9 + 10)
    assert task_flops(4, 10, 2, 8, backward=False) == 4 * 8 * 2 * (7 + 8 + 9 + 10)


@pytest.mark.parametrize("mode", ["distinct", "shared"])
@pytest.mark.parametrize("n", [16, 128, 4096])
def test_shard_chunk_generator(mode, n):
    b = W.shard_chunk(n, mode, seed=1)
    assert b.total_q == 32768 and b.n_tasks == 32768 // n
    assert np.all(b.task_q_len == n) and np.all(b.task_kv_len == b.task_q_pos + n)
    if mode == "distinct":
        assert b.n_docs == b.n_tasks and np.all(b.task_q_pos % 16 == 0) and b.task_q_pos.max() <= 16384
        assert np.all(b.doc_kv_len[b.task_doc] == b.task_kv_len)
    else:
        assert b.n_docs == 2 and b.total_kv == 32768
        for d in range(2):  # the shards of a document tile it exactly
            pos = np.sort(b.task_q_pos[b.task_doc == d])
            assert np.array_equal(pos, np.arange(0, 16384, n))
    # query rows of the tasks tile packed Q without overlap
    order = np.argsort(b.task_q_start)
    assert np.array_equal(b.task_q_start[order], np.arange(0, 32768, n))
    assert W.shard_chunk(n, mode, seed=1).task_q_pos.tolist() == b.task_q_pos.tolist()
    assert mode == "shared" or W.shard_chunk(n, mode, seed=2).task_q_pos.tolist() != b.task_q_pos.tolist()

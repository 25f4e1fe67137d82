"""GPU parity of the shared-window plans (2 or 4 partitions per workgroup behind one graph
stream) against the CPU oracle: every output, element by element, bit-exact."""
import numpy as np
import pytest

from workloads import make_workload, random_layered_dag
from test_gpu_parity import _check, _custom, _oracle, gpu  # noqa: F401

pytestmark = pytest.mark.gpu

COLUMN, WINDOW, SHARED2, SHARED4 = 1, 2, 3, 4


def test_large_sparse_full_shared(gpu, oracle):
    """The benchmark workload at full size, all columns, under both group sizes."""
    _check(gpu, oracle, make_workload("large_sparse"), plans=(SHARED2, SHARED4), out_layouts=(1,))


def test_tiny_and_mlp_shared(gpu, oracle):
    _check(gpu, oracle, make_workload("tiny"), plans=(SHARED2, SHARED4), layouts=(0, 1))
    _check(gpu, oracle, make_workload("mlp"), plans=(SHARED2, SHARED4))
    _check(gpu, oracle, make_workload("mlp", shards=1, P=130), plans=(SHARED2, SHARED4), layouts=(0, 1))


@pytest.mark.parametrize("P", [1, 2, 3, 5, 7, 9, 66, 131])
def test_last_group_not_full(gpu, oracle, P):
    w = make_workload("large_sparse", P=P, levels=40, width=70)
    _check(gpu, oracle, w, plans=(SHARED2, SHARED4), layouts=(0, 1), what=f"ragged P={P}")


def test_paper_scale_fifty_devices(gpu, oracle):
    # 20 KB of cost tables beside a small ring, one slice per tick
    w = make_workload("paper_scale", P=37)
    _check(gpu, oracle, w, plans=(SHARED2, SHARED4), layouts=(0, 1))


def test_wide_levels_and_long_ring(gpu, oracle):
    # 13 slices per tick against at most 8 compute wavefronts; a ring of ~9,000 slots takes
    # 8-byte entries and leaves room for two partitions per workgroup only
    from gpu_util import run_gpu
    w = make_workload("large_sparse", P=21, levels=30, width=800)
    g = gpu.CpGraph.from_workload(w)
    assert g.info["window_ok"] == 1 and g.info["window_slots_b"] > 8192
    g.close()
    _check(gpu, oracle, w, plans=(SHARED2,), layouts=(0, 1))
    with pytest.raises(gpu.CpError) as e:
        run_gpu(w, SHARED4)
    assert e.value.code == -12


def test_comm_heavy_scaled_rows_of_forty_edges(gpu, oracle):
    # rows of 40 edges next to rows of 2-4, 8-byte entries (volumes up to 1e7)
    w = make_workload("comm_heavy", P=70, levels=5, width=600, hub_degree=40)
    _check(gpu, oracle, w, plans=(SHARED2, SHARED4))


def test_graphs_with_far_reads(gpu, oracle):
    """Neighbours too old for the ring come back from the output rows, for all partitions of a
    workgroup at once: the inception workload (one far wavefront), a batch that leaves the last
    workgroup short, both layouts."""
    w = make_workload("inception", P=22)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    assert g.info["window_far_b"] > 0 and g.info["window_far_t"] > 0
    g.close()
    _check(gpu, oracle, w, plans=(SHARED2, SHARED4), layouts=(0, 1))


def test_far_reads_on_wide_ticks(gpu, oracle):
    """Far reads beside ticks of eight slices (several far wavefronts, two stores per compute
    wavefront and tick in some shapes)."""
    import test_gpu_parity as T
    rng = np.random.default_rng(84)
    n, level, src, dst = T._with_long_edges(rng, [600] * 300, extra=5000, min_span=40)
    w = T._custom("long-edges", n, src, dst, rng.integers(1, 3000, size=len(src)), rng.integers(1, 500, size=n),
                  [1, 2, 4, 4], rng.integers(1, 40, size=(4, 4)), rng.integers(0, 4, size=(37, n), dtype=np.uint8), level)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    info = g.info
    g.close()
    assert info["window_ok"] == 1 and info["window_far_b"] > 0 and info["window_far_t"] > 0
    _check(gpu, oracle, w, plans=(SHARED2, SHARED4), layouts=(0, 1))


def test_cp_alone_and_b_alone(gpu, oracle):
    import torch
    w = make_workload("large_sparse", P=13, levels=60, width=200)
    ref = _oracle(oracle, w)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    a = torch.from_numpy(w.assignments).to("cuda:0")
    for plan in (SHARED2, SHARED4):
        out = gpu.cp_eval(g, a, w.speeds, w.bandwidth, want=("cp",), plan=plan)
        assert "b" not in out and np.array_equal(out["cp"].cpu().numpy(), ref["cp"])
        out = gpu.cp_eval(g, a, w.speeds, w.bandwidth, want=("b",), plan=plan, out_layout=1)
        assert np.array_equal(out["b"].cpu().numpy().astype(np.int64), ref["b"])
        out = gpu.cp_eval(g, a, w.speeds, w.bandwidth, want=("tl",), plan=plan, out_layout=1)
        assert np.array_equal(out["tl"].cpu().numpy().astype(np.int64), ref["tl"])
    g.close()


def test_bad_device_id_is_reported(gpu):
    import torch
    w = make_workload("large_sparse", P=6, levels=20, width=70)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    bad = w.assignments.copy()
    bad[4, w.n // 2] = w.k
    a = torch.from_numpy(bad).to("cuda:0")
    for plan in (SHARED2, SHARED4):
        out = gpu.cp_eval(g, a, w.speeds, w.bandwidth, plan=plan, check_status=False)
        torch.cuda.synchronize()
        assert int(out["status"].item()) == 1
    g.close()


@pytest.mark.parametrize("block", range(3))
def test_random_shapes_shared(gpu, oracle, block):
    """Layered DAGs of random depth, width, degree and edge span with random device counts,
    batch sizes and weight ranges, wherever the shared-window plans can run them."""
    from gpu_util import assert_equal_to_oracle, run_gpu
    ran = 0
    for seed in range(block * 8, block * 8 + 8):
        rng = np.random.default_rng(9700 + seed)
        depth = int(rng.integers(2, 80))
        widths = rng.integers(1, int(rng.choice([3, 20, 90, 300, 700])) + 1, size=depth)
        n, level, src, dst = random_layered_dag(rng, widths, int(rng.integers(0, 2)), int(rng.integers(2, 9)),
                                                int(rng.integers(1, max(2, min(depth, 12)))))
        k = int(rng.choice([1, 2, 3, 7, 16, 33, 64]))
        P = int(rng.choice([1, 3, 4, 6, 64, 67, 130]))
        tmax = int(rng.choice([1, 50, 70000, 2**31]))
        cmax = int(rng.choice([1, 99, 10**6]))
        B = rng.integers(1, int(rng.choice([2, 64, 10**5])) + 1, size=(k, k))
        w = _custom(f"random-{seed}", n, src, dst, rng.integers(0, tmax + 1, size=len(src)),
                    rng.integers(0, cmax + 1, size=n), rng.integers(1, int(rng.choice([2, 17, 5000])) + 1, size=k), B,
                    rng.integers(0, k, size=(P, n), dtype=np.uint8), level)
        ref = _oracle(oracle, w)
        g = gpu.CpGraph.from_workload(w, device="cuda:0")
        for plan in (SHARED2, SHARED4):
            for ol in (0, 1):
                for layout in (0, 1):
                    try:
                        res = run_gpu(w, plan, layout=layout, graph=g, out_layout=ol)
                    except gpu.CpError as e:
                        assert e.code in (-12, -8), (seed, plan, e.code)
                        continue
                    ran += 1
                    assert_equal_to_oracle(res, ref, what=f"seed={seed} plan={plan} layout={layout} out={ol} "
                                                          f"n={n} k={k} P={P}")
        g.close()
    assert ran > 0

"""GPU parity of the streamed resident-window plan (compute wavefronts fetch their own slices
into registers two ticks ahead) against the CPU oracle: every output, element by element."""
import numpy as np
import pytest

from workloads import make_workload, random_layered_dag
from test_gpu_parity import _check, _custom, _oracle, gpu  # noqa: F401

pytestmark = pytest.mark.gpu

STREAMED = 6


def test_large_sparse_full_streamed(gpu, oracle):
    """The benchmark workload at full size, all columns; partition-major outputs take the t
    sweep that writes the mask itself, vertex-major outputs the separate mask pass."""
    _check(gpu, oracle, make_workload("large_sparse"), plans=(STREAMED,), out_layouts=(1, 0))


def test_small_workloads_streamed(gpu, oracle):
    _check(gpu, oracle, make_workload("tiny"), plans=(STREAMED,), layouts=(0, 1))
    _check(gpu, oracle, make_workload("mlp"), plans=(STREAMED,))
    _check(gpu, oracle, make_workload("mlp", shards=1, P=130), plans=(STREAMED,), layouts=(0, 1))
    _check(gpu, oracle, make_workload("paper_scale", P=37), plans=(STREAMED,), layouts=(0, 1))


@pytest.mark.parametrize("P", [1, 2, 9, 65, 257])
def test_batches_and_short_sweeps(gpu, oracle, P):
    # 40 ticks, then 3 and 1: the sweep loop runs on to a multiple of eight ticks
    _check(gpu, oracle, make_workload("large_sparse", P=P, levels=40, width=70), plans=(STREAMED,), layouts=(0, 1))
    _check(gpu, oracle, make_workload("large_sparse", P=P, levels=3, width=200), plans=(STREAMED,))
    _check(gpu, oracle, make_workload("large_sparse", P=P, levels=1, width=30), plans=(STREAMED,))


@pytest.mark.parametrize("width,P", [(7, 3), (8, 5), (25, 64), (500, 4)])
def test_mask_rows_for_aligned_and_unaligned_sizes(gpu, oracle, width, P):
    # n * P not a multiple of 16 sends the mask to the separate pass; 500 x 4 takes the fused one
    w = make_workload("large_sparse", P=P, levels=9, width=width)
    _check(gpu, oracle, w, plans=(STREAMED,), out_layouts=(1,))


def test_rows_wider_than_the_entry_registers(gpu, oracle):
    # out-degrees up to 30: sixteen entries per lane in registers, the rest fetched on the spot;
    # in-degrees pile up likewise in the other sweep
    rng = np.random.default_rng(77)
    n, level, src, dst = random_layered_dag(rng, [150] * 30, 1, 30, 3)
    k = 6
    w = _custom("wide-rows", n, src, dst, rng.integers(0, 5000, size=len(src)), rng.integers(1, 900, size=n),
                rng.integers(1, 9, size=k), rng.integers(1, 40, size=(k, k)),
                rng.integers(0, k, size=(70, n), dtype=np.uint8), level)
    g = gpu.CpGraph.from_workload(w)
    assert g.info["window_ok"] == 1 and g.info["max_out_degree"] > 16 and g.info["max_in_degree"] > 16
    g.close()
    _check(gpu, oracle, w, plans=(STREAMED,), layouts=(0, 1))


def test_graphs_it_cannot_run_are_refused(gpu):
    from gpu_util import run_gpu
    for w in (make_workload("inception", P=8),                                             # far reads
              make_workload("comm_heavy", P=8, levels=5, width=600, hub_degree=40)):       # 8-byte entries
        g = gpu.CpGraph.from_workload(w, device="cuda:0")
        with pytest.raises(gpu.CpError) as e:
            run_gpu(w, STREAMED, graph=g)
        assert e.value.code == -12
        g.close()


def test_cp_alone_and_bad_device_id(gpu, oracle):
    import torch
    w = make_workload("large_sparse", P=13, levels=60, width=200)
    ref = _oracle(oracle, w)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    a = torch.from_numpy(w.assignments).to("cuda:0")
    out = gpu.cp_eval(g, a, w.speeds, w.bandwidth, want=("cp",), plan=STREAMED)
    assert "b" not in out and np.array_equal(out["cp"].cpu().numpy(), ref["cp"])
    bad = w.assignments.copy()
    bad[4, w.n // 2] = w.k
    out = gpu.cp_eval(g, torch.from_numpy(bad).to("cuda:0"), w.speeds, w.bandwidth, plan=STREAMED, check_status=False)
    torch.cuda.synchronize()
    assert int(out["status"].item()) == 1
    g.close()

"""GPU parity of the resident-window plan's pair launch (the b-level and the t-level sweep in
one launch, a workgroup of each side by side on a compute unit) against the CPU oracle:
every output, element by element, bit-exact; the stage profile shows that the pair ran."""
import numpy as np
import pytest

from workloads import make_workload
from test_gpu_parity import _oracle, gpu  # noqa: F401

pytestmark = pytest.mark.gpu

WINDOW = 2


def _wide_deep(P):
    # 500 vertices per level with edges over up to ten levels: a ring of 5,500 slots, so that a
    # workgroup of either sweep fills half a compute unit's LDS, as on the benchmark workload
    return make_workload("large_sparse", P=P, levels=120, width=500)


def _eval(gpu, g, w, a, layout, want):
    import torch
    prof = gpu.CpProfile(1)
    d_a = torch.from_numpy(np.ascontiguousarray(a if layout == 0 else a.T)).to("cuda:0")
    out = gpu.cp_eval(g, d_a, w.speeds, w.bandwidth, want=want, plan=WINDOW, assign_layout=layout, out_layout=1,
                      profile=prof)
    torch.cuda.synchronize()
    _, launches = prof.read(0)
    return out, launches


@pytest.mark.parametrize("P", [1, 3, 64, 70])
def test_pair_launch_all_outputs(gpu, oracle, P):
    from paper_1711_01912_amd import binding
    w = _wide_deep(P)
    ref = _oracle(oracle, w)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    shape = g.window_shape(w.k)
    assert shape["partitions_per_workgroup"] == 1 and shape["lds_bytes"] > 64 * 1024, shape
    for layout in (0, 1):                    # vertex-major assignments go through the gathered ids
        out, launches = _eval(gpu, g, w, w.assignments, layout, ("cp", "b", "tl", "mask"))
        assert launches == (1, 0), launches  # one launch ran both sweeps
        assert np.array_equal(out["cp"].cpu().numpy(), ref["cp"])
        assert np.array_equal(out["b"].cpu().numpy().astype(np.int64), ref["b"])
        assert np.array_equal(out["tl"].cpu().numpy().astype(np.int64), ref["tl"])
        assert np.array_equal(binding.mask_to_bool(out["mask"], w.n), ref["mask"])
    g.close()


def test_pair_launch_partial_outputs(gpu, oracle):
    """CP and tl without b (the b sweep then stores nothing), b and tl without CP; one sweep
    alone and rows per vertex keep the launch per sweep."""
    import torch
    w = _wide_deep(37)
    ref = _oracle(oracle, w)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    out, launches = _eval(gpu, g, w, w.assignments, 0, ("cp", "tl"))
    assert launches == (1, 0) and "b" not in out
    assert np.array_equal(out["cp"].cpu().numpy(), ref["cp"])
    assert np.array_equal(out["tl"].cpu().numpy().astype(np.int64), ref["tl"])
    out, launches = _eval(gpu, g, w, w.assignments, 0, ("b", "tl"))
    assert launches == (1, 0)
    assert np.array_equal(out["b"].cpu().numpy().astype(np.int64), ref["b"])
    assert np.array_equal(out["tl"].cpu().numpy().astype(np.int64), ref["tl"])
    out, launches = _eval(gpu, g, w, w.assignments, 0, ("cp", "b"))
    assert launches[0] == 1 and np.array_equal(out["b"].cpu().numpy().astype(np.int64), ref["b"])
    prof = gpu.CpProfile(1)
    a = torch.from_numpy(w.assignments).to("cuda:0")
    out = gpu.cp_eval(g, a, w.speeds, w.bandwidth, plan=WINDOW, out_layout=0, profile=prof)
    torch.cuda.synchronize()
    assert prof.read(0)[1] == (1, 1)
    assert np.array_equal(out["tl"].cpu().numpy().T.astype(np.int64), ref["tl"])
    g.close()


def test_pair_launch_reports_a_bad_device_id(gpu):
    import torch
    w = _wide_deep(5)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    bad = w.assignments.copy()
    bad[3, w.n // 2] = w.k
    with pytest.raises(ValueError):
        gpu.cp_eval(g, torch.from_numpy(bad).to("cuda:0"), w.speeds, w.bandwidth, plan=WINDOW, out_layout=1)
    g.close()

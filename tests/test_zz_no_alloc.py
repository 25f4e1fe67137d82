"""cp_eval_static (the entry point that allocates nothing: its scratch is a fixed array inside
the library) against cp_eval, element by element, on calls in a row that share the array."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _both(cpe, g, a, w, **kw):
    import torch
    ref = cpe.cp_eval(g, a, w.speeds, w.bandwidth, **kw)
    got = cpe.cp_eval_static(g, a, w.speeds, w.bandwidth, **kw)
    torch.cuda.synchronize()
    for key in ("cp", "b", "tl", "mask", "status"):
        assert torch.equal(got[key], ref[key]), key
    return ref


def test_static_scratch_matches_workspace_calls_in_a_row(oracle):
    import torch
    import paper_1711_01912_amd as cpe
    from workloads import make_workload

    big = make_workload("mlp")                 # 2,016 vertices x 1,024 partitions
    small = make_workload("tiny")              # 64 vertices x 16 partitions
    g_big = cpe.CpGraph.from_workload(big, device="cuda:0")
    g_small = cpe.CpGraph.from_workload(small, device="cuda:0")
    a_big = torch.from_numpy(big.assignments).to("cuda:0")
    a_small = torch.from_numpy(small.assignments).to("cuda:0")

    # first call: the wave-column plan on partition-major rows and outputs keeps the transposed
    # device ids and two sweep arrays in the scratch (2 + 2 * 8 MB) beside the cost tables
    ref_big = _both(cpe, g_big, a_big, big, plan=cpe.PLAN_WAVE_COLUMN, out_layout=cpe.OUT_PARTITION_MAJOR)
    # second call, smaller input, same array: whatever the first left behind must not show
    ref_small = _both(cpe, g_small, a_small, small, plan=cpe.PLAN_WAVE_COLUMN, out_layout=cpe.OUT_PARTITION_MAJOR)
    # the resident-window plan, with the device ids gathered into the scratch (vertex-major input)
    a_small_t = a_small.t().contiguous()
    _both(cpe, g_small, a_small_t, small, plan=cpe.PLAN_RESIDENT_WINDOW, assign_layout=1)
    _both(cpe, g_big, a_big[:200].contiguous(), big, plan=cpe.PLAN_RESIDENT_WINDOW,
          out_layout=cpe.OUT_PARTITION_MAJOR)
    _both(cpe, g_big, a_big, big)

    # and both agree with the oracle
    for w, ref in ((big, ref_big), (small, ref_small)):
        exp = oracle.evaluate_workload(w)
        assert np.array_equal(ref["cp"].cpu().numpy(), exp["cp"])
        assert np.array_equal(ref["b"].cpu().numpy().astype(np.int64), exp["b"])
        assert np.array_equal(ref["tl"].cpu().numpy().astype(np.int64), exp["tl"])


def test_static_scratch_limits():
    import torch
    import paper_1711_01912_amd as cpe
    from workloads import make_workload

    w = make_workload("inception", P=2048)     # 19,772 x 2,048 device ids = 40 MB to transpose
    g = cpe.CpGraph.from_workload(w, device="cuda:0")
    a = torch.from_numpy(w.assignments).to("cuda:0")
    with pytest.raises(cpe.CpError) as e:
        cpe.cp_eval_static(g, a, w.speeds, w.bandwidth, plan=cpe.PLAN_WAVE_COLUMN)
    assert e.value.code == -9      # CP_ERR_WORKSPACE
    # more devices than the kernel-argument tables carry
    k = 65
    s = np.ones(k, dtype=np.int64)
    bw = np.ones((k, k), dtype=np.int64)
    with pytest.raises(cpe.CpError) as e:
        cpe.cp_eval_static(g, a, s, bw)
    assert e.value.code == -2          # CP_ERR_SIZE

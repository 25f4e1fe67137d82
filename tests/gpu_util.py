"""Shared helpers of the GPU parity tests: run both sides on one workload and
compare every output element by element."""
import numpy as np


def run_gpu(w, plan, tick_bytes=None, want=("cp", "b", "tl", "mask"), layout=0, graph=None,
            speeds=None, bandwidth=None, assignments=None, out_layout=0):
    """Returns host arrays in the oracle's orientation ([P][n]) whatever the two layouts."""
    import torch
    import paper_1711_01912_amd as cpe
    from paper_1711_01912_amd import binding
    g = graph if graph is not None else cpe.CpGraph.from_workload(w, device="cuda:0")
    a_host = w.assignments if assignments is None else assignments
    P = a_host.shape[0]
    a = torch.from_numpy(np.ascontiguousarray(a_host if layout == 0 else a_host.T)).to("cuda:0")
    out = cpe.cp_eval(g, a, w.speeds if speeds is None else speeds,
                      w.bandwidth if bandwidth is None else bandwidth,
                      want=want, plan=plan, tick_bytes=tick_bytes, assign_layout=layout, out_layout=out_layout)
    orient = (lambda x: x.T) if out_layout == 0 else (lambda x: x)
    res = {}
    if "cp" in out:
        res["cp"] = out["cp"].cpu().numpy()
    if "b" in out:
        res["b"] = orient(out["b"].cpu().numpy())
        assert res["b"].shape == (P, w.n)
    if "tl" in out:
        res["tl"] = orient(out["tl"].cpu().numpy())
    if "mask" in out and "mask" in want:
        res["mask"] = orient(binding.mask_to_bool(out["mask"], P if out_layout == 0 else w.n))
    return res


def assert_equal_to_oracle(res, ref, what=""):
    """Both sides as [P][n]."""
    assert np.array_equal(res["cp"], ref["cp"]), f"{what}: CP differs"
    for key in ("b", "tl"):
        if key in res:
            got = res[key]
            bad = np.nonzero(got != ref[key])
            assert bad[0].size == 0, (f"{what}: {key} differs at {bad[0].size} places, first "
                                      f"(partition {bad[0][0]}, vertex {bad[1][0]}): "
                                      f"{got[bad[0][0], bad[1][0]]} vs {ref[key][bad[0][0], bad[1][0]]}")
    if "mask" in res:
        assert np.array_equal(res["mask"], ref["mask"]), f"{what}: mask differs"

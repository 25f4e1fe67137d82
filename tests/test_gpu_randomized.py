"""Bounded randomized comparison of every GPU entry point with the CPU oracle: seeded graph
shapes, device models, batch sizes, weight widths, layouts and plans; bit-exact; stops at
the first difference."""
import numpy as np
import pytest

from workloads import build_csr, random_layered_dag
from workloads.dags import _finish

pytestmark = pytest.mark.gpu

PLANS = (1, 2, 3, 4, 5, 6)    # wave-column, resident window, shared window x2 / x4, column slices, streamed window


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1711_01912_amd as cpe
    cpe.load_library()
    return cpe


def _draw(rng, layers_hi, width_hi, ks, Ps, cmaxs, tmaxs, c_lo=0, spans=(1, 2, 3, 6, 12, 30)):
    layers = int(rng.integers(1, layers_hi))
    width = int(rng.integers(1, int(rng.choice([4, 20, width_hi])) + 1))
    deg_hi = int(rng.integers(1, 9))
    span_hi = int(rng.choice(spans))
    k = int(rng.choice(ks))
    P = int(rng.choice(Ps))
    n, level, src, dst = random_layered_dag(rng, [width] * layers, 1, deg_hi, span_hi)
    cmax, tmax = int(rng.choice(cmaxs)), int(rng.choice(tmaxs))
    t = rng.integers(0, tmax + 1, size=len(src))
    c = rng.integers(min(c_lo, cmax), cmax + 1, size=n)
    speeds = rng.integers(1, int(rng.choice([1, 3, 100])) + 1, size=k)
    bw = rng.integers(1, int(rng.choice([1, 4, 60, 300])) + 1, size=(k, k))
    a = rng.integers(0, k, size=(P, n)).astype(np.uint8)
    w = _finish("random", build_csr(n, src, dst, t, level), c, k, speeds, bw, a)
    what = dict(layers=layers, width=width, deg_hi=deg_hi, span_hi=span_hi, k=k, P=P, cmax=cmax, tmax=tmax)
    return w, what


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_randomized_evaluation_all_plans(gpu, oracle, seed):
    from gpu_util import assert_equal_to_oracle, run_gpu
    rng = np.random.default_rng(seed)
    ran = {p: 0 for p in PLANS}
    for it in range(120):
        w, what = _draw(rng, 60, 300, [1, 2, 3, 5, 8, 16, 21, 32, 33, 50, 64, 100], [1, 2, 7, 33, 64, 65, 130, 300],
                        [1, 100, 5000, 70000], [0, 1, 100, 20000, 100000])
        ref = oracle.evaluate_workload(w, threads=16)
        g = gpu.CpGraph.from_workload(w, device="cuda:0")
        for plan in PLANS:
            layout, ol = int(rng.integers(0, 2)), int(rng.integers(0, 2))
            try:
                res = run_gpu(w, plan, layout=layout, graph=g, out_layout=ol)
            except gpu.CpError as e:
                # every plan but the wave-column one may refuse a graph or a cost model
                assert plan != 1 and e.code == -12, (seed, it, plan, e.code, what)
                continue
            ran[plan] += 1
            assert_equal_to_oracle(res, ref, what=f"seed {seed} case {it} plan {plan} layout {layout} out {ol} {what}")
        g.close()
    assert all(ran[p] > 30 for p in PLANS), ran


@pytest.mark.parametrize("seed", [21, 22])
def test_randomized_consumers(gpu, oracle, seed):
    """Critical path, priority lists, the seed partition and four search moves."""
    import test_gpu_parity as T
    rng = np.random.default_rng(seed)
    for it in range(60):
        w, what = _draw(rng, 40, 120, [1, 2, 3, 5, 8, 16, 33, 50, 64], [1, 2, 7, 33, 70], [1, 3, 100, 5000],
                        [0, 1, 3, 100, 20000], spans=(1, 2, 3, 6, 12))
        try:
            T._check_paths(gpu, oracle, w, layout=int(rng.integers(0, 2)))
            T._check_pct_order(gpu, oracle, w, layout=int(rng.integers(0, 2)))
            if w.k >= 2:
                T._check_search(gpu, oracle, w, w.assignments[0], max_moves=4, chunk=int(rng.choice([3, 64, 256])))
            g = gpu.CpGraph.from_workload(w, device="cuda:0")
            seed_part = gpu.cp_seed_partition(g, w.speeds).cpu().numpy()
            ref = oracle.seed(w.n, w.succ_ptr, w.succ_idx, w.c, w.speeds, max_len=w.L)
            g.close()
            assert np.array_equal(seed_part, ref), "seed partition"
        except AssertionError as e:
            raise AssertionError(f"seed {seed} case {it} {what}: {e}") from e


@pytest.mark.parametrize("seed", [31, 32])
def test_randomized_simulation(gpu, oracle, seed):
    """The list-scheduling simulation under PCT, FIFO and FIFO with a random tie order."""
    import torch
    rng = np.random.default_rng(seed)
    for it in range(60):
        w, what = _draw(rng, 40, 120, [1, 2, 3, 5, 8, 13, 16, 21, 32, 33, 50, 64], [1, 2, 7, 33, 64, 200],
                        [1, 5, 100, 5000], [0, 1, 100, 20000], c_lo=1, spans=(1, 2, 3, 4, 5))
        a = w.assignments
        if rng.random() < 0.2:
            a = np.ascontiguousarray(np.broadcast_to(a[:, :1], a.shape))   # one device per partition
        g = gpu.CpGraph.from_workload(w, device="cuda:0")
        layout = int(rng.integers(0, 2))
        d_a = torch.from_numpy(np.ascontiguousarray(a if layout == 0 else a.T)).to("cuda:0")
        ev = gpu.cp_eval(g, d_a, w.speeds, w.bandwidth, want=("cp", "b"), assign_layout=layout, out_layout=layout)
        ref_ev = oracle.evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth, a,
                                 want=("cp", "b"), threads=16)
        tie = rng.permutation(w.n).astype(np.int32)
        for name, pol, kw, okw in (("pct", 1, dict(b=ev["b"], b_layout=layout), dict(b=ref_ev["b"])),
                                   ("fifo", 0, {}, {}),
                                   ("fifo+tie", 0, dict(tie=torch.from_numpy(tie).to("cuda:0")), dict(tie=tie))):
            m, s = gpu.cp_simulate(g, d_a, w.speeds, w.bandwidth, pol, assign_layout=layout, **kw)
            ref = oracle.simulate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth, a, pol,
                                  threads=16, **okw)
            assert np.array_equal(m.cpu().numpy(), ref["makespan"]), f"seed {seed} case {it} {name} {what}: makespan"
            assert np.array_equal(s.cpu().numpy(), ref["start"]), f"seed {seed} case {it} {name} {what}: start times"
        g.close()

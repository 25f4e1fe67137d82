"""GPU parity of cp_simulate (list scheduling under FIFO and PCT), called through the C ABI,
against the CPU oracle: every start time and every makespan, bit-exact."""
import sys

import numpy as np
import pytest

from workloads import build_csr, make_workload, random_layered_dag
from workloads.dags import _finish

pytestmark = pytest.mark.gpu

FIFO, PCT = 0, 1


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1711_01912_amd as cpe
    cpe.load_library()
    return cpe


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _oracle_sim(oracle, w, a, policy, b=None, tie=None):
    return oracle.simulate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth, a, policy,
                           b=b, tie=tie, threads=16)


def _check(gpu, oracle, w, a=None, tie_seed=1, layouts=(0, 1), what=""):
    """Both policies; FIFO with and without tie ranks; the assignments and b in both layouts."""
    import torch
    a = w.assignments if a is None else a
    P = a.shape[0]
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    ref_eval = oracle.evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth, a,
                               want=("cp", "b"), threads=16)
    tie = np.random.default_rng(tie_seed).permutation(w.n).astype(np.int32)
    refs = {"pct": _oracle_sim(oracle, w, a, PCT, b=ref_eval["b"]),
            "fifo": _oracle_sim(oracle, w, a, FIFO),
            "fifo_tie": _oracle_sim(oracle, w, a, FIFO, tie=tie)}
    d_tie = torch.from_numpy(tie).to("cuda:0")
    for layout in layouts:
        d_a = torch.from_numpy(np.ascontiguousarray(a if layout == 0 else a.T)).to("cuda:0")
        ev = gpu.cp_eval(g, d_a, w.speeds, w.bandwidth, want=("cp", "b"), assign_layout=layout, out_layout=layout)
        for name, kw in (("pct", dict(policy=PCT, b=ev["b"], b_layout=layout)),
                         ("fifo", dict(policy=FIFO)),
                         ("fifo_tie", dict(policy=FIFO, tie=d_tie))):
            _say(f"cp_simulate {what or w.name} n={w.n} P={P} k={w.k} {name} layout={layout}")
            policy = kw.pop("policy")
            makespan, start = gpu.cp_simulate(g, d_a, w.speeds, w.bandwidth, policy, assign_layout=layout, **kw)
            got_m = makespan.cpu().numpy()
            got_s = start.cpu().numpy()
            ref = refs[name]
            bad = np.nonzero(got_s != ref["start"])
            assert bad[0].size == 0, (f"{what} {name} layout={layout}: start differs at {bad[0].size} places, first "
                                      f"(partition {bad[0][0]}, vertex {bad[1][0]}): "
                                      f"{got_s[bad[0][0], bad[1][0]]} vs {ref['start'][bad[0][0], bad[1][0]]}")
            assert np.array_equal(got_m, ref["makespan"]), f"{what} {name} layout={layout}: makespan differs"
            assert (got_m >= ref_eval["cp"]).all()
    g.close()
    return refs


def _random_workload(seed, layers, width, k, P, deg_hi=4, span_hi=4, cmax=100, tmax=100, s=(10, 100), B=(10, 60),
                     cmin=1, tmin=1):
    rng = np.random.default_rng(seed)
    n, level, src, dst = random_layered_dag(rng, [width] * layers, 1, deg_hi, span_hi)
    t = rng.integers(tmin, tmax + 1, size=len(src))
    c = rng.integers(cmin, cmax + 1, size=n)
    csr = build_csr(n, src, dst, t, level)
    speeds = rng.integers(s[0], s[1] + 1, size=k)
    bandwidth = rng.integers(B[0], B[1] + 1, size=(k, k))
    a = rng.integers(0, k, size=(P, n)).astype(np.uint8)
    return _finish(f"random{seed}", csr, c, k, speeds, bandwidth, a)


def test_tiny(gpu, oracle):
    _check(gpu, oracle, make_workload("tiny"))


def test_worked_example(gpu, oracle):
    """The schedule worked by hand in tests/golden (through the oracle's pin of it)."""
    src = np.array([0, 0, 1, 2, 3, 4])
    dst = np.array([3, 2, 4, 5, 5, 5])
    t = np.array([2, 5, 4, 1, 1, 2])
    csr = build_csr(6, src, dst, t)
    a = np.array([[0, 0, 0, 1, 1, 0]], dtype=np.uint8)
    w = _finish("worked", csr, np.array([2, 3, 4, 2, 6, 2]), 2, np.array([1, 2]), np.full((2, 2), 2), a)
    refs = _check(gpu, oracle, w, what="worked example")
    assert refs["pct"]["makespan"][0] == 12 and refs["fifo"]["makespan"][0] == 13


@pytest.mark.parametrize("seed,layers,width,k,P", [(1, 12, 8, 4, 5), (2, 30, 10, 8, 9), (3, 8, 60, 16, 4),
                                                   (4, 50, 4, 50, 7), (5, 20, 20, 3, 3), (6, 6, 100, 64, 3),
                                                   (7, 40, 12, 1, 2)])
def test_random_shapes(gpu, oracle, seed, layers, width, k, P):
    _check(gpu, oracle, _random_workload(seed, layers, width, k, P), tie_seed=seed)


def test_paper_scale_graph_on_fifty_devices(gpu, oracle):
    """The size of the paper's largest graph (Table 1: 5,271 vertices, average degree 1.75) with
    the simulation's parameter ranges (section 5.1), 50 devices, many partitions."""
    w = _random_workload(11, 251, 21, 50, 192, deg_hi=3, span_hi=3)
    assert w.n == 5271
    _check(gpu, oracle, w, layouts=(0,))


def test_equal_costs_make_many_ties(gpu, oracle):
    """All weights equal: every decision is a tie, and many devices decide at the same time."""
    w = _random_workload(12, 15, 30, 6, 6, cmax=1, tmax=1, s=(1, 1), B=(1, 1))
    _check(gpu, oracle, w)


def test_wide_lookahead(gpu, oracle):
    """Long minimum execution and transfer times: devices far apart in time decide together."""
    w = _random_workload(13, 20, 16, 8, 6, cmin=9000, cmax=10000, tmin=5000, tmax=6000)
    _check(gpu, oracle, w)


def test_hubs_and_skewed_devices(gpu, oracle):
    """comm_heavy's hubs (a thousand successors) and a partition that puts nearly everything on one device."""
    w = make_workload("comm_heavy", P=4, levels=6, width=600, hub_degree=300)
    a = w.assignments.copy()
    a[1, :] = 0
    a[1, ::97] = 3
    _check(gpu, oracle, w, a=a, layouts=(0,))


def test_isolated_vertices_and_a_single_vertex(gpu, oracle):
    n = 70
    csr = build_csr(n, np.array([], dtype=np.int64), np.array([], dtype=np.int64), np.array([], dtype=np.int64))
    rng = np.random.default_rng(14)
    a = rng.integers(0, 3, size=(3, n)).astype(np.uint8)
    w = _finish("isolated", csr, rng.integers(1, 50, size=n), 3, np.array([1, 2, 3]), np.full((3, 3), 5), a)
    _check(gpu, oracle, w)
    csr = build_csr(1, np.array([], dtype=np.int64), np.array([], dtype=np.int64), np.array([], dtype=np.int64))
    w = _finish("single", csr, np.array([7]), 2, np.array([2, 3]), np.full((2, 2), 5), np.array([[1], [0]], dtype=np.uint8))
    refs = _check(gpu, oracle, w)
    assert refs["pct"]["makespan"].tolist() == [3, 4]


def test_large_sparse_reduced(gpu, oracle):
    w = make_workload("large_sparse", P=24, levels=300, width=100)
    _check(gpu, oracle, w, layouts=(0,))


def test_inception_sample(gpu, oracle):
    w = make_workload("inception", P=16)
    _check(gpu, oracle, w, layouts=(0,))


def test_status_and_errors(gpu, oracle):
    import torch
    w = make_workload("tiny")
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    a = w.assignments.copy()
    a[3, 5] = w.k            # a device that does not exist
    d_a = torch.from_numpy(a).to("cuda:0")
    with pytest.raises(ValueError):
        gpu.cp_simulate(g, d_a, w.speeds, w.bandwidth, FIFO)
    makespan, _ = gpu.cp_simulate(g, d_a, w.speeds, w.bandwidth, FIFO, check_status=False)
    ref = _oracle_sim(oracle, w, np.delete(w.assignments, 3, axis=0), FIFO)
    got = makespan.cpu().numpy()
    assert got[3] == -1 and np.array_equal(np.delete(got, 3), ref["makespan"])
    d_a = torch.from_numpy(w.assignments).to("cuda:0")
    tie = torch.arange(w.n, dtype=torch.int32, device="cuda:0")
    tie[4] = 5               # rank 5 twice, rank 4 never
    with pytest.raises(ValueError):
        gpu.cp_simulate(g, d_a, w.speeds, w.bandwidth, FIFO, tie=tie)
    tie[4] = w.n             # out of range
    with pytest.raises(ValueError):
        gpu.cp_simulate(g, d_a, w.speeds, w.bandwidth, FIFO, tie=tie)
    b = torch.full((w.P, w.n), -5, dtype=torch.int32, device="cuda:0")
    with pytest.raises(ValueError):
        gpu.cp_simulate(g, d_a, w.speeds, w.bandwidth, PCT, b=b, b_layout=1)
    g.close()
    # a vertex that costs nothing is refused on the host
    w0 = make_workload("tiny")
    w0.c = w0.c.copy()
    w0.c[0] = 0
    g0 = gpu.CpGraph.from_workload(w0, device="cuda:0")
    with pytest.raises(gpu.CpError) as e:
        gpu.cp_simulate(g0, d_a, w.speeds, w.bandwidth, FIFO)
    assert e.value.code == -12
    g0.close()
    # times that could pass 2^31 are refused: 64 vertices of 2^26 ticks each on a device of speed 1
    w1 = make_workload("tiny")
    w1.c = np.full(w1.n, 2**26, dtype=np.int64)
    g1 = gpu.CpGraph.from_workload(w1, device="cuda:0")
    with pytest.raises(gpu.CpError) as e:
        gpu.cp_simulate(g1, d_a, w.speeds, w.bandwidth, FIFO)
    assert e.value.code == -8
    g1.close()


def test_partitions_sharing_a_wavefront(gpu, oracle):
    """A batch large enough that partitions with few devices are simulated several per wavefront
    (three here: 24,600 partitions of a small graph on 5 devices), with a ragged last wavefront and
    one partition that names a device that does not exist."""
    import torch
    w = _random_workload(21, 9, 6, 5, 24600, deg_hi=3, span_hi=2)
    a = w.assignments.copy()
    a[12345, 7] = 5
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    d_a = torch.from_numpy(a).to("cuda:0")
    ev = gpu.cp_eval(g, torch.from_numpy(w.assignments).to("cuda:0"), w.speeds, w.bandwidth, want=("cp", "b"),
                     out_layout=1)
    good = np.delete(np.arange(w.P), 12345)
    b_ref = oracle.evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth, w.assignments[good],
                            want=("cp", "b"), threads=16)["b"]
    for policy, kw in ((PCT, dict(b=ev["b"], b_layout=1)), (FIFO, {})):
        _say(f"cp_simulate shared wavefronts policy={policy}")
        makespan, start = gpu.cp_simulate(g, d_a, w.speeds, w.bandwidth, policy, check_status=False, **kw)
        ref = _oracle_sim(oracle, w, w.assignments[good], policy, b=b_ref if policy == PCT else None)
        got_m = makespan.cpu().numpy()
        assert got_m[12345] == -1
        assert np.array_equal(got_m[good], ref["makespan"])
        assert np.array_equal(start.cpu().numpy()[good], ref["start"])
    g.close()


def test_large_sparse_full_size(gpu, oracle):
    """The bench graph at full size (1,000,000 vertices, 16 devices), a few partitions: every start time."""
    import torch
    w = make_workload("large_sparse", P=6)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    d_a = torch.from_numpy(w.assignments).to("cuda:0")
    ev = gpu.cp_eval(g, d_a, w.speeds, w.bandwidth, want=("cp", "b"), out_layout=1)
    b_ref = ev["b"].cpu().numpy().astype(np.int64)      # parity of b itself is test_gpu_parity's subject
    for policy, kw in ((PCT, dict(b=ev["b"], b_layout=1)), (FIFO, {})):
        _say(f"cp_simulate large_sparse full size policy={policy}")
        makespan, start = gpu.cp_simulate(g, d_a, w.speeds, w.bandwidth, policy, **kw)
        ref = _oracle_sim(oracle, w, w.assignments, policy, b=b_ref if policy == PCT else None)
        assert np.array_equal(makespan.cpu().numpy(), ref["makespan"])
        assert np.array_equal(start.cpu().numpy(), ref["start"])
    g.close()


def test_other_weight_and_tick_types(gpu, oracle):
    """b handed over as int64; weights past 32 bits (plain 64-bit division in the kernel); 32-bit
    weights whose divisors have no exact multiply-shift form."""
    import torch
    # (a) int64 b from the wave-column plan
    w = _random_workload(31, 14, 9, 6, 5)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    d_a = torch.from_numpy(w.assignments).to("cuda:0")
    ev = gpu.cp_eval(g, d_a, w.speeds, w.bandwidth, want=("cp", "b"), tick_bytes=8, plan=1)
    assert ev["b"].dtype == torch.int64
    ref_b = oracle.evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth, w.assignments,
                            want=("cp", "b"), threads=4)["b"]
    _say("cp_simulate with int64 b")
    makespan, start = gpu.cp_simulate(g, d_a, w.speeds, w.bandwidth, PCT, b=ev["b"], b_layout=0)
    ref = _oracle_sim(oracle, w, w.assignments, PCT, b=ref_b)
    assert np.array_equal(start.cpu().numpy(), ref["start"]) and np.array_equal(makespan.cpu().numpy(), ref["makespan"])
    g.close()
    # (b) weights of 33..35 bits over speeds and rates of ~30 bits: every time stays small
    rng = np.random.default_rng(32)
    w = _random_workload(32, 10, 8, 4, 4)
    w.c = rng.integers(2**32, 2**34, size=w.n)
    w.succ_t = rng.integers(2**32, 2**35, size=w.succ_t.shape[0])
    w.speeds = rng.integers(2**28, 2**30, size=4)
    w.bandwidth = rng.integers(2**28, 2**30, size=(4, 4))
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    assert g.info["max_c"] >= 2**32
    g.close()
    _check(gpu, oracle, w, what="wide weights")
    # (c) 32-bit weights, divisors near 10^9: no exact multiply-shift constant exists for them
    w = _random_workload(33, 10, 8, 4, 4)
    w.c = rng.integers(2 * 10**9, 4 * 10**9, size=w.n)
    w.succ_t = rng.integers(2 * 10**9, 4 * 10**9, size=w.succ_t.shape[0])
    w.speeds = rng.integers(10**9, 10**9 + 50, size=4)
    w.bandwidth = rng.integers(10**9, 10**9 + 50, size=(4, 4))
    _check(gpu, oracle, w, what="no multiply-shift")


def test_hub_rows_in_shared_wavefronts(gpu, oracle):
    """A vertex with 40 successors is shared out over the whole wavefront, here a wavefront that
    holds two partitions (16,400 partitions on 7 devices)."""
    rng = np.random.default_rng(41)
    n = 48
    src = [0] * 40 + list(range(1, 41)) + [41, 42, 43, 44, 45, 46]
    dst = list(range(1, 41)) + [41] * 40 + [42, 43, 44, 45, 46, 47]
    t = rng.integers(1, 200, size=len(src))
    csr = build_csr(n, np.array(src), np.array(dst), t)
    k = 7
    a = rng.integers(0, k, size=(16400, n)).astype(np.uint8)
    w = _finish("hub", csr, rng.integers(1, 60, size=n), k, rng.integers(1, 9, size=k), rng.integers(1, 9, size=(k, k)), a)
    _check(gpu, oracle, w, layouts=(0,))


def test_many_random_configurations(gpu, oracle):
    """Sixty graphs with random shape, device count (1 .. 64), batch, weight ranges (zero transfer
    volumes, equal weights, long minimum times), device models and layouts; all three policies."""
    import torch
    rng = np.random.default_rng(51)
    for it in range(60):
        layers, width = int(rng.integers(1, 40)), int(rng.integers(1, 50))
        k = int(rng.choice([1, 2, 3, 5, 8, 13, 16, 21, 32, 33, 50, 64]))
        P = int(rng.choice([1, 2, 7, 33, 64, 200]))
        n, level, src, dst = random_layered_dag(rng, [width] * layers, 1, int(rng.integers(1, 9)), int(rng.integers(1, 6)))
        cmax, tmax = int(rng.choice([1, 5, 100, 5000])), int(rng.choice([0, 1, 100, 20000]))
        t = rng.integers(int(rng.integers(0, tmax + 1)), tmax + 1, size=len(src))
        c = rng.integers(int(rng.integers(1, cmax + 1)), cmax + 1, size=n)
        speeds = rng.integers(1, int(rng.choice([1, 3, 100])) + 1, size=k)
        bw = rng.integers(1, int(rng.choice([1, 4, 60])) + 1, size=(k, k))
        a = rng.integers(0, k, size=(P, n)).astype(np.uint8)
        if rng.random() < 0.2:
            a[:, :] = a[:, :1]          # one device per partition
        w = _finish("random", build_csr(n, src, dst, t, level), c, k, speeds, bw, a)
        if it % 20 == 0:
            _say(f"cp_simulate random configuration {it}: n={n} k={k} P={P}")
        _check(gpu, oracle, w, tie_seed=it, layouts=(int(rng.integers(0, 2)),), what=f"random configuration {it}")

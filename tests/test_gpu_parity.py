"""GPU parity: the HIP library, called through the C ABI, against the CPU oracle,
element by element and bit-exact (integer ticks), on the same seeded inputs."""
import numpy as np
import pytest

from workloads import build_csr, make_workload, random_layered_dag
from workloads.dags import Workload, _finish

pytestmark = pytest.mark.gpu

COLUMN, WINDOW = 1, 2


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1711_01912_amd as cpe
    cpe.load_library()
    return cpe


def _oracle(oracle, w, **kw):
    return oracle.evaluate_workload(w, threads=16, **kw)


def _check(gpu, oracle, w, plans=(COLUMN, WINDOW), ticks=(None,), layouts=(0,), out_layouts=(0, 1), what=None):
    from gpu_util import assert_equal_to_oracle, run_gpu
    ref = _oracle(oracle, w)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    for plan in plans:
        for tb in ticks:
            for layout in layouts:
                for ol in out_layouts:
                    res = run_gpu(w, plan, tick_bytes=tb, layout=layout, graph=g, out_layout=ol)
                    assert_equal_to_oracle(res, ref, what=f"{what or w.name} plan={plan} ticks={tb} "
                                                          f"layout={layout} out_layout={ol}")
    g.close()
    return ref


def _custom(name, n, src, dst, t, c, speeds, bandwidth, assignments, level=None):
    csr = build_csr(n, src, dst, t, level)
    return _finish(name, csr, c, len(speeds), speeds, bandwidth, assignments)


# ------------------------------------------------------------------ the five workloads

def test_tiny_all_variants(gpu, oracle):
    from gpu_util import run_gpu
    w = make_workload("tiny")
    _check(gpu, oracle, w, ticks=(4,), layouts=(0, 1))
    _check(gpu, oracle, w, plans=(COLUMN,), ticks=(8,), layouts=(0, 1))
    # this graph's window ring was packed for 32-bit ticks: 64-bit ticks must be refused there
    with pytest.raises(gpu.CpError) as e:
        run_gpu(w, WINDOW, tick_bytes=8)
    assert e.value.code == -12


@pytest.mark.parametrize("P", [300, 258, 1028])
def test_batches_that_end_inside_a_mask_word(gpu, oracle, P):
    """Batches that are a multiple of four but not of 64 (the 16-byte mask kernel's last word of a
    vertex-major row holds 44 / 2 / 4 partitions; the assignments are transposed four ids at a
    time) and one that is not a multiple of four (258: the plain kernels), both plans and layouts."""
    _check(gpu, oracle, make_workload("mlp", P=P), layouts=(0, 1))


def test_window_plan_with_64_bit_ticks(gpu, oracle):
    """A raw path bound past 2^31 with 32-bit weights: the window plan runs on int64 ticks."""
    w = make_workload("large_sparse", P=40, levels=300, width=40)
    w.c = w.c * 2**18
    g = gpu.CpGraph.from_workload(w)
    assert g.info["min_tick_bytes"] == 8 and g.info["window_ok"] == 1
    g.close()
    _check(gpu, oracle, w, ticks=(8,))


def test_mlp_full(gpu, oracle):
    _check(gpu, oracle, make_workload("mlp"))


def test_mlp_literal_single_shard(gpu, oracle):
    _check(gpu, oracle, make_workload("mlp", shards=1, P=130))


def test_inception_full(gpu, oracle):
    _check(gpu, oracle, make_workload("inception"))


def test_large_sparse_full(gpu, oracle):
    """The benchmark workload at full size, all columns, in both plans."""
    _check(gpu, oracle, make_workload("large_sparse"))


def test_comm_heavy_full(gpu, oracle):
    w = make_workload("comm_heavy")
    _check(gpu, oracle, w, plans=(COLUMN,))


def test_comm_heavy_scaled_hub_rows(gpu, oracle):
    # hub rows (300 >= the hub threshold) take a whole workgroup in the wave-column plan;
    # levels this wide do not fit the other plan's LDS stage, which must say so
    from gpu_util import run_gpu
    w = make_workload("comm_heavy", P=70, levels=5, width=3000, hub_degree=300)
    _check(gpu, oracle, w, plans=(COLUMN,))
    with pytest.raises(gpu.CpError) as e:
        run_gpu(w, WINDOW)
    assert e.value.code == -12


def test_comm_heavy_scaled_both_plans(gpu, oracle):
    # rows of 40 edges next to rows of 2-4, 8-byte entries (volumes up to 1e7)
    w = make_workload("comm_heavy", P=70, levels=5, width=600, hub_degree=40)
    _check(gpu, oracle, w)


def test_levels_wider_than_the_compute_wavefronts(gpu, oracle):
    # 19 slices of 64 vertices per level against at most 8 compute wavefronts
    rng = np.random.default_rng(7)
    n, level, src, dst = random_layered_dag(rng, [1200] * 9, 1, 3, 2)
    k = 5
    w = _custom("wide-levels", n, src, dst, rng.integers(1, 10**4, size=len(src)),
                rng.integers(1, 10**3, size=n), rng.integers(1, 9, size=k),
                rng.integers(1, 50, size=(k, k)), rng.integers(0, k, size=(70, n), dtype=np.uint8), level)
    g = gpu.CpGraph.from_workload(w)
    assert g.info["window_ok"] == 1 and g.info["max_level_width"] == 1200
    g.close()
    _check(gpu, oracle, w)


# ------------------------------------------------------------------ edge cases

@pytest.mark.parametrize("P", [1, 2, 63, 64, 65, 127, 130])
def test_ragged_batches(gpu, oracle, P):
    w = make_workload("large_sparse", P=P, levels=40, width=70)
    _check(gpu, oracle, w, what=f"ragged P={P}")


def test_single_vertex_and_edgeless(gpu, oracle):
    a = np.array([[0], [1], [1]], dtype=np.uint8)
    w = _custom("one", 1, [], [], [], [7], [2, 3], [[1, 5], [4, 1]], a)
    _check(gpu, oracle, w)
    rng = np.random.default_rng(0)
    a = rng.integers(0, 3, size=(5, 200), dtype=np.uint8)
    w = _custom("antichain", 200, [], [], [], rng.integers(0, 50, size=200), [1, 2, 5],
                rng.integers(1, 9, size=(3, 3)), a)
    _check(gpu, oracle, w)


def test_zero_costs_and_multi_edges(gpu, oracle):
    rng = np.random.default_rng(1)
    n, level, src, dst = random_layered_dag(rng, [9] * 12, 1, 4, 3)
    # duplicate a third of the edges with other volumes
    dup = rng.random(len(src)) < 0.33
    src = np.concatenate([src, src[dup]])
    dst = np.concatenate([dst, dst[dup]])
    t = rng.integers(0, 3, size=len(src)) * rng.integers(0, 1000, size=len(src))
    c = rng.integers(0, 2, size=n) * rng.integers(0, 100, size=n)
    a = rng.integers(0, 4, size=(37, n), dtype=np.uint8)
    B = rng.integers(1, 30, size=(4, 4))
    w = _custom("zeros-multi", n, src, dst, t, c, [1, 2, 3, 4], B, a, level)
    _check(gpu, oracle, w)


def test_asymmetric_bandwidth(gpu, oracle):
    w = make_workload("inception", P=100, modules=5, groups=3)
    rng = np.random.default_rng(2)
    w.bandwidth = rng.integers(1, 100, size=(w.k, w.k)).astype(np.int64)
    assert not np.array_equal(w.bandwidth, w.bandwidth.T)
    _check(gpu, oracle, w)


def test_paper_parameter_ranges_fifty_devices(gpu, oracle):
    """50 devices with the simulation's ranges (section 5.1)."""
    rng = np.random.default_rng(3)
    n, level, src, dst = random_layered_dag(rng, [7] * 50, 1, 2, 3)
    k = 50
    w = _custom("paper-ranges", n, src, dst, rng.integers(1, 101, size=len(src)),
                rng.integers(1, 101, size=n), rng.integers(10, 101, size=k),
                rng.integers(10, 61, size=(k, k)), rng.integers(0, k, size=(96, n), dtype=np.uint8), level)
    _check(gpu, oracle, w)


def test_partitions_sharing_a_workgroup(gpu, oracle):
    """Large cost tables beside a small ring: the window plan puts several partitions into one
    workgroup.  A batch that does not fill the last workgroup, both layouts, both sweeps."""
    for P in (37, 130):
        w = make_workload("paper_scale", P=P)
        _check(gpu, oracle, w, plans=(WINDOW,), layouts=(0, 1), what=f"paper_scale P={P}")


def test_many_devices_take_the_plain_division_path(gpu, oracle):
    """k = 200 exceeds the LDS-table limit: plain divisors from global memory."""
    rng = np.random.default_rng(4)
    n, level, src, dst = random_layered_dag(rng, [11] * 14, 1, 3, 2)
    k = 200
    w = _custom("k200", n, src, dst, rng.integers(1, 10**4, size=len(src)),
                rng.integers(1, 10**3, size=n), rng.integers(1, 40, size=k),
                rng.integers(1, 90, size=(k, k)), rng.integers(0, k, size=(70, n), dtype=np.uint8), level)
    _check(gpu, oracle, w, plans=(COLUMN,))
    with pytest.raises(gpu.CpError) as e:
        from gpu_util import run_gpu
        run_gpu(w, WINDOW)
    assert e.value.code == -12


def test_wide_weights_take_the_64_bit_path(gpu, oracle):
    """Volumes above 2^32 and a path bound above 2^31: int64 ticks, plain division."""
    rng = np.random.default_rng(5)
    n, level, src, dst = random_layered_dag(rng, [8] * 10, 1, 3, 2)
    t = rng.integers(1, 2**45, size=len(src))
    c = rng.integers(1, 2**40, size=n)
    B = rng.integers(1, 2**20, size=(3, 3))
    a = rng.integers(0, 3, size=(66, n), dtype=np.uint8)
    w = _custom("wide", n, src, dst, t, c, [1, 3, 2**33], B, a, level)
    g = gpu.CpGraph.from_workload(w)
    assert g.info["min_tick_bytes"] == 8
    g.close()
    _check(gpu, oracle, w, plans=(COLUMN,))


def test_narrow_weights_with_inexact_constants_fall_back(gpu, oracle):
    """Weights fit 32 bits but a divisor does not admit the exact 32-bit form."""
    rng = np.random.default_rng(6)
    n, level, src, dst = random_layered_dag(rng, [8] * 10, 1, 3, 2)
    t = rng.integers(2**31, 2**32, size=len(src))
    c = rng.integers(1, 1000, size=n)
    B = np.array([[1, 3, 7], [11, 1, 641], [6700417, 5, 1]])
    assert gpu.cost_magic(3, int(t.max())) is None
    a = rng.integers(0, 3, size=(40, n), dtype=np.uint8)
    w = _custom("inexact", n, src, dst, t, c, [1, 2, 3], B, a, level)
    _check(gpu, oracle, w, plans=(COLUMN,), ticks=(8,))


def test_tick_width_request_is_checked(gpu, oracle):
    import torch
    w = make_workload("tiny")
    w.c = w.c * 2**26            # pushes the raw path bound past 2^31
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    assert g.info["min_tick_bytes"] == 8
    a = torch.from_numpy(w.assignments).to("cuda:0")
    with pytest.raises(gpu.CpError) as e:
        gpu.cp_eval(g, a, w.speeds, w.bandwidth, tick_bytes=4)
    assert e.value.code == -8
    g.close()
    _check(gpu, oracle, w, plans=(COLUMN,), ticks=(8,))


def test_bad_device_id_is_reported_not_fatal(gpu):
    import torch
    w = make_workload("tiny")
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    bad = w.assignments.copy()
    bad[3, 10] = 9
    a = torch.from_numpy(bad).to("cuda:0")
    for plan in (COLUMN, WINDOW):
        with pytest.raises(ValueError):
            gpu.cp_eval(g, a, w.speeds, w.bandwidth, plan=plan)
    # a good call afterwards clears the status word
    out = gpu.cp_eval(g, torch.from_numpy(w.assignments).to("cuda:0"), w.speeds, w.bandwidth)
    assert int(out["status"].item()) == 0
    g.close()


def test_rejected_cost_models(gpu):
    import torch
    w = make_workload("tiny")
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    a = torch.from_numpy(w.assignments).to("cuda:0")
    with pytest.raises(gpu.CpError) as e:
        gpu.cp_eval(g, a, [1, 0], w.bandwidth)
    assert e.value.code == -6
    with pytest.raises(gpu.CpError) as e:
        gpu.cp_eval(g, a, w.speeds, [[0, 0], [3, 0]])
    assert e.value.code == -7
    gpu.cp_eval(g, a, w.speeds, [[0, 1], [3, -5]])   # the diagonal is never read
    g.close()


def test_partial_outputs_and_determinism(gpu, oracle):
    from gpu_util import run_gpu
    w = make_workload("large_sparse", P=100, levels=60, width=90)
    ref = _oracle(oracle, w)
    for plan in (COLUMN, WINDOW):
        r1 = run_gpu(w, plan, want=("b",))
        assert np.array_equal(r1["b"], ref["b"]) and "tl" not in r1
        r2 = run_gpu(w, plan, want=("cp",))
        assert np.array_equal(r2["cp"], ref["cp"])
        assert ("b" in r2) == (plan == COLUMN)         # the window sweep needs no b array for CP alone
        r3 = run_gpu(w, plan, want=("tl",))
        assert np.array_equal(r3["tl"], ref["tl"])
        r4 = run_gpu(w, plan)
        r5 = run_gpu(w, plan)
        for key in ("cp", "b", "tl", "mask"):
            assert np.array_equal(r4[key], r5[key])


def test_one_column_equals_its_column_in_a_batch(gpu):
    from gpu_util import run_gpu
    w = make_workload("mlp", P=200, layers=8, shards=3)
    full = run_gpu(w, WINDOW)
    for plan in (COLUMN, WINDOW):
        one = run_gpu(w, plan, assignments=w.assignments[77:78])
        assert np.array_equal(one["b"][0], full["b"][77])
        assert np.array_equal(one["tl"][0], full["tl"][77])
        assert one["cp"][0] == full["cp"][77]


# ------------------------------------------------------------------ one critical path per partition

def _check_paths(gpu, oracle, w, layout=0):
    import torch
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    a_host = w.assignments if layout == 0 else np.ascontiguousarray(w.assignments.T)
    a = torch.from_numpy(a_host).to("cuda:0")
    ref_p, ref_l = oracle.critical_path(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth,
                                        w.assignments, max_len=w.L)
    for ol in (0, 1):
        out = gpu.cp_eval(g, a, w.speeds, w.bandwidth, want=("cp", "b"), assign_layout=layout, out_layout=ol)
        paths, lens = gpu.cp_critical_path(g, a, w.speeds, w.bandwidth, out["b"], out["cp"],
                                           assign_layout=layout, b_layout=ol)
        assert np.array_equal(lens.cpu().numpy(), ref_l)
        assert np.array_equal(paths.cpu().numpy(), ref_p)
    g.close()


def test_critical_path_tiny_and_mlp(gpu, oracle):
    _check_paths(gpu, oracle, make_workload("tiny"))
    _check_paths(gpu, oracle, make_workload("tiny"), layout=1)
    _check_paths(gpu, oracle, make_workload("mlp", P=96))


def test_critical_path_with_ties_and_hubs(gpu, oracle):
    rng = np.random.default_rng(21)
    n, level, src, dst = random_layered_dag(rng, [6] * 12, 1, 4, 3)
    w = _custom("ties", n, src, dst, rng.integers(0, 3, size=len(src)), rng.integers(1, 3, size=n),
                [1, 2], [[1, 2], [1, 1]], rng.integers(0, 2, size=(70, n), dtype=np.uint8), level)
    _check_paths(gpu, oracle, w)
    # rows longer than one wavefront
    _check_paths(gpu, oracle, make_workload("comm_heavy", P=12, levels=5, width=600, hub_degree=300))


def test_critical_path_large_sparse_full(gpu, oracle):
    _check_paths(gpu, oracle, make_workload("large_sparse"))


def test_critical_path_64_bit_weights(gpu, oracle):
    rng = np.random.default_rng(22)
    n, level, src, dst = random_layered_dag(rng, [8] * 10, 1, 3, 2)
    w = _custom("wide-path", n, src, dst, rng.integers(1, 2**45, size=len(src)), rng.integers(1, 2**40, size=n),
                [1, 3, 2**33], rng.integers(1, 2**20, size=(3, 3)), rng.integers(0, 3, size=(20, n), dtype=np.uint8),
                level)
    _check_paths(gpu, oracle, w)


# ------------------------------------------------------------------ ranks of section 3.2

@pytest.mark.parametrize("name,kw", [("tiny", {}), ("mlp", {}), ("inception", {}), ("comm_heavy", {}),
                                     ("large_sparse", {})])
def test_ranks(gpu, oracle, name, kw):
    w = make_workload(name, P=1, **kw)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    up, down, total = gpu.cp_ranks(g)
    ref = oracle.ranks(w.n, w.succ_ptr, w.succ_idx, w.c)
    for got, exp, what in zip((up, down, total), ref, ("upRank", "downRank", "totalRank")):
        assert np.array_equal(got.cpu().numpy(), exp), what
    g.close()


def test_ranks_with_wide_weights(gpu, oracle):
    rng = np.random.default_rng(31)
    n, level, src, dst = random_layered_dag(rng, [70] * 9, 1, 3, 2)
    w = _custom("wide-ranks", n, src, dst, np.ones(len(src), dtype=np.int64), rng.integers(1, 2**40, size=n),
                [1], [[1]], np.zeros((1, n), dtype=np.uint8), level)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    assert g.info["min_tick_bytes"] == 8
    got = gpu.cp_ranks(g)
    ref = oracle.ranks(w.n, w.succ_ptr, w.succ_idx, w.c)
    for a, b in zip(got, ref):
        assert np.array_equal(a.cpu().numpy(), b)
    g.close()


# ------------------------------------------------------------------ PCT priority lists (section 4.1)

def _check_pct_order(gpu, oracle, w, layout=0, max_b="cp", sample=None):
    import torch
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    a_host = w.assignments if layout == 0 else np.ascontiguousarray(w.assignments.T)
    a = torch.from_numpy(a_host).to("cuda:0")
    rows = slice(0, w.P) if sample is None else slice(0, sample)
    ref_b = oracle.evaluate_workload(w, want=("b",), threads=8, partitions=rows)["b"]
    ref_order, ref_seg = oracle.pct_order(w.k, w.assignments[rows], ref_b, threads=8)
    for ol in (0, 1):
        out = gpu.cp_eval(g, a, w.speeds, w.bandwidth, want=("cp", "b"), assign_layout=layout, out_layout=ol)
        bound = int(out["cp"].max().item()) if max_b == "cp" else max_b
        order, seg = gpu.cp_pct_order(g, a, w.k, out["b"], max_b=bound, assign_layout=layout, b_layout=ol)
        b_host = out["b"].cpu().numpy()
        b_host = np.ascontiguousarray((b_host.T if ol == 0 else b_host)[rows]).astype(np.int64)
        assert np.array_equal(b_host, ref_b)
        assert np.array_equal(seg.cpu().numpy()[rows], ref_seg)
        assert np.array_equal(order.cpu().numpy()[rows], ref_order)
    g.close()


def test_pct_order_small(gpu, oracle):
    _check_pct_order(gpu, oracle, make_workload("tiny"))
    _check_pct_order(gpu, oracle, make_workload("tiny"), layout=1)
    _check_pct_order(gpu, oracle, make_workload("tiny"), max_b=0)            # the graph's own bound
    _check_pct_order(gpu, oracle, make_workload("mlp", P=70))
    _check_pct_order(gpu, oracle, make_workload("mlp", P=70), layout=1)


def test_pct_order_several_tiles_and_a_ragged_tail(gpu, oracle):
    # partitions of up to 20,480 vertices are sorted inside LDS by one workgroup: 19,772 takes 20
    # items per thread, 8,196 takes 9 of 16
    _check_pct_order(gpu, oracle, make_workload("inception", P=33))
    _check_pct_order(gpu, oracle, make_workload("comm_heavy", P=9, levels=4, width=2049))
    # above that and below 65,536 vertices: digit passes over tiles of 4,096 items, here 6 + 3,424
    w = make_workload("comm_heavy", P=5, levels=4, width=7000)
    assert 20480 < w.n < 65536
    _check_pct_order(gpu, oracle, w)
    _check_pct_order(gpu, oracle, w, layout=1)


def test_pct_order_many_ties_and_one_device(gpu, oracle):
    rng = np.random.default_rng(41)
    n, level, src, dst = random_layered_dag(rng, [700] * 8, 1, 3, 2)
    w = _custom("ties", n, src, dst, np.zeros(len(src), dtype=np.int64), np.ones(n, dtype=np.int64), [1, 1, 1],
                np.ones((3, 3), dtype=np.int64), rng.integers(0, 3, size=(5, n), dtype=np.uint8), level)
    _check_pct_order(gpu, oracle, w)                                         # b takes 8 values only
    w1 = _custom("one-device", n, src, dst, rng.integers(0, 50, size=len(src)), rng.integers(1, 50, size=n), [2],
                 [[1]], np.zeros((3, n), dtype=np.uint8), level)
    _check_pct_order(gpu, oracle, w1)


def test_pct_order_64_bit_keys(gpu, oracle):
    rng = np.random.default_rng(42)
    n, level, src, dst = random_layered_dag(rng, [600] * 9, 1, 3, 2)
    w = _custom("wide-order", n, src, dst, rng.integers(1, 2**45, size=len(src)), rng.integers(1, 2**40, size=n),
                [1, 3, 2**33], rng.integers(1, 2**20, size=(3, 3)), rng.integers(0, 3, size=(7, n), dtype=np.uint8),
                level)
    _check_pct_order(gpu, oracle, w)
    _check_pct_order(gpu, oracle, w, max_b=0)


def test_pct_order_large_sparse_full(gpu, oracle):
    _check_pct_order(gpu, oracle, make_workload("large_sparse"), sample=24)


def test_pct_order_buckets_of_the_leading_digit(gpu, oracle):
    """Partitions of 65,536 vertices or more with keys of more than 17 bits: one pass on the
    leading 9 bits, then every bucket sorted inside LDS."""
    _check_pct_order(gpu, oracle, make_workload("large_sparse", P=5, levels=300, width=300))
    _check_pct_order(gpu, oracle, make_workload("large_sparse", P=3, levels=300, width=300), layout=1)
    _check_pct_order(gpu, oracle, make_workload("comm_heavy", P=3, levels=20, width=4000))
    w = make_workload("large_sparse", P=3, levels=299, width=301)         # rows that are not 16-byte aligned
    assert w.n % 4 != 0
    _check_pct_order(gpu, oracle, w)
    # 31-bit keys (a path bound near 2^28, 8 devices): three passes inside a bucket, the first of
    # them with too many key bits left to travel in one word with the vertex number
    rng = np.random.default_rng(44)
    n, level, src, dst = random_layered_dag(rng, [700] * 100, 1, 3, 2)
    wide = _custom("wide-keys", n, src, dst, rng.integers(0, 2**20, size=len(src)), rng.integers(1, 2**21, size=n),
                   [1] * 8, np.ones((8, 8), dtype=np.int64), rng.integers(0, 8, size=(3, n), dtype=np.uint8), level)
    _check_pct_order(gpu, oracle, wide)
    # 18-bit keys (two devices, a path bound of 17 bits): the shortest keys on the bucket path,
    # nine bits left for the buckets, the second pass inside a bucket sorts on one bit
    rng = np.random.default_rng(45)
    n, level, src, dst = random_layered_dag(rng, [700] * 100, 1, 3, 2)
    narrow = _custom("narrow-keys", n, src, dst, rng.integers(0, 600, size=len(src)), rng.integers(1, 1200, size=n),
                     [1, 2], np.ones((2, 2), dtype=np.int64), rng.integers(0, 2, size=(3, n), dtype=np.uint8), level)
    _check_pct_order(gpu, oracle, narrow)


def test_pct_order_buckets_too_large_for_lds(gpu, oracle):
    """70,000 vertices without edges on one device and a generous bound: every key has the same
    leading bits, one bucket holds the whole partition, and the ordinary passes take over."""
    rng = np.random.default_rng(43)
    n = 70000
    w = _custom("one-bucket", n, np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64),
                rng.integers(1, 200, size=n), [1], [[1]], np.zeros((2, n), dtype=np.uint8),
                np.zeros(n, dtype=np.int64))
    _check_pct_order(gpu, oracle, w, max_b=2**24)
    # ... and two devices with everything but a handful of vertices on one of them
    a = np.zeros((2, n), dtype=np.uint8)
    a[:, ::1000] = 1
    w2 = _custom("lopsided", n, np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64),
                 rng.integers(1, 200, size=n), [1, 2], [[1, 1], [1, 1]], a, np.zeros(n, dtype=np.int64))
    _check_pct_order(gpu, oracle, w2, max_b=2**23)


def test_pct_order_buckets_from_rows_of_b(gpu, oracle):
    """Rows of b per partition on the bucket path: the leading pass builds its keys from b and
    the device ids directly.  64-bit ticks give the same lists; a bound that is too small and a
    device id >= k are still reported."""
    import torch
    w = make_workload("large_sparse", P=4, levels=300, width=300)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    a = torch.from_numpy(w.assignments).to("cuda:0")
    out = gpu.cp_eval(g, a, w.speeds, w.bandwidth, want=("cp", "b"), out_layout=1)
    bound = int(out["cp"].max().item())
    ref_order, ref_seg = oracle.pct_order(w.k, w.assignments, out["b"].cpu().numpy().astype(np.int64), threads=8)
    order, seg = gpu.cp_pct_order(g, a, w.k, out["b"].to(torch.int64), max_b=bound, b_layout=1)
    assert np.array_equal(order.cpu().numpy(), ref_order) and np.array_equal(seg.cpu().numpy(), ref_seg)
    with pytest.raises(ValueError):
        gpu.cp_pct_order(g, a, w.k, out["b"], max_b=bound - 1, b_layout=1)
    bad = a.clone()
    bad[2, w.n - 5] = w.k
    with pytest.raises(ValueError):
        gpu.cp_pct_order(g, bad, w.k, out["b"], max_b=bound, b_layout=1)
    g.close()


def test_pct_order_reports_a_bound_that_is_too_small(gpu):
    import torch
    w = make_workload("tiny")
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    a = torch.from_numpy(w.assignments).to("cuda:0")
    out = gpu.cp_eval(g, a, w.speeds, w.bandwidth, want=("cp", "b"))
    with pytest.raises(ValueError):
        gpu.cp_pct_order(g, a, w.k, out["b"], max_b=int(out["cp"].max().item()) - 1)
    g.close()


# ------------------------------------------------------------------ placement constraints (section 2)

@pytest.mark.parametrize("layout", [0, 1])
def test_validate_against_the_oracle(gpu, oracle, layout):
    import torch
    rng = np.random.default_rng(51)
    w = make_workload("inception", P=300)
    # constraints that one hidden placement satisfies: pairs inside its device classes, pins to its devices
    hidden = rng.integers(0, w.k, size=w.n).astype(np.uint8)
    u = rng.integers(0, w.n, size=1000)
    v = np.array([rng.choice(np.nonzero(hidden == hidden[x])[0]) for x in u])
    pairs = np.stack([u, v], axis=1).astype(np.int32)
    pv = rng.integers(0, w.n, size=700)
    pins = np.stack([pv, hidden[pv]], axis=1).astype(np.int32)
    a = w.assignments.copy()
    a[:20] = hidden                                   # valid
    for j in range(20, 40):                           # a few constraints broken
        a[j] = hidden
        flip = rng.integers(0, w.n, size=j - 19)
        a[j, flip] = (a[j, flip] + 1) % w.k
    ref_valid, ref_broken = oracle.validate(w.k, a, pairs, pins)
    assert 0 < ref_valid.sum() < w.P
    a_dev = torch.from_numpy(np.ascontiguousarray(a if layout == 0 else a.T)).to("cuda:0")
    valid, broken = gpu.cp_validate(a_dev, w.k, torch.from_numpy(pairs).to("cuda:0"),
                                    torch.from_numpy(pins).to("cuda:0"), assign_layout=layout)
    assert np.array_equal(valid.cpu().numpy(), ref_valid)
    assert np.array_equal(broken.cpu().numpy(), ref_broken)
    # no constraints at all; pairs only; pins only
    for pr, pn in ((None, None), (pairs, None), (None, pins)):
        rv, rb = oracle.validate(w.k, a, pr if pr is not None else [], pn if pn is not None else [])
        v, b = gpu.cp_validate(a_dev, w.k, None if pr is None else torch.from_numpy(pr).to("cuda:0"),
                               None if pn is None else torch.from_numpy(pn).to("cuda:0"), assign_layout=layout)
        assert np.array_equal(v.cpu().numpy(), rv) and np.array_equal(b.cpu().numpy(), rb)


def test_validate_reports_an_index_out_of_range(gpu):
    import torch
    a = torch.zeros((3, 10), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(ValueError):
        gpu.cp_validate(a, 2, torch.tensor([[0, 10]], dtype=torch.int32, device="cuda:0"))
    with pytest.raises(ValueError):
        gpu.cp_validate(a, 2, None, torch.tensor([[0, 2]], dtype=torch.int32, device="cuda:0"))


# ------------------------------------------------------------------ critical-path move search

def _check_search(gpu, oracle, w, start, pairs=(), pins=(), max_moves=1000, chunk=256):
    import torch
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    ref_a, ref_trace, ref_moves = oracle.search(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth,
                                                start, max_len=w.L, pairs=pairs, pins=pins, max_moves=max_moves,
                                                threads=8)
    to_dev = lambda x: torch.from_numpy(np.asarray(x, dtype=np.int32).reshape(-1, 2)).to("cuda:0") if len(x) else None
    got = gpu.cp_search(g, torch.from_numpy(np.ascontiguousarray(start)).to("cuda:0"), w.speeds, w.bandwidth,
                        pairs=to_dev(pairs), pins=to_dev(pins), max_moves=max_moves, chunk=chunk)
    assert got["cp_trace"].tolist() == ref_trace.tolist()
    assert got["moves"].tolist() == ref_moves.tolist()
    assert np.array_equal(got["assignment"].cpu().numpy(), ref_a)
    g.close()
    return got


def test_search_tiny_and_mlp(gpu, oracle):
    w = make_workload("tiny")
    got = _check_search(gpu, oracle, w, w.assignments[0])
    assert len(got["moves"]) >= 2
    _check_search(gpu, oracle, w, w.assignments[1], chunk=3)              # many ragged chunks
    v0 = int(got["moves"][0][0])
    _check_search(gpu, oracle, w, w.assignments[0], pins=[[v0, int(w.assignments[0][v0])]], pairs=[[0, 1]])
    _check_search(gpu, oracle, w, w.assignments[0], max_moves=1)
    w = make_workload("mlp", P=2)                                          # n = 2016: rows are 16-byte multiples
    _check_search(gpu, oracle, w, w.assignments[0], max_moves=6, chunk=200)


def test_search_under_the_wave_column_plan(gpu, oracle):
    # hub rows rule the window plan out: candidates are evaluated with b kept
    w = make_workload("comm_heavy", P=2, levels=5, width=300, hub_degree=280)
    _check_search(gpu, oracle, w, w.assignments[0], max_moves=3, chunk=16)


# ------------------------------------------------------------------ Critical Path partitioning strategy (section 3.2.2)

@pytest.mark.parametrize("name,kw", [("tiny", {}), ("mlp", {}), ("inception", {}), ("large_sparse", {"levels": 300}),
                                     ("comm_heavy", {"levels": 6, "width": 900, "hub_degree": 300})])
def test_seed_partition(gpu, oracle, name, kw):
    w = make_workload(name, P=1, **kw)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    got = gpu.cp_seed_partition(g, w.speeds)
    ref = oracle.seed(w.n, w.succ_ptr, w.succ_idx, w.c, w.speeds, max_len=w.L)
    assert np.array_equal(got.cpu().numpy(), ref)
    g.close()


def test_seed_partition_wide_weights_and_many_devices(gpu, oracle):
    rng = np.random.default_rng(61)
    n, level, src, dst = random_layered_dag(rng, [33] * 7, 1, 3, 2)
    c = rng.integers(1, 2**40, size=n)
    w = _custom("wide-seed", n, src, dst, np.ones(len(src), dtype=np.int64), c, [1, 3, 2**33, 2**33, 5],
                np.ones((5, 5), dtype=np.int64), np.zeros((1, n), dtype=np.uint8), level)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    got = gpu.cp_seed_partition(g, w.speeds)
    assert np.array_equal(got.cpu().numpy(), oracle.seed(w.n, w.succ_ptr, w.succ_idx, w.c, w.speeds, max_len=w.L))
    g.close()
    # 64 devices with many equal speeds: ties go to the lowest number
    speeds = np.array([7] * 20 + [9] * 20 + [3] * 24)
    w = make_workload("mlp", P=1)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    got = gpu.cp_seed_partition(g, speeds)
    assert np.array_equal(got.cpu().numpy(), oracle.seed(w.n, w.succ_ptr, w.succ_idx, w.c, speeds, max_len=w.L))
    g.close()


def test_seed_then_search(gpu, oracle):
    """The strategy's partition as the start of the search, end to end against the oracle."""
    w = make_workload("mlp", P=1)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    start = gpu.cp_seed_partition(g, w.speeds)
    got = gpu.cp_search(g, start, w.speeds, w.bandwidth, max_moves=8, chunk=128)
    ref_start = oracle.seed(w.n, w.succ_ptr, w.succ_idx, w.c, w.speeds, max_len=w.L)
    ref_a, ref_trace, ref_moves = oracle.search(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth,
                                                ref_start, max_len=w.L, max_moves=8, threads=8)
    assert got["cp_trace"].tolist() == ref_trace.tolist() and got["moves"].tolist() == ref_moves.tolist()
    assert np.array_equal(got["assignment"].cpu().numpy(), ref_a)
    g.close()


# ------------------------------------------------------------------ mask written by the t sweep, and its fallbacks

@pytest.mark.parametrize("width,P", [(7, 3), (8, 5), (8, 4), (25, 64), (16, 1)])
def test_mask_rows_for_aligned_and_unaligned_sizes(gpu, oracle, width, P):
    """Partition-major masks under the window plan: with n * P * 4 a multiple of 16 the t sweep
    writes the bits itself, otherwise the separate pass does; n is not a multiple of 64 in
    either case, so the last mask word of a row is partly used."""
    rng = np.random.default_rng(71 + width)
    n, level, src, dst = random_layered_dag(rng, [width] * 11, 1, 3, 2)
    w = _custom("mask-rows", n, src, dst, rng.integers(0, 40, size=len(src)), rng.integers(1, 30, size=n), [1, 2, 3],
                [[1, 2, 3], [2, 1, 2], [4, 3, 1]], rng.integers(0, 3, size=(P, n), dtype=np.uint8), level)
    _check(gpu, oracle, w, plans=(WINDOW,), out_layouts=(1,))


def test_mask_rows_when_ids_are_gathered(gpu, oracle):
    """Vertices numbered against the level order: the ids of a level are spread over the whole
    range, so they are gathered first and the t sweep does not write the mask."""
    rng = np.random.default_rng(72)
    n, level, src, dst = random_layered_dag(rng, [600] * 12, 1, 3, 2)
    perm = rng.permutation(n)
    w = _custom("scrambled", n, perm[src], perm[dst], rng.integers(1, 50, size=len(src)),
                rng.integers(1, 30, size=n), [1, 2], [[1, 3], [2, 1]],
                rng.integers(0, 2, size=(16, n), dtype=np.uint8), None)
    _check(gpu, oracle, w, plans=(WINDOW, COLUMN), out_layouts=(0, 1))


def test_search_degenerate_calls(gpu, oracle):
    import torch
    w = make_workload("tiny")
    # no moves allowed: the trace is the start's CP alone; a chunk larger than the neighbourhood
    _check_search(gpu, oracle, w, w.assignments[2], max_moves=0)
    _check_search(gpu, oracle, w, w.assignments[2], chunk=100000)
    # one device: nothing can move
    w1 = _custom("one-device", w.n, np.repeat(np.arange(w.n), np.diff(w.succ_ptr)), w.succ_idx, w.succ_t, w.c, [3],
                 [[1]], np.zeros((1, w.n), dtype=np.uint8))
    got = _check_search(gpu, oracle, w1, w1.assignments[0])
    assert len(got["moves"]) == 0 and got["evaluated"] == 0
    # every vertex pinned where it is: all candidates are invalid, the search stops at once
    pins = np.stack([np.arange(w.n), w.assignments[0]], axis=1)
    got = _check_search(gpu, oracle, w, w.assignments[0], pins=pins.tolist())
    assert len(got["moves"]) == 0 and got["evaluated"] > 0
    # a start with a device id out of range is refused
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    bad = torch.from_numpy(w.assignments[0].copy()).to("cuda:0")
    bad[5] = 7
    with pytest.raises(gpu.CpError) as e:
        gpu.cp_search(g, bad, w.speeds, w.bandwidth)
    assert e.value.code == -12
    g.close()


# ------------------------------------------------------------------ far reads of the resident-window plan

def _with_long_edges(rng, widths, extra, min_span):
    n, level, src, dst = random_layered_dag(rng, widths, 1, 4, 6)
    L = len(widths)
    off = np.concatenate([[0], np.cumsum(widths)])
    lo = rng.integers(0, L - min_span, size=extra)
    hi = rng.integers(lo + min_span, L)                 # uniformly over the levels far enough ahead
    u = off[lo] + rng.integers(0, np.asarray(widths)[lo])
    v = off[hi] + rng.integers(0, np.asarray(widths)[hi])
    pairs = np.unique(np.stack([np.concatenate([src, u]), np.concatenate([dst, v])], axis=1), axis=0)
    return n, level, pairs[:, 0], pairs[:, 1]


def test_long_edges_do_not_rule_the_window_plan_out(gpu, oracle):
    """A deep narrow graph with edges that span most of its depth: their far ends do not fit an
    LDS ring, so the window plan reads them back from the output array."""
    rng = np.random.default_rng(81)
    n, level, src, dst = _with_long_edges(rng, [700] * 400, extra=6000, min_span=40)
    w = _custom("long-edges", n, src, dst, rng.integers(1, 3000, size=len(src)), rng.integers(1, 500, size=n),
                [1, 2, 4, 4], rng.integers(1, 40, size=(4, 4)), rng.integers(0, 4, size=(70, n), dtype=np.uint8), level)
    g = gpu.CpGraph.from_workload(w)
    info = g.info
    shapes = [g.window_shape(4, tsweep=ts) for ts in (False, True)]
    g.close()
    assert info["window_ok"] == 1 and info["window_far_b"] > 0 and info["window_far_t"] > 0
    # wide ticks: eight slices on fewer compute wavefronts, two output stores per wavefront and tick,
    # the larger of the two store counts the far reads' ordering allows for
    assert all(sh["far_waves"] > 0 and sh["stores_per_tick"] == 2 for sh in shapes), shapes
    _check(gpu, oracle, w, plans=(WINDOW, COLUMN), layouts=(0, 1))
    # CP alone still needs the b array on such a graph
    from gpu_util import run_gpu
    r = run_gpu(w, WINDOW, want=("cp",))
    assert "b" in r and np.array_equal(r["cp"], _oracle(oracle, w, want=("cp",))["cp"])


def test_far_reads_with_few_levels_and_mirror_edges(gpu, oracle):
    """A forward chain mirrored by a backward chain with an edge from every forward vertex to
    its twin (the shape of a training graph), deep enough that the twins are far apart."""
    depth, width = 1500, 20
    n = 2 * depth * width
    fwd = np.arange(depth * width).reshape(depth, width)
    bwd = fwd[::-1] + depth * width
    src = np.concatenate([fwd[:-1].ravel(), bwd[:-1].ravel(), fwd.ravel(), fwd[-1]])
    dst = np.concatenate([fwd[1:].ravel(), bwd[1:].ravel(), bwd[::-1].ravel(), bwd[0]])
    rng = np.random.default_rng(82)
    level = np.concatenate([np.repeat(np.arange(depth), width), np.repeat(np.arange(2 * depth - 1, depth - 1, -1), width)])
    w = _custom("mirror", n, src, dst, rng.integers(1, 200, size=len(src)), rng.integers(1, 60, size=n), [2, 3, 5],
                rng.integers(1, 9, size=(3, 3)), rng.integers(0, 3, size=(130, n), dtype=np.uint8), level)
    g = gpu.CpGraph.from_workload(w)
    info = g.info
    shapes = [g.window_shape(3, tsweep=ts) for ts in (False, True)]
    g.close()
    assert info["window_ok"] == 1 and info["window_far_b"] > 0
    # narrow ticks: one slice, one output store per compute wavefront and tick
    assert all(sh["far_waves"] > 0 and sh["stores_per_tick"] == 1 for sh in shapes), shapes
    _check(gpu, oracle, w)
    _check_paths(gpu, oracle, w)


def _chain_and_wide_level(width):
    """A chain of six vertices, one per level, and `width` vertices without edges in a seventh
    level: the widest tick of either sweep is far wider than any edge's span."""
    n = 6 + width
    src, dst = np.arange(5), np.arange(1, 6)
    level = np.concatenate([np.arange(6), np.full(width, 6)])
    return n, level, src, dst


@pytest.mark.parametrize("shape", ["no-edges", "wide-level"])
def test_ticks_wider_than_any_edge_span(gpu, oracle, shape):
    """The ring of the window plans is sized by the edges' spans; a tick whose vertices have no
    edges still publishes into it and must find room (279 vertices without a single edge once
    overwrote the staged device ids)."""
    from gpu_util import assert_equal_to_oracle, run_gpu
    rng = np.random.default_rng(83)
    if shape == "no-edges":
        n, level, src, dst = 279, np.zeros(279, dtype=np.int64), np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64)
    else:
        n, level, src, dst = _chain_and_wide_level(300)
    k = 50
    w = _custom(shape, n, src, dst, rng.integers(1, 100, size=len(src)), rng.integers(1, 5000, size=n),
                rng.integers(1, 100, size=k), rng.integers(1, 5, size=(k, k)),
                rng.integers(0, k, size=(5, n), dtype=np.uint8), level)
    ref = _oracle(oracle, w)
    g = gpu.CpGraph.from_workload(w, device="cuda:0")
    info = g.info
    assert info["window_ok"] == 1
    assert min(info["window_slots_b"], info["window_slots_t"]) >= min(info["max_level_width"], 512)
    ran = 0
    for plan in (1, 2, 3, 4, 5, 6):
        for layout in (0, 1):
            for ol in (0, 1):
                try:
                    res = run_gpu(w, plan, layout=layout, graph=g, out_layout=ol)
                except gpu.CpError as e:
                    assert plan != 1 and e.code == -12, (plan, e.code)
                    continue
                ran += 1
                assert_equal_to_oracle(res, ref, what=f"{shape} plan={plan} layout={layout} out={ol}")
    g.close()
    assert ran >= 12


# ------------------------------------------------------------------ many small random shapes

@pytest.mark.parametrize("block", range(4))
def test_random_shapes(gpu, oracle, block):
    """Layered DAGs of random depth, width, degree and edge span, with random device counts,
    batch sizes and weight ranges: every output of every plan that can run them, both layouts."""
    from gpu_util import assert_equal_to_oracle, run_gpu
    for seed in range(block * 6, block * 6 + 6):
        rng = np.random.default_rng(9000 + seed)
        depth = int(rng.integers(2, 60))
        widths = rng.integers(1, int(rng.choice([3, 20, 90, 300])) + 1, size=depth)
        n, level, src, dst = random_layered_dag(rng, widths, int(rng.integers(0, 2)), int(rng.integers(2, 9)),
                                                int(rng.integers(1, max(2, depth))))
        k = int(rng.choice([1, 2, 3, 7, 16, 33]))
        P = int(rng.choice([1, 5, 64, 65, 130]))
        tmax = int(rng.choice([1, 50, 70000, 2**31]))
        cmax = int(rng.choice([1, 99, 10**6]))
        B = rng.integers(1, int(rng.choice([2, 64, 10**5])) + 1, size=(k, k))
        w = _custom(f"random-{seed}", n, src, dst, rng.integers(0, tmax + 1, size=len(src)),
                    rng.integers(0, cmax + 1, size=n), rng.integers(1, int(rng.choice([2, 17, 5000])) + 1, size=k), B,
                    rng.integers(0, k, size=(P, n), dtype=np.uint8), level)
        ref = _oracle(oracle, w)
        g = gpu.CpGraph.from_workload(w, device="cuda:0")
        plans = [COLUMN] + ([WINDOW] if g.info["window_ok"] else [])
        for plan in plans:
            for ol in (0, 1):
                for layout in (0, 1):
                    try:
                        res = run_gpu(w, plan, layout=layout, graph=g, out_layout=ol)
                    except gpu.CpError as e:
                        # the window plan also needs cost tables in the 32-bit form and room in LDS for k
                        assert plan == WINDOW and e.code == -12, (seed, plan, e.code)
                        continue
                    assert_equal_to_oracle(res, ref, what=f"seed={seed} plan={plan} layout={layout} out={ol} "
                                                          f"n={n} k={k} P={P}")
        g.close()


@pytest.mark.parametrize("seed", range(4))
def test_random_deep_shapes_with_long_spans(gpu, oracle, seed):
    """Deep graphs whose edges may span the whole depth: the window plan runs them with far reads."""
    rng = np.random.default_rng(9500 + seed)
    depth = int(rng.integers(250, 600))
    widths = rng.integers(20, 110, size=depth)
    n, level, src, dst = random_layered_dag(rng, widths, 1, 3, depth - 1)
    k = int(rng.choice([2, 5, 16]))
    P = int(rng.choice([3, 64, 200]))
    w = _custom(f"deep-{seed}", n, src, dst, rng.integers(0, 3000, size=len(src)), rng.integers(1, 400, size=n),
                rng.integers(1, 9, size=k), rng.integers(1, 50, size=(k, k)),
                rng.integers(0, k, size=(P, n), dtype=np.uint8), level)
    g = gpu.CpGraph.from_workload(w)
    info = g.info
    g.close()
    if info["window_ok"]:
        assert info["window_far_b"] > 0 or info["window_slots_b"] < 20000
    _check(gpu, oracle, w, plans=(COLUMN,) + ((WINDOW,) if info["window_ok"] else ()), layouts=(0, 1))

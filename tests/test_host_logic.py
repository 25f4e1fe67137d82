"""CPU-only checks of the library's host side: it loads, exports what the header
declares, validates graphs, reports graph facts, and builds exact division
constants.  No kernel is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_1711_01912_amd as cpe
from paper_1711_01912_amd import binding
from workloads import build_csr, make_workload, random_layered_dag

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_1711_01912_amd.build import build_library
    build_library(force=False)
    return cpe.load_library()


def test_library_exports_every_declared_symbol(lib):
    text = open(os.path.join(ROOT, "include", "cpeval.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(cp_[a-z_]+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_error_strings(lib):
    seen = set()
    for code in range(0, -14, -1):
        s = cpe.error_string(code)
        assert s and s != "unknown error code"
        seen.add(s)
    assert len(seen) == 14
    assert cpe.error_string(-99) == "unknown error code"


def _graph_args(w):
    return dict(n=w.n, succ_ptr=w.succ_ptr.copy(), succ_idx=w.succ_idx.copy(), succ_t=w.succ_t.copy(),
                pred_ptr=w.pred_ptr.copy(), pred_idx=w.pred_idx.copy(), pred_eid=w.pred_eid.copy(),
                c=w.c.copy(), level_ptr=w.level_ptr.copy(), level_vtx=w.level_vtx.copy())


def _create_rc(**a):
    try:
        cpe.CpGraph(**a).close()
        return 0
    except cpe.CpError as e:
        return e.code


def test_create_accepts_every_workload_recipe(lib):
    for name, kw in [("tiny", {}), ("mlp", dict(P=4, layers=4, shards=2)),
                     ("inception", dict(P=4, modules=3, groups=2)),
                     ("large_sparse", dict(P=4, levels=30, width=20)),
                     ("comm_heavy", dict(P=4, levels=4, width=400, hub_degree=300))]:
        w = make_workload(name, **kw)
        g = cpe.CpGraph.from_workload(w)
        info = g.info
        assert (info["n"], info["m"], info["L"]) == (w.n, w.m, w.L)
        assert info["max_out_degree"] == int(np.diff(w.succ_ptr).max())
        assert info["max_in_degree"] == int(np.diff(w.pred_ptr).max())
        assert info["max_level_width"] == int(np.diff(w.level_ptr).max())
        assert info["num_sources"] == int((np.diff(w.pred_ptr) == 0).sum())
        assert info["num_sinks"] == int((np.diff(w.succ_ptr) == 0).sum())
        assert info["max_c"] == int(w.c.max()) and info["max_t"] == int(w.succ_t.max())
        assert info["uploaded"] == 0 and info["blob_bytes"] % 256 == 0
        g.close()


def test_raw_path_bound_is_the_unit_speed_critical_path(lib, oracle):
    """U0 is the critical path with w = c and x = t: one device per vertex pair
    cannot be arranged in general, so compare on a chain-free bound instead: it
    must dominate CP for any speeds/bandwidth >= 1 and equal the longest raw path."""
    w = make_workload("large_sparse", P=6, levels=25, width=12)
    g = cpe.CpGraph.from_workload(w)
    u0 = g.info["raw_path_bound"]
    # longest raw path by plain DP in level order
    best = np.zeros(w.n, dtype=np.int64)
    for l in range(w.L - 1, -1, -1):
        for v in w.level_vtx[w.level_ptr[l]:w.level_ptr[l + 1]]:
            e0, e1 = w.succ_ptr[v], w.succ_ptr[v + 1]
            m = 0 if e0 == e1 else int((w.succ_t[e0:e1] + best[w.succ_idx[e0:e1]]).max())
            best[v] = w.c[v] + m
    assert u0 == int(best.max())
    out = oracle.evaluate_workload(w)
    assert (out["cp"] <= u0).all()
    assert g.info["min_tick_bytes"] == 4


def test_create_rejects_bad_graphs(lib):
    w = make_workload("tiny")
    base = _graph_args(w)
    assert _create_rc(**base) == 0

    a = dict(base); a["succ_ptr"] = base["succ_ptr"].copy(); a["succ_ptr"][3] = a["succ_ptr"][4] + 1
    assert _create_rc(**a) == -3                       # non-monotone ptr
    a = dict(base); a["succ_idx"] = base["succ_idx"].copy(); a["succ_idx"][0] = w.n
    assert _create_rc(**a) == -3                       # index out of range
    a = dict(base); a["pred_eid"] = base["pred_eid"].copy(); a["pred_eid"][0] = a["pred_eid"][1]
    assert _create_rc(**a) == -3                       # eid not a permutation
    a = dict(base); a["pred_idx"] = base["pred_idx"].copy()
    a["pred_idx"][0] = (a["pred_idx"][0] + 1) % w.n
    assert _create_rc(**a) == -3                       # pred disagrees with succ
    a = dict(base); a["level_vtx"] = base["level_vtx"].copy(); a["level_vtx"][0] = a["level_vtx"][1]
    assert _create_rc(**a) == -4                       # not a permutation
    a = dict(base); a["level_vtx"] = base["level_vtx"][::-1].copy()
    assert _create_rc(**a) == -4                       # edges go down
    a = dict(base); a["c"] = base["c"].copy(); a["c"][5] = -1
    assert _create_rc(**a) == -5
    a = dict(base); a["succ_t"] = base["succ_t"].copy(); a["succ_t"][7] = -3
    assert _create_rc(**a) == -5
    a = dict(base); a["c"] = base["c"].copy(); a["c"][:] = 2**61
    assert _create_rc(**a) == -8                       # raw path bound >= 2^62
    a = dict(base); a["n"] = 0
    assert _create_rc(**a) == -2
    a = dict(base); a["c"] = None
    assert _create_rc(**a) == -1


def test_cycle_is_rejected_through_the_level_check(lib):
    # 0 -> 1 -> 0 cannot be levelled
    csr = dict(n=2, succ_ptr=[0, 1, 2], succ_idx=[1, 0], succ_t=[1, 1],
               pred_ptr=[0, 1, 2], pred_idx=[1, 0], pred_eid=[1, 0], c=[1, 1],
               level_ptr=[0, 1, 2], level_vtx=[0, 1])
    assert _create_rc(**csr) == -4


def test_edgeless_and_wide_tick_graphs(lib):
    g = cpe.CpGraph(5, [0] * 6, None, None, [0] * 6, None, None, [3, 1, 4, 1, 5], [0, 5], [0, 1, 2, 3, 4])
    assert g.info["m"] == 0 and g.info["num_sources"] == 5 and g.info["raw_path_bound"] == 5
    g.close()
    csr = build_csr(3, [0, 1], [1, 2], [2**40, 5])
    g = cpe.CpGraph(3, csr["succ_ptr"], csr["succ_idx"], csr["succ_t"], csr["pred_ptr"],
                    csr["pred_idx"], csr["pred_eid"], [1, 1, 1], csr["level_ptr"], csr["level_vtx"])
    assert g.info["min_tick_bytes"] == 8 and g.info["window_ok"] == 0
    assert g.info["auto_plan"] == cpe.PLAN_WAVE_COLUMN
    g.close()


def test_plan_selection_facts(lib):
    w = make_workload("large_sparse", P=4, levels=40, width=30)
    g = cpe.CpGraph.from_workload(w)
    info = g.info
    assert info["window_ok"] == 1 and info["auto_plan"] == cpe.PLAN_RESIDENT_WINDOW
    # the ring must cover at least one level plus the longest edge span (10 levels here)
    assert 30 <= info["window_slots_b"] <= 11 * 30
    assert 30 <= info["window_slots_t"] <= 11 * 30
    g.close()
    w = make_workload("comm_heavy", P=4, levels=4, width=400, hub_degree=300)
    g = cpe.CpGraph.from_workload(w)
    assert g.info["auto_plan"] == cpe.PLAN_WAVE_COLUMN   # hub rows
    g.close()


def test_workspace_bytes_and_eval_argument_errors(lib):
    w = make_workload("tiny")
    g = cpe.CpGraph.from_workload(w)
    # cost tables, then either the transposed ids (wave-column) or the ids gathered into
    # sweep order for each direction (resident-window: 8 levels padded to 64 positions)
    assert binding.workspace_bytes(g, 16, 2, plan=cpe.PLAN_RESIDENT_WINDOW) == 256 + 2 * 16 * 8 * 64
    assert binding.workspace_bytes(g, 16, 2, plan=cpe.PLAN_WAVE_COLUMN) == 256 + 1024
    assert binding.workspace_bytes(g, 16, 2) == 256 + 2 * 16 * 8 * 64
    # partition-major outputs of the wave-column plan pass through two vertex-major scratch arrays
    assert binding.workspace_bytes(g, 16, 2, plan=cpe.PLAN_WAVE_COLUMN, out_layout=cpe.OUT_PARTITION_MAJOR,
                                   tick_bytes=4) == 256 + 1024 + 2 * 64 * 16 * 4
    assert binding.workspace_bytes(g, 16, 2, plan=cpe.PLAN_RESIDENT_WINDOW, out_layout=cpe.OUT_PARTITION_MAJOR,
                                   tick_bytes=4) == 256 + 2 * 16 * 8 * 64
    with pytest.raises(cpe.CpError) as e:
        binding.workspace_bytes(g, 0, 2)
    assert e.value.code == -2
    with pytest.raises(cpe.CpError) as e:
        binding.workspace_bytes(g, 4, 256)
    assert e.value.code == -2

    s = np.array([1, 2], dtype=np.int64)
    B = np.array([[1, 10], [10, 1]], dtype=np.int64)
    dummy = C.c_void_p(256)   # never dereferenced: every call below fails before any use
    i64p = C.POINTER(C.c_int64)

    def call(batch=4, k=2, assign=dummy, layout=0, sp=s, bw=B, ws=dummy, cp=dummy, b=dummy, tl=dummy,
             mask=dummy, tick=4, plan=0, status=dummy, out_layout=0):
        return lib.cp_eval(g._handle, batch, k, assign, layout, sp.ctypes.data_as(i64p),
                           bw.ctypes.data_as(i64p), ws, 1 << 20, None, cp, b, tl, mask, tick, out_layout, plan,
                           status, None)

    assert call(batch=0) == -2
    assert call(k=0) == -2
    assert call(layout=7) == -12
    assert call(plan=9) == -12
    assert call(tick=2) == -12
    assert call(out_layout=2) == -12
    assert call(assign=C.c_void_p()) == -1
    assert call(status=C.c_void_p()) == -1
    assert call(b=C.c_void_p()) == -12            # cp needs b
    assert call(tl=C.c_void_p()) == -12           # mask needs tl
    assert call() == -11                          # everything fine, but the graph was never uploaded
    g.close()


@pytest.mark.parametrize("amax", [0, 1, 999, 10**4, 10**7, 2**31, 2**32 - 1])
def test_multiply_shift_constants_are_exact(lib, amax):
    rng = np.random.default_rng(amax % 1000)
    divisors = list(range(1, 70)) + [100, 255, 256, 257, 1000, 4095, 4096, 65535, 65536, 65537,
                                     10**6, 2**31 - 1, 2**31, 2**32 - 1]
    divisors += [int(x) for x in rng.integers(1, 2**32, size=40)]
    found = 0
    for d in divisors:
        mg = cpe.cost_magic(d, amax)
        if mg is None:
            continue
        found += 1
        mul, dm1 = mg
        assert dm1 == d - 1
        # dividends around every multiple boundary near the ends, plus random ones
        cands = {0, 1, amax, max(0, amax - 1)}
        for q in (1, 2, 3, amax // d, max(0, amax // d - 1)):
            for delta in (-1, 0, 1):
                cands.add(q * d + delta)
        cands |= {int(x) for x in rng.integers(0, amax + 1, size=200)}
        for a in cands:
            if 0 <= a <= amax:
                n_ = a + dm1
                assert n_ < 2**32
                assert (n_ * mul + n_) >> 32 == -(-a // d), (a, d)
    if amax <= 10**7:
        assert found >= 69   # every small divisor must take the fast path for small weights


def test_multiply_shift_exhaustive_small_range(lib):
    for d in range(1, 130):
        mul, dm1 = cpe.cost_magic(d, 5000)
        a = np.arange(0, 5001, dtype=np.uint64)
        n_ = a + np.uint64(dm1)
        got = (n_ * np.uint64(mul) + n_) >> np.uint64(32)
        assert (got == (a + np.uint64(d - 1)) // np.uint64(d)).all()


def test_four_byte_table_entries_are_exact(lib):
    """Every dividend of the range, every divisor up to 256: the 4-byte form equals ceil(a / d)
    wherever the library offers it, and it is offered for the benchmark's ranges."""
    offered = 0
    for amax in (0, 1, 1000, 10_000, 70_000, 2**20, 2**24 - 1):
        if amax <= 70_000:
            a = np.arange(0, amax + 1, dtype=np.uint64)
        else:
            rng = np.random.default_rng(amax)
            a = np.unique(np.concatenate([np.arange(0, 3000), np.arange(amax - 3000, amax + 1),
                                          rng.integers(0, amax + 1, size=20000)])).astype(np.uint64)
        for d in range(1, 258):
            e = cpe.cost_compact(d, amax)
            if e is None:
                assert d > 256 or (amax + d - 1) * 257 * d >= 2**32, (d, amax)   # only where exactness is not provable
                continue
            offered += 1
            assert e & 0xff == d - 1
            if amax > 70_000:                       # multiples of d near the top of the range as well
                top = (np.uint64(amax) // np.uint64(d)) * np.uint64(d)
                aa = np.unique(np.concatenate([a, top - np.arange(0, 3, dtype=np.uint64) * np.uint64(d),
                                               top + np.uint64(1) - np.arange(0, 3, dtype=np.uint64) * np.uint64(d)]))
                aa = aa[aa <= np.uint64(amax)]
            else:
                aa = a
            n_ = aa + np.uint64(e & 0xff)
            got = (n_ * np.uint64(e | 0xff) + n_) >> np.uint64(32)
            assert (got == (aa + np.uint64(d - 1)) // np.uint64(d)).all(), (d, amax)
    assert offered > 1000
    # the large sparse workload's ranges: volumes up to 10,000 over rates up to 64, work up to 1,000 over speeds up to 16
    assert all(cpe.cost_compact(d, 10_000) is not None for d in range(1, 65))
    assert cpe.cost_compact(257, 100) is None and cpe.cost_compact(3, 2**24) is None
    # a free transfer's entry 0 gives 0 ticks for every volume below 2^24
    a = np.array([0, 1, 12345, 2**24 - 1], dtype=np.uint64)
    assert (((a * np.uint64(0xff) + a) >> np.uint64(32)) == 0).all()


def test_consumer_entry_points_check_their_arguments(lib):
    """cp_critical_path, cp_pct_order and cp_ranks reject bad arguments before touching the GPU."""
    w = make_workload("tiny")
    g = cpe.CpGraph.from_workload(w)
    s = np.array([1, 2], dtype=np.int64)
    B = np.array([[1, 10], [10, 1]], dtype=np.int64)
    dummy = C.c_void_p(256)
    i64p = C.POINTER(C.c_int64)
    sp, bp = s.ctypes.data_as(i64p), B.ctypes.data_as(i64p)

    def path(batch=4, k=2, assign=dummy, layout=0, b=dummy, cp=dummy, tick=4, b_layout=0, ws=dummy, max_len=8,
             out=dummy):
        return lib.cp_critical_path(g._handle, batch, k, assign, layout, sp, bp, b, cp, tick, b_layout, ws, 1 << 20,
                                    None, max_len, out, dummy, dummy)

    assert path(batch=0) == -2
    assert path(layout=3) == -12
    assert path(b_layout=2) == -12
    assert path(tick=5) == -12
    assert path(b=C.c_void_p()) == -1
    assert path() == -11                           # not uploaded

    need = C.c_size_t(0)
    assert lib.cp_pct_order_workspace_bytes(g._handle, 16, 2, 0, C.byref(need)) == 0
    # two key arrays and one list of 16 x 64 32-bit items, counts for 512 digits x 1 tile x 16 partitions,
    # one aligned slot for the flag of the bucket path
    assert need.value == 3 * 16 * 64 * 4 + 16 * 512 * 4 + 256
    assert lib.cp_pct_order_workspace_bytes(g._handle, 16, 2, -1, C.byref(need)) == -12
    assert lib.cp_pct_order_workspace_bytes(g._handle, 0, 2, 0, C.byref(need)) == -2
    assert lib.cp_pct_order_workspace_bytes(g._handle, 16, 2, 0, None) == -1
    # 62 bits of b plus 8 device bits do not fit one 64-bit key
    assert lib.cp_pct_order_workspace_bytes(g._handle, 16, 255, 2**62, C.byref(need)) == -8
    # a bound past 32 bits: 64-bit keys
    assert lib.cp_pct_order_workspace_bytes(g._handle, 16, 2, 2**40, C.byref(need)) == 0
    assert need.value == 2 * 16 * 64 * 8 + 16 * 64 * 4 + 16 * 512 * 4 + 256

    def order(batch=4, k=2, assign=dummy, layout=0, b=dummy, tick=4, b_layout=0, max_b=0, ws=dummy, out=dummy):
        return lib.cp_pct_order(g._handle, batch, k, assign, layout, b, tick, b_layout, max_b, ws, 1 << 20, None,
                                out, dummy, dummy)

    assert order(batch=0) == -2
    assert order(b_layout=5) == -12
    assert order(max_b=-3) == -12
    assert order(out=C.c_void_p()) == -1
    assert order() == -11

    assert lib.cp_ranks_workspace_bytes(g._handle, C.byref(need)) == 0 and need.value > 0
    assert lib.cp_ranks(g._handle, dummy, 1 << 20, None, None, None, None) == -1
    assert lib.cp_ranks(g._handle, dummy, 1 << 20, None, dummy, dummy, dummy) == -11
    plan = C.c_int(0)
    assert lib.cp_eval_choose_plan(g._handle, 16, 2, sp, bp, 4, C.byref(plan)) == 0
    assert plan.value in (cpe.PLAN_WAVE_COLUMN, cpe.PLAN_RESIDENT_WINDOW)
    assert lib.cp_eval_choose_plan(g._handle, 16, 2, sp, bp, 3, C.byref(plan)) == -12
    g.close()


def test_simulate_checks_its_arguments(lib):
    """cp_simulate rejects bad arguments before touching the GPU."""
    w = make_workload("tiny")
    g = cpe.CpGraph.from_workload(w)
    s = np.array([1, 2], dtype=np.int64)
    B = np.array([[1, 10], [10, 1]], dtype=np.int64)
    dummy = C.c_void_p(256)
    null = C.c_void_p()
    i64p = C.POINTER(C.c_int64)
    sp, bp = s.ctypes.data_as(i64p), B.ctypes.data_as(i64p)
    n = w.n
    need = C.c_size_t(0)
    assert lib.cp_simulate_workspace_bytes(g._handle, 16, 2, 1, 0, C.byref(need)) == 0
    per_i32 = -(-16 * n * 4 // 256) * 256
    per_u64 = -(-16 * n * 8 // 256) * 256
    tab = -(-(2 * 2 * 2 + 2) * 8 // 256) * 256
    assert need.value == tab + 3 * per_i32 + 2 * per_u64            # PCT: two heaps
    assert lib.cp_simulate_workspace_bytes(g._handle, 16, 2, 0, 1, C.byref(need)) == 0
    assert need.value == tab + -(-n * 4 // 256) * 256 + 3 * per_i32 + per_u64   # FIFO with tie ranks
    assert lib.cp_simulate_workspace_bytes(g._handle, 16, 65, 0, 0, C.byref(need)) == -2
    assert lib.cp_simulate_workspace_bytes(g._handle, 0, 2, 0, 0, C.byref(need)) == -2
    assert lib.cp_simulate_workspace_bytes(g._handle, 16, 2, 2, 0, C.byref(need)) == -12
    assert lib.cp_simulate_workspace_bytes(g._handle, 16, 2, 0, 0, None) == -1

    def sim(batch=4, k=2, assign=dummy, layout=0, policy=1, b=dummy, tick=4, b_layout=0, tie=null, ws=dummy,
            out=dummy, status=dummy):
        return lib.cp_simulate(g._handle, batch, k, assign, layout, sp, bp, policy, b, tick, b_layout, tie, ws,
                               1 << 24, None, out, null, status)

    assert sim(batch=0) == -2
    assert sim(k=65) == -2
    assert sim(policy=7) == -12
    assert sim(layout=2) == -12
    assert sim(b=null) == -1                 # PCT needs b
    assert sim(b_layout=3) == -12
    assert sim(tick=5) == -12
    assert sim(out=null) == -1
    assert sim(policy=0, b=null) == -11      # FIFO needs no b; the graph is not uploaded
    assert sim() == -11
    g.close()


def test_packing_deep_graphs_with_long_spans(lib):
    """Deep graphs whose edges span the whole depth are packed for the resident-window plan
    with far reads: a short ring plus a bounded number of far reads per tick."""
    from workloads import random_layered_dag
    from workloads.dags import _finish
    for seed in range(3):
        rng = np.random.default_rng(9500 + seed)
        depth = int(rng.integers(250, 600))
        widths = rng.integers(20, 110, size=depth)
        n, level, src, dst = random_layered_dag(rng, widths, 1, 3, depth - 1)
        csr = build_csr(n, src, dst, rng.integers(0, 3000, size=len(src)), level)
        w = _finish(f"deep-{seed}", csr, rng.integers(1, 400, size=n), 2, [1, 2], [[1, 3], [3, 1]],
                    np.zeros((1, n), dtype=np.uint8))
        g = cpe.CpGraph.from_workload(w)
        info = g.info
        assert info["window_ok"] == 1
        assert 0 < info["window_far_b"] <= 256 and info["window_far_b"] % 64 == 0
        assert 0 < info["window_far_t"] <= 256
        assert info["window_slots_b"] < n // 2 and info["window_slots_t"] < n // 2
        g.close()
    # without long edges nothing is a far read
    w = make_workload("large_sparse", P=1, levels=100, width=80)
    g = cpe.CpGraph.from_workload(w)
    assert g.info["window_far_b"] == 0 and g.info["window_far_t"] == 0
    g.close()


def test_window_ring_holds_the_widest_tick():
    """Vertices without edges still take ring slots when they are published: the ring is never
    shorter than the widest tick, whatever the edges' spans."""
    import paper_1711_01912_amd as cpe
    from workloads import build_csr
    from workloads.dags import _finish
    for width in (70, 279, 600):
        n = 6 + width                      # a chain of six and a level of `width` vertices without edges
        src, dst = np.arange(5), np.arange(1, 6)
        level = np.concatenate([np.arange(6), np.full(width, 6)])
        w = _finish("wide-level", build_csr(n, src, dst, np.ones(5, dtype=np.int64), level), np.ones(n, dtype=np.int64),
                    2, [1, 1], [[1, 1], [1, 1]], np.zeros((1, n), dtype=np.uint8))
        g = cpe.CpGraph.from_workload(w)
        info = g.info
        g.close()
        assert info["window_ok"] == 1
        assert min(info["window_slots_b"], info["window_slots_t"]) >= min(width, 512), info

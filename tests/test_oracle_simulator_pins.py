"""Pins for the oracle's list-scheduling simulation: a schedule worked by hand, a
tick-by-tick brute force, a checker that verifies a finished schedule against the
paper's scheduling criteria, closed forms and bounds.  Nothing here calls the GPU
path and no expected value comes from it."""
import os

import numpy as np
import pytest

from oracle import brute_force
from workloads import build_csr, make_workload, random_layered_dag

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
FIFO, PCT = 0, 1


def _edges(csr):
    n = csr["n"]
    src = np.repeat(np.arange(n), np.diff(csr["succ_ptr"]))
    return [(int(u), int(v), int(t)) for u, v, t in zip(src, csr["succ_idx"], csr["succ_t"])]


def _sim(oracle, csr, c, s, B, a, policy, b=None, tie=None):
    a = np.atleast_2d(np.asarray(a, dtype=np.uint8))
    return oracle.simulate(csr["n"], csr["succ_ptr"], csr["succ_idx"], csr["succ_t"], c, s, B, a, policy,
                           b=b, tie=tie)


def _b(oracle, csr, c, s, B, a):
    a = np.atleast_2d(np.asarray(a, dtype=np.uint8))
    return oracle.evaluate(csr["n"], csr["succ_ptr"], csr["succ_idx"], csr["succ_t"], c, s, B, a,
                           want=("cp", "b", "tl"))


def _dag(seed, layers, width, deg_hi=3, span_hi=2, tmax=100, cmax=100):
    rng = np.random.default_rng(seed)
    n, level, src, dst = random_layered_dag(rng, [width] * layers, 1, deg_hi, span_hi)
    t = rng.integers(0, tmax + 1, size=len(src))
    c = rng.integers(1, cmax + 1, size=n)
    return build_csr(n, src, dst, t, level), c, rng


def _devices(rng, k, s_hi=100, b_hi=60):
    s = rng.integers(1, s_hi + 1, size=k)
    B = rng.integers(1, b_hi + 1, size=(k, k))
    return s, B


# ----------------------------------------------------------------- worked by hand

def _worked_example():
    rows = {}
    edges = []
    with open(os.path.join(GOLDEN, "list_schedule_worked_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            if key == "edge":
                edges.append(tuple(int(x) for x in vals))
            else:
                rows[key] = [int(x) for x in vals]
    return rows, edges


def test_worked_example(oracle):
    rows, edges = _worked_example()
    n, k = rows["n"][0], rows["k"][0]
    src = [e[0] for e in edges]
    dst = [e[1] for e in edges]
    t = [e[2] for e in edges]
    csr = build_csr(n, np.array(src), np.array(dst), np.array(t))
    s = np.array(rows["speeds"])
    B = np.full((k, k), rows["rate"][0])
    a = np.array(rows["device"], dtype=np.uint8)
    c = np.array(rows["c"])
    b = _b(oracle, csr, c, s, B, a)["b"]
    assert b[0].tolist() == [8, 11, 6, 4, 6, 2]          # the b values the hand schedule uses
    got = _sim(oracle, csr, c, s, B, a, PCT, b=b)
    assert got["start"][0].tolist() == rows["pct_start"]
    assert got["makespan"][0] == rows["pct_makespan"][0]
    got = _sim(oracle, csr, c, s, B, a, FIFO)
    assert got["start"][0].tolist() == rows["fifo_start"]
    assert got["makespan"][0] == rows["fifo_makespan"][0]
    got = _sim(oracle, csr, c, s, B, a, FIFO, tie=np.arange(n)[::-1])
    assert got["start"][0].tolist() == rows["fifo_reversed_start"]
    assert got["makespan"][0] == rows["fifo_reversed_makespan"][0]


# ----------------------------------------------------------------- tick-by-tick brute force

@pytest.mark.parametrize("seed", range(40))
def test_against_tick_by_tick_brute_force(oracle, seed):
    layers, width = [(3, 2), (4, 3), (5, 3), (3, 5)][seed % 4]
    csr, c, rng = _dag(100 + seed, layers, width, deg_hi=3, span_hi=3, tmax=40, cmax=30)
    n = csr["n"]
    k = [1, 2, 3, 5][(seed // 4) % 4]
    s, B = _devices(rng, k, s_hi=6, b_hi=8)
    a = rng.integers(0, k, size=n).astype(np.uint8)
    edges = _edges(csr)
    b = _b(oracle, csr, c, s, B, a)["b"]
    # ties with repeated values, so that the last tie-break (the vertex number) is used too
    tie = rng.integers(0, 3, size=n).astype(np.int32)
    want_m, want_s = brute_force.list_schedule_by_ticks(n, edges, c, s, B, a, "pct", b=b[0])
    got = _sim(oracle, csr, c, s, B, a, PCT, b=b)
    assert got["start"][0].tolist() == want_s and got["makespan"][0] == want_m
    for tt in (None, tie):
        want_m, want_s = brute_force.list_schedule_by_ticks(n, edges, c, s, B, a, "fifo", tie=tt)
        got = _sim(oracle, csr, c, s, B, a, FIFO, tie=tt)
        assert got["start"][0].tolist() == want_s and got["makespan"][0] == want_m


# ----------------------------------------------------------------- checker of a finished schedule

def check_schedule(csr, c, s, B, a, start, policy, b=None, tie=None):
    """Verify a finished schedule against the scheduling criteria of section 4 and the
    policy, from the start times alone.  Raises AssertionError with the reason."""
    n = csr["n"]
    a = np.asarray(a)
    start = np.asarray(start, dtype=np.int64)
    assert (start >= 0).all(), "criterion (1): every vertex runs"
    w = -(-np.asarray(c, dtype=np.int64) // np.asarray(s, dtype=np.int64)[a])
    finish = start + w
    src = np.repeat(np.arange(n), np.diff(csr["succ_ptr"]))
    dst = np.asarray(csr["succ_idx"])
    t = np.asarray(csr["succ_t"], dtype=np.int64)
    rate = np.asarray(B, dtype=np.int64)[a[src], a[dst]]
    x = np.where(a[src] == a[dst], 0, -(-t // rate))
    ready = np.zeros(n, dtype=np.int64)
    np.maximum.at(ready, dst, finish[src] + x)
    assert (start >= ready).all(), "criterion (4): inputs computed and transferred"
    for d in range(len(s)):
        mine = np.flatnonzero(a == d)
        mine = mine[np.argsort(start[mine], kind="stable")]
        free = 0
        todo = set(mine.tolist())
        for v in mine:
            now = start[v]
            assert now >= free, "criteria (2), (3): one vertex at a time, no interruption"
            first = min(ready[u] for u in todo)
            assert now == max(free, first), "criterion (6): idle only while nothing is executable"
            able = [u for u in todo if ready[u] <= now]
            if policy == PCT:
                best = min(able, key=lambda u: (-b[u], u))
            else:
                best = min(able, key=lambda u: (ready[u], u if tie is None else tie[u], u))
            assert best == v, "policy: another executable vertex had precedence"
            todo.remove(v)
            free = finish[v]
    return int(finish.max())


@pytest.mark.parametrize("seed,layers,width,k", [(1, 12, 8, 4), (2, 30, 10, 8), (3, 8, 60, 16), (4, 50, 4, 50),
                                                 (5, 20, 20, 3)])
def test_schedules_satisfy_the_criteria(oracle, seed, layers, width, k):
    csr, c, rng = _dag(seed, layers, width, deg_hi=4, span_hi=4)
    n = csr["n"]
    s = rng.integers(10, 101, size=k)
    B = rng.integers(10, 61, size=(k, k))
    P = 3
    a = rng.integers(0, k, size=(P, n)).astype(np.uint8)
    ev = _b(oracle, csr, c, s, B, a)
    tie = rng.permutation(n).astype(np.int32)
    pct = _sim(oracle, csr, c, s, B, a, PCT, b=ev["b"])
    fifo = _sim(oracle, csr, c, s, B, a, FIFO, tie=tie)
    for j in range(P):
        assert check_schedule(csr, c, s, B, a[j], pct["start"][j], PCT, b=ev["b"][j]) == pct["makespan"][j]
        assert check_schedule(csr, c, s, B, a[j], fifo["start"][j], FIFO, tie=tie) == fifo["makespan"][j]
        for got in (pct, fifo):
            w = -(-c // s[a[j]])
            load = np.bincount(a[j], weights=w, minlength=k).max()
            assert got["makespan"][j] >= ev["cp"][j]          # no schedule beats the critical path
            assert got["makespan"][j] >= load                 # nor the busiest device's work


def test_checker_rejects_wrong_schedules(oracle):
    """The checker itself must notice a late start, an overlap and a wrong choice."""
    csr, c, rng = _dag(9, 10, 6)
    n, k = csr["n"], 3
    s, B = _devices(rng, k)
    a = rng.integers(0, k, size=n).astype(np.uint8)
    b = _b(oracle, csr, c, s, B, a)["b"]
    good = _sim(oracle, csr, c, s, B, a, PCT, b=b)["start"][0]
    check_schedule(csr, c, s, B, a, good, PCT, b=b[0])
    late = good.copy()
    late[int(np.argmax(good))] += 1
    with pytest.raises(AssertionError):
        check_schedule(csr, c, s, B, a, late, PCT, b=b[0])
    early = good.copy()
    early[int(np.argmax(good))] -= 1
    with pytest.raises(AssertionError):
        check_schedule(csr, c, s, B, a, early, PCT, b=b[0])
    with pytest.raises(AssertionError):                     # a FIFO schedule is not a PCT schedule here
        fifo = _sim(oracle, csr, c, s, B, a, FIFO)["start"][0]
        assert not np.array_equal(fifo, good)
        check_schedule(csr, c, s, B, a, fifo, PCT, b=b[0])


# ----------------------------------------------------------------- closed forms and symmetries

def test_one_device_runs_everything_back_to_back(oracle):
    csr, c, rng = _dag(11, 9, 7)
    n = csr["n"]
    s = np.array([7])
    B = np.array([[1]])
    a = np.zeros(n, dtype=np.uint8)
    b = _b(oracle, csr, c, s, B, a)["b"]
    for policy in (FIFO, PCT):
        got = _sim(oracle, csr, c, s, B, a, policy, b=b)
        assert got["makespan"][0] == int((-(-c // 7)).sum())


def test_a_device_per_vertex_runs_at_the_critical_path(oracle):
    """Without contention every vertex starts as soon as its inputs are there: start = tl
    and the makespan is the critical-path time (section 4.1's rationale)."""
    csr, c, rng = _dag(12, 6, 5, deg_hi=3, span_hi=3)
    n = csr["n"]
    assert n <= 64
    s = rng.integers(1, 20, size=n)
    B = rng.integers(1, 20, size=(n, n))
    a = rng.permutation(n).astype(np.uint8)
    ev = _b(oracle, csr, c, s, B, a)
    for policy in (FIFO, PCT):
        got = _sim(oracle, csr, c, s, B, a, policy, b=ev["b"])
        assert np.array_equal(got["start"][0], ev["tl"][0])
        assert got["makespan"][0] == ev["cp"][0]


def test_a_chain_runs_at_the_critical_path(oracle):
    n = 40
    rng = np.random.default_rng(13)
    csr = build_csr(n, np.arange(n - 1), np.arange(1, n), rng.integers(0, 50, size=n - 1))
    c = rng.integers(1, 50, size=n)
    s, B = _devices(rng, 4)
    a = rng.integers(0, 4, size=(5, n)).astype(np.uint8)
    ev = _b(oracle, csr, c, s, B, a)
    for policy in (FIFO, PCT):
        got = _sim(oracle, csr, c, s, B, a, policy, b=ev["b"])
        assert np.array_equal(got["makespan"], ev["cp"])
        assert np.array_equal(got["start"], ev["tl"])


def test_independent_vertices_fill_devices_in_priority_order(oracle):
    """No edges, one device: PCT runs the vertices by descending b = w, FIFO by tie."""
    n = 12
    rng = np.random.default_rng(14)
    csr = build_csr(n, np.array([], dtype=np.int64), np.array([], dtype=np.int64), np.array([], dtype=np.int64))
    c = rng.permutation(n) + 1
    s = np.array([1])
    B = np.array([[1]])
    a = np.zeros(n, dtype=np.uint8)
    b = c[None, :].astype(np.int64)
    got = _sim(oracle, csr, c, s, B, a, PCT, b=b)["start"][0]
    order = np.argsort(got)
    assert c[order].tolist() == sorted(c.tolist(), reverse=True)
    tie = rng.permutation(n).astype(np.int32)
    got = _sim(oracle, csr, c, s, B, a, FIFO, tie=tie)["start"][0]
    assert tie[np.argsort(got)].tolist() == list(range(n))


def test_unit_rates_scale_with_the_weights(oracle):
    csr, c, rng = _dag(15, 8, 6)
    n, k = csr["n"], 3
    s = np.ones(k, dtype=np.int64)
    B = np.ones((k, k), dtype=np.int64)
    a = rng.integers(0, k, size=(2, n)).astype(np.uint8)
    b = _b(oracle, csr, c, s, B, a)["b"]
    base = _sim(oracle, csr, c, s, B, a, PCT, b=b)
    big = dict(csr)
    big["succ_t"] = np.asarray(csr["succ_t"]) * 7
    scaled = _sim(oracle, big, c * 7, s, B, a, PCT, b=b * 7)
    assert np.array_equal(scaled["start"], base["start"] * 7)
    assert np.array_equal(scaled["makespan"], base["makespan"] * 7)


def test_relabelling_devices_changes_nothing(oracle):
    csr, c, rng = _dag(16, 10, 6)
    n, k = csr["n"], 4
    s, B = _devices(rng, k)
    a = rng.integers(0, k, size=n).astype(np.uint8)
    perm = rng.permutation(k)
    inv = np.argsort(perm)
    a2 = perm[a].astype(np.uint8)
    s2, B2 = s[inv], B[np.ix_(inv, inv)]
    b = _b(oracle, csr, c, s, B, a)["b"]
    for policy in (FIFO, PCT):
        one = _sim(oracle, csr, c, s, B, a, policy, b=b)
        two = _sim(oracle, csr, c, s2, B2, a2, policy, b=b)
        assert np.array_equal(one["start"], two["start"])


def test_zero_cost_vertices_are_refused(oracle):
    csr, c, rng = _dag(17, 4, 3)
    c = c.copy()
    c[2] = 0
    s, B = _devices(rng, 2)
    a = np.zeros(csr["n"], dtype=np.uint8)
    with pytest.raises(ValueError):
        _sim(oracle, csr, c, s, B, a, FIFO)


def test_paper_like_workload_orders_the_strategies(oracle):
    """On the paper-sized synthetic graph PCT is never behind the critical-path bound and the
    makespan is within the trivial upper bound (everything in sequence)."""
    wl = make_workload("tiny")
    csr = {"n": wl.n, "succ_ptr": wl.succ_ptr, "succ_idx": wl.succ_idx, "succ_t": wl.succ_t}
    c = np.maximum(wl.c, 1)
    ev = _b(oracle, csr, c, wl.speeds, wl.bandwidth, wl.assignments)
    got = _sim(oracle, csr, c, wl.speeds, wl.bandwidth, wl.assignments, PCT, b=ev["b"])
    assert (got["makespan"] >= ev["cp"]).all()
    a = wl.assignments
    w = -(-c[None, :] // wl.speeds[a])
    assert (got["makespan"] <= w.sum(axis=1) + ev["cp"]).all()


@pytest.mark.parametrize("seed", range(6))
def test_makespan_never_exceeds_busy_time_plus_the_longest_transfer_chain(oracle, seed):
    """At any moment before the end some device is busy, or all of them wait for a transfer on one
    chain of dependent vertices: makespan <= sum of w + the largest sum of x along a path."""
    csr, c, rng = _dag(200 + seed, 12, 9, deg_hi=4, span_hi=4, tmax=5000, cmax=20)
    n, k = csr["n"], 5
    s = rng.integers(1, 4, size=k)
    B = rng.integers(1, 6, size=(k, k))
    a = rng.integers(0, k, size=(4, n)).astype(np.uint8)
    ev = _b(oracle, csr, c, s, B, a)
    chain = oracle.evaluate(n, csr["succ_ptr"], csr["succ_idx"], csr["succ_t"], np.zeros(n, dtype=np.int64), s, B, a,
                            want=("cp",))["cp"]
    busy = (-(-c[None, :] // s[a])).sum(axis=1)
    for policy in (FIFO, PCT):
        got = _sim(oracle, csr, c, s, B, a, policy, b=ev["b"])["makespan"]
        assert (got <= busy + chain).all()
        assert (got >= ev["cp"]).all()

"""Pins for the CPU oracle: values the paper prints, brute force, closed forms,
a library shortest-path routine, invariants, symmetries.  None of these calls
the GPU path, and no expected value comes from it."""
import itertools
import os
from fractions import Fraction
from math import ceil

import numpy as np
import pytest

from oracle import brute_force
from workloads import build_csr, make_workload, random_layered_dag

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def _edges(csr):
    n = csr["n"]
    src = np.repeat(np.arange(n), np.diff(csr["succ_ptr"]))
    return [(int(u), int(v), int(t)) for u, v, t in zip(src, csr["succ_idx"], csr["succ_t"])]


def _eval(oracle, csr, c, s, B, a, **kw):
    return oracle.evaluate(csr["n"], csr["succ_ptr"], csr["succ_idx"], csr["succ_t"], c, s, B,
                           np.atleast_2d(np.asarray(a, dtype=np.uint8)), **kw)


def _small_dag(seed, layers=4, width=3, deg_hi=3, span_hi=2, tmax=1000, cmax=100):
    rng = np.random.default_rng(seed)
    n, level, src, dst = random_layered_dag(rng, [width] * layers, 1, deg_hi, span_hi)
    t = rng.integers(0, tmax + 1, size=len(src))
    c = rng.integers(0, cmax + 1, size=n)
    return build_csr(n, src, dst, t, level), c, rng


# ----------------------------------------------------------------- single terms

def test_vertex_cost_paper_example(oracle):
    for c, s, want in _read_table("vertex_cost_example.txt"):
        assert oracle.vertex_cost(int(c), int(s)) == int(want)


@pytest.mark.parametrize("c,s,want", [(10, 3, 4), (0, 5, 0), (1, 16, 1), (16, 16, 1), (17, 16, 2),
                                      (999, 1, 999), (10**12 + 1, 10**6, 10**6 + 1)])
def test_vertex_cost_rounds_up(oracle, c, s, want):
    assert oracle.vertex_cost(c, s) == want


def test_edge_cost_terms(oracle):
    B = np.array([[7, 10, 3], [20, 7, 4], [5, 6, 7]])
    # same device: free, whatever the volume and the diagonal say
    for d in range(3):
        assert oracle.edge_cost(10**9, d, d, B) == 0
    assert oracle.edge_cost(1000, 0, 1, B) == 100      # row = source vertex's device
    assert oracle.edge_cost(1000, 1, 0, B) == 50       # asymmetric: the other direction differs
    assert oracle.edge_cost(1000, 0, 2, B) == 334
    assert oracle.edge_cost(1000, 2, 0, B) == 200
    assert oracle.edge_cost(0, 0, 1, B) == 0
    assert oracle.edge_cost(1, 1, 2, B) == 1


def test_terms_against_exact_rationals(oracle):
    rng = np.random.default_rng(5)
    for _ in range(300):
        a = int(rng.integers(0, 10**9))
        d = int(rng.integers(1, 10**5))
        assert oracle.vertex_cost(a, d) == ceil(Fraction(a, d))


# ----------------------------------------------------------------- brute force

@pytest.mark.parametrize("seed", range(6))
def test_brute_force_all_partitions_two_devices(oracle, seed):
    """n = 8, k = 2: every one of the 2^8 partitions, every output."""
    csr, c, rng = _small_dag(seed, layers=4, width=2, deg_hi=2)
    n = csr["n"]
    s = np.array([1, 3])
    B = np.array([[1, 7], [13, 1]])  # asymmetric on purpose
    parts = np.array(list(itertools.product([0, 1], repeat=n)), dtype=np.uint8)
    got = _eval(oracle, csr, c, s, B, parts)
    edges = _edges(csr)
    for j, p in enumerate(parts):
        cp, b, tl = brute_force.evaluate(n, edges, c, s, B, p)
        assert got["cp"][j] == cp
        assert got["b"][j].tolist() == b
        assert got["tl"][j].tolist() == tl
        assert got["mask"][j].tolist() == [tl[v] + b[v] == cp for v in range(n)]


@pytest.mark.parametrize("seed", range(8))
def test_brute_force_random_partitions(oracle, seed):
    csr, c, rng = _small_dag(100 + seed, layers=5, width=3, deg_hi=3, span_hi=3)
    n = csr["n"]
    k = 3
    s = rng.integers(1, 9, size=k)
    B = rng.integers(1, 40, size=(k, k))
    parts = rng.integers(0, k, size=(12, n), dtype=np.uint8)
    got = _eval(oracle, csr, c, s, B, parts)
    edges = _edges(csr)
    for j, p in enumerate(parts):
        cp, b, tl = brute_force.evaluate(n, edges, c, s, B, p)
        assert got["cp"][j] == cp
        assert got["b"][j].tolist() == b
        assert got["tl"][j].tolist() == tl


def test_brute_force_multi_edges(oracle):
    """Parallel edges u->v with different volumes: the costlier one decides."""
    src, dst, t = [0, 0, 0, 1, 1], [1, 1, 2, 2, 2], [10, 500, 30, 5, 900]
    csr = build_csr(3, src, dst, t)
    c = np.array([4, 0, 9])
    s = np.array([1, 2])
    B = np.array([[1, 10], [3, 1]])
    parts = np.array(list(itertools.product([0, 1], repeat=3)), dtype=np.uint8)
    got = _eval(oracle, csr, c, s, B, parts)
    for j, p in enumerate(parts):
        cp, b, tl = brute_force.evaluate(3, list(zip(src, dst, t)), c, s, B, p)
        assert (got["cp"][j], got["b"][j].tolist(), got["tl"][j].tolist()) == (cp, b, tl)


def test_brute_force_tiny_workload(oracle):
    w = make_workload("tiny")
    got = oracle.evaluate_workload(w, partitions=[0, 7])
    edges = _edges(dict(n=w.n, succ_ptr=w.succ_ptr, succ_idx=w.succ_idx, succ_t=w.succ_t))
    for row, j in enumerate([0, 7]):
        cp, b, tl = brute_force.evaluate(w.n, edges, w.c, w.speeds, w.bandwidth, w.assignments[j])
        assert got["cp"][row] == cp
        assert got["b"][row].tolist() == b
        assert got["tl"][row].tolist() == tl


# ----------------------------------------------------------------- closed forms

def _chain(n, t):
    return build_csr(n, list(range(n - 1)), list(range(1, n)), t)


def test_chain_one_device_is_sum_of_costs(oracle):
    rng = np.random.default_rng(1)
    n = 40
    c = rng.integers(0, 100, size=n)
    csr = _chain(n, rng.integers(0, 1000, size=n - 1))
    s = np.array([7, 3])
    B = np.array([[1, 2], [2, 1]])
    got = _eval(oracle, csr, c, s, B, [[1] * n])
    w = [ceil(Fraction(int(ci), 3)) for ci in c]
    assert got["cp"][0] == sum(w)
    assert got["b"][0].tolist() == [sum(w[i:]) for i in range(n)]
    assert got["tl"][0].tolist() == [sum(w[:i]) for i in range(n)]
    assert got["mask"][0].all()


def test_chain_alternating_devices_adds_every_transfer(oracle):
    rng = np.random.default_rng(2)
    n = 31
    c = rng.integers(1, 100, size=n)
    t = rng.integers(1, 1000, size=n - 1)
    csr = _chain(n, t)
    s = np.array([2, 5])
    B = np.array([[99, 4], [9, 99]])
    p = [i % 2 for i in range(n)]
    got = _eval(oracle, csr, c, s, B, [p])
    w = [ceil(Fraction(int(c[i]), int(s[p[i]]))) for i in range(n)]
    x = [ceil(Fraction(int(t[i]), int(B[p[i]][p[i + 1]]))) for i in range(n - 1)]
    assert got["cp"][0] == sum(w) + sum(x)
    assert got["b"][0][0] == sum(w) + sum(x)
    assert got["tl"][0][n - 1] == sum(w[:-1]) + sum(x)
    assert got["b"][0][n - 1] == w[-1]


def test_antichain_is_max_single_vertex(oracle):
    n = 17
    c = np.arange(3, 3 + n) * 5 % 37
    csr = build_csr(n, [], [], [])
    s = np.array([2, 3])
    B = np.array([[1, 1], [1, 1]])
    p = np.array([i % 2 for i in range(n)], dtype=np.uint8)
    got = _eval(oracle, csr, c, s, B, [p])
    w = np.array([ceil(Fraction(int(c[i]), int(s[p[i]]))) for i in range(n)])
    assert got["cp"][0] == w.max()
    assert (got["b"][0] == w).all()
    assert (got["tl"][0] == 0).all()
    assert (got["mask"][0] == (w == w.max())).all()


def test_fork_join_takes_longer_arm(oracle):
    # 0 -> 1 -> 2 -> 5 and 0 -> 3 -> 4 -> 5
    src, dst = [0, 1, 2, 0, 3, 4], [1, 2, 5, 3, 4, 5]
    t = [10, 10, 10, 10, 10, 10]
    c = np.array([5, 20, 20, 30, 30, 5])
    csr = build_csr(6, src, dst, t)
    s = np.array([1])
    B = np.array([[1]])
    got = _eval(oracle, csr, c, s, B, [[0] * 6])
    assert got["cp"][0] == 5 + 30 + 30 + 5
    assert got["mask"][0].tolist() == [True, False, False, True, True, True]
    assert got["tl"][0].tolist() == [0, 5, 25, 5, 35, 65]
    assert got["b"][0].tolist() == [70, 45, 25, 65, 35, 5]


def test_hand_worked_two_device_example(oracle):
    """Diamond 0->{1,2}->3, hand-computed.  s = (1, 4); B[0][1] = 10, B[1][0] = 2.
    p = (0, 1, 0, 1):  w = (8, ceil(10/4)=3, 6, ceil(7/4)=2)
    x(0->1) = ceil(25/10) = 3, x(0->2) = 0, x(1->3) = 0, x(2->3) = ceil(95/10) = 10
    b(3)=2, b(1)=3+0+2=5, b(2)=6+10+2=18, b(0)=8+max(3+5, 0+18)=26
    tl(0)=0, tl(1)=8+3=11, tl(2)=8, tl(3)=max(11+3+0, 8+6+10)=24."""
    csr = build_csr(4, [0, 0, 1, 2], [1, 2, 3, 3], [25, 40, 1000, 95])
    c = np.array([8, 10, 6, 7])
    got = _eval(oracle, csr, c, np.array([1, 4]), np.array([[1, 10], [2, 1]]), [[0, 1, 0, 1]])
    assert got["b"][0].tolist() == [26, 5, 18, 2]
    assert got["tl"][0].tolist() == [0, 11, 8, 24]
    assert got["cp"][0] == 26
    assert got["mask"][0].tolist() == [True, False, True, True]


# ----------------------------------------------------------------- library routine

def test_against_library_shortest_path(oracle):
    """Weights are kept >= 1 so that no explicit zero sits in the sparse matrix."""
    rng = np.random.default_rng(11)
    n, level, src, dst = random_layered_dag(rng, [12] * 15, 1, 4, 4)
    t = rng.integers(1, 5000, size=len(src))
    c = rng.integers(1, 500, size=n)
    csr = build_csr(n, src, dst, t, level)
    k = 4
    s = rng.integers(1, 9, size=k)
    B = rng.integers(1, 64, size=(k, k))
    parts = rng.integers(0, k, size=(3, n), dtype=np.uint8)
    got = _eval(oracle, csr, c, s, B, parts)
    from scipy.sparse import csr_matrix
    from scipy.sparse.csgraph import bellman_ford
    for j, p in enumerate(parts):
        w = np.array([ceil(Fraction(int(c[v]), int(s[p[v]]))) for v in range(n)], dtype=np.int64)
        es = np.repeat(np.arange(n), np.diff(csr["succ_ptr"]))
        ed = csr["succ_idx"].astype(np.int64)
        x = np.array([0 if p[u] == p[v] else ceil(Fraction(int(tt), int(B[p[u]][p[v]])))
                      for u, v, tt in zip(es, ed, csr["succ_t"])], dtype=np.int64)
        T = n
        # forward: edge u->v weighs w(u)+x; v->T weighs w(v): longest v->T is b(v)
        g = csr_matrix((-np.concatenate([w[es] + x, w]).astype(float),
                        (np.concatenate([es, np.arange(n)]), np.concatenate([ed, np.full(n, T)]))),
                       shape=(n + 1, n + 1))
        b = -bellman_ford(g, directed=True, indices=np.arange(n))[:, T]
        assert (got["b"][j] == b.astype(np.int64)).all()
        # reversed: edge v->u weighs w(v)+x(u,v); u->T weighs w(u): longest v->T is tl(v)+w(v)
        gr = csr_matrix((-np.concatenate([w[ed] + x, w]).astype(float),
                         (np.concatenate([ed, np.arange(n)]), np.concatenate([es, np.full(n, T)]))),
                        shape=(n + 1, n + 1))
        f = -bellman_ford(gr, directed=True, indices=np.arange(n))[:, T]
        assert (got["tl"][j] == f.astype(np.int64) - w).all()
        assert got["cp"][j] == int(b.max())


def test_one_unit_speed_device_gives_the_papers_ranks(oracle):
    """k = 1, s = 1: b is the upward rank and tl + c the downward rank of
    section 3.2 (longest summed complexity), checked against networkx on the
    vertex-split graph."""
    nx = pytest.importorskip("networkx")
    rng = np.random.default_rng(3)
    n, level, src, dst = random_layered_dag(rng, [6] * 10, 1, 3, 3)
    c = rng.integers(1, 100, size=n)
    csr = build_csr(n, src, dst, rng.integers(1, 10**6, size=len(src)), level)
    got = _eval(oracle, csr, c, np.array([1]), np.array([[1]]), [[0] * n])
    g = nx.DiGraph()
    for v in range(n):
        g.add_edge(("in", v), ("out", v), weight=int(c[v]))
    for u, v in zip(src, dst):
        g.add_edge(("out", int(u)), ("in", int(v)), weight=0)
    assert got["cp"][0] == nx.dag_longest_path_length(g, weight="weight")
    order = list(nx.topological_sort(g))
    up = {}
    for node in reversed(order):
        best = 0
        for _, nb, d in g.out_edges(node, data=True):
            best = max(best, d["weight"] + up[nb])
        up[node] = best
    assert got["b"][0].tolist() == [up[("in", v)] for v in range(n)]


def test_unit_cost_graph_counts_the_longest_chain(oracle):
    """c = 1, s = 1, one device (the reduction's instance in the NP-completeness
    proof): CP is the number of vertices on the longest chain, i.e. the number of
    levels of the longest-path layering."""
    rng = np.random.default_rng(4)
    n, level, src, dst = random_layered_dag(rng, [5] * 9, 1, 2, 3)
    csr = build_csr(n, src, dst, np.zeros(len(src), dtype=np.int64))  # ASAP levels
    got = _eval(oracle, csr, np.ones(n, dtype=np.int64), np.array([1]), np.array([[1]]), [[0] * n])
    assert got["cp"][0] == csr["L"]
    assert (got["tl"][0] == csr["level"]).all()


# ----------------------------------------------------------------- invariants

def _check_invariants(w, out, parts):
    n = w.n
    src = np.repeat(np.arange(n), np.diff(w.succ_ptr))
    dst = w.succ_idx
    outdeg = np.diff(w.succ_ptr)
    indeg = np.diff(w.pred_ptr)
    for row, j in enumerate(parts):
        p = w.assignments[j].astype(np.int64)
        wv = -(-w.c // w.speeds[p])
        xe = np.where(p[src] == p[dst], 0, -(-w.succ_t // w.bandwidth[p[src], p[dst]]))
        b, tl, cp, mask = out["b"][row], out["tl"][row], out["cp"][row], out["mask"][row]
        assert (b >= 0).all() and (tl >= 0).all()
        assert b.max() == cp == (tl + wv).max() == (tl + b).max()
        assert (tl + b <= cp).all()
        assert cp >= wv.max()
        assert cp <= wv.sum() + xe.sum()
        assert mask.any()
        assert (mask == (tl + b == cp)).all()
        assert (mask & (indeg == 0)).any() and (mask & (outdeg == 0)).any()
        # every edge respects both recurrences as inequalities ...
        assert (b[src] >= wv[src] + xe + b[dst]).all()
        assert (tl[dst] >= tl[src] + wv[src] + xe).all()
        # ... and every masked non-sink has a masked successor that attains its maximum
        tight = mask[src] & mask[dst] & (b[src] == wv[src] + xe + b[dst])
        has_tight = np.zeros(n, dtype=bool)
        has_tight[src[tight]] = True
        assert (has_tight | ~mask | (outdeg == 0)).all()


@pytest.mark.parametrize("name,kw", [
    ("tiny", {}),
    ("mlp", dict(P=24, layers=6, shards=3)),
    ("inception", dict(P=16, modules=4, groups=3)),
    ("large_sparse", dict(P=8, levels=60, width=40)),
    ("comm_heavy", dict(P=8, levels=6, width=300, hub_degree=100)),
])
def test_invariants_on_workloads(oracle, name, kw):
    w = make_workload(name, **kw)
    out = oracle.evaluate_workload(w)
    _check_invariants(w, out, range(w.P))


def test_duality_between_the_two_sweeps(oracle):
    """tl on G equals (b - w) on the edge-reversed graph with B transposed."""
    w = make_workload("inception", P=6, modules=3, groups=2)
    rng = np.random.default_rng(8)
    B = rng.integers(1, 50, size=(w.k, w.k))  # asymmetric
    out = oracle.evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, B, w.assignments)
    src = np.repeat(np.arange(w.n), np.diff(w.succ_ptr))
    rev = build_csr(w.n, w.succ_idx, src, w.succ_t)
    outr = oracle.evaluate(w.n, rev["succ_ptr"], rev["succ_idx"], rev["succ_t"], w.c, w.speeds,
                           B.T.copy(), w.assignments)
    wv = -(-w.c[None, :] // w.speeds[w.assignments.astype(np.int64)])
    assert (out["tl"] == outr["b"] - wv).all()
    assert (out["b"] == outr["tl"] + wv).all()
    assert (out["cp"] == outr["cp"]).all()


# ----------------------------------------------------------------- symmetries

def test_batch_permutation_and_single_column(oracle):
    w = make_workload("mlp", P=20, layers=5, shards=2)
    out = oracle.evaluate_workload(w)
    perm = np.random.default_rng(0).permutation(w.P)
    outp = oracle.evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth,
                           w.assignments[perm])
    assert (outp["cp"] == out["cp"][perm]).all()
    assert (outp["b"] == out["b"][perm]).all()
    one = oracle.evaluate_workload(w, partitions=[13])
    assert one["cp"][0] == out["cp"][13] and (one["tl"][0] == out["tl"][13]).all()


def test_device_relabelling_leaves_results_unchanged(oracle):
    w = make_workload("large_sparse", P=10, levels=30, width=20)
    rng = np.random.default_rng(9)
    B = rng.integers(1, 64, size=(w.k, w.k))
    out = oracle.evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, B, w.assignments)
    perm = rng.permutation(w.k)          # new label of old device d is perm[d]
    s2 = np.empty_like(w.speeds)
    s2[perm] = w.speeds
    B2 = np.empty_like(B)
    B2[np.ix_(perm, perm)] = B
    a2 = perm[w.assignments.astype(np.int64)].astype(np.uint8)
    out2 = oracle.evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, s2, B2, a2)
    for key in ("cp", "b", "tl", "mask"):
        assert (out[key] == out2[key]).all()


def test_explicit_final_sink_does_not_change_cp(oracle):
    """Section 2: a zero-cost vertex joined to every sink by zero-cost edges starts
    exactly when the computation finishes."""
    w = make_workload("tiny")
    out = oracle.evaluate_workload(w)
    src = np.repeat(np.arange(w.n), np.diff(w.succ_ptr))
    sinks = np.nonzero(np.diff(w.succ_ptr) == 0)[0]
    T = w.n
    csr = build_csr(w.n + 1, np.concatenate([src, sinks]),
                    np.concatenate([w.succ_idx, np.full(len(sinks), T)]),
                    np.concatenate([w.succ_t, np.zeros(len(sinks), dtype=np.int64)]))
    c2 = np.concatenate([w.c, [0]])
    a2 = np.concatenate([w.assignments, np.zeros((w.P, 1), dtype=np.uint8)], axis=1)
    out2 = oracle.evaluate(w.n + 1, csr["succ_ptr"], csr["succ_idx"], csr["succ_t"], c2,
                           w.speeds, w.bandwidth, a2)
    assert (out2["cp"] == out["cp"]).all()
    assert (out2["tl"][:, T] == out["cp"]).all()   # its start time is the finishing time
    assert (out2["b"][:, :w.n] == out["b"]).all()


def test_all_on_one_device_ignores_bandwidth(oracle):
    w = make_workload("tiny")
    a = np.ones((1, w.n), dtype=np.uint8)
    o1 = oracle.evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth, a)
    o2 = oracle.evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds,
                         np.array([[1, 1], [1, 1]]), a)
    assert (o1["b"] == o2["b"]).all() and (o1["tl"] == o2["tl"]).all()


def test_faster_devices_and_links_never_hurt(oracle):
    w = make_workload("inception", P=12, modules=3, groups=2)
    base = oracle.evaluate_workload(w)
    rng = np.random.default_rng(10)
    for _ in range(4):
        s2 = w.speeds + rng.integers(0, 3, size=w.k)
        B2 = w.bandwidth + rng.integers(0, 30, size=(w.k, w.k))
        out = oracle.evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, s2, B2, w.assignments)
        assert (out["cp"] <= base["cp"]).all()
        assert (out["b"] <= base["b"]).all() and (out["tl"] <= base["tl"]).all()


def test_paper_parameter_ranges_smoke(oracle):
    """A graph the size of the paper's smallest network with the simulation's
    parameter ranges (section 5.1): 50 devices."""
    rows = {r[0]: (int(r[1]), int(r[2])) for r in _read_table("simulation_parameter_ranges.txt")}
    rng = np.random.default_rng(12)
    n, level, src, dst = random_layered_dag(rng, [7] * 50, 1, 2, 3)
    k = rows["devices"][0]
    csr = build_csr(n, src, dst, rng.integers(rows["tensor_bytes"][0], rows["tensor_bytes"][1] + 1,
                                              size=len(src)), level)
    c = rng.integers(rows["vertex_ops"][0], rows["vertex_ops"][1] + 1, size=n)
    s = rng.integers(rows["speed"][0], rows["speed"][1] + 1, size=k)
    B = rng.integers(rows["rate"][0], rows["rate"][1] + 1, size=(k, k))
    parts = rng.integers(0, k, size=(4, n), dtype=np.uint8)
    got = _eval(oracle, csr, c, s, B, parts)
    # every vertex takes 1..10 ticks and every transfer 0..10 ticks, and a path has
    # at most L vertices: that bounds CP from above; the longest-path layering has a
    # chain of L vertices of at least one tick each, which bounds it from below
    asap = build_csr(n, src, dst, np.zeros(len(src), dtype=np.int64))
    assert (got["cp"] >= asap["L"]).all()
    assert (got["cp"] <= csr["L"] * 10 + (csr["L"] - 1) * 10).all()


def test_rejects_cycles_and_bad_ids(oracle):
    csr = dict(n=2, succ_ptr=np.array([0, 1, 2], dtype=np.int32),
               succ_idx=np.array([1, 0], dtype=np.int32), succ_t=np.array([1, 1]))
    with pytest.raises(ValueError):
        _eval(oracle, csr, np.array([1, 1]), np.array([1]), np.array([[1]]), [[0, 0]])
    ok = build_csr(2, [0], [1], [1])
    with pytest.raises(ValueError):
        _eval(oracle, ok, np.array([1, 1]), np.array([1]), np.array([[1]]), [[0, 1]])


# ----------------------------------------------------------------- one critical path

@pytest.mark.parametrize("seed", range(6))
def test_critical_path_is_the_lexicographically_smallest_one(oracle, seed):
    """Brute force lists every source-to-sink path of maximal cost; the oracle must
    return the smallest vertex sequence among them (small weights force ties)."""
    rng = np.random.default_rng(200 + seed)
    n, level, src, dst = random_layered_dag(rng, [3] * 5, 1, 3, 2)
    t = rng.integers(0, 3, size=len(src))
    c = rng.integers(1, 3, size=n)
    csr = build_csr(n, src, dst, t, level)
    s = np.array([1, 2])
    B = np.array([[1, 2], [1, 1]])
    parts = rng.integers(0, 2, size=(10, n), dtype=np.uint8)
    paths, lens = oracle.critical_path(n, csr["succ_ptr"], csr["succ_idx"], csr["succ_t"], c, s, B,
                                       parts, max_len=csr["L"])
    got = _eval(oracle, csr, c, s, B, parts)
    edges = _edges(csr)
    ties = 0
    for j, p in enumerate(parts):
        best, found = brute_force.critical_paths(n, edges, c, s, B, p)
        assert best == got["cp"][j]
        ties += len(found) > 1
        assert paths[j, :lens[j]].tolist() == min(found)
        assert (paths[j, lens[j]:] == -1).all()
        assert got["mask"][j][paths[j, :lens[j]]].all()      # every vertex of it is critical
    assert ties > 0


def test_critical_path_of_a_chain_and_of_an_antichain(oracle):
    csr = _chain(6, [1, 2, 3, 4, 5])
    paths, lens = oracle.critical_path(6, csr["succ_ptr"], csr["succ_idx"], csr["succ_t"], np.ones(6),
                                       np.array([1]), np.array([[1]]), np.zeros((1, 6), dtype=np.uint8), 6)
    assert lens[0] == 6 and paths[0].tolist() == [0, 1, 2, 3, 4, 5]
    csr = build_csr(4, [], [], [])
    paths, lens = oracle.critical_path(4, csr["succ_ptr"], csr["succ_idx"], csr["succ_t"],
                                       np.array([3, 9, 9, 1]), np.array([1]), np.array([[1]]),
                                       np.zeros((1, 4), dtype=np.uint8), 2)
    assert lens[0] == 1 and paths[0].tolist() == [1, -1]     # lowest id among the costliest


# ------------------------------------------------------------------ ranks of section 3.2

@pytest.mark.parametrize("seed", range(4))
def test_ranks_against_path_enumeration(oracle, seed):
    """upRank(v) is the largest sum of c over a path that starts at v, downRank(v) the
    largest over a path that ends at v (both count v), by listing every path."""
    rng = np.random.default_rng(300 + seed)
    n, level, src, dst = random_layered_dag(rng, [3, 4, 2, 4, 3], 1, 3, 2)
    c = rng.integers(1, 50, size=n)
    csr = build_csr(n, src, dst, np.ones(len(src), dtype=np.int64), level)
    up, down, total = oracle.ranks(n, csr["succ_ptr"], csr["succ_idx"], c)
    exp_up = [0] * n
    exp_down = [0] * n
    for path in brute_force.all_paths(n, _edges(csr)):
        cost = sum(int(c[v]) for v, _ in path)
        exp_up[path[0][0]] = max(exp_up[path[0][0]], cost)
        exp_down[path[-1][0]] = max(exp_down[path[-1][0]], cost)
    assert up.tolist() == exp_up
    assert down.tolist() == exp_down
    assert total.tolist() == [a + b for a, b in zip(exp_up, exp_down)]


def test_ranks_closed_forms(oracle):
    # chain: suffix and prefix sums
    c = np.array([5, 1, 7, 2, 3])
    csr = _chain(5, [9, 9, 9, 9])
    up, down, total = oracle.ranks(5, csr["succ_ptr"], csr["succ_idx"], c)
    assert up.tolist() == np.cumsum(c[::-1])[::-1].tolist()
    assert down.tolist() == np.cumsum(c).tolist()
    assert total.tolist() == (c.sum() + c).tolist()       # every vertex lies on the one path; c counted twice
    # diamond 0 -> {1, 2} -> 3 with a heavy and a light arm
    csr = build_csr(4, [0, 0, 1, 2], [1, 2, 3, 3], [1, 1, 1, 1])
    up, down, total = oracle.ranks(4, csr["succ_ptr"], csr["succ_idx"], np.array([1, 10, 2, 4]))
    assert up.tolist() == [15, 14, 6, 4]
    assert down.tolist() == [1, 11, 3, 15]
    assert total.tolist() == [16, 25, 9, 19]
    # no edges: both ranks are c
    csr = build_csr(3, [], [], [])
    up, down, total = oracle.ranks(3, csr["succ_ptr"], csr["succ_idx"], np.array([4, 0, 9]))
    assert up.tolist() == [4, 0, 9] and down.tolist() == [4, 0, 9] and total.tolist() == [8, 0, 18]


def test_ranks_are_the_one_device_unit_speed_evaluation(oracle):
    """With one device of speed 1 nothing is transferred and w = c: upRank is the b-level,
    downRank the t-level plus c (the rank equations add the vertex's own c)."""
    w = make_workload("mlp", P=1)
    up, down, total = oracle.ranks(w.n, w.succ_ptr, w.succ_idx, w.c)
    got = oracle.evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, np.array([1]), np.array([[1]]),
                          np.zeros((1, w.n), dtype=np.uint8))
    assert np.array_equal(up, got["b"][0])
    assert np.array_equal(down, got["tl"][0] + w.c)
    assert up.max() == got["cp"][0] == down.max()


# ------------------------------------------------------------------ PCT priority order (section 4.1)

def test_pct_order_hand_example(oracle):
    # two devices; device 0 holds {0, 2, 3, 5}, device 1 holds {1, 4}
    a = np.array([[0, 1, 0, 0, 1, 0]], dtype=np.uint8)
    b = np.array([[7, 3, 9, 7, 3, 1]])
    order, seg = oracle.pct_order(2, a, b)
    assert order[0].tolist() == [2, 0, 3, 5, 1, 4]        # 9, then the two 7s by vertex number, then 1 | 3, 3
    assert seg[0].tolist() == [0, 4, 6]
    # an unused device has an empty range
    order, seg = oracle.pct_order(3, np.array([[2, 0, 2]], dtype=np.uint8), np.array([[5, 5, 6]]))
    assert order[0].tolist() == [1, 2, 0] and seg[0].tolist() == [0, 1, 1, 3]


@pytest.mark.parametrize("seed", range(3))
def test_pct_order_by_counting_ranks(oracle, seed):
    """Position of v = number of vertices that must come before it (lower device, or the
    same device and higher b, or the same b and lower number), counted pair by pair."""
    rng = np.random.default_rng(400 + seed)
    n, k, P = 60, 3, 5
    a = rng.integers(0, k, size=(P, n), dtype=np.uint8)
    b = rng.integers(0, 8, size=(P, n))                   # many ties
    order, seg = oracle.pct_order(k, a, b)
    for j in range(P):
        pos = np.empty(n, dtype=np.int64)
        pos[order[j]] = np.arange(n)
        for v in range(n):
            before = sum(1 for u in range(n) if u != v and (
                a[j, u] < a[j, v] or (a[j, u] == a[j, v] and (b[j, u] > b[j, v] or (b[j, u] == b[j, v] and u < v)))))
            assert pos[v] == before
        assert seg[j].tolist() == [int((a[j] < d).sum()) for d in range(k + 1)]


def test_pct_order_against_lexsort_and_precedence(oracle):
    """numpy's lexsort under the same key; and since every vertex here costs at least one
    tick, b strictly decreases along an edge, so a device's list never runs a vertex before
    one of its predecessors on that device (requirement 4 of section 4)."""
    w = make_workload("mlp", P=6)
    got = oracle.evaluate_workload(w, want=("b",))
    order, seg = oracle.pct_order(w.k, w.assignments, got["b"])
    ids = np.arange(w.n)
    src = np.repeat(ids, np.diff(w.succ_ptr))
    for j in range(w.P):
        assert np.array_equal(order[j], np.lexsort((ids, -got["b"][j], w.assignments[j])))
        pos = np.empty(w.n, dtype=np.int64)
        pos[order[j]] = ids
        same = w.assignments[j][src] == w.assignments[j][w.succ_idx]
        assert (pos[src][same] < pos[w.succ_idx][same]).all()
        assert np.array_equal(np.diff(seg[j]), np.bincount(w.assignments[j], minlength=w.k))


# ------------------------------------------------------------------ placement constraints (section 2)

def test_validate_hand_example(oracle):
    # vertices 0 and 3 must share a device, so must 1 and 2; vertex 4 must sit on device 1
    pairs = [[0, 3], [1, 2]]
    pins = [[4, 1]]
    a = np.array([[0, 1, 1, 0, 1],      # all three hold
                  [0, 1, 1, 0, 0],      # the device constraint is broken
                  [0, 1, 0, 1, 1],      # both pairs are broken
                  [2, 2, 2, 2, 1]], dtype=np.uint8)
    valid, broken = oracle.validate(3, a, pairs, pins)
    assert valid.tolist() == [1, 0, 0, 1] and broken.tolist() == [0, 1, 2, 0]
    # no constraints: everything is valid
    valid, broken = oracle.validate(3, a, [], [])
    assert valid.tolist() == [1, 1, 1, 1] and broken.tolist() == [0, 0, 0, 0]


def test_validate_against_set_formulation(oracle):
    """The same through the relations as sets: p must be constant on every pair and map
    every constrained vertex to its device."""
    rng = np.random.default_rng(500)
    n, k, P = 40, 4, 60
    pairs = rng.integers(0, n, size=(12, 2))
    pins = np.stack([rng.integers(0, n, size=6), rng.integers(0, k, size=6)], axis=1)
    a = rng.integers(0, k, size=(P, n), dtype=np.uint8)
    a[:10, pairs[:, 1]] = a[:10, pairs[:, 0]]          # make some partitions satisfy the pairs ...
    for _ in range(3):                                   # (chains of pairs need a few rounds)
        a[:10, pairs[:, 1]] = a[:10, pairs[:, 0]]
    valid, broken = oracle.validate(k, a, pairs, pins)
    for j in range(P):
        exp = sum(int(a[j, u] != a[j, v]) for u, v in pairs) + sum(int(a[j, v] != d) for v, d in pins)
        assert broken[j] == exp and valid[j] == (exp == 0)
    # symmetric relation: swapping the two ends of every pair changes nothing
    v2, b2 = oracle.validate(k, a, pairs[:, ::-1], pins)
    assert np.array_equal(v2, valid) and np.array_equal(b2, broken)
    # a partition that puts everything on the device every pin names is valid when all pins agree
    one = np.full((1, n), 2, dtype=np.uint8)
    assert oracle.validate(k, one, pairs, [[3, 2], [7, 2]])[0].tolist() == [1]
    assert oracle.validate(k, one, pairs, [[3, 2], [7, 1]])[0].tolist() == [0]
    with pytest.raises(ValueError):
        oracle.validate(k, one, [[0, n]], [])
    with pytest.raises(ValueError):
        oracle.validate(k, one, [], [[0, k]])


# ------------------------------------------------------------------ critical-path move search

def test_neighbours_are_all_single_moves_of_path_vertices(oracle):
    base = np.array([0, 2, 1, 1, 0], dtype=np.uint8)
    out = oracle.neighbours(3, base, [3, 0])
    assert out.tolist() == [[0, 2, 1, 0, 0], [0, 2, 1, 2, 0],        # vertex 3 (on 1) -> 0, 2
                            [1, 2, 1, 1, 0], [2, 2, 1, 1, 0]]        # vertex 0 (on 0) -> 1, 2
    rng = np.random.default_rng(600)
    n, k = 30, 5
    base = rng.integers(0, k, size=n, dtype=np.uint8)
    path = rng.permutation(n)[:7]
    out = oracle.neighbours(k, base, path)
    seen = set()
    for row in out:
        diff = np.nonzero(row != base)[0]
        assert len(diff) == 1 and diff[0] in path
        seen.add((int(diff[0]), int(row[diff[0]])))
    assert seen == {(int(v), d) for v in path for d in range(k) if d != base[v]}
    assert oracle.neighbours(1, np.zeros(4, dtype=np.uint8), [1, 2]).shape == (0, 4)


def test_argmin_takes_the_first_of_the_smallest_valid(oracle):
    assert oracle.argmin([5, 3, 9, 3]) == (1, 3)
    assert oracle.argmin([5, 3, 9, 3], [1, 0, 1, 1]) == (3, 3)
    assert oracle.argmin([5, 3, 9, 3], [1, 0, 1, 0]) == (0, 5)
    assert oracle.argmin([5, 3], [0, 0]) == (-1, None)
    assert oracle.argmin([]) == (-1, None)


@pytest.mark.parametrize("seed", range(3))
def test_search_descends_to_a_local_optimum(oracle, seed):
    """Every move lowers CP; at the end no single move of a critical-path vertex does
    (checked move by move with the brute-force evaluator); the result is never better
    than the true optimum over all k^n partitions."""
    rng = np.random.default_rng(700 + seed)
    n, level, src, dst = random_layered_dag(rng, [2, 3, 2, 2], 1, 2, 2)
    t = rng.integers(1, 30, size=len(src))
    c = rng.integers(1, 20, size=n)
    csr = build_csr(n, src, dst, t, level)
    s = np.array([1, 3])
    B = np.array([[1, 2], [4, 1]])
    start = rng.integers(0, 2, size=n, dtype=np.uint8)
    final, trace, moves = oracle.search(n, csr["succ_ptr"], csr["succ_idx"], csr["succ_t"], c, s, B, start,
                                        max_len=csr["L"])
    assert (np.diff(trace) < 0).all() and len(moves) == len(trace) - 1
    edges = _edges(csr)
    replay = start.copy()
    for (v, d), cp_after in zip(moves, trace[1:]):
        replay[v] = d
        assert brute_force.evaluate(n, edges, c, s, B, replay)[0] == cp_after
    assert np.array_equal(replay, final)
    best, found = brute_force.critical_paths(n, edges, c, s, B, final)
    assert best == trace[-1]
    for v in min(found):
        other = final.copy()
        other[v] = 1 - other[v]
        assert brute_force.evaluate(n, edges, c, s, B, other)[0] >= best
    optimum = min(brute_force.evaluate(n, edges, c, s, B, np.array([(code >> i) & 1 for i in range(n)]))[0]
                  for code in range(2 ** n))
    assert optimum <= trace[-1] <= trace[0]


def test_search_respects_constraints_and_the_move_limit(oracle):
    w = make_workload("tiny")
    start = w.assignments[0]
    free, trace_free, moves_free = oracle.search(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds,
                                                 w.bandwidth, start, max_len=w.L)
    assert len(moves_free) >= 2
    # pin the first vertex that moved to where it started: that move is no longer allowed
    v0 = int(moves_free[0][0])
    pinned, trace_pin, moves_pin = oracle.search(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds,
                                                 w.bandwidth, start, max_len=w.L, pins=[[v0, int(start[v0])]])
    assert pinned[v0] == start[v0] and all(int(m[0]) != v0 for m in moves_pin)
    assert trace_pin[0] == trace_free[0]
    one, trace_one, moves_one = oracle.search(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth,
                                              start, max_len=w.L, max_moves=1)
    assert len(moves_one) == 1 and trace_one.tolist() == trace_free[:2].tolist()
    assert np.array_equal(moves_one[0], moves_free[0])


# ------------------------------------------------------------------ Critical Path partitioning strategy (section 3.2.2)

def test_seed_hand_example(oracle):
    # 0 -> 1 -> 3 and 0 -> 2 -> 3 with c = 4, 9, 2, 4: the critical path is 0, 1, 3 (4 + 9 + 4);
    # vertex 4 is isolated with c = 6.  Devices: speeds 2, 4, 4 -> fastest is device 1.
    csr = build_csr(5, [0, 0, 1, 2], [1, 2, 3, 3], [7, 7, 7, 7])
    got = oracle.seed(5, csr["succ_ptr"], csr["succ_idx"], [4, 9, 2, 4, 6], [2, 4, 4], max_len=3)
    # path on device 1: load = ceil(4/4) + ceil(9/4) + ceil(4/4) = 1 + 3 + 1 = 5
    # vertex 2: device 0: 0 + ceil(2/2) = 1; device 1: 5 + 1 = 6; device 2: 0 + 1 = 1 -> device 0 (lowest number)
    # vertex 4: device 0: 1 + ceil(6/2) = 4; device 1: 5 + 2 = 7; device 2: 0 + 2 = 2 -> device 2
    assert got.tolist() == [1, 1, 0, 1, 2]


@pytest.mark.parametrize("seed", range(3))
def test_seed_step_by_step(oracle, seed):
    """The critical path (device-free ranks: the one-device critical path) sits on the fastest
    device; replaying the remaining vertices in order, the chosen device is a cheapest one
    for the loads at that moment, and no lower-numbered device is as cheap."""
    rng = np.random.default_rng(800 + seed)
    n, level, src, dst = random_layered_dag(rng, [5] * 8, 1, 3, 2)
    c = rng.integers(1, 40, size=n)
    csr = build_csr(n, src, dst, rng.integers(1, 9, size=len(src)), level)
    speeds = np.array([3, 7, 2, 7])
    got = oracle.seed(n, csr["succ_ptr"], csr["succ_idx"], c, speeds, max_len=csr["L"])
    paths, lens = oracle.critical_path(n, csr["succ_ptr"], csr["succ_idx"], np.zeros(len(src), dtype=np.int64), c,
                                       np.array([1]), np.array([[1]]), np.zeros((1, n), dtype=np.uint8), csr["L"])
    path = paths[0, :lens[0]]
    up, down, total = oracle.ranks(n, csr["succ_ptr"], csr["succ_idx"], c)
    assert sum(int(c[v]) for v in path) == up.max()            # it is a longest path of the rank equations
    assert (got[path] == 1).all()                               # device 1: first of the two fastest
    load = [0] * 4
    load[1] = sum(-(-int(c[v]) // 7) for v in path)
    on_path = set(int(v) for v in path)
    for v in range(n):
        if v in on_path:
            continue
        cost = [load[d] + -(-int(c[v]) // int(speeds[d])) for d in range(4)]
        d = int(got[v])
        assert cost[d] == min(cost) and all(cost[e] > cost[d] for e in range(d))
        load[d] = cost[d]


def test_seed_degenerate_cases(oracle):
    # one device: everything on it; no edges: the "path" is the costliest vertex alone
    csr = build_csr(4, [], [], [])
    assert oracle.seed(4, csr["succ_ptr"], csr["succ_idx"], [3, 9, 9, 1], [5], max_len=1).tolist() == [0, 0, 0, 0]
    got = oracle.seed(4, csr["succ_ptr"], csr["succ_idx"], [3, 9, 9, 1], [1, 1], max_len=1)
    # path = vertex 1 (lowest number among the costliest) on device 0 (lowest number among the fastest): load 9
    # vertex 0 -> device 1 (3 < 12); vertex 2 -> device 1 (3 + 9 = 12 < 18); vertex 3 -> device 0 (10 < 13)
    assert got.tolist() == [1, 0, 1, 0]

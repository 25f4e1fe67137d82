"""TEST INFRASTRUCTURE: brute-force path enumeration, used only to pin the oracle.

Every directed path of a tiny DAG is listed explicitly and its cost summed term
by term; no recurrence, no topological order.  Costs are taken from the model's
definition (paper, section 2 and section 4.1) with exact rational arithmetic and
an explicit round-up, independent of the C oracle's integer formula.
"""
from __future__ import annotations

from fractions import Fraction
from math import ceil


def _w(c, s, p, v):
    return ceil(Fraction(int(c[v]), int(s[p[v]])))


def _x(t_e, bandwidth, p, u, v):
    if p[u] == p[v]:
        return 0
    return ceil(Fraction(int(t_e), int(bandwidth[p[u]][p[v]])))


def all_paths(n, edges):
    """Yield every directed path with at least one vertex as a list of
    (vertex, edge-index-or-None) steps; edges is a list of (u, v, t)."""
    out = [[] for _ in range(n)]
    for ei, (u, v, _t) in enumerate(edges):
        out[u].append((v, ei))

    def extend(path):
        yield path
        last = path[-1][0]
        for (v, ei) in out[last]:
            yield from extend(path + [(v, ei)])

    for start in range(n):
        yield from extend([(start, None)])


def evaluate(n, edges, c, speeds, bandwidth, p, max_paths=2_000_000):
    """Return (CP, b[n], tl[n]) for one partition p by enumerating all paths.

    b(v)  = largest cost of a path that starts at v (all its vertices and edges).
    tl(v) = largest cost of a path that ends at v, not counting v itself.
    CP    = largest cost of any path.
    """
    b = [0] * n
    tl = [0] * n
    cp = 0
    count = 0
    for path in all_paths(n, edges):
        count += 1
        if count > max_paths:
            raise RuntimeError("too many paths for brute force")
        cost = 0
        for (v, ei) in path:
            if ei is not None:
                u_, v_, t_ = edges[ei]
                cost += _x(t_, bandwidth, p, u_, v_)
            cost += _w(c, speeds, p, v)
        first, last = path[0][0], path[-1][0]
        b[first] = max(b[first], cost)
        tl[last] = max(tl[last], cost - _w(c, speeds, p, last))
        cp = max(cp, cost)
    return cp, b, tl


def critical_paths(n, edges, c, speeds, bandwidth, p):
    """Every source-to-sink path whose cost equals the largest path cost, as lists
    of vertices (explicit enumeration)."""
    has_pred = [False] * n
    has_succ = [False] * n
    for (u, v, _t) in edges:
        has_pred[v] = True
        has_succ[u] = True
    best, found = -1, []
    for path in all_paths(n, edges):
        first, last = path[0][0], path[-1][0]
        if has_pred[first] or has_succ[last]:
            continue
        cost = 0
        for (v, ei) in path:
            if ei is not None:
                u_, v_, t_ = edges[ei]
                cost += _x(t_, bandwidth, p, u_, v_)
            cost += _w(c, speeds, p, v)
        verts = [v for (v, _e) in path]
        if cost > best:
            best, found = cost, [verts]
        elif cost == best:
            found.append(verts)
    return best, found

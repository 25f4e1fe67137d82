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


def list_schedule_by_ticks(n, edges, c, speeds, bandwidth, p, policy, b=None, tie=None, horizon=100_000):
    """Time-stepped list scheduling of one partition p, used only to pin the oracle's event loop.

    The clock advances one tick at a time (no event queue, no ready lists).  At every tick
    each free device looks at all its unstarted vertices, keeps those whose every input
    tensor has arrived (paper, section 4, criterion (4)) and starts one at once (criteria
    (2), (3), (6)): under "pct" the one with the largest b, lowest vertex number among
    equals (section 4.1); under "fifo" the one that became executable first, the smaller
    tie value (vertex number if tie is None) among equals (section 5.1).  Returns
    (makespan, start[n]).  Every vertex must take at least one tick.
    """
    k = len(speeds)
    w = [_w(c, speeds, p, v) for v in range(n)]
    assert all(x >= 1 for x in w)
    preds = [[] for _ in range(n)]
    for (u, v, t) in edges:
        preds[v].append((u, _x(t, bandwidth, p, u, v)))
    start = [None] * n
    free_at = [0] * k
    now = 0
    left = n
    while left:
        if now > horizon:
            raise RuntimeError("no progress: cycle or horizon too short")
        started_now = []
        for d in range(k):
            if free_at[d] > now:
                continue
            executable = []
            for v in range(n):
                if p[v] != d or start[v] is not None:
                    continue
                arrivals = [None if start[u] is None else start[u] + w[u] + x for (u, x) in preds[v]]
                if any(a is None or a > now for a in arrivals):
                    continue
                executable.append((v, max(arrivals, default=0)))
            if not executable:
                continue
            if policy == "pct":
                v = min(executable, key=lambda it: (-b[it[0]], it[0]))[0]
            else:
                v = min(executable, key=lambda it: (it[1], it[0] if tie is None else tie[it[0]], it[0]))[0]
            started_now.append((v, d))
        # a vertex started at this tick finishes later than this tick, so the devices'
        # decisions at one tick do not depend on each other: apply them together
        for (v, d) in started_now:
            start[v] = now
            free_at[d] = now + w[v]
            left -= 1
        now += 1
    return max(free_at), start

"""Seeded generators for the five synthetic workloads and for small random DAGs.

Everything here is input construction: graph topology, integer weights, device
speeds, a bandwidth matrix and candidate partitions.  Nothing here evaluates a
cost or a path.

Conventions (problem statement of the paper, section 2): a DAG G=(V,E) with
n vertices and m edges, vertex complexity c(v), edge volume t(e), k devices with
speed s[i], bandwidth matrix B[i][j] (row = device of the edge's source vertex),
and P candidate partition functions p: V -> D stored as ``assignments[P][n]``.
All weights are non-negative integers ("ticks" come out of integer ceil
division downstream).

The paper's own three TensorFlow graphs (Table 1) are not available; these
workloads stand in for them and borrow their shape: layered forward+backward
graphs, sparse, heterogeneous device speeds and link rates (section 5.1).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 171101912  # + i for workload i = 1..5; assignments use seed + 1000

CONFIG_NAMES = ("tiny", "mlp", "inception", "large_sparse", "comm_heavy")


@dataclass
class Workload:
    name: str
    n: int
    m: int
    L: int
    succ_ptr: np.ndarray  # int32 [n+1]
    succ_idx: np.ndarray  # int32 [m]   head vertex of each out-edge
    succ_t: np.ndarray    # int64 [m]   t(e), in successor-CSR order
    pred_ptr: np.ndarray  # int32 [n+1]
    pred_idx: np.ndarray  # int32 [m]   tail vertex of each in-edge
    pred_eid: np.ndarray  # int32 [m]   position of that edge in the successor arrays
    c: np.ndarray         # int64 [n]
    level: np.ndarray     # int32 [n]   topological level of each vertex
    level_ptr: np.ndarray  # int32 [L+1]
    level_vtx: np.ndarray  # int32 [n]  vertices grouped by level
    k: int
    speeds: np.ndarray     # int64 [k]
    bandwidth: np.ndarray  # int64 [k][k]
    assignments: np.ndarray  # uint8 [P][n]
    meta: dict = field(default_factory=dict)

    @property
    def P(self) -> int:
        return int(self.assignments.shape[0])

    @property
    def max_out_degree(self) -> int:
        return int(np.diff(self.succ_ptr).max()) if self.n else 0

    def describe(self) -> dict:
        return {
            "workload": self.name, "n": self.n, "m": self.m, "L": self.L,
            "max_out_degree": self.max_out_degree, "P": self.P, "k": self.k,
        }


# --------------------------------------------------------------------------
# structure helpers
# --------------------------------------------------------------------------

def asap_levels(n: int, src: np.ndarray, dst: np.ndarray) -> np.ndarray:
    """Longest-distance-from-a-source layering (every edge goes to a strictly
    higher level).  Raises ValueError on a cycle."""
    level = np.zeros(n, dtype=np.int64)
    if len(src) == 0:
        return level.astype(np.int32)
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    for _ in range(n + 1):
        cand = level[src] + 1
        new = level.copy()
        np.maximum.at(new, dst, cand)
        if np.array_equal(new, level):
            return level.astype(np.int32)
        level = new
    raise ValueError("graph has a cycle")


def build_csr(n: int, src, dst, t, level=None) -> dict:
    """Successor CSR, predecessor CSR (with edge ids into the successor arrays)
    and the level index, from an edge list."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    t = np.asarray(t, dtype=np.int64)
    m = int(len(src))
    if level is None:
        level = asap_levels(n, src, dst)
    level = np.asarray(level, dtype=np.int32)

    order = np.lexsort((dst, src))  # by src, then dst
    s_src, s_dst, s_t = src[order], dst[order], t[order]
    succ_ptr = np.concatenate([[0], np.cumsum(np.bincount(s_src, minlength=n))])

    porder = np.lexsort((s_src, s_dst))  # by dst, then src; indexes the succ arrays
    pred_ptr = np.concatenate([[0], np.cumsum(np.bincount(s_dst, minlength=n))])

    L = int(level.max()) + 1 if n else 0
    lorder = np.argsort(level, kind="stable")
    level_ptr = np.concatenate([[0], np.cumsum(np.bincount(level, minlength=L))])
    return dict(
        n=n, m=m, L=L,
        succ_ptr=succ_ptr.astype(np.int32), succ_idx=s_dst.astype(np.int32), succ_t=s_t.copy(),
        pred_ptr=pred_ptr.astype(np.int32), pred_idx=s_src[porder].astype(np.int32),
        pred_eid=porder.astype(np.int32),
        level=level, level_ptr=level_ptr.astype(np.int32), level_vtx=lorder.astype(np.int32),
    )


def _dedupe(n, src, dst, t):
    """Keep the first of any repeated (src, dst) pair."""
    key = src.astype(np.int64) * n + dst.astype(np.int64)
    _, first = np.unique(key, return_index=True)
    first.sort()
    return src[first], dst[first], t[first]


def random_layered_dag(rng, widths, deg_lo, deg_hi, span_hi, overflow="resample"):
    """Vertices are numbered level by level.  A vertex in level l (not the last)
    draws d in U{deg_lo..deg_hi} out-edges; each goes ``span`` in U{1..span_hi}
    levels down to a uniformly drawn vertex there.  A span running past the last
    level is clamped to it (overflow="clamp") or drawn uniformly over the levels
    that remain (overflow="resample").  Returns (n, level, src, dst) with
    duplicate (src, dst) pairs removed."""
    widths = np.asarray(widths, dtype=np.int64)
    L = len(widths)
    off = np.concatenate([[0], np.cumsum(widths)])
    n = int(off[-1])
    level = np.repeat(np.arange(L, dtype=np.int64), widths)
    has_out = np.nonzero(level < L - 1)[0]
    deg = rng.integers(deg_lo, deg_hi + 1, size=len(has_out))
    src = np.repeat(has_out, deg)
    lsrc = level[src]
    room = (L - 1) - lsrc
    if overflow == "clamp":
        span = np.minimum(rng.integers(1, span_hi + 1, size=len(src)), room)
    else:
        span = 1 + np.floor(rng.random(len(src)) * np.minimum(span_hi, room)).astype(np.int64)
    ldst = lsrc + span
    dst = off[ldst] + np.floor(rng.random(len(src)) * widths[ldst]).astype(np.int64)
    key = src * n + dst
    _, first = np.unique(key, return_index=True)
    first.sort()
    return n, level.astype(np.int32), src[first], dst[first]


def _sym_int_matrix(rng, k, lo, hi):
    a = rng.integers(lo, hi + 1, size=(k, k)).astype(np.int64)
    b = np.triu(a, 1)
    b = b + b.T
    np.fill_diagonal(b, lo)  # the diagonal is never used: same-device transfers are free
    return b


def _uniform_assignments(rng, P, n, k):
    return rng.integers(0, k, size=(P, n), dtype=np.uint8)


def _block_assignments(rng, P, level_vtx, k):
    """Vertices in level order cut into k contiguous blocks at random cut
    points; block i goes to a randomly relabelled device."""
    n = len(level_vtx)
    out = np.empty((P, n), dtype=np.uint8)
    pos = np.arange(n)
    for j in range(P):
        cuts = np.sort(rng.integers(0, n + 1, size=k - 1))
        block = np.searchsorted(cuts, pos, side="right")
        relabel = rng.permutation(k).astype(np.uint8)
        out[j, level_vtx] = relabel[block]
    return out


def _finish(name, csr, c, k, speeds, bandwidth, assignments, **meta) -> Workload:
    return Workload(
        name=name, n=csr["n"], m=csr["m"], L=csr["L"],
        succ_ptr=csr["succ_ptr"], succ_idx=csr["succ_idx"], succ_t=csr["succ_t"],
        pred_ptr=csr["pred_ptr"], pred_idx=csr["pred_idx"], pred_eid=csr["pred_eid"],
        c=np.asarray(c, dtype=np.int64), level=csr["level"],
        level_ptr=csr["level_ptr"], level_vtx=csr["level_vtx"],
        k=int(k), speeds=np.asarray(speeds, dtype=np.int64),
        bandwidth=np.ascontiguousarray(bandwidth, dtype=np.int64),
        assignments=np.ascontiguousarray(assignments, dtype=np.uint8), meta=meta,
    )


# --------------------------------------------------------------------------
# the five workloads
# --------------------------------------------------------------------------

def _tiny(seed, P=16, layers=8, width=8):
    rng = np.random.default_rng(seed)
    n, level, src, dst = random_layered_dag(rng, [width] * layers, 1, 3, 2, overflow="clamp")
    t = rng.integers(1, 1001, size=len(src))
    c = rng.integers(1, 101, size=n)
    k = 2
    speeds = np.array([1, 2])
    bandwidth = np.array([[10, 10], [10, 10]])
    csr = build_csr(n, src, dst, t, level)
    arng = np.random.default_rng(seed + 1000)
    return _finish("tiny", csr, c, k, speeds, bandwidth, _uniform_assignments(arng, P, n, k))


def _mirror_with_twins(n_fwd, fsrc, fdst, ft):
    """Forward graph on ids [0, n_fwd); backward twin of x is x + n_fwd.  Every
    forward edge a->b gets the reversed backward edge b'->a' of the same volume,
    and every forward vertex x gets a gradient edge x->x'."""
    fsrc = np.asarray(fsrc, dtype=np.int64)
    fdst = np.asarray(fdst, dtype=np.int64)
    ft = np.asarray(ft, dtype=np.int64)
    bsrc, bdst = fdst + n_fwd, fsrc + n_fwd
    x = np.arange(n_fwd, dtype=np.int64)
    return (np.concatenate([fsrc, bsrc, x]), np.concatenate([fdst, bdst, x + n_fwd]),
            np.concatenate([ft, ft]), x)


def _mlp(seed, P=1024, layers=32, shards=7):
    """Forward chain of `layers` layers; each layer is matmul -> bias -> act plus
    a loss-branch vertex fed by act; every op is split into `shards` parallel
    shards and a matmul shard depends on all act shards of the layer before.
    Backward mirror with gradient edges, and one weight-update vertex per
    (layer, shard) fed by the backward matmul."""
    rng = np.random.default_rng(seed)
    g = shards
    widths = [256, 512, 1024, 2048, 4096]
    MM, BI, AC, LB = 0, 1, 2, 3

    def vid(layer, op, sh):
        return (layer * 4 + op) * g + sh

    n_fwd = layers * 4 * g
    fsrc, fdst, flayer = [], [], []
    for l in range(layers):
        for sh in range(g):
            fsrc += [vid(l, MM, sh), vid(l, BI, sh), vid(l, AC, sh)]
            fdst += [vid(l, BI, sh), vid(l, AC, sh), vid(l, LB, sh)]
            flayer += [l, l, l]
            if l + 1 < layers:
                for sh2 in range(g):
                    fsrc.append(vid(l, AC, sh))
                    fdst.append(vid(l + 1, MM, sh2))
                    flayer.append(l)
    flayer = np.asarray(flayer)
    ft = 4 * np.asarray(widths)[flayer % len(widths)]
    src, dst, t_fb, twins = _mirror_with_twins(n_fwd, fsrc, fdst, ft)
    # gradient (twin) edges carry the activation of the layer they belong to
    twin_layer = (twins // (4 * g))
    t_twin = 4 * np.asarray(widths)[twin_layer % len(widths)]
    # weight updates
    upd_src, upd_dst, upd_t = [], [], []
    nxt = 2 * n_fwd
    for l in range(layers):
        for sh in range(g):
            upd_src.append(vid(l, MM, sh) + n_fwd)
            upd_dst.append(nxt)
            upd_t.append(4 * widths[l % len(widths)])
            nxt += 1
    n = nxt
    src = np.concatenate([src, upd_src])
    dst = np.concatenate([dst, upd_dst])
    t = np.concatenate([t_fb, t_twin, upd_t])
    c = rng.integers(10, 1001, size=n)
    k = 4
    speeds = np.array([1, 8, 8, 8])
    bandwidth = _sym_int_matrix(rng, k, 5, 50)
    csr = build_csr(n, src, dst, t)
    arng = np.random.default_rng(seed + 1000)
    half = P // 2
    a = np.concatenate([_uniform_assignments(arng, half, n, k),
                        _block_assignments(arng, P - half, csr["level_vtx"], k)])
    return _finish("mlp", csr, c, k, speeds, bandwidth, a, shards=g, layers=layers)


def _inception(seed, P=4096, modules=50, groups=14, target_out_degree=2.5):
    """`modules` modules in sequence; a module is split -> 4 branches -> concat,
    a branch being `groups` parallel chains of one depth drawn from U{2..5};
    random forward skip edges inside a module raise the average out-degree to
    the target; backward mirror with gradient edges."""
    rng = np.random.default_rng(seed)
    fsrc, fdst = [], []
    module_of = []
    pos_in_module = []  # a coarse forward position used to orient skip edges
    nxt = 0
    prev_concat = -1
    for mod in range(modules):
        split = nxt
        nxt += 1
        module_of.append(mod)
        pos_in_module.append(0)
        if prev_concat >= 0:
            fsrc.append(prev_concat)
            fdst.append(split)
        tails = []
        for _ in range(4):
            depth = int(rng.integers(2, 6))
            for _ in range(groups):
                prev = split
                for d in range(depth):
                    v = nxt
                    nxt += 1
                    module_of.append(mod)
                    pos_in_module.append(1 + d)
                    fsrc.append(prev)
                    fdst.append(v)
                    prev = v
                tails.append(prev)
        concat = nxt
        nxt += 1
        module_of.append(mod)
        pos_in_module.append(6)
        for tl in tails:
            fsrc.append(tl)
            fdst.append(concat)
        prev_concat = concat
    n_fwd = nxt
    module_of = np.asarray(module_of)
    pos_in_module = np.asarray(pos_in_module)
    fsrc = np.asarray(fsrc, dtype=np.int64)
    fdst = np.asarray(fdst, dtype=np.int64)
    # skip edges: total edges wanted = target * n, with n = 2 n_fwd and the
    # mirror doubling every forward edge, plus n_fwd gradient edges
    want_fwd = int((target_out_degree * 2 * n_fwd - n_fwd) / 2)
    need = max(0, want_fwd - len(fsrc))
    by_module = [np.nonzero(module_of == mod)[0] for mod in range(modules)]
    extra_s, extra_d = [], []
    have = set((fsrc * n_fwd + fdst).tolist())
    tries = 0
    while len(extra_s) < need and tries < 50 * need + 1000:
        tries += 1
        members = by_module[int(rng.integers(0, modules))]
        a, b = rng.choice(members, size=2, replace=False)
        if pos_in_module[a] == pos_in_module[b]:
            continue
        if pos_in_module[a] > pos_in_module[b]:
            a, b = b, a
        key = int(a) * n_fwd + int(b)
        if key in have:
            continue
        have.add(key)
        extra_s.append(int(a))
        extra_d.append(int(b))
    fsrc = np.concatenate([fsrc, np.asarray(extra_s, dtype=np.int64)])
    fdst = np.concatenate([fdst, np.asarray(extra_d, dtype=np.int64)])
    ft = np.maximum(1, np.rint(rng.lognormal(8.0, 1.5, size=len(fsrc)))).astype(np.int64)
    src, dst, t_fb, twins = _mirror_with_twins(n_fwd, fsrc, fdst, ft)
    t_twin = np.maximum(1, np.rint(rng.lognormal(8.0, 1.5, size=len(twins)))).astype(np.int64)
    t = np.concatenate([t_fb, t_twin])
    n = 2 * n_fwd
    c = np.maximum(1, np.rint(rng.lognormal(4.0, 1.0, size=n))).astype(np.int64)
    k = 8
    speeds = rng.choice(np.array([1, 2, 4, 8]), size=k)
    bandwidth = _sym_int_matrix(rng, k, 1, 100)
    csr = build_csr(n, src, dst, t)
    arng = np.random.default_rng(seed + 1000)
    return _finish("inception", csr, c, k, speeds, bandwidth,
                   _uniform_assignments(arng, P, n, k), modules=modules, groups=groups)


def _large_sparse(seed, P=256, levels=2000, width=500):
    rng = np.random.default_rng(seed)
    n, level, src, dst = random_layered_dag(rng, [width] * levels, 1, 7, 10, overflow="resample")
    t = rng.integers(1, 10001, size=len(src))
    c = rng.integers(1, 1001, size=n)
    k = 16
    speeds = rng.integers(1, 17, size=k)
    bandwidth = _sym_int_matrix(rng, k, 1, 64)
    csr = build_csr(n, src, dst, t, level)
    arng = np.random.default_rng(seed + 1000)
    return _finish("large_sparse", csr, c, k, speeds, bandwidth,
                   _uniform_assignments(arng, P, n, k))


def _comm_heavy(seed, P=1024, levels=20, width=10000, hub_fraction=0.01, hub_degree=1000):
    rng = np.random.default_rng(seed)
    n = levels * width
    level = np.repeat(np.arange(levels, dtype=np.int64), width)
    hub_degree = min(hub_degree, width)
    is_hub = np.zeros(n, dtype=bool)
    is_hub[rng.choice(n, size=max(1, int(round(hub_fraction * n))), replace=False)] = True
    inner = level < levels - 1
    # ordinary vertices: 2..4 successors in the next level
    ordinary = np.nonzero(inner & ~is_hub)[0]
    deg = rng.integers(2, 5, size=len(ordinary))
    o_src = np.repeat(ordinary, deg)
    o_dst = (level[o_src] + 1) * width + np.floor(rng.random(len(o_src)) * width).astype(np.int64)
    o_src, o_dst, _ = _dedupe(n, o_src, o_dst, np.zeros(len(o_src), dtype=np.int64))
    # hubs: hub_degree distinct successors in the next level
    hubs = np.nonzero(inner & is_hub)[0]
    h_src = np.repeat(hubs, hub_degree)
    h_dst = np.empty(len(h_src), dtype=np.int64)
    for i, h in enumerate(hubs):
        h_dst[i * hub_degree:(i + 1) * hub_degree] = (
            (level[h] + 1) * width + rng.choice(width, size=hub_degree, replace=False))
    src = np.concatenate([o_src, h_src])
    dst = np.concatenate([o_dst, h_dst])
    u = rng.random(len(src))
    t = np.minimum(1e7, np.floor(100.0 * (1.0 - u) ** (-1.0 / 1.2))).astype(np.int64)
    c = rng.integers(1, 51, size=n)
    k = 8
    speeds = np.array([1, 1, 4, 4, 8, 8, 16, 16])
    bandwidth = _sym_int_matrix(rng, k, 1, 20)
    csr = build_csr(n, src, dst, t, level.astype(np.int32))
    arng = np.random.default_rng(seed + 1000)
    return _finish("comm_heavy", csr, c, k, speeds, bandwidth,
                   _uniform_assignments(arng, P, n, k), hubs=int(len(hubs)))


def _paper_scale(seed, P=4096, levels=251, width=21, k=50):
    """The size of the largest graph of the paper's evaluation (Table 1: 5,271 vertices, 9,214
    edges, average degree 1.75) on the simulated cluster of section 5.1: 50 devices, speeds
    10..100, transfer rates 10..60, tensor sizes 1..100, vertex operations 1..100, all uniform.
    The graph itself is a random layered DAG, not the paper's network."""
    rng = np.random.default_rng(seed)
    n, level, src, dst = random_layered_dag(rng, [width] * levels, 1, 3, 3, overflow="resample")
    t = rng.integers(1, 101, size=len(src))
    c = rng.integers(1, 101, size=n)
    speeds = rng.integers(10, 101, size=k)
    bandwidth = rng.integers(10, 61, size=(k, k))
    csr = build_csr(n, src, dst, t, level)
    arng = np.random.default_rng(seed + 1000)
    return _finish("paper_scale", csr, c, k, speeds, bandwidth, _uniform_assignments(arng, P, n, k))


_BUILDERS = {
    "paper_scale": (6, _paper_scale),
    "tiny": (1, _tiny),
    "mlp": (2, _mlp),
    "inception": (3, _inception),
    "large_sparse": (4, _large_sparse),
    "comm_heavy": (5, _comm_heavy),
}


def make_workload(name: str, **overrides) -> Workload:
    """Build one of the five named workloads (or "paper_scale", the scheduling simulation's own size).  Keyword overrides (P, levels,
    width, layers, shards, modules, groups, ...) give scaled-down variants of the
    same recipe for tests; `seed` replaces the default seed."""
    idx, fn = _BUILDERS[name]
    seed = overrides.pop("seed", BASE_SEED + idx)
    return fn(seed, **overrides)

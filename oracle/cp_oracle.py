"""TEST INFRASTRUCTURE: ctypes access to the C oracle (``cp_oracle.c``).

The arithmetic lives in the C file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import build_oracle

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build_oracle(force=False))
        i64p, i32p, u8p = C.POINTER(C.c_int64), C.POINTER(C.c_int32), C.POINTER(C.c_uint8)
        lib.cp_oracle_ceil_div.restype = C.c_int64
        lib.cp_oracle_ceil_div.argtypes = [C.c_int64, C.c_int64]
        lib.cp_oracle_vertex_cost.restype = C.c_int64
        lib.cp_oracle_vertex_cost.argtypes = [C.c_int64, C.c_int64]
        lib.cp_oracle_edge_cost.restype = C.c_int64
        lib.cp_oracle_edge_cost.argtypes = [C.c_int64, C.c_int, C.c_int, i64p, C.c_int]
        lib.cp_oracle_topo_order.restype = C.c_int
        lib.cp_oracle_topo_order.argtypes = [C.c_int32, i32p, i32p, i32p]
        lib.cp_oracle_eval.restype = C.c_int
        lib.cp_oracle_eval.argtypes = [C.c_int32, i32p, i32p, i64p, i64p, C.c_int, i64p, i64p,
                                       C.c_int32, u8p, i64p, i64p, i64p, u8p, C.c_int,
                                       C.POINTER(C.c_int)]
        lib.cp_oracle_critical_path.restype = C.c_int
        lib.cp_oracle_critical_path.argtypes = [C.c_int32, i32p, i32p, i64p, i64p, C.c_int, i64p, i64p,
                                                C.c_int32, u8p, C.c_int32, i32p, i32p]
        lib.cp_oracle_ranks.restype = C.c_int
        lib.cp_oracle_ranks.argtypes = [C.c_int32, i32p, i32p, i64p, i64p, i64p, i64p]
        lib.cp_oracle_pct_order.restype = C.c_int
        lib.cp_oracle_pct_order.argtypes = [C.c_int32, C.c_int, C.c_int32, u8p, i64p, i32p, i32p, C.c_int]
        lib.cp_oracle_validate.restype = C.c_int
        lib.cp_oracle_validate.argtypes = [C.c_int32, C.c_int, C.c_int32, u8p, C.c_int64, i32p, C.c_int64, i32p,
                                           u8p, i32p]
        lib.cp_oracle_neighbours.restype = C.c_int
        lib.cp_oracle_neighbours.argtypes = [C.c_int32, C.c_int, u8p, C.c_int32, i32p, u8p]
        lib.cp_oracle_argmin.restype = None
        lib.cp_oracle_argmin.argtypes = [C.c_int32, i64p, u8p, i32p, i64p]
        lib.cp_oracle_search.restype = C.c_int
        lib.cp_oracle_search.argtypes = [C.c_int32, i32p, i32p, i64p, i64p, C.c_int, i64p, i64p, u8p, C.c_int64,
                                         i32p, C.c_int64, i32p, C.c_int32, C.c_int32, i64p, i32p, C.c_int]
        lib.cp_oracle_seed.restype = C.c_int
        lib.cp_oracle_seed.argtypes = [C.c_int32, i32p, i32p, i64p, C.c_int, i64p, C.c_int32, u8p]
        lib.cp_oracle_simulate.restype = C.c_int
        lib.cp_oracle_simulate.argtypes = [C.c_int32, i32p, i32p, i64p, i64p, C.c_int, i64p, i64p, C.c_int32, u8p,
                                           C.c_int, i64p, i32p, i64p, i64p, C.c_int, C.POINTER(C.c_int)]
        _lib = lib
    return _lib


def _ptr(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def vertex_cost(c: int, s: int) -> int:
    return int(_load().cp_oracle_vertex_cost(int(c), int(s)))


def edge_cost(t: int, pu: int, pv: int, bandwidth) -> int:
    bw = np.ascontiguousarray(bandwidth, dtype=np.int64)
    return int(_load().cp_oracle_edge_cost(int(t), int(pu), int(pv), _ptr(bw, C.c_int64), bw.shape[0]))


def topo_order(n, succ_ptr, succ_idx):
    sp = np.ascontiguousarray(succ_ptr, dtype=np.int32)
    si = np.ascontiguousarray(succ_idx, dtype=np.int32)
    if si.size == 0:
        si = np.zeros(1, dtype=np.int32)
    order = np.empty(n + 1, dtype=np.int32)
    rc = _load().cp_oracle_topo_order(n, _ptr(sp, C.c_int32), _ptr(si, C.c_int32), _ptr(order, C.c_int32))
    if rc:
        raise ValueError("graph has a cycle")
    return order[:n]


def evaluate(n, succ_ptr, succ_idx, succ_t, c, speeds, bandwidth, assignments,
             want=("cp", "b", "tl", "mask"), threads=1):
    """Evaluate every row of ``assignments[P][n]``.

    Returns a dict with ``cp`` int64 [P] and, if asked for, ``b``, ``tl`` int64
    [P][n] and ``mask`` bool [P][n] (partition-major), plus ``threads`` = the
    number of threads that ran.
    """
    lib = _load()
    sp = np.ascontiguousarray(succ_ptr, dtype=np.int32)
    si = np.ascontiguousarray(succ_idx, dtype=np.int32)
    st = np.ascontiguousarray(succ_t, dtype=np.int64)
    if si.size == 0:  # keep the pointers valid for m = 0
        si = np.zeros(1, dtype=np.int32)
        st = np.zeros(1, dtype=np.int64)
    cc = np.ascontiguousarray(c, dtype=np.int64)
    s = np.ascontiguousarray(speeds, dtype=np.int64)
    bw = np.ascontiguousarray(bandwidth, dtype=np.int64)
    a = np.ascontiguousarray(assignments, dtype=np.uint8)
    k = int(s.shape[0])
    assert bw.shape == (k, k), "bandwidth must be k x k"
    assert a.ndim == 2 and a.shape[1] == n, "assignments must be [P][n]"
    assert sp.shape[0] == n + 1
    P = int(a.shape[0])
    cp = np.zeros(P, dtype=np.int64)
    b = np.zeros((P, n), dtype=np.int64) if "b" in want else None
    tl = np.zeros((P, n), dtype=np.int64) if "tl" in want else None
    mask = np.zeros((P, n), dtype=np.uint8) if "mask" in want else None
    used = C.c_int(0)
    null64 = C.POINTER(C.c_int64)()
    null8 = C.POINTER(C.c_uint8)()
    rc = lib.cp_oracle_eval(
        n, _ptr(sp, C.c_int32), _ptr(si, C.c_int32), _ptr(st, C.c_int64), _ptr(cc, C.c_int64),
        k, _ptr(s, C.c_int64), _ptr(bw, C.c_int64), P, _ptr(a, C.c_uint8), _ptr(cp, C.c_int64),
        _ptr(b, C.c_int64) if b is not None else null64,
        _ptr(tl, C.c_int64) if tl is not None else null64,
        _ptr(mask, C.c_uint8) if mask is not None else null8,
        int(threads), C.byref(used))
    if rc == -1:
        raise ValueError("graph has a cycle")
    if rc == -3:
        raise ValueError("bad argument (device id >= k, speed < 1, bandwidth < 1 or negative weight)")
    if rc:
        raise MemoryError("oracle ran out of memory")
    out = {"cp": cp, "threads": int(used.value)}
    if b is not None:
        out["b"] = b
    if tl is not None:
        out["tl"] = tl
    if mask is not None:
        out["mask"] = mask.astype(bool)
    return out


def evaluate_workload(w, want=("cp", "b", "tl", "mask"), threads=1, partitions=None):
    a = w.assignments if partitions is None else w.assignments[partitions]
    return evaluate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth, a,
                    want=want, threads=threads)


def critical_path(n, succ_ptr, succ_idx, succ_t, c, speeds, bandwidth, assignments, max_len):
    """One critical path per row of ``assignments``: the lexicographically smallest
    source-to-sink vertex sequence of cost CP.  Returns (paths int32 [P][max_len]
    padded with -1, lengths int32 [P])."""
    lib = _load()
    sp = np.ascontiguousarray(succ_ptr, dtype=np.int32)
    si = np.ascontiguousarray(succ_idx, dtype=np.int32)
    st = np.ascontiguousarray(succ_t, dtype=np.int64)
    if si.size == 0:
        si = np.zeros(1, dtype=np.int32)
        st = np.zeros(1, dtype=np.int64)
    cc = np.ascontiguousarray(c, dtype=np.int64)
    s = np.ascontiguousarray(speeds, dtype=np.int64)
    bw = np.ascontiguousarray(bandwidth, dtype=np.int64)
    a = np.ascontiguousarray(assignments, dtype=np.uint8)
    P = int(a.shape[0])
    paths = np.full((P, max_len), -1, dtype=np.int32)
    lens = np.zeros(P, dtype=np.int32)
    rc = lib.cp_oracle_critical_path(n, _ptr(sp, C.c_int32), _ptr(si, C.c_int32), _ptr(st, C.c_int64),
                                     _ptr(cc, C.c_int64), int(s.shape[0]), _ptr(s, C.c_int64),
                                     _ptr(bw, C.c_int64), P, _ptr(a, C.c_uint8), int(max_len),
                                     _ptr(paths, C.c_int32), _ptr(lens, C.c_int32))
    if rc:
        raise ValueError(f"critical_path failed with code {rc}")
    return paths, lens


def ranks(n, succ_ptr, succ_idx, c):
    """upRank, downRank and totalRank of section 3.2 (each int64 [n])."""
    lib = _load()
    sp = np.ascontiguousarray(succ_ptr, dtype=np.int32)
    si = np.ascontiguousarray(succ_idx, dtype=np.int32)
    if si.size == 0:
        si = np.zeros(1, dtype=np.int32)
    cc = np.ascontiguousarray(c, dtype=np.int64)
    up = np.zeros(n, dtype=np.int64)
    down = np.zeros(n, dtype=np.int64)
    total = np.zeros(n, dtype=np.int64)
    rc = lib.cp_oracle_ranks(n, _ptr(sp, C.c_int32), _ptr(si, C.c_int32), _ptr(cc, C.c_int64),
                             _ptr(up, C.c_int64), _ptr(down, C.c_int64), _ptr(total, C.c_int64))
    if rc:
        raise ValueError(f"ranks failed with code {rc}")
    return up, down, total


def pct_order(k, assignments, b, threads=0):
    """PCT priority lists (section 4.1): per row of ``assignments`` [P][n] and ``b`` [P][n],
    the vertices grouped by device and, inside a device, by descending b then ascending
    vertex number.  Returns (order int32 [P][n], seg int32 [P][k+1])."""
    lib = _load()
    a = np.ascontiguousarray(assignments, dtype=np.uint8)
    bb = np.ascontiguousarray(b, dtype=np.int64)
    P, n = a.shape
    assert bb.shape == (P, n)
    order = np.zeros((P, n), dtype=np.int32)
    seg = np.zeros((P, k + 1), dtype=np.int32)
    rc = lib.cp_oracle_pct_order(n, int(k), P, _ptr(a, C.c_uint8), _ptr(bb, C.c_int64), _ptr(order, C.c_int32),
                                 _ptr(seg, C.c_int32), int(threads))
    if rc:
        raise ValueError(f"pct_order failed with code {rc}")
    return order, seg


def validate(k, assignments, pairs, pins):
    """Section 2's collocation pairs (each [v_i, v_j]) and device constraints (each
    [v_i, d_j]) checked for every row of ``assignments``.  Returns (valid uint8 [P],
    violations int32 [P])."""
    lib = _load()
    a = np.ascontiguousarray(assignments, dtype=np.uint8)
    P, n = a.shape
    pr = np.ascontiguousarray(np.asarray(pairs, dtype=np.int32).reshape(-1, 2))
    pn = np.ascontiguousarray(np.asarray(pins, dtype=np.int32).reshape(-1, 2))
    pr_arg = pr if pr.size else np.zeros((1, 2), dtype=np.int32)
    pn_arg = pn if pn.size else np.zeros((1, 2), dtype=np.int32)
    valid = np.zeros(P, dtype=np.uint8)
    broken = np.zeros(P, dtype=np.int32)
    rc = lib.cp_oracle_validate(n, int(k), P, _ptr(a, C.c_uint8), pr.shape[0], _ptr(pr_arg, C.c_int32),
                                pn.shape[0], _ptr(pn_arg, C.c_int32), _ptr(valid, C.c_uint8),
                                _ptr(broken, C.c_int32))
    if rc:
        raise ValueError(f"validate failed with code {rc}")
    return valid, broken


def neighbours(k, base, path):
    """All partitions that differ from ``base`` in exactly one vertex of ``path``:
    uint8 [len(path) * (k-1)][n], candidate i*(k-1)+r moves path[i] to the r-th device
    other than its own."""
    lib = _load()
    b = np.ascontiguousarray(base, dtype=np.uint8)
    pth = np.ascontiguousarray(path, dtype=np.int32)
    out = np.zeros((len(pth) * (k - 1), b.shape[0]), dtype=np.uint8)
    if out.size:
        rc = lib.cp_oracle_neighbours(b.shape[0], int(k), _ptr(b, C.c_uint8), len(pth), _ptr(pth, C.c_int32),
                                      _ptr(out, C.c_uint8))
        if rc:
            raise ValueError(f"neighbours failed with code {rc}")
    return out


def argmin(cp, valid=None):
    """(index, value) of the lowest-index minimum of ``cp`` over the valid entries;
    (-1, None) when there is none."""
    lib = _load()
    c = np.ascontiguousarray(cp, dtype=np.int64)
    idx = C.c_int32(-1)
    val = C.c_int64(0)
    vptr = None
    if valid is not None:
        v = np.ascontiguousarray(valid, dtype=np.uint8)
        vptr = _ptr(v, C.c_uint8)
    lib.cp_oracle_argmin(len(c), _ptr(c if len(c) else np.zeros(1, dtype=np.int64), C.c_int64), vptr,
                         C.byref(idx), C.byref(val))
    return (int(idx.value), int(val.value)) if idx.value >= 0 else (-1, None)


def search(n, succ_ptr, succ_idx, succ_t, c, speeds, bandwidth, start, max_len, pairs=(), pins=(),
           max_moves=1000, threads=1):
    """Critical-path move search from ``start`` (uint8 [n]).  Returns (assignment,
    cp_trace int64 [moves+1], moves int32 [moves][2] = {vertex, new device})."""
    lib = _load()
    sp = np.ascontiguousarray(succ_ptr, dtype=np.int32)
    si = np.ascontiguousarray(succ_idx, dtype=np.int32)
    st = np.ascontiguousarray(succ_t, dtype=np.int64)
    if si.size == 0:
        si = np.zeros(1, dtype=np.int32)
        st = np.zeros(1, dtype=np.int64)
    cc = np.ascontiguousarray(c, dtype=np.int64)
    s = np.ascontiguousarray(speeds, dtype=np.int64)
    bw = np.ascontiguousarray(bandwidth, dtype=np.int64)
    a = np.array(start, dtype=np.uint8).copy()
    pr = np.ascontiguousarray(np.asarray(pairs, dtype=np.int32).reshape(-1, 2))
    pn = np.ascontiguousarray(np.asarray(pins, dtype=np.int32).reshape(-1, 2))
    pr_arg = pr if pr.size else np.zeros((1, 2), dtype=np.int32)
    pn_arg = pn if pn.size else np.zeros((1, 2), dtype=np.int32)
    trace = np.zeros(max_moves + 1, dtype=np.int64)
    moves = np.zeros((max(max_moves, 1), 2), dtype=np.int32)
    rc = lib.cp_oracle_search(n, _ptr(sp, C.c_int32), _ptr(si, C.c_int32), _ptr(st, C.c_int64),
                              _ptr(cc, C.c_int64), int(s.shape[0]), _ptr(s, C.c_int64), _ptr(bw, C.c_int64),
                              _ptr(a, C.c_uint8), pr.shape[0], _ptr(pr_arg, C.c_int32), pn.shape[0],
                              _ptr(pn_arg, C.c_int32), int(max_moves), int(max_len), _ptr(trace, C.c_int64),
                              _ptr(moves, C.c_int32), int(threads))
    if rc < 0:
        raise ValueError(f"search failed with code {rc}")
    return a, trace[:rc + 1].copy(), moves[:rc].copy()


def seed(n, succ_ptr, succ_idx, c, speeds, max_len):
    """The paper's Critical Path partitioning strategy (section 3.2.2): uint8 [n]."""
    lib = _load()
    sp = np.ascontiguousarray(succ_ptr, dtype=np.int32)
    si = np.ascontiguousarray(succ_idx, dtype=np.int32)
    if si.size == 0:
        si = np.zeros(1, dtype=np.int32)
    cc = np.ascontiguousarray(c, dtype=np.int64)
    s = np.ascontiguousarray(speeds, dtype=np.int64)
    out = np.zeros(n, dtype=np.uint8)
    rc = lib.cp_oracle_seed(n, _ptr(sp, C.c_int32), _ptr(si, C.c_int32), _ptr(cc, C.c_int64), int(s.shape[0]),
                            _ptr(s, C.c_int64), int(max_len), _ptr(out, C.c_uint8))
    if rc:
        raise ValueError(f"seed failed with code {rc}")
    return out


FIFO, PCT = 0, 1


def simulate(n, succ_ptr, succ_idx, succ_t, c, speeds, bandwidth, assignments, policy, b=None, tie=None,
             want_start=True, threads=1):
    """List-scheduling simulation (paper, section 4 criteria, section 4.1 PCT, section 5.1 FIFO) of
    every row of ``assignments[P][n]``.  ``b`` int64 [P][n] is needed for PCT, ``tie`` int32 [n]
    (optional) orders FIFO's equal ready times.  Returns {"makespan": int64 [P], "start": int64
    [P][n] (if asked for), "threads": threads that ran}."""
    lib = _load()
    sp = np.ascontiguousarray(succ_ptr, dtype=np.int32)
    si = np.ascontiguousarray(succ_idx, dtype=np.int32)
    st = np.ascontiguousarray(succ_t, dtype=np.int64)
    if si.size == 0:
        si = np.zeros(1, dtype=np.int32)
        st = np.zeros(1, dtype=np.int64)
    cc = np.ascontiguousarray(c, dtype=np.int64)
    s = np.ascontiguousarray(speeds, dtype=np.int64)
    bw = np.ascontiguousarray(bandwidth, dtype=np.int64)
    a = np.ascontiguousarray(assignments, dtype=np.uint8)
    k = int(s.shape[0])
    assert bw.shape == (k, k) and a.ndim == 2 and a.shape[1] == n and sp.shape[0] == n + 1
    P = int(a.shape[0])
    bb = None
    if b is not None:
        bb = np.ascontiguousarray(b, dtype=np.int64)
        assert bb.shape == (P, n)
    tt = None
    if tie is not None:
        tt = np.ascontiguousarray(tie, dtype=np.int32)
        assert tt.shape == (n,)
    makespan = np.zeros(P, dtype=np.int64)
    start = np.zeros((P, n), dtype=np.int64) if want_start else None
    used = C.c_int(0)
    rc = lib.cp_oracle_simulate(
        n, _ptr(sp, C.c_int32), _ptr(si, C.c_int32), _ptr(st, C.c_int64), _ptr(cc, C.c_int64),
        k, _ptr(s, C.c_int64), _ptr(bw, C.c_int64), P, _ptr(a, C.c_uint8), int(policy),
        _ptr(bb, C.c_int64) if bb is not None else C.POINTER(C.c_int64)(),
        _ptr(tt, C.c_int32) if tt is not None else C.POINTER(C.c_int32)(),
        _ptr(makespan, C.c_int64),
        _ptr(start, C.c_int64) if start is not None else C.POINTER(C.c_int64)(),
        int(threads), C.byref(used))
    if rc == -1:
        raise ValueError("graph has a cycle")
    if rc == -3:
        raise ValueError("bad argument (see cp_oracle_simulate)")
    if rc:
        raise MemoryError("oracle ran out of memory")
    out = {"makespan": makespan, "threads": int(used.value)}
    if start is not None:
        out["start"] = start
    return out

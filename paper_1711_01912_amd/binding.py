"""ctypes binding of the C ABI in ``include/cpeval.h``.

Names follow the C entry points.  Nothing is computed here: tensors are
allocated with torch, pointers and sizes are handed to the library, and every
step of the evaluation runs in the library's kernels.  If the shared library is
missing the import of this module still works (so that the build can be checked
without a GPU), but any call raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcpeval.so")

TICK_I32, TICK_I64 = 4, 8
ASSIGN_PARTITION_MAJOR, ASSIGN_VERTEX_MAJOR = 0, 1
OUT_VERTEX_MAJOR, OUT_PARTITION_MAJOR = 0, 1
PLAN_AUTO, PLAN_WAVE_COLUMN, PLAN_RESIDENT_WINDOW, PLAN_SHARED_WINDOW_2, PLAN_SHARED_WINDOW_4 = 0, 1, 2, 3, 4
PLAN_COLUMN_SLICE, PLAN_STREAMED_WINDOW = 5, 6
NUM_STAGES = 5
STAGE_NAMES = ("prep", "blevel", "cp", "tlevel", "mask")
STATUS_BAD_DEVICE_ID = 1

EXPORTS = (
    "cp_graph_create", "cp_graph_get_info", "cp_graph_upload", "cp_graph_destroy",
    "cp_eval_workspace_bytes", "cp_eval_choose_plan", "cp_eval", "cp_eval_static", "cp_critical_path", "cp_ranks_workspace_bytes", "cp_ranks",
    "cp_pct_order_workspace_bytes", "cp_pct_order", "cp_validate",
    "cp_search_workspace_bytes", "cp_search", "cp_seed_workspace_bytes", "cp_seed_partition",
    "cp_simulate_workspace_bytes", "cp_simulate",
    "cp_profile_create", "cp_profile_reset",
    "cp_profile_count", "cp_profile_read", "cp_profile_destroy", "cp_cost_magic",
    "cp_error_string", "cp_cost_compact", "cp_window_shape",
)


class GraphInfo(C.Structure):
    _fields_ = [
        ("n", C.c_int32), ("L", C.c_int32), ("m", C.c_int64),
        ("max_out_degree", C.c_int32), ("max_in_degree", C.c_int32), ("max_level_width", C.c_int32),
        ("num_sources", C.c_int32), ("num_sinks", C.c_int32),
        ("max_c", C.c_int64), ("max_t", C.c_int64), ("raw_path_bound", C.c_int64),
        ("min_tick_bytes", C.c_int32), ("window_ok", C.c_int32),
        ("window_slots_b", C.c_int32), ("window_slots_t", C.c_int32),
        ("window_packet_bytes_b", C.c_int32), ("window_packet_bytes_t", C.c_int32),
        ("window_far_b", C.c_int32), ("window_far_t", C.c_int32),
        ("window_ticks_b", C.c_int32), ("window_ticks_t", C.c_int32),
        ("window_slices_b", C.c_int32), ("window_slices_t", C.c_int32),
        ("auto_plan", C.c_int32), ("uploaded", C.c_int32), ("blob_bytes", C.c_uint64),
    ]

    def as_dict(self):
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


class CpError(RuntimeError):
    def __init__(self, code, where):
        self.code = int(code)
        super().__init__(f"{where}: {error_string(code)} (code {code})")


_lib = None


def load_library():
    """Load ``libcpeval.so`` from the package directory; fails loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    # PyTorch first: it brings its own HIP runtime, and device memory handed over by torch must
    # belong to the runtime this library calls.  The library's dependency then resolves to it.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    i32p, i64p, u8p = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_uint8)
    vp = C.c_void_p
    lib.cp_graph_create.restype = C.c_int
    lib.cp_graph_create.argtypes = [C.c_int32, C.c_int64, C.c_int32, i32p, i32p, i64p, i32p, i32p,
                                    i32p, i64p, i32p, i32p, C.POINTER(vp)]
    lib.cp_graph_get_info.restype = C.c_int
    lib.cp_graph_get_info.argtypes = [vp, C.POINTER(GraphInfo)]
    lib.cp_graph_upload.restype = C.c_int
    lib.cp_graph_upload.argtypes = [vp, vp, C.c_size_t, vp]
    lib.cp_graph_destroy.restype = None
    lib.cp_graph_destroy.argtypes = [vp]
    lib.cp_eval_workspace_bytes.restype = C.c_int
    lib.cp_eval_workspace_bytes.argtypes = [vp, C.c_int32, C.c_int32, C.c_int, C.c_int, C.c_int, C.c_int,
                                            C.POINTER(C.c_size_t)]
    lib.cp_eval_choose_plan.restype = C.c_int
    lib.cp_eval_choose_plan.argtypes = [vp, C.c_int32, C.c_int32, i64p, i64p, C.c_int, C.POINTER(C.c_int)]
    lib.cp_eval.restype = C.c_int
    lib.cp_eval.argtypes = [vp, C.c_int32, C.c_int32, vp, C.c_int, i64p, i64p, vp, C.c_size_t, vp,
                            vp, vp, vp, vp, C.c_int, C.c_int, C.c_int, vp, vp]
    lib.cp_eval_static.restype = C.c_int
    lib.cp_eval_static.argtypes = [vp, C.c_int32, C.c_int32, vp, C.c_int, i64p, i64p, vp,
                                   vp, vp, vp, vp, C.c_int, C.c_int, C.c_int, vp]
    lib.cp_critical_path.restype = C.c_int
    lib.cp_critical_path.argtypes = [vp, C.c_int32, C.c_int32, vp, C.c_int, i64p, i64p, vp, vp, C.c_int, C.c_int,
                                     vp, C.c_size_t, vp, C.c_int32, vp, vp, vp]
    lib.cp_pct_order_workspace_bytes.restype = C.c_int
    lib.cp_pct_order_workspace_bytes.argtypes = [vp, C.c_int32, C.c_int32, C.c_int64, C.POINTER(C.c_size_t)]
    lib.cp_pct_order.restype = C.c_int
    lib.cp_pct_order.argtypes = [vp, C.c_int32, C.c_int32, vp, C.c_int, vp, C.c_int, C.c_int, C.c_int64,
                                 vp, C.c_size_t, vp, vp, vp, vp]
    lib.cp_validate.restype = C.c_int
    lib.cp_validate.argtypes = [C.c_int32, C.c_int32, C.c_int32, vp, C.c_int, C.c_int64, vp, C.c_int64, vp, vp,
                                vp, vp, vp]
    lib.cp_seed_workspace_bytes.restype = C.c_int
    lib.cp_seed_workspace_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
    lib.cp_seed_partition.restype = C.c_int
    lib.cp_seed_partition.argtypes = [vp, C.c_int32, i64p, vp, C.c_size_t, vp, vp, vp]
    lib.cp_search_workspace_bytes.restype = C.c_int
    lib.cp_search_workspace_bytes.argtypes = [vp, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
    lib.cp_search.restype = C.c_int
    lib.cp_search.argtypes = [vp, C.c_int32, i64p, i64p, vp, C.c_int64, vp, C.c_int64, vp, C.c_int32, C.c_int32,
                              vp, C.c_size_t, vp, i64p, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                              C.POINTER(C.c_int64)]
    lib.cp_simulate_workspace_bytes.restype = C.c_int
    lib.cp_simulate_workspace_bytes.argtypes = [vp, C.c_int32, C.c_int32, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    lib.cp_simulate.restype = C.c_int
    lib.cp_simulate.argtypes = [vp, C.c_int32, C.c_int32, vp, C.c_int, i64p, i64p, C.c_int, vp, C.c_int, C.c_int,
                                vp, vp, C.c_size_t, vp, vp, vp, vp]
    lib.cp_ranks_workspace_bytes.restype = C.c_int
    lib.cp_ranks_workspace_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
    lib.cp_ranks.restype = C.c_int
    lib.cp_ranks.argtypes = [vp, vp, C.c_size_t, vp, vp, vp, vp]
    lib.cp_profile_create.restype = C.c_int
    lib.cp_profile_create.argtypes = [C.c_int32, C.POINTER(vp)]
    lib.cp_profile_reset.restype = C.c_int
    lib.cp_profile_reset.argtypes = [vp]
    lib.cp_profile_count.restype = C.c_int
    lib.cp_profile_count.argtypes = [vp, i32p]
    lib.cp_profile_read.restype = C.c_int
    lib.cp_profile_read.argtypes = [vp, C.c_int32, C.POINTER(C.c_float), i32p]
    lib.cp_profile_destroy.restype = None
    lib.cp_profile_destroy.argtypes = [vp]
    lib.cp_cost_magic.restype = C.c_int
    lib.cp_cost_magic.argtypes = [C.c_int64, C.c_int64, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
    lib.cp_error_string.restype = C.c_char_p
    lib.cp_window_shape.restype = C.c_int
    lib.cp_window_shape.argtypes = [C.c_void_p, C.c_int32, C.c_int, C.c_int, C.POINTER(C.c_int32)]
    lib.cp_cost_compact.restype = C.c_int
    lib.cp_cost_compact.argtypes = [C.c_int64, C.c_int64, C.POINTER(C.c_uint32)]
    lib.cp_error_string.argtypes = [C.c_int]
    _lib = lib
    return lib


def error_string(code: int) -> str:
    return load_library().cp_error_string(int(code)).decode()


def cost_magic(divisor: int, max_dividend: int):
    """(mul, dm1) of the exact multiply-shift form, or None if there is none."""
    mul, dm1 = C.c_uint32(0), C.c_uint32(0)
    rc = load_library().cp_cost_magic(int(divisor), int(max_dividend), C.byref(mul), C.byref(dm1))
    if rc < 0:
        raise CpError(rc, "cp_cost_magic")
    return (int(mul.value), int(dm1.value)) if rc == 1 else None


def cost_compact(divisor: int, max_dividend: int):
    """The 4-byte table entry for ceil(a / divisor), 0 <= a <= max_dividend, or None where that form is not exact."""
    e = C.c_uint32(0)
    rc = load_library().cp_cost_compact(int(divisor), int(max_dividend), C.byref(e))
    if rc < 0:
        raise CpError(rc, "cp_cost_compact")
    return int(e.value) if rc == 1 else None


def _np_ptr(a, ctype):
    if a is None:
        return C.POINTER(ctype)()
    return a.ctypes.data_as(C.POINTER(ctype))


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(int(s.cuda_stream))


class CpGraph:
    """cp_graph_create (+ cp_graph_upload when a device is given)."""

    def __init__(self, n, succ_ptr, succ_idx, succ_t, pred_ptr, pred_idx, pred_eid, c,
                 level_ptr, level_vtx, device=None, m=None, L=None):
        lib = load_library()
        self._lib = lib
        self._handle = C.c_void_p()
        self.blob = None
        a32 = lambda x: None if x is None else np.ascontiguousarray(x, dtype=np.int32)
        a64 = lambda x: None if x is None else np.ascontiguousarray(x, dtype=np.int64)
        sp, si, st = a32(succ_ptr), a32(succ_idx), a64(succ_t)
        pp, pi, pe = a32(pred_ptr), a32(pred_idx), a32(pred_eid)
        cc, lp, lv = a64(c), a32(level_ptr), a32(level_vtx)
        if m is None:
            m = 0 if si is None else int(si.shape[0])
        if L is None:
            L = int(lp.shape[0]) - 1
        rc = lib.cp_graph_create(int(n), int(m), int(L), _np_ptr(sp, C.c_int32), _np_ptr(si, C.c_int32),
                                 _np_ptr(st, C.c_int64), _np_ptr(pp, C.c_int32), _np_ptr(pi, C.c_int32),
                                 _np_ptr(pe, C.c_int32), _np_ptr(cc, C.c_int64), _np_ptr(lp, C.c_int32),
                                 _np_ptr(lv, C.c_int32), C.byref(self._handle))
        if rc:
            self._handle = C.c_void_p()
            raise CpError(rc, "cp_graph_create")
        if device is not None:
            self.upload(device)

    @classmethod
    def from_workload(cls, w, device=None):
        return cls(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.pred_ptr, w.pred_idx, w.pred_eid,
                   w.c, w.level_ptr, w.level_vtx, device=device)

    @property
    def info(self) -> dict:
        gi = GraphInfo()
        rc = self._lib.cp_graph_get_info(self._handle, C.byref(gi))
        if rc:
            raise CpError(rc, "cp_graph_get_info")
        return gi.as_dict()

    def window_shape(self, k: int, tsweep: bool = False, tick_dtype: int = TICK_I32) -> dict:
        """cp_window_shape: the resident-window plan's workgroup shape for one sweep, or None where the plan
        does not apply."""
        out = (C.c_int32 * 8)()
        rc = self._lib.cp_window_shape(self._handle, int(k), int(tick_dtype), int(bool(tsweep)), out)
        if rc == -12:
            return None
        if rc:
            raise CpError(rc, "cp_window_shape")
        names = ("loads_per_lane", "loader_waves", "far_waves", "compute_waves", "prefetch_ticks",
                 "partitions_per_workgroup", "stores_per_tick", "lds_bytes")
        return dict(zip(names, (int(v) for v in out)))

    def upload(self, device="cuda:0", stream=None):
        import torch
        nbytes = self.info["blob_bytes"]
        self.blob = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        rc = self._lib.cp_graph_upload(self._handle, C.c_void_p(self.blob.data_ptr()),
                                       C.c_size_t(self.blob.numel()), _stream_ptr(stream))
        if rc:
            raise CpError(rc, "cp_graph_upload")
        return self

    def close(self):
        if getattr(self, "_handle", None) is not None and self._handle:
            self._lib.cp_graph_destroy(self._handle)
            self._handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class CpProfile:
    """cp_profile_*: per-stage HIP-event timing of cp_eval calls."""

    def __init__(self, slots: int):
        self._lib = load_library()
        self._handle = C.c_void_p()
        rc = self._lib.cp_profile_create(int(slots), C.byref(self._handle))
        if rc:
            raise CpError(rc, "cp_profile_create")

    def reset(self):
        rc = self._lib.cp_profile_reset(self._handle)
        if rc:
            raise CpError(rc, "cp_profile_reset")

    def count(self) -> int:
        out = C.c_int32(0)
        rc = self._lib.cp_profile_count(self._handle, C.byref(out))
        if rc:
            raise CpError(rc, "cp_profile_count")
        return int(out.value)

    def read(self, slot: int):
        """(ms per stage as a dict, (b-level launches, t-level launches)); synchronise first."""
        ms = (C.c_float * NUM_STAGES)()
        launches = (C.c_int32 * 2)()
        rc = self._lib.cp_profile_read(self._handle, int(slot), ms, launches)
        if rc:
            raise CpError(rc, "cp_profile_read")
        return {STAGE_NAMES[i]: float(ms[i]) for i in range(NUM_STAGES)}, (int(launches[0]), int(launches[1]))

    def close(self):
        if getattr(self, "_handle", None) is not None and self._handle:
            self._lib.cp_profile_destroy(self._handle)
            self._handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def workspace_bytes(graph: CpGraph, batch: int, k: int, assign_layout=ASSIGN_PARTITION_MAJOR,
                    plan=PLAN_AUTO, out_layout=OUT_VERTEX_MAJOR, tick_bytes=None) -> int:
    out = C.c_size_t(0)
    if tick_bytes is None:
        tick_bytes = graph.info["min_tick_bytes"]
    rc = load_library().cp_eval_workspace_bytes(graph._handle, int(batch), int(k), int(assign_layout),
                                                int(plan), int(out_layout), int(tick_bytes), C.byref(out))
    if rc:
        raise CpError(rc, "cp_eval_workspace_bytes")
    return int(out.value)


def choose_plan(graph: CpGraph, batch: int, speeds, bandwidth, tick_bytes=None) -> int:
    """The plan PLAN_AUTO resolves to for this batch and cost model on the current device."""
    s = np.ascontiguousarray(speeds, dtype=np.int64)
    bw = np.ascontiguousarray(bandwidth, dtype=np.int64)
    if tick_bytes is None:
        tick_bytes = graph.info["min_tick_bytes"]
    plan = C.c_int(0)
    rc = load_library().cp_eval_choose_plan(graph._handle, int(batch), int(s.shape[0]), _np_ptr(s, C.c_int64),
                                            _np_ptr(bw, C.c_int64), int(tick_bytes), C.byref(plan))
    if rc:
        raise CpError(rc, "cp_eval_choose_plan")
    return int(plan.value)


def cp_eval(graph: CpGraph, assignments, speeds, bandwidth, *, want=("cp", "b", "tl", "mask"),
            tick_bytes=None, plan=PLAN_AUTO, assign_layout=ASSIGN_PARTITION_MAJOR,
            out_layout=OUT_VERTEX_MAJOR, out=None, workspace=None, profile: CpProfile | None = None,
            stream=None, check_status=True, static=False):
    """cp_eval on torch tensors.

    ``assignments``: uint8 CUDA tensor, [batch][n] (or [n][batch] with
    ``assign_layout=ASSIGN_VERTEX_MAJOR``).  Returns a dict with the requested
    tensors: ``cp`` int64 [batch]; ``b``, ``tl`` int32/int64 [n][batch];
    ``mask`` uint64-as-int64 words [n][ceil(batch/64)] (with
    ``out_layout=OUT_PARTITION_MAJOR``: [batch][n] and [batch][ceil(n/64)]); plus
    ``status`` (int32 tensor).  ``out`` may carry preallocated tensors under the same keys and
    ``workspace`` a preallocated uint8 tensor.  With ``check_status`` the stream
    is synchronised and a bad device id raises.  ``static=True`` goes through
    ``cp_eval_static`` (the library's fixed scratch array instead of a workspace).
    """
    import torch
    lib = load_library()
    info = graph.info
    n = info["n"]
    assert assignments.is_cuda and assignments.dtype == torch.uint8 and assignments.is_contiguous()
    if assign_layout == ASSIGN_PARTITION_MAJOR:
        batch = int(assignments.shape[0])
        assert int(assignments.shape[1]) == n
    else:
        batch = int(assignments.shape[1])
        assert int(assignments.shape[0]) == n
    s = np.ascontiguousarray(speeds, dtype=np.int64)
    bw = np.ascontiguousarray(bandwidth, dtype=np.int64)
    k = int(s.shape[0])
    assert bw.shape == (k, k)
    if tick_bytes is None:
        tick_bytes = info["min_tick_bytes"]
    tdt = torch.int32 if tick_bytes == 4 else torch.int64
    dev = assignments.device
    out = dict(out) if out else {}
    want = set(want)
    if "mask" in want:
        want |= {"cp", "b", "tl"}
    if "cp" in want and "b" not in want:
        # CP alone: the resident-window plan needs no b array for it
        used = plan if plan != PLAN_AUTO else choose_plan(graph, batch, s, bw, tick_bytes)
        if used not in (PLAN_RESIDENT_WINDOW, PLAN_SHARED_WINDOW_2, PLAN_SHARED_WINDOW_4, PLAN_STREAMED_WINDOW) or info["window_far_b"] > 0:
            want.add("b")
    rows, cols = (n, batch) if out_layout == OUT_VERTEX_MAJOR else (batch, n)
    if "cp" in want and "cp" not in out:
        out["cp"] = torch.empty(batch, dtype=torch.int64, device=dev)
    if "b" in want and "b" not in out:
        out["b"] = torch.empty((rows, cols), dtype=tdt, device=dev)
    if "tl" in want and "tl" not in out:
        out["tl"] = torch.empty((rows, cols), dtype=tdt, device=dev)
    if "mask" in want and "mask" not in out:
        out["mask"] = torch.empty((rows, (cols + 63) // 64), dtype=torch.int64, device=dev)
    if "status" not in out:
        out["status"] = torch.empty(1, dtype=torch.int32, device=dev)
    ptr = lambda key: C.c_void_p(out[key].data_ptr()) if key in want else C.c_void_p()
    if static:
        assert workspace is None and profile is None
        rc = lib.cp_eval_static(graph._handle, batch, k, C.c_void_p(assignments.data_ptr()), int(assign_layout),
                                _np_ptr(s, C.c_int64), _np_ptr(bw, C.c_int64), _stream_ptr(stream),
                                ptr("cp"), ptr("b"), ptr("tl"), ptr("mask"), int(tick_bytes), int(out_layout),
                                int(plan), C.c_void_p(out["status"].data_ptr()))
        if rc:
            raise CpError(rc, "cp_eval_static")
    else:
        if workspace is None:
            workspace = torch.empty(workspace_bytes(graph, batch, k, assign_layout, plan, out_layout, tick_bytes),
                                    dtype=torch.uint8, device=dev)
        rc = lib.cp_eval(graph._handle, batch, k, C.c_void_p(assignments.data_ptr()), int(assign_layout),
                         _np_ptr(s, C.c_int64), _np_ptr(bw, C.c_int64),
                         C.c_void_p(workspace.data_ptr()), C.c_size_t(workspace.numel()), _stream_ptr(stream),
                         ptr("cp"), ptr("b"), ptr("tl"), ptr("mask"), int(tick_bytes), int(out_layout), int(plan),
                         C.c_void_p(out["status"].data_ptr()),
                         C.c_void_p(profile._handle.value) if profile is not None else C.c_void_p())
        if rc:
            raise CpError(rc, "cp_eval")
        out["_workspace"] = workspace  # keep it alive until the caller drops the result
    if check_status:
        torch.cuda.synchronize(dev)
        st = int(out["status"].item())
        if st == STATUS_BAD_DEVICE_ID:
            raise ValueError("assignments holds a device id >= k")
    return out


def cp_eval_static(graph: CpGraph, assignments, speeds, bandwidth, **kw):
    """cp_eval_static on torch tensors: cp_eval without a workspace (the library's fixed
    scratch array; the call itself allocates nothing on the device).  Same keywords as
    cp_eval except ``workspace`` and ``profile``; pass ``out`` to keep torch from allocating
    the results."""
    return cp_eval(graph, assignments, speeds, bandwidth, static=True, **kw)


def cp_critical_path(graph: CpGraph, assignments, speeds, bandwidth, b, cp, *,
                     assign_layout=ASSIGN_PARTITION_MAJOR, b_layout=OUT_VERTEX_MAJOR, workspace=None,
                     stream=None, check_status=True):
    """cp_critical_path on torch tensors: ``b`` and ``cp`` are outputs of cp_eval for the
    same assignments and cost model.  Returns (paths int32 [batch][L] padded with -1,
    lengths int32 [batch])."""
    import torch
    lib = load_library()
    info = graph.info
    s = np.ascontiguousarray(speeds, dtype=np.int64)
    bw = np.ascontiguousarray(bandwidth, dtype=np.int64)
    k = int(s.shape[0])
    batch = int(cp.shape[0])
    dev = assignments.device
    max_len = info["L"]
    paths = torch.empty((batch, max_len), dtype=torch.int32, device=dev)
    lens = torch.empty(batch, dtype=torch.int32, device=dev)
    status = torch.empty(1, dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = torch.empty(workspace_bytes(graph, batch, k, assign_layout), dtype=torch.uint8, device=dev)
    tick = 4 if b.dtype == torch.int32 else 8
    rc = lib.cp_critical_path(graph._handle, batch, k, C.c_void_p(assignments.data_ptr()), int(assign_layout),
                              _np_ptr(s, C.c_int64), _np_ptr(bw, C.c_int64), C.c_void_p(b.data_ptr()),
                              C.c_void_p(cp.data_ptr()), tick, int(b_layout), C.c_void_p(workspace.data_ptr()),
                              C.c_size_t(workspace.numel()), _stream_ptr(stream), max_len,
                              C.c_void_p(paths.data_ptr()), C.c_void_p(lens.data_ptr()),
                              C.c_void_p(status.data_ptr()))
    if rc:
        raise CpError(rc, "cp_critical_path")
    if check_status:
        torch.cuda.synchronize(dev)
        if int(status.item()) == STATUS_BAD_DEVICE_ID:
            raise ValueError("assignments holds a device id >= k")
    return paths, lens


STATUS_B_OUT_OF_RANGE = 2


def cp_pct_order(graph: CpGraph, assignments, k: int, b, *, max_b: int = 0,
                 assign_layout=ASSIGN_PARTITION_MAJOR, b_layout=OUT_VERTEX_MAJOR, workspace=None, out=None,
                 stream=None, check_status=True):
    """cp_pct_order on torch tensors: ``b`` is cp_eval's b-level output for the same
    assignments.  Returns (order int32 [batch][n], seg int32 [batch][k+1])."""
    import torch
    lib = load_library()
    n = graph.info["n"]
    batch = int(b.shape[1] if b_layout == OUT_VERTEX_MAJOR else b.shape[0])
    dev = b.device
    if workspace is None:
        need = C.c_size_t(0)
        rc = lib.cp_pct_order_workspace_bytes(graph._handle, batch, int(k), int(max_b), C.byref(need))
        if rc:
            raise CpError(rc, "cp_pct_order_workspace_bytes")
        workspace = torch.empty(need.value, dtype=torch.uint8, device=dev)
    if out is None:
        out = {"order": torch.empty((batch, n), dtype=torch.int32, device=dev),
               "seg": torch.empty((batch, int(k) + 1), dtype=torch.int32, device=dev),
               "status": torch.empty(1, dtype=torch.int32, device=dev)}
    tick = 4 if b.dtype == torch.int32 else 8
    rc = lib.cp_pct_order(graph._handle, batch, int(k), C.c_void_p(assignments.data_ptr()), int(assign_layout),
                          C.c_void_p(b.data_ptr()), tick, int(b_layout), int(max_b),
                          C.c_void_p(workspace.data_ptr()),
                          C.c_size_t(workspace.numel()), _stream_ptr(stream), C.c_void_p(out["order"].data_ptr()),
                          C.c_void_p(out["seg"].data_ptr()), C.c_void_p(out["status"].data_ptr()))
    if rc:
        raise CpError(rc, "cp_pct_order")
    if check_status:
        torch.cuda.synchronize(dev)
        st = int(out["status"].item())
        if st & STATUS_BAD_DEVICE_ID:
            raise ValueError("assignments holds a device id >= k")
        if st & STATUS_B_OUT_OF_RANGE:
            raise ValueError("some b lies outside [0, max_b]")
    return out["order"], out["seg"]


STATUS_BAD_CONSTRAINT = 4


def cp_validate(assignments, k: int, pairs=None, pins=None, *, assign_layout=ASSIGN_PARTITION_MAJOR,
                stream=None, check_status=True):
    """cp_validate on torch tensors: ``pairs`` int32 [*][2] vertices that must share a
    device, ``pins`` int32 [*][2] = {vertex, device}; both on the device of
    ``assignments`` (or None).  Returns (valid uint8 [batch], violations int32 [batch])."""
    import torch
    lib = load_library()
    dev = assignments.device
    if assign_layout == ASSIGN_PARTITION_MAJOR:
        batch, n = (int(x) for x in assignments.shape)
    else:
        n, batch = (int(x) for x in assignments.shape)

    def arg(t):
        if t is None or t.numel() == 0:
            return 0, C.c_void_p()
        assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous() and t.shape[-1] == 2
        return int(t.numel() // 2), C.c_void_p(t.data_ptr())

    n_pairs, p_pairs = arg(pairs)
    n_pins, p_pins = arg(pins)
    valid = torch.empty(batch, dtype=torch.uint8, device=dev)
    broken = torch.empty(batch, dtype=torch.int32, device=dev)
    status = torch.empty(1, dtype=torch.int32, device=dev)
    rc = lib.cp_validate(n, batch, int(k), C.c_void_p(assignments.data_ptr()), int(assign_layout), n_pairs, p_pairs,
                         n_pins, p_pins, _stream_ptr(stream), C.c_void_p(valid.data_ptr()),
                         C.c_void_p(broken.data_ptr()), C.c_void_p(status.data_ptr()))
    if rc:
        raise CpError(rc, "cp_validate")
    if check_status:
        torch.cuda.synchronize(dev)
        if int(status.item()) & STATUS_BAD_CONSTRAINT:
            raise ValueError("a constraint names a vertex >= n or a device >= k")
    return valid, broken


POLICY_FIFO, POLICY_PCT = 0, 1
STATUS_BAD_TIE, STATUS_INCOMPLETE = 8, 16


def cp_simulate(graph: CpGraph, assignments, speeds, bandwidth, policy, *, b=None, tie=None,
                assign_layout=ASSIGN_PARTITION_MAJOR, b_layout=OUT_VERTEX_MAJOR, want_start=True,
                workspace=None, stream=None, check_status=True):
    """cp_simulate on torch tensors: ``assignments`` uint8 on the GPU, ``b`` cp_eval's b-level
    output for them (POLICY_PCT), ``tie`` an int32 permutation [n] on the GPU or None
    (POLICY_FIFO).  Returns (makespan int64 [batch], start int32 [batch][n] or None)."""
    import torch
    lib = load_library()
    dev = assignments.device
    n = graph.info["n"]
    batch = int(assignments.shape[0] if assign_layout == ASSIGN_PARTITION_MAJOR else assignments.shape[1])
    s = np.ascontiguousarray(speeds, dtype=np.int64)
    bw = np.ascontiguousarray(bandwidth, dtype=np.int64)
    k = int(s.shape[0])
    if workspace is None:
        need = C.c_size_t(0)
        rc = lib.cp_simulate_workspace_bytes(graph._handle, batch, k, int(policy), int(tie is not None),
                                             C.byref(need))
        if rc:
            raise CpError(rc, "cp_simulate_workspace_bytes")
        workspace = torch.empty(need.value, dtype=torch.uint8, device=dev)
    makespan = torch.empty(batch, dtype=torch.int64, device=dev)
    start = torch.empty((batch, n), dtype=torch.int32, device=dev) if want_start else None
    status = torch.empty(1, dtype=torch.int32, device=dev)
    tick = 4
    if b is not None:
        tick = 4 if b.dtype == torch.int32 else 8
    rc = lib.cp_simulate(graph._handle, batch, k, C.c_void_p(assignments.data_ptr()), int(assign_layout),
                         _np_ptr(s, C.c_int64), _np_ptr(bw, C.c_int64), int(policy),
                         C.c_void_p(b.data_ptr()) if b is not None else C.c_void_p(), tick, int(b_layout),
                         C.c_void_p(tie.data_ptr()) if tie is not None else C.c_void_p(),
                         C.c_void_p(workspace.data_ptr()), C.c_size_t(workspace.numel()), _stream_ptr(stream),
                         C.c_void_p(makespan.data_ptr()),
                         C.c_void_p(start.data_ptr()) if start is not None else C.c_void_p(),
                         C.c_void_p(status.data_ptr()))
    if rc:
        raise CpError(rc, "cp_simulate")
    if check_status:
        torch.cuda.synchronize(dev)
        st = int(status.item())
        if st & STATUS_BAD_DEVICE_ID:
            raise ValueError("assignments holds a device id >= k")
        if st & STATUS_B_OUT_OF_RANGE:
            raise ValueError("some b lies outside [0, 2^31)")
        if st & STATUS_BAD_TIE:
            raise ValueError("tie is not a permutation of 0 .. n-1")
        if st & STATUS_INCOMPLETE:
            raise RuntimeError("a partition ended with vertices that never started")
    return makespan, start


def cp_seed_partition(graph: CpGraph, speeds, *, stream=None):
    """cp_seed_partition on the graph's device: the paper's Critical Path strategy, uint8 [n]."""
    import torch
    lib = load_library()
    dev = graph.blob.device
    s = np.ascontiguousarray(speeds, dtype=np.int64)
    need = C.c_size_t(0)
    rc = lib.cp_seed_workspace_bytes(graph._handle, C.byref(need))
    if rc:
        raise CpError(rc, "cp_seed_workspace_bytes")
    ws = torch.empty(need.value, dtype=torch.uint8, device=dev)
    out = torch.empty(graph.info["n"], dtype=torch.uint8, device=dev)
    status = torch.empty(1, dtype=torch.int32, device=dev)
    rc = lib.cp_seed_partition(graph._handle, int(s.shape[0]), _np_ptr(s, C.c_int64), C.c_void_p(ws.data_ptr()),
                               C.c_size_t(ws.numel()), _stream_ptr(stream), C.c_void_p(out.data_ptr()),
                               C.c_void_p(status.data_ptr()))
    if rc:
        raise CpError(rc, "cp_seed_partition")
    torch.cuda.synchronize(dev)          # the workspace is released on return
    return out


def cp_search(graph: CpGraph, start, speeds, bandwidth, *, pairs=None, pins=None, max_moves=1000, chunk=1024,
              stream=None):
    """cp_search on torch tensors: ``start`` is a uint8 CUDA tensor [n].  Returns a dict
    with ``assignment`` (new tensor), ``cp_trace`` (int64 numpy, CP of the start and after
    each move), ``moves`` (int32 numpy [moves][2]) and ``evaluated`` (candidates)."""
    import torch
    lib = load_library()
    dev = start.device
    s = np.ascontiguousarray(speeds, dtype=np.int64)
    bw = np.ascontiguousarray(bandwidth, dtype=np.int64)
    k = int(s.shape[0])
    a = start.clone().contiguous()

    def arg(t):
        if t is None or t.numel() == 0:
            return 0, C.c_void_p()
        assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous() and t.shape[-1] == 2
        return int(t.numel() // 2), C.c_void_p(t.data_ptr())

    n_pairs, p_pairs = arg(pairs)
    n_pins, p_pins = arg(pins)
    need = C.c_size_t(0)
    rc = lib.cp_search_workspace_bytes(graph._handle, k, int(chunk), C.byref(need))
    if rc:
        raise CpError(rc, "cp_search_workspace_bytes")
    ws = torch.empty(need.value, dtype=torch.uint8, device=dev)
    trace = np.zeros(max_moves + 1, dtype=np.int64)
    moves = np.zeros((max(max_moves, 1), 2), dtype=np.int32)
    done = C.c_int32(0)
    seen = C.c_int64(0)
    rc = lib.cp_search(graph._handle, k, _np_ptr(s, C.c_int64), _np_ptr(bw, C.c_int64), C.c_void_p(a.data_ptr()),
                       n_pairs, p_pairs, n_pins, p_pins, int(max_moves), int(chunk), C.c_void_p(ws.data_ptr()),
                       C.c_size_t(ws.numel()), _stream_ptr(stream), _np_ptr(trace, C.c_int64),
                       _np_ptr(moves, C.c_int32), C.byref(done), C.byref(seen))
    if rc:
        raise CpError(rc, "cp_search")
    return {"assignment": a, "cp_trace": trace[:done.value + 1].copy(), "moves": moves[:done.value].copy(),
            "evaluated": int(seen.value)}


def cp_ranks(graph: CpGraph, *, stream=None):
    """cp_ranks on the graph's device: returns (upRank, downRank, totalRank), int64 [n] each."""
    import torch
    lib = load_library()
    dev = graph.blob.device
    n = graph.info["n"]
    need = C.c_size_t(0)
    rc = lib.cp_ranks_workspace_bytes(graph._handle, C.byref(need))
    if rc:
        raise CpError(rc, "cp_ranks_workspace_bytes")
    ws = torch.empty(need.value, dtype=torch.uint8, device=dev)
    up, down, total = (torch.empty(n, dtype=torch.int64, device=dev) for _ in range(3))
    rc = lib.cp_ranks(graph._handle, C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()), _stream_ptr(stream),
                      C.c_void_p(up.data_ptr()), C.c_void_p(down.data_ptr()), C.c_void_p(total.data_ptr()))
    if rc:
        raise CpError(rc, "cp_ranks")
    torch.cuda.synchronize(dev)      # the workspace is released on return
    return up, down, total


def mask_to_bool(mask_words, batch: int) -> np.ndarray:
    """Unpack mask words [n][ceil(batch/64)] (host numpy or torch) into bool [n][batch]."""
    a = mask_words.cpu().numpy() if hasattr(mask_words, "cpu") else np.asarray(mask_words)
    a = np.ascontiguousarray(a).view(np.uint64)
    bits = np.unpackbits(a.view(np.uint8).reshape(a.shape[0], -1), axis=1, bitorder="little")
    return bits[:, :batch].astype(bool)

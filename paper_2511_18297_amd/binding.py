"""ctypes binding of libgroot.so: argument marshalling only.

Function names are those of ``include/groot.h``.  Host arrays are numpy, device
arrays are torch CUDA tensors (used for their memory and their stream, nothing
else); every step of the path runs inside the library.  There is no fallback:
if the shared library has not been built, importing fails.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgroot.so")

GROOT_OK, GROOT_EINVAL, GROOT_ENOMEM, GROOT_EHIP, GROOT_ERANGE = range(5)
GROOT_SYMMETRIC, GROOT_SELF_LOOPS, GROOT_NORM_MEAN = 1, 2, 4
GROOT_DEFAULT_FLAGS = GROOT_SYMMETRIC | GROOT_SELF_LOOPS | GROOT_NORM_MEAN
GROOT_REGROW = 1
GROOT_PHASE_LD, GROOT_PHASE_HD, GROOT_PHASE_FINISH, GROOT_PHASE_ALL = 1, 2, 4, 7

EXPORTS = [
    "groot_graph_build", "groot_graph_from_csr", "groot_graph_transpose", "groot_graph_view", "groot_graph_free",
    "groot_spmm_plan", "groot_plan_view", "groot_plan_upload", "groot_spmm_execute",
    "groot_spmm_execute_phases", "groot_spmm_execute_rows", "groot_plan_use_global_columns", "groot_sage_layer_forward", "groot_sage_layer_forward_io", "groot_sage_layer_backward_data", "groot_rows_over_degree", "groot_sage_layer_backward_weights", "groot_sage_layer_backward_weights_workspace", "groot_plan_lists_device", "groot_plan_lists_device_static", "groot_plan_query", "groot_plan_hd_pieces", "groot_feature_placement", "groot_plan_free", "groot_partition_regrow", "groot_parts_view",
    "groot_parts_count", "groot_parts_free", "groot_partition_regrow_device", "groot_dev_part_view",
    "groot_dev_part_plan", "groot_dev_part_download", "groot_dev_part_free", "groot_rows_gather", "groot_rows_scatter",
    "groot_set_tuning", "groot_last_error",
]

# an alternative build of the library (same ABI), for experiments
LIB_PATH = os.environ.get("GROOT_LIBRARY", LIB_PATH)
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_18297_amd.build` "
                      "(or __graft_entry__.build()); there is no fallback path")

# torch is imported first on purpose: it carries its own HIP runtime
# (libamdhip64.so.7) and the process must hold exactly one.  Loaded afterwards,
# libgroot.so binds to that same runtime through the shared soname, so device
# pointers and streams made by torch are valid inside the library.
import torch  # noqa: E402,F401

_lib = ctypes.CDLL(LIB_PATH)

_vp = ctypes.c_void_p
_i64, _i32, _u32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32
_pp = ctypes.POINTER(ctypes.c_void_p)
_pi64 = ctypes.POINTER(ctypes.c_int64)

_lib.groot_graph_build.argtypes = [_i64, _vp, _vp, _vp, _i32, _u32, _pp]
_lib.groot_graph_from_csr.argtypes = [_i64, _vp, _vp, _vp, _pp]
_lib.groot_graph_transpose.argtypes = [_vp, _pp]
_lib.groot_graph_view.argtypes = [_vp, _pi64, _pi64, _pp, _pp, _pp, _pp]
_lib.groot_graph_free.argtypes = [_vp]
_lib.groot_graph_free.restype = None
_lib.groot_spmm_plan.argtypes = [_vp, _i32, _pp]
_lib.groot_plan_view.argtypes = [_vp, _pi64, _pi64, _pp, _pp, _pp, _pp, _pp]
_lib.groot_plan_upload.argtypes = [_vp, _i32]
_lib.groot_spmm_execute.argtypes = [_vp, _vp, _vp, _i32, _vp]
_lib.groot_spmm_execute_phases.argtypes = [_vp, _vp, _vp, _i32, _u32, _vp]
_lib.groot_spmm_execute_rows.argtypes = [_vp, _vp, _vp, _i32, _i64, _vp, _vp]
_lib.groot_plan_use_global_columns.argtypes = [_vp, _vp, _i64, _vp]
_lib.groot_sage_layer_forward.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _vp, _i32, _vp]
_lib.groot_sage_layer_forward_io.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _vp, _i32, _i32, _vp]
_lib.groot_sage_layer_backward_data.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp]
_lib.groot_rows_over_degree.argtypes = [_vp, _vp, _vp, _i32, _vp]
_lib.groot_sage_layer_backward_weights_workspace.argtypes = [_vp, _i32, _i32, ctypes.POINTER(ctypes.c_size_t)]
_lib.groot_sage_layer_backward_weights.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, ctypes.c_size_t, _vp]
_lib.groot_plan_lists_device.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.groot_plan_lists_device_static.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.groot_plan_query.argtypes = [_vp, ctypes.c_char_p, _pi64]
_lib.groot_plan_hd_pieces.argtypes = [_vp, _i64, _vp, _vp, _vp, _vp]
_lib.groot_feature_placement.argtypes = [_vp, _vp, ctypes.c_size_t, _i32, _vp, ctypes.POINTER(ctypes.c_size_t),
                                         ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_float),
                                         ctypes.POINTER(ctypes.c_float)]
_lib.groot_plan_free.argtypes = [_vp]
_lib.groot_plan_free.restype = None
_lib.groot_partition_regrow.argtypes = [_vp, _i32, _vp, _u32, _pp]
_lib.groot_parts_view.argtypes = [_vp, _i32, _pi64, _pi64, _pi64, _pp, _pp]
_lib.groot_parts_count.argtypes = [_vp]
_lib.groot_parts_count.restype = _i32
_lib.groot_parts_free.argtypes = [_vp]
_lib.groot_parts_free.restype = None
_lib.groot_partition_regrow_device.argtypes = [_vp, _i32, _vp, _u32, _i32, _vp, _pp]
_lib.groot_dev_part_view.argtypes = [_vp, _pi64, _pi64, _pi64, _pi64, _pp, _pp, _pp, _pp]
_lib.groot_dev_part_plan.argtypes = [_vp, _i32, _i32, _vp, _pp]
_lib.groot_dev_part_download.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp]
_lib.groot_dev_part_free.argtypes = [_vp]
_lib.groot_dev_part_free.restype = None
_lib.groot_rows_gather.argtypes = [_vp, _i64, _vp, _vp, _i32, _vp]
_lib.groot_rows_scatter.argtypes = [_vp, _i64, _vp, _vp, _i32, _vp]
_lib.groot_set_tuning.argtypes = [ctypes.c_char_p, _i64]
_lib.groot_last_error.argtypes = []
_lib.groot_last_error.restype = ctypes.c_char_p


class GrootError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"groot status {status}: {message}")
        self.status = status


def groot_last_error() -> str:
    return _lib.groot_last_error().decode()


def _check(status: int) -> None:
    if status != GROOT_OK:
        raise GrootError(status, groot_last_error())


def _host(a, dtype):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data


def _view(ptr, count, dtype, owner):
    """numpy view (no copy) of library-owned host memory; the array keeps the
    owning Python object alive through the buffer it is built on"""
    if not ptr or count == 0:
        return np.empty(0, dtype=dtype)
    buf = (ctypes.c_char * (count * np.dtype(dtype).itemsize)).from_address(ptr)
    buf._owner = owner
    arr = np.frombuffer(buf, dtype=dtype, count=count)
    arr.flags.writeable = False
    return arr


class Graph:
    """Owner of a groot_graph handle (or a borrowed sub-graph of a Parts object)."""

    def __init__(self, handle, owner=None):
        self.handle = handle
        self._owner = owner          # keeps the parent alive for borrowed handles

    def __del__(self):
        if getattr(self, "handle", None) and self._owner is None and _lib is not None:
            _lib.groot_graph_free(self.handle)
            self.handle = None


class Plan:
    def __init__(self, handle, graph: Graph):
        self.handle = handle
        self.graph = graph           # the plan borrows its graph

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:   # module globals are cleared at interpreter exit
            _lib.groot_plan_free(self.handle)
            self.handle = None


class DevPart:
    """Owner of a groot_dev_part handle (one part of a partition, in device memory)."""

    def __init__(self, handle, plan):
        self.handle = handle
        self.plan = plan             # the plan whose graph was partitioned

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.groot_dev_part_free(self.handle)
            self.handle = None


class RawDeviceArray:
    """A library-owned device array: pointer, element count and dtype; accepted wherever a CUDA tensor of ids is."""

    def __init__(self, ptr, count, dtype, owner):
        self.device_pointer = ptr
        self.shape = (count,)
        self.dtype = np.dtype(dtype)
        self._owner = owner


class Parts:
    def __init__(self, handle, graph: Graph):
        self.handle = handle
        self.graph = graph

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.groot_parts_free(self.handle)
            self.handle = None


def groot_graph_build(type_, fanin0, fanin1, batch: int = 1, flags: int = GROOT_DEFAULT_FLAGS) -> Graph:
    t, tp = _host(type_, np.uint8)
    a, ap = _host(fanin0, np.int32)
    b, bp = _host(fanin1, np.int32)
    n1 = 0 if t is None else t.shape[0]
    out = ctypes.c_void_p()
    _check(_lib.groot_graph_build(n1, tp, ap, bp, batch, flags, ctypes.byref(out)))
    return Graph(out.value)


def groot_graph_from_csr(rowptr, col, val) -> Graph:
    r, rp = _host(rowptr, np.int64)
    c, cp = _host(col, np.int32)
    v, vp = _host(val, np.float32)
    n = 0 if r is None else r.shape[0] - 1
    out = ctypes.c_void_p()
    _check(_lib.groot_graph_from_csr(n, rp, cp, vp, ctypes.byref(out)))
    return Graph(out.value)


def groot_graph_transpose(g: Graph) -> Graph:
    out = ctypes.c_void_p()
    _check(_lib.groot_graph_transpose(g.handle, ctypes.byref(out)))
    return Graph(out.value)


def groot_graph_view(g: Graph) -> dict:
    n, nnz = _i64(0), _i64(0)
    rp, col, val, pol = (ctypes.c_void_p() for _ in range(4))
    _check(_lib.groot_graph_view(g.handle, ctypes.byref(n), ctypes.byref(nnz), ctypes.byref(rp),
                                 ctypes.byref(col), ctypes.byref(val), ctypes.byref(pol)))
    return dict(n=n.value, nnz=nnz.value,
                rowptr=_view(rp.value, n.value + 1, np.int64, g), col=_view(col.value, nnz.value, np.int32, g),
                val=_view(val.value, nnz.value, np.float32, g),
                pol=_view(pol.value, nnz.value, np.uint8, g) if pol.value else None)


def groot_spmm_plan(g: Graph, degree_threshold: int) -> Plan:
    out = ctypes.c_void_p()
    _check(_lib.groot_spmm_plan(g.handle, degree_threshold, ctypes.byref(out)))
    pl = Plan(out.value, g)
    pl.degree_threshold = degree_threshold
    n = _i64(0)
    _check(_lib.groot_graph_view(g.handle, ctypes.byref(n), None, None, None, None, None))
    pl.n_rows = n.value
    return pl


def groot_plan_view(pl: Plan) -> dict:
    n_hd, n_ld = _i64(0), _i64(0)
    rc, hd, ld, by, off = (ctypes.c_void_p() for _ in range(5))
    _check(_lib.groot_plan_view(pl.handle, ctypes.byref(n_hd), ctypes.byref(n_ld), ctypes.byref(rc),
                                ctypes.byref(hd), ctypes.byref(ld), ctypes.byref(by), ctypes.byref(off)))
    n = n_hd.value + n_ld.value
    return dict(n_hd=n_hd.value, n_ld=n_ld.value, row_class=_view(rc.value, n, np.uint8, pl),
                hd_rows=_view(hd.value, n_hd.value, np.int32, pl), ld_rows=_view(ld.value, n_ld.value, np.int32, pl),
                ld_rows_by_degree=_view(by.value, n_ld.value, np.int32, pl),
                ld_deg_offsets=_view(off.value, pl.degree_threshold + 1, np.int64, pl))


def groot_plan_upload(pl: Plan, max_F: int) -> None:
    _check(_lib.groot_plan_upload(pl.handle, max_F))


def _dev_ptr(t, what):
    import torch

    if isinstance(t, RawDeviceArray):
        return t.device_pointer
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{what} must be a contiguous CUDA tensor")
    return t.data_ptr()


def _stream_handle(stream):
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def _plan_rows(pl: Plan) -> int:
    """rows of the plan's graph (sub-graph rows for a plan built from a device part)"""
    return pl.n_rows


def _feature_rows(pl: Plan) -> int:
    """rows of the feature matrix the plan's columns index (the whole graph's once its columns are global)"""
    return getattr(pl, "n_cols", pl.n_rows)


def _features(t, what, rows, F):
    """The C ABI cannot know buffer sizes: a float32 CUDA tensor that holds at least rows x F elements, or TypeError /
    ValueError before anything is launched (a kernel that runs off a short buffer faults the GPU)."""
    import torch

    ptr = _dev_ptr(t, what)
    if t.dtype != torch.float32:
        raise TypeError(f"{what} must be float32")
    if t.dim() == 2 and t.shape[1] != F:
        raise ValueError(f"{what} has {t.shape[1]} columns, F = {F}")
    if t.numel() < rows * F:
        raise ValueError(f"{what} holds {t.numel()} elements, {rows} rows x F = {F} are needed")
    return ptr


def groot_spmm_execute(pl: Plan, X, Y, F: int = None, stream=None) -> None:
    F = X.shape[1] if F is None else F
    _check(_lib.groot_spmm_execute(pl.handle, _features(X, "X", _feature_rows(pl), F),
                                   _features(Y, "Y", _plan_rows(pl), F), F, _stream_handle(stream)))


def groot_spmm_execute_phases(pl: Plan, X, Y, F: int, phases: int, stream=None) -> None:
    _check(_lib.groot_spmm_execute_phases(pl.handle, _features(X, "X", _feature_rows(pl), F),
                                          _features(Y, "Y", _plan_rows(pl), F), F, phases, _stream_handle(stream)))


def groot_plan_use_global_columns(pl: Plan, global_id, n_global: int, stream=None) -> None:
    """global_id: the part's int64 ids on the device (tensor or library-owned array), one per row of the plan."""
    if global_id.shape[0] < _plan_rows(pl):
        raise ValueError("global_id must have one entry per row of the plan")
    _check(_lib.groot_plan_use_global_columns(pl.handle, _ids(global_id, "global_id"), n_global, _stream_handle(stream)))
    pl.n_cols = n_global


def groot_spmm_execute_rows(pl: Plan, X, Y, F: int, n_rows: int, out_ids=None, stream=None) -> None:
    """Y must hold every row that out_ids names (not checked: the ids live on the device); without out_ids it
    must hold n_rows rows."""
    import torch

    _features(X, "X", _feature_rows(pl), F)
    _features(Y, "Y", n_rows if out_ids is None else 0, F)
    if isinstance(out_ids, RawDeviceArray):
        if out_ids.dtype != np.int64 or out_ids.shape[0] < n_rows:
            raise TypeError("out_ids must be int64 with at least n_rows entries")
    elif out_ids is not None and (out_ids.dtype != torch.int64 or out_ids.numel() < n_rows):
        raise TypeError("out_ids must be int64 with at least n_rows entries")
    _check(_lib.groot_spmm_execute_rows(pl.handle, _dev_ptr(X, "X"), _dev_ptr(Y, "Y"), F, n_rows,
                                        None if out_ids is None else _dev_ptr(out_ids, "out_ids"),
                                        _stream_handle(stream)))


def groot_sage_layer_forward(pl: Plan, X, Wn, Ws, bias, relu: bool, H, F: int = None, stream=None) -> None:
    F = X.shape[1] if F is None else F
    n = _plan_rows(pl)
    _check(_lib.groot_sage_layer_forward(pl.handle, _features(X, "X", n, F), _features(Wn, "Wn", F, F),
                                         _features(Ws, "Ws", F, F),
                                         None if bias is None else _features(bias, "bias", 1, F), 1 if relu else 0,
                                         _features(H, "H", n, F), F, _stream_handle(stream)))


def groot_sage_layer_forward_io(pl: Plan, X, Wn, Ws, bias, relu: bool, H, F_in: int = None, F_out: int = None,
                                stream=None) -> None:
    """X [N, F_in], Wn and Ws [F_in, F_out], bias [F_out] or None, H [N, F_out]."""
    F_in = X.shape[1] if F_in is None else F_in
    F_out = H.shape[1] if F_out is None else F_out
    n = _plan_rows(pl)
    _check(_lib.groot_sage_layer_forward_io(pl.handle, _features(X, "X", n, F_in), _features(Wn, "Wn", F_in, F_out),
                                            _features(Ws, "Ws", F_in, F_out),
                                            None if bias is None else _features(bias, "bias", 1, F_out),
                                            1 if relu else 0, _features(H, "H", n, F_out), F_in, F_out,
                                            _stream_handle(stream)))


def groot_sage_layer_backward_data(pl: Plan, dZ_over_deg, WnT, WsT, dX, F_out: int = None, F_in: int = None,
                                   stream=None) -> None:
    """dZ_over_deg [N, F_out] (row i of dZ divided by the stored length of row i), WnT and WsT [F_out, F_in]
    (the forward layer's weights transposed), dX [N, F_in]."""
    F_out = dZ_over_deg.shape[1] if F_out is None else F_out
    F_in = dX.shape[1] if F_in is None else F_in
    n = _plan_rows(pl)
    _check(_lib.groot_sage_layer_backward_data(pl.handle, _features(dZ_over_deg, "dZ_over_deg", n, F_out),
                                               _features(WnT, "WnT", F_out, F_in), _features(WsT, "WsT", F_out, F_in),
                                               _features(dX, "dX", n, F_in), F_out, F_in, _stream_handle(stream)))


def groot_sage_layer_backward_weights_workspace(pl: Plan, F_in: int, F_out: int = None) -> int:
    """Bytes of device workspace that groot_sage_layer_backward_weights needs for X of width F_in and dZ of width
    F_out (default: F_in)."""
    b = ctypes.c_size_t(0)
    _check(_lib.groot_sage_layer_backward_weights_workspace(pl.handle, F_in, F_in if F_out is None else F_out,
                                                            ctypes.byref(b)))
    return b.value


def groot_sage_layer_backward_weights(pl: Plan, X, dZ, dWn, dWs, workspace, F_in: int = None, F_out: int = None,
                                      stream=None) -> None:
    """X [N, F_in], dZ [N, F_out], dWn and dWs [F_in, F_out] (overwritten); workspace: a contiguous device tensor of
    at least groot_sage_layer_backward_weights_workspace(pl, F_in, F_out) bytes."""
    F_in = X.shape[1] if F_in is None else F_in
    F_out = dZ.shape[1] if F_out is None else F_out
    n = _plan_rows(pl)
    _check(_lib.groot_sage_layer_backward_weights(pl.handle, _features(X, "X", n, F_in), _features(dZ, "dZ", n, F_out),
                                                  _features(dWn, "dWn", F_in, F_out), _features(dWs, "dWs", F_in, F_out),
                                                  F_in, F_out, _dev_ptr(workspace, "workspace"),
                                                  workspace.numel() * workspace.element_size(), _stream_handle(stream)))


def groot_rows_over_degree(pl: Plan, Z, out, F: int = None, stream=None) -> None:
    """out[i, :] = Z[i, :] / stored length of row i; out may be Z."""
    F = Z.shape[1] if F is None else F
    n = _plan_rows(pl)
    _check(_lib.groot_rows_over_degree(pl.handle, _features(Z, "Z", n, F), _features(out, "out", n, F), F,
                                       _stream_handle(stream)))


def groot_plan_lists_device(pl: Plan, row_class, hd_rows, ld_rows, ld_rows_by_degree, ld_deg_offsets, counts,
                            stream=None, _entry=None) -> None:
    """Caller-allocated CUDA tensors: uint8[N], int32[N] x3, int64[T+1], int64[2]."""
    import torch

    n = _plan_rows(pl)
    for t, dt, size, what in ((row_class, torch.uint8, n, "row_class"), (hd_rows, torch.int32, n, "hd_rows"),
                              (ld_rows, torch.int32, n, "ld_rows"), (ld_rows_by_degree, torch.int32, n, "ld_rows_by_degree"),
                              (ld_deg_offsets, torch.int64, pl.degree_threshold + 1, "ld_deg_offsets"),
                              (counts, torch.int64, 2, "counts")):
        if t.dtype != dt or t.numel() < max(size, 1):
            raise TypeError(f"{what} must be {dt} with at least {max(size, 1)} elements")
    entry = _entry or _lib.groot_plan_lists_device
    _check(entry(pl.handle, _dev_ptr(row_class, "row_class"), _dev_ptr(hd_rows, "hd_rows"),
                 _dev_ptr(ld_rows, "ld_rows"), _dev_ptr(ld_rows_by_degree, "ld_rows_by_degree"),
                 _dev_ptr(ld_deg_offsets, "ld_deg_offsets"), _dev_ptr(counts, "counts"), _stream_handle(stream)))


def groot_plan_lists_device_static(pl: Plan, row_class, hd_rows, ld_rows, ld_rows_by_degree, ld_deg_offsets, counts,
                                   stream=None) -> None:
    """The same lists without any allocation or synchronisation inside the call (fixed scratch in the library)."""
    groot_plan_lists_device(pl, row_class, hd_rows, ld_rows, ld_rows_by_degree, ld_deg_offsets, counts, stream,
                            _entry=_lib.groot_plan_lists_device_static)


def groot_plan_query(pl: Plan, what: str) -> int:
    out = _i64(0)
    _check(_lib.groot_plan_query(pl.handle, what.encode(), ctypes.byref(out)))
    return out.value


def groot_plan_hd_pieces(pl: Plan) -> dict:
    n = groot_plan_query(pl, "hd_pieces")
    out = {"begin": np.empty(n, np.int64), "len": np.empty(n, np.int32), "row": np.empty(n, np.int32),
           "slot": np.empty(n, np.int32)}
    _check(_lib.groot_plan_hd_pieces(pl.handle, n, *(out[k].ctypes.data for k in ("begin", "len", "row", "slot"))))
    return out


def groot_feature_placement(pl: Plan, arena, F: int, stream=None) -> dict:
    """arena: a contiguous float32 CUDA tensor (its contents are overwritten) -> byte offsets of X and Y in it"""
    import torch

    ptr = _dev_ptr(arena, "arena")
    if arena.dtype != torch.float32:
        raise TypeError("arena must be float32")
    x, y = ctypes.c_size_t(0), ctypes.c_size_t(0)
    best, first = ctypes.c_float(0), ctypes.c_float(0)
    _check(_lib.groot_feature_placement(pl.handle, ptr, arena.numel() * 4, F, _stream_handle(stream), ctypes.byref(x),
                                        ctypes.byref(y), ctypes.byref(best), ctypes.byref(first)))
    return {"x_offset": x.value, "y_offset": y.value, "best_ms": best.value, "first_ms": first.value}


def groot_partition_regrow(g: Graph, num_parts: int, part_of=None, flags: int = GROOT_REGROW) -> Parts:
    p, pp = _host(part_of, np.int32)
    if p is not None and p.shape[0] != groot_graph_view(g)["n"]:
        raise ValueError("part_of must have one entry per node")
    out = ctypes.c_void_p()
    _check(_lib.groot_partition_regrow(g.handle, num_parts, pp, flags, ctypes.byref(out)))
    return Parts(out.value, g)


def groot_parts_count(parts: Parts) -> int:
    return _lib.groot_parts_count(parts.handle)


def groot_parts_view(parts: Parts, p: int) -> dict:
    a, b, c = _i64(0), _i64(0), _i64(0)
    gid, sub = ctypes.c_void_p(), ctypes.c_void_p()
    _check(_lib.groot_parts_view(parts.handle, p, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c),
                                 ctypes.byref(gid), ctypes.byref(sub)))
    return dict(n_owned=a.value, n_halo=b.value, n_crossing=c.value,
                global_id=_view(gid.value, a.value + b.value, np.int64, parts), sub=Graph(sub.value, owner=parts))


def groot_partition_regrow_device(pl: Plan, num_parts: int, p: int, part_of=None, flags: int = GROOT_REGROW,
                                  stream=None) -> DevPart:
    """part_of: None (built-in rule) or a CUDA int32 tensor with one entry per node."""
    import torch

    pp = None
    if part_of is not None:
        if not isinstance(part_of, torch.Tensor) or part_of.dtype != torch.int32:
            raise TypeError("part_of must be a CUDA int32 tensor")
        n = pl.n_rows if pl.graph is None else groot_graph_view(pl.graph)["n"]
        if part_of.numel() != n:
            raise ValueError("part_of must have one entry per node")
        pp = _dev_ptr(part_of, "part_of")
    out = ctypes.c_void_p()
    _check(_lib.groot_partition_regrow_device(pl.handle, num_parts, pp, flags, p, _stream_handle(stream),
                                              ctypes.byref(out)))
    return DevPart(out.value, pl)


def groot_dev_part_view(part: DevPart) -> dict:
    a, b, c, z = _i64(0), _i64(0), _i64(0), _i64(0)
    gid, rp, col, val = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
    _check(_lib.groot_dev_part_view(part.handle, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(z),
                                    ctypes.byref(gid), ctypes.byref(rp), ctypes.byref(col), ctypes.byref(val)))
    n = a.value + b.value

    def arr(ptr, count, dtype):
        return RawDeviceArray(ptr.value, count, dtype, part) if ptr.value else None
    return dict(n_owned=a.value, n_halo=b.value, n_crossing=c.value, nnz=z.value,
                global_id=arr(gid, n, np.int64), rowptr=arr(rp, n + 1, np.int64), col=arr(col, z.value, np.int32),
                val=arr(val, z.value, np.float32))


def groot_dev_part_download(part: DevPart, stream=None) -> dict:
    """Host copies (numpy) of whatever the part still holds."""
    v = groot_dev_part_view(part)
    n = v["n_owned"] + v["n_halo"]
    out = dict(global_id=np.empty(n, np.int64))
    if v["rowptr"] is not None:
        out["rowptr"] = np.empty(n + 1, np.int64)
        out["col"] = np.empty(v["nnz"], np.int32)
    if v["val"] is not None:
        out["val"] = np.empty(v["nnz"], np.float32)

    def ptr(name):
        return out[name].ctypes.data if name in out else None
    _check(_lib.groot_dev_part_download(part.handle, ptr("global_id"), ptr("rowptr"), ptr("col"), ptr("val"),
                                        _stream_handle(stream)))
    return out


def groot_dev_part_plan(part: DevPart, degree_threshold: int, max_F: int, stream=None) -> Plan:
    out = ctypes.c_void_p()
    _check(_lib.groot_dev_part_plan(part.handle, degree_threshold, max_F, _stream_handle(stream), ctypes.byref(out)))
    pl = Plan(out.value, None)
    pl.degree_threshold = degree_threshold
    v = groot_dev_part_view(part)
    pl.n_rows = v["n_owned"] + v["n_halo"]
    return pl


def _ids(ids, what="ids"):
    import torch

    if (ids.dtype != np.int64) if isinstance(ids, RawDeviceArray) else (ids.dtype != torch.int64):
        raise TypeError(f"{what} must be int64")
    return _dev_ptr(ids, what)


def groot_rows_gather(ids, X, out, F: int = None, stream=None) -> None:
    """X must hold every row that ids names (not checked: the ids live on the device)."""
    F = X.shape[1] if F is None else F
    _check(_lib.groot_rows_gather(_ids(ids), ids.shape[0], _features(X, "X", 0, F), _features(out, "out", ids.shape[0], F),
                                  F, _stream_handle(stream)))


def groot_rows_scatter(ids, inp, Y, F: int = None, stream=None) -> None:
    """Y must hold every row that ids names (not checked: the ids live on the device)."""
    F = Y.shape[1] if F is None else F
    _check(_lib.groot_rows_scatter(_ids(ids), ids.shape[0], _features(inp, "in", ids.shape[0], F), _features(Y, "Y", 0, F),
                                   F, _stream_handle(stream)))


def groot_set_tuning(name: str, value: int) -> None:
    _check(_lib.groot_set_tuning(name.encode(), value))

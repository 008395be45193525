"""CPU oracle -- TEST INFRASTRUCTURE ONLY.

ctypes access to ``groot_oracle.c`` (plain C, fp64 where floating point) plus
two numpy pieces: the dense statement of A_hat X used on tiny graphs and the
GraphSAGE-mean forward pass.  Only ``tests/``, ``__graft_entry__.smoke`` and
the ``cpu_baseline`` leg of ``bench.py`` may import this package; it imports
nothing from the HIP library or its binding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "groot_oracle.c")
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

SYMMETRIC, SELF_LOOPS, NORM_MEAN = 1, 2, 4
DEFAULT_FLAGS = SYMMETRIC | SELF_LOOPS | NORM_MEAN
REGROW = 1

_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_u64p = ctypes.POINTER(ctypes.c_uint64)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", _LIB_PATH, _SRC, "-lm"],
                       check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        I64, I32, U32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32
        lib.orc_aig_simulate.restype = I32
        lib.orc_aig_simulate.argtypes = [I64, _u8p, _i32p, _i32p, _u64p, _u64p]
        lib.orc_csr_nnz.restype = I64
        lib.orc_csr_nnz.argtypes = [I64, _u8p, _i32p, _i32p, I32, U32]
        lib.orc_csr_build.restype = I32
        lib.orc_csr_build.argtypes = [I64, _u8p, _i32p, _i32p, I32, U32, _i64p, _i32p, _f32p, _u8p]
        lib.orc_spmm_f64.restype = None
        lib.orc_spmm_f64.argtypes = [I64, _i64p, _i32p, _f32p, _f32p, I32, _f64p, _f64p]
        lib.orc_spmm_t_f64.restype = None
        lib.orc_spmm_t_f64.argtypes = [I64, _i64p, _i32p, _f32p, _f32p, I32, _f64p, _f64p]
        lib.orc_csr_transpose.restype = None
        lib.orc_csr_transpose.argtypes = [I64, _i64p, _i32p, _f32p, _i64p, _i32p, _f32p]
        lib.orc_plan.restype = I32
        lib.orc_plan.argtypes = [I64, _i64p, I32, _u8p, _i32p, _i32p, _i32p, _i64p, _i64p, _i64p]
        lib.orc_part_of_default.restype = None
        lib.orc_part_of_default.argtypes = [I64, I64, I32, _i32p]
        lib.orc_regrow_sizes.restype = I32
        lib.orc_regrow_sizes.argtypes = [I64, _i64p, _i32p, _i32p, I32, U32, _i64p, _i64p, _i64p, _i64p]
        lib.orc_regrow_fill.restype = I32
        lib.orc_regrow_fill.argtypes = [I64, _i64p, _i32p, _f32p, _i32p, I32, U32, I32, _i64p, _i64p, _i32p, _f32p]
        _lib = lib
    return _lib


def _p(a, t):
    return a.ctypes.data_as(t)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def aig_simulate(type_, fanin0, fanin1, pi_words):
    """64 input patterns at once: returns the uint64 word of every node."""
    lib = _load()
    type_, fanin0, fanin1 = _c(type_, np.uint8), _c(fanin0, np.int32), _c(fanin1, np.int32)
    pi_words = _c(pi_words, np.uint64)
    out = np.zeros(type_.shape[0], dtype=np.uint64)
    rc = lib.orc_aig_simulate(type_.shape[0], _p(type_, _u8p), _p(fanin0, _i32p), _p(fanin1, _i32p),
                              _p(pi_words, _u64p), _p(out, _u64p))
    if rc != 0:
        raise ValueError("AIG is not in topological order")
    return out


def csr_build(type_, fanin0, fanin1, batch=1, flags=DEFAULT_FLAGS):
    """-> rowptr int64 [N+1], col int32, val float32, pol uint8"""
    lib = _load()
    type_, fanin0, fanin1 = _c(type_, np.uint8), _c(fanin0, np.int32), _c(fanin1, np.int32)
    n1 = type_.shape[0]
    args = (n1, _p(type_, _u8p), _p(fanin0, _i32p), _p(fanin1, _i32p), batch, flags)
    nnz = lib.orc_csr_nnz(*args)
    if nnz < 0:
        raise MemoryError
    rowptr = np.zeros(n1 * batch + 1, dtype=np.int64)
    col = np.empty(nnz, dtype=np.int32)
    val = np.empty(nnz, dtype=np.float32)
    pol = np.empty(nnz, dtype=np.uint8)
    if lib.orc_csr_build(*args, _p(rowptr, _i64p), _p(col, _i32p), _p(val, _f32p), _p(pol, _u8p)) != 0:
        raise MemoryError
    return rowptr, col, val, pol


def spmm_f64(rowptr, col, val, X, want_abs=True):
    """-> (Y fp64 [N,F], S fp64 [N,F] or None); S = sum_p |val_p * X[col_p,k]|"""
    lib = _load()
    rowptr, col, val = _c(rowptr, np.int64), _c(col, np.int32), _c(val, np.float32)
    X = _c(X, np.float32)
    n, F = rowptr.shape[0] - 1, X.shape[1]
    Y = np.empty((n, F), dtype=np.float64)
    S = np.empty((n, F), dtype=np.float64) if want_abs else None
    lib.orc_spmm_f64(n, _p(rowptr, _i64p), _p(col, _i32p), _p(val, _f32p), _p(X, _f32p), F,
                     _p(Y, _f64p), _p(S, _f64p) if want_abs else None)
    return Y, S


def spmm_t_f64(rowptr, col, val, G, want_abs=True):
    """(A_hat^T G) by the scatter definition -> (fp64 [N,F], sum of |terms| or None)"""
    lib = _load()
    rowptr, col, val = _c(rowptr, np.int64), _c(col, np.int32), _c(val, np.float32)
    G = _c(G, np.float32)
    n, F = rowptr.shape[0] - 1, G.shape[1]
    out = np.empty((n, F), dtype=np.float64)
    S = np.empty((n, F), dtype=np.float64) if want_abs else None
    lib.orc_spmm_t_f64(n, _p(rowptr, _i64p), _p(col, _i32p), _p(val, _f32p), _p(G, _f32p), F,
                       _p(out, _f64p), _p(S, _f64p) if want_abs else None)
    return out, S


def csr_transpose(rowptr, col, val):
    """A_hat^T as (rowptr, col, val)"""
    lib = _load()
    rowptr, col, val = _c(rowptr, np.int64), _c(col, np.int32), _c(val, np.float32)
    n = rowptr.shape[0] - 1
    t_rowptr = np.empty(n + 1, dtype=np.int64)
    t_col = np.empty(col.shape[0], dtype=np.int32)
    t_val = np.empty(col.shape[0], dtype=np.float32)
    lib.orc_csr_transpose(n, _p(rowptr, _i64p), _p(col, _i32p), _p(val, _f32p), _p(t_rowptr, _i64p),
                          _p(t_col, _i32p), _p(t_val, _f32p))
    return t_rowptr, t_col, t_val


def plan(rowptr, T):
    """-> dict(row_class, hd_rows, ld_rows, ld_rows_by_degree, ld_deg_offsets)"""
    lib = _load()
    rowptr = _c(rowptr, np.int64)
    n = rowptr.shape[0] - 1
    row_class = np.empty(n, dtype=np.uint8)
    hd = np.empty(n, dtype=np.int32)
    ld = np.empty(n, dtype=np.int32)
    by = np.empty(n, dtype=np.int32)
    off = np.empty(T + 1, dtype=np.int64)
    n_hd, n_ld = ctypes.c_int64(0), ctypes.c_int64(0)
    rc = lib.orc_plan(n, _p(rowptr, _i64p), T, _p(row_class, _u8p), _p(hd, _i32p), _p(ld, _i32p),
                      _p(by, _i32p), _p(off, _i64p), ctypes.byref(n_hd), ctypes.byref(n_ld))
    if rc != 0:
        raise ValueError("bad plan arguments")
    return dict(row_class=row_class, hd_rows=hd[:n_hd.value].copy(), ld_rows=ld[:n_ld.value].copy(),
                ld_rows_by_degree=by[:n_ld.value].copy(), ld_deg_offsets=off)


def part_of_default(n, n1, P):
    lib = _load()
    out = np.empty(n, dtype=np.int32)
    lib.orc_part_of_default(n, n1, P, _p(out, _i32p))
    return out


def regrow_part(rowptr, col, val, part_of, p, flags=REGROW, weight_mode=1):
    """One part of Algorithm 1 -> dict(n_owned, n_halo, n_crossing, global_id,
    rowptr, col, val) with local ids (owned ascending, then boundary ascending)."""
    lib = _load()
    rowptr, col, val = _c(rowptr, np.int64), _c(col, np.int32), _c(val, np.float32)
    part_of = _c(part_of, np.int32)
    n = rowptr.shape[0] - 1
    a, b, c, d = (ctypes.c_int64(0) for _ in range(4))
    if lib.orc_regrow_sizes(n, _p(rowptr, _i64p), _p(col, _i32p), _p(part_of, _i32p), p, flags,
                            ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(d)) != 0:
        raise MemoryError
    tot = a.value + b.value
    gid = np.empty(tot, dtype=np.int64)
    srp = np.empty(tot + 1, dtype=np.int64)
    scol = np.empty(d.value, dtype=np.int32)
    sval = np.empty(d.value, dtype=np.float32)
    if lib.orc_regrow_fill(n, _p(rowptr, _i64p), _p(col, _i32p), _p(val, _f32p), _p(part_of, _i32p), p, flags,
                           weight_mode, _p(gid, _i64p), _p(srp, _i64p), _p(scol, _i32p), _p(sval, _f32p)) != 0:
        raise MemoryError
    return dict(n_owned=a.value, n_halo=b.value, n_crossing=c.value, global_id=gid,
                rowptr=srp, col=scol, val=sval)


def dense_adjacency(rowptr, col, val):
    """A_hat as a dense fp64 matrix (tiny graphs only)."""
    n = len(rowptr) - 1
    A = np.zeros((n, n), dtype=np.float64)
    for i in range(n):
        for p in range(rowptr[i], rowptr[i + 1]):
            A[i, col[p]] += float(val[p])
    return A


def sage_layer_f64(rowptr, col, val, X, Wn, Ws, b, relu):
    """One GraphSAGE-mean layer in fp64 (Section "GNN and Edge Re-growth After Partition": the layer
    aggregates the neighbours' features, then transforms): act((A_hat X) Wn + X Ws + b), act = ReLU applied
    after the bias, or the identity; also returns A_hat X and its sum of absolute terms (for the error
    scale).  Pinned by the dense layer on the 18- and 51-node multipliers, the Wn = I / Ws = I reductions
    and a closed-form case where ReLU clips."""
    A, S = spmm_f64(rowptr, col, val, X)
    H = A @ Wn.astype(np.float64) + np.asarray(X, dtype=np.float64) @ Ws.astype(np.float64)
    if b is not None:
        H = H + b.astype(np.float64)
    return (np.maximum(H, 0.0) if relu else H), A, S


def sage_layer_backward_data_f64(rowptr, col, val, dZ, Wn, Ws):
    """Gradient of a GraphSAGE-mean layer with respect to its input, in fp64 (Section "GNN and Edge Re-growth
    After Partition": the model is trained).  For Z = (A_hat X) Wn + X Ws + b and dZ the gradient of the loss
    at Z, the chain rule gives dX = A_hat^T (dZ Wn^T) + dZ Ws^T; written here as (A_hat^T dZ) Wn^T + dZ Ws^T
    so that the transposed aggregation takes the fp32 input itself.  Returns dX, A_hat^T dZ and the latter's
    sum of absolute terms (for the error scale).  Pinned by automatic differentiation of the dense layer on
    the 18- and 51-node multipliers, by central differences, and by the adjoint identity <dZ, J V> = <J^T dZ, V>."""
    T, S = spmm_t_f64(rowptr, col, val, dZ)
    dX = T @ Wn.astype(np.float64).T + np.asarray(dZ, dtype=np.float64) @ Ws.astype(np.float64).T
    return dX, T, S


def sage_layer_backward_weights_f64(rowptr, col, val, X, dZ):
    """Gradients of a GraphSAGE-mean layer with respect to its two weight matrices, in fp64: for
    Z = (A_hat X) Wn + X Ws + b and dZ the gradient of the loss at Z, dWn = (A_hat X)^T dZ and dWs = X^T dZ
    (chain rule; Section "GNN and Edge Re-growth After Partition": the model is trained).  Also returns the
    sums of absolute terms of the two products, with the aggregation's own sum of absolute terms in the first
    (for the error scale).  Pinned by automatic differentiation of the dense layer on the 18- and 51-node
    multipliers and by the identity <dWn, V> + <dWs, U> = <dZ, (A_hat X) V + X U>."""
    A, S = spmm_f64(rowptr, col, val, X)
    X64, dZ64 = np.asarray(X, dtype=np.float64), np.asarray(dZ, dtype=np.float64)
    return A.T @ dZ64, X64.T @ dZ64, S.T @ np.abs(dZ64), np.abs(X64).T @ np.abs(dZ64)


def sage_forward_f64(rowptr, col, val, X, W1n, W1s, b1, W2n, W2s, b2):
    """Two GraphSAGE-mean layers (Section "GNN and Edge Re-growth After
    Partition": the layer aggregates neighbour features, then transforms):
        H1 = relu((A_hat X) W1n + X W1s + b1),  H2 = (A_hat H1) W2n + H1 W2s + b2.
    The aggregation input of layer 2 is H1 rounded to fp32, as the library
    receives it.  The paper gives no hyper-parameters (width, depth, where the
    activation sits): those are this build's reading; the arithmetic is pinned
    as two applications of the pinned layer."""
    X64 = np.asarray(X, dtype=np.float64)
    A1, _ = spmm_f64(rowptr, col, val, X, want_abs=False)
    H1 = np.maximum(A1 @ W1n.astype(np.float64) + X64 @ W1s.astype(np.float64) + b1.astype(np.float64), 0.0)
    H1f = H1.astype(np.float32)
    A2, _ = spmm_f64(rowptr, col, val, H1f, want_abs=False)
    H2 = A2 @ W2n.astype(np.float64) + H1f.astype(np.float64) @ W2s.astype(np.float64) + b2.astype(np.float64)
    return H1f, H2

"""Seeded synthetic inputs shared by the HIP library's callers and the CPU oracle.

Nothing in this package performs the method's arithmetic (no adjacency
building, no normalisation of an AIG graph, no SpMM, no planning, no
partitioning).  It only produces inputs:

* ``csa_multiplier_aig(n)``   the And-Inverter Graph of an n-bit carry-save
  array multiplier (stand-in for the paper's ABC-generated CSA datasets;
  Section "Converting Netlists into Transitional Graph");
* ``uniform_features``        counter-based U(-1,1) feature matrices that can be
  produced on the host or directly in device memory, block by block;
* ``aig_node_features``       the first eight structural feature columns used
  by the smallest workload (node type one-hot plus edge-polarity counts, in
  the spirit of Section "Node Features and Node Label creation");
* ``stress_graph``            a CSR matrix with an exaggerated polarized degree
  distribution (Section "Kernel Design - GROOT-GPU").

The C sources beside this file are compiled with gcc into
``libworkloads.so`` on first use (or by ``__graft_entry__.build``).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libworkloads.so")
_SOURCES = [os.path.join(_HERE, "csa_aig.c"), os.path.join(_HERE, "stress.c"), os.path.join(_HERE, "booth_aig.c")]
_lib = None

PI, AND, PO = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the C generators (host only, gcc)."""
    newest = max(os.path.getmtime(s) for s in _SOURCES)
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < newest:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", _LIB_PATH] + _SOURCES + ["-lm"]
        subprocess.run(cmd, check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        f32p = ctypes.POINTER(ctypes.c_float)
        lib.wl_csa_num_nodes.restype = ctypes.c_int64
        lib.wl_csa_num_nodes.argtypes = [ctypes.c_int32]
        lib.wl_csa_generate.restype = ctypes.c_int64
        lib.wl_csa_generate.argtypes = [ctypes.c_int32, u8p, i32p, i32p, i32p]
        lib.wl_csa_generate_labeled.restype = ctypes.c_int64
        lib.wl_csa_generate_labeled.argtypes = [ctypes.c_int32, u8p, i32p, i32p, i32p, u8p]
        lib.wl_booth_generate.restype = ctypes.c_int64
        lib.wl_booth_generate.argtypes = [ctypes.c_int32, u8p, i32p, i32p, i32p]
        lib.wl_stress_rowptr.restype = ctypes.c_int64
        lib.wl_stress_rowptr.argtypes = [ctypes.c_uint64] + [ctypes.c_int64] * 4 + [i64p]
        lib.wl_stress_fill.restype = ctypes.c_int32
        lib.wl_stress_fill.argtypes = [ctypes.c_uint64] + [ctypes.c_int64] * 4 + [i64p, i32p, f32p]
        lib.wl_stress_is_heavy.restype = ctypes.c_int32
        lib.wl_stress_is_heavy.argtypes = [ctypes.c_uint64, ctypes.c_int64]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


@dataclass
class Aig:
    """An AIG in literal form.  ``fanin = 2*source_id + inverted``; PIs hold -1."""
    n_bits: int
    type: np.ndarray       # uint8 [N1]  0 = PI, 1 = AND, 2 = PO
    fanin0: np.ndarray     # int32 [N1]
    fanin1: np.ndarray     # int32 [N1]
    po_driver: np.ndarray  # int32 [2n] literal driving each product bit m_k
    label: np.ndarray      # uint8 [N1] the paper's node classes: 4 PI, 3 AND, 2 XOR, 1 MAJ, 0 PO

    @property
    def num_nodes(self) -> int:
        return int(self.type.shape[0])


def csa_multiplier_aig(n_bits: int) -> Aig:
    lib = _load()
    n1 = int(lib.wl_csa_num_nodes(n_bits))
    typ = np.empty(n1, dtype=np.uint8)
    f0 = np.empty(n1, dtype=np.int32)
    f1 = np.empty(n1, dtype=np.int32)
    po = np.empty(2 * n_bits, dtype=np.int32)
    label = np.empty(n1, dtype=np.uint8)
    got = lib.wl_csa_generate_labeled(n_bits, _ptr(typ, ctypes.c_uint8), _ptr(f0, ctypes.c_int32),
                                      _ptr(f1, ctypes.c_int32), _ptr(po, ctypes.c_int32),
                                      _ptr(label, ctypes.c_uint8))
    if got != n1:
        raise RuntimeError(f"CSA generator wrote {got} nodes, expected {n1}")
    return Aig(n_bits, typ, f0, f1, po, label)


def booth_multiplier_aig(n_bits: int) -> Aig:
    """Radix-4 Booth multiplier (unsigned, n_bits even): the degree profile of the paper's Booth dataset.
    Labels: 4 = PI, 3 = AND, 0 = PO (no XOR / MAJ roots are marked)."""
    lib = _load()
    n1 = int(lib.wl_booth_generate(n_bits, None, None, None, None))
    if n1 < 0:
        raise ValueError("n_bits must be even, 2..2048")
    typ = np.empty(n1, dtype=np.uint8)
    f0 = np.empty(n1, dtype=np.int32)
    f1 = np.empty(n1, dtype=np.int32)
    po = np.empty(2 * n_bits, dtype=np.int32)
    got = lib.wl_booth_generate(n_bits, _ptr(typ, ctypes.c_uint8), _ptr(f0, ctypes.c_int32),
                                _ptr(f1, ctypes.c_int32), _ptr(po, ctypes.c_int32))
    if got != n1:
        raise RuntimeError(f"Booth generator wrote {got} nodes, expected {n1}")
    label = np.where(typ == 0, 4, np.where(typ == 1, 3, 0)).astype(np.uint8)
    return Aig(n_bits, typ, f0, f1, po, label)


# ----------------------------------------------------------------------------
# counter-based uniform features
# ----------------------------------------------------------------------------
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_GOLD = 0x9E3779B97F4A7C15


def _s64(v: int) -> int:
    """two's-complement reinterpretation of a 64-bit pattern as a signed int"""
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >= (1 << 63) else v


def _mix64_int(z: int) -> int:
    mask = (1 << 64) - 1
    z = (z + _GOLD) & mask
    z = ((z ^ (z >> 30)) * _M1) & mask
    z = ((z ^ (z >> 27)) * _M2) & mask
    return z ^ (z >> 31)


def _mix64_torch(z):
    """The same 64-bit mixer on an int64 torch tensor (wrapping arithmetic,
    logical shifts emulated by masking the sign-extended bits)."""
    z = z + _s64(_GOLD)
    z = (z ^ ((z >> 30) & ((1 << 34) - 1))) * _s64(_M1)
    z = (z ^ ((z >> 27) & ((1 << 37) - 1))) * _s64(_M2)
    return z ^ ((z >> 31) & ((1 << 33) - 1))


def uniform_features(seed: int, row_begin: int, row_end: int, F: int, device="cpu", out=None,
                     block_rows: int = 1 << 20):
    """fp32 [row_end-row_begin, F] with x[r,k] = ((h >> 40) * 2^-23) - 1 where
    h = mix64(mix64(seed) + r*F + k) and r is the GLOBAL row index: every
    element is a pure function of (seed, r, k), lies on a 2^-23 grid in
    [-1, 1) and is therefore exact in fp32.  Works on any torch device."""
    import torch

    n = row_end - row_begin
    if out is None:
        out = torch.empty((n, F), dtype=torch.float32, device=device)
    base = _s64(_mix64_int(seed & ((1 << 64) - 1)))
    k = torch.arange(F, dtype=torch.int64, device=out.device)
    for b0 in range(0, n, block_rows):
        b1 = min(n, b0 + block_rows)
        r = torch.arange(row_begin + b0, row_begin + b1, dtype=torch.int64, device=out.device)
        ctr = (r * F)[:, None] + k[None, :] + base
        h = _mix64_torch(ctr)
        top = (h >> 40) & ((1 << 24) - 1)
        out[b0:b1] = top.to(torch.float32) * (2.0 ** -23) - 1.0
    return out


def uniform_features_numpy(seed: int, row_begin: int, row_end: int, F: int) -> np.ndarray:
    """uint64 numpy statement of the same generator (used to cross-check the
    torch form; small sizes)."""
    base = np.uint64(_mix64_int(seed & ((1 << 64) - 1)))
    r = np.arange(row_begin, row_end, dtype=np.uint64)
    ctr = r[:, None] * np.uint64(F) + np.arange(F, dtype=np.uint64)[None, :] + base
    with np.errstate(over="ignore"):
        z = ctr + np.uint64(_GOLD)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_M1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_M2)
        h = z ^ (z >> np.uint64(31))
    top = (h >> np.uint64(40)).astype(np.float64)
    return (top * 2.0 ** -23 - 1.0).astype(np.float32)


def paper_node_features(aig: Aig) -> np.ndarray:
    """The paper's 4-bit node feature vector (Section "Node Features and Node Label creation") as
    float32 [N1, 4]: PI 0000; internal AND node 1 1 L R with L / R = left / right input inverted;
    PO 0 X 1 1 with X = the edge from its driver is inverted.  (The text gives the PO encoding as
    "0X" plus inherited polarity and prints 0011 for a PO with a non-inverted input; this is the
    reading under which all four printed examples -- nodes 1, 5, 10, 15 of the two-bit multiplier --
    come out as printed.)"""
    n1 = aig.num_nodes
    x = np.zeros((n1, 4), dtype=np.float32)
    is_and, is_po = aig.type == AND, aig.type == PO
    x[is_and, 0] = 1.0
    x[is_and, 1] = 1.0
    x[is_and, 2] = (aig.fanin0[is_and] & 1).astype(np.float32)
    x[is_and, 3] = (aig.fanin1[is_and] & 1).astype(np.float32)
    x[is_po, 1] = (aig.fanin0[is_po] & 1).astype(np.float32)
    x[is_po, 2] = 1.0
    x[is_po, 3] = 1.0
    return x


def aig_node_features(aig: Aig, seed: int, F: int) -> np.ndarray:
    """Feature matrix of the smallest workload: columns 0-2 one-hot node type
    (PI / AND / PO); 3 = inverted fanin records; 4 = non-inverted fanin
    records; 5 = inverted fanout records; 6 = non-inverted fanout records;
    7 = 1; remaining columns U(-1,1).  All structural values are small
    integers, exact in fp32."""
    if F < 8:
        raise ValueError("need F >= 8")
    n1 = aig.num_nodes
    x = uniform_features_numpy(seed, 0, n1, F)
    x[:, :8] = 0.0
    x[np.arange(n1), aig.type.astype(np.int64)] = 1.0
    for f in (aig.fanin0, aig.fanin1):
        has = f >= 0
        inv = (f & 1).astype(bool) & has
        x[:, 3] += inv
        x[:, 4] += has & ~inv
        src = (f[has] >> 1).astype(np.int64)
        np.add.at(x[:, 5], src, (f[has] & 1).astype(np.float32))
        np.add.at(x[:, 6], src, 1.0 - (f[has] & 1).astype(np.float32))
    x[:, 7] = 1.0
    return x


# ----------------------------------------------------------------------------
# polarized stress graph
# ----------------------------------------------------------------------------
@dataclass
class Csr:
    n: int
    rowptr: np.ndarray  # int64 [n+1]
    col: np.ndarray     # int32 [nnz]
    val: np.ndarray     # float32 [nnz]


def stress_graph(seed: int, n: int, window: int = 4096, dmin: int = 64, dmax: int = 262144,
                 verbose: bool = False) -> Csr:
    """1 % heavy rows (Zipf(1.2) draws clipped to [dmin, dmax], uniform
    columns), 99 % light rows (2-4 neighbours within +-window), self-loops,
    weights 1/row length.  Directed."""
    if n < 2 * window + 2 or window < 4 or n >= 2 ** 31 or dmin < 1 or dmax < dmin:
        raise ValueError("bad stress graph parameters")
    lib = _load()
    rowptr = np.zeros(n + 1, dtype=np.int64)
    nnz = lib.wl_stress_rowptr(seed, n, window, dmin, dmax, _ptr(rowptr, ctypes.c_int64))
    if nnz < 0:
        raise MemoryError("stress graph generation failed")
    if verbose:
        print(f"stress graph: row lengths done, {nnz} stored entries", flush=True)
    col = np.empty(nnz, dtype=np.int32)
    val = np.empty(nnz, dtype=np.float32)
    rc = lib.wl_stress_fill(seed, n, window, dmin, dmax, _ptr(rowptr, ctypes.c_int64),
                            _ptr(col, ctypes.c_int32), _ptr(val, ctypes.c_float))
    if rc != 0:
        raise RuntimeError("stress graph fill failed")
    return Csr(n, rowptr, col, val)


def stress_is_heavy(seed: int, row: int) -> bool:
    return bool(_load().wl_stress_is_heavy(seed, row))


# ----------------------------------------------------------------------------
# 4-LUT-mapped carry-save multiplier (graph shape only)
# ----------------------------------------------------------------------------
def lut4_csa_graph(n_bits: int, batch: int = 1) -> Csr:
    """Shape of a carry-save array multiplier after mapping to 4-input LUTs (stand-in for the paper's
    FPGA-mapped dataset, which needs ABC): every array cell (i, j) becomes two LUT nodes, sum and carry,
    with the same four fanins a_j, b_i, sum(i-1, j+1), carry(i-1, j) (those that exist); a last row of
    n sum/carry LUT pairs forms the ripple adder; 2n primary outputs have one fanin each.  No logic
    functions are modelled: only the adjacency.  Node order: a_0.., b_0.., cells row by row (sum, carry
    interleaved), adder row, outputs.  Returns the symmetric adjacency with self-loops, mean-normalised
    (weights fl(1/row length)), replicated block-diagonally `batch` times.
    Degree profile: 2n primary-input rows of 2n+1 entries (the high-degree class), interior LUT rows of
    7 entries (4 fanins, 2 fanouts, itself): longer than an AIG's 4-5."""
    import scipy.sparse as sp

    n = n_bits
    if n < 2 or n > 2048 or batch < 1:
        raise ValueError("bad LUT graph parameters")
    a = np.arange(n)
    b = n + np.arange(n)
    cell0 = 2 * n
    i, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    s_id = cell0 + 2 * (i * n + j)
    c_id = s_id + 1
    src, dst = [], []

    def edges(frm, to, mask=None):
        frm, to = np.broadcast_arrays(frm, to)
        if mask is not None:
            frm, to = frm[mask], to[mask]
        src.append(np.asarray(frm).ravel())
        dst.append(np.asarray(to).ravel())

    for out in (s_id, c_id):
        edges(a[j], out)
        edges(b[i], out)
        up = (i > 0) & (j + 1 < n)
        edges(np.where(up, s_id - 2 * n + 2, 0), out, up)            # sum(i-1, j+1)
        edges(np.where(i > 0, c_id - 2 * n, 0), out, i > 0)          # carry(i-1, j)
    add0 = cell0 + 2 * n * n
    k = np.arange(n)
    for out in (add0 + 2 * k, add0 + 2 * k + 1):                      # adder bit k: sum and carry LUTs
        edges(np.where(k + 1 < n, s_id[n - 1, np.minimum(k + 1, n - 1)], 0), out, k + 1 < n)
        edges(c_id[n - 1, k], out)
        edges(np.where(k > 0, add0 + 2 * (k - 1) + 1, 0), out, k > 0)
    po0 = add0 + 2 * n
    edges(s_id[:, 0], po0 + np.arange(n))                             # low product bits leave the array's first column
    edges(add0 + 2 * k, po0 + n + k)
    n1 = po0 + 2 * n
    return _symmetric_mean_csr(src, dst, int(n1), batch)


def _symmetric_mean_csr(src, dst, n1: int, batch: int) -> Csr:
    """Directed edge lists -> symmetric adjacency with self-loops, mean-normalised (weights fl(1/row length)),
    replicated block-diagonally `batch` times."""
    import scipy.sparse as sp

    src = np.concatenate(src).astype(np.int64)
    dst = np.concatenate(dst).astype(np.int64)
    ones = np.ones(src.shape[0], dtype=np.int8)
    adj = sp.coo_matrix((ones, (src, dst)), shape=(n1, n1)).tocsr()
    adj = ((adj + adj.T + sp.identity(n1, dtype=np.int8, format="csr")) > 0).astype(np.int8).tocsr()
    adj.sort_indices()
    rp1 = adj.indptr.astype(np.int64)
    col1 = adj.indices.astype(np.int64)
    deg = np.diff(rp1)
    val1 = np.repeat(np.float32(1.0) / deg.astype(np.float32), deg).astype(np.float32)
    nnz1 = int(rp1[-1])
    rowptr = np.concatenate([[0]] + [rp1[1:] + c * nnz1 for c in range(batch)]).astype(np.int64)
    col = np.concatenate([col1 + c * n1 for c in range(batch)]).astype(np.int32)
    val = np.tile(val1, batch)
    return Csr(int(n1) * batch, rowptr, col, val)


def cellmap_csa_graph(n_bits: int, batch: int = 1) -> Csr:
    """Shape of a carry-save array multiplier after mapping to standard cells (stand-in for the paper's
    technology-mapped dataset, which needs ABC and a cell library): every array cell (i, j) becomes an AND2
    cell (fanins a_j, b_i) and a full-adder cell (fanins: that AND2, the adder of cell (i-1, j+1) for its sum
    and the adder of cell (i-1, j) for its carry, those that exist); a last row of n full adders forms the
    ripple adder; 2n primary outputs have one fanin each.  A cell is one node whatever its number of output
    pins; no logic is modelled, only the adjacency.  Node order: a_0.., b_0.., cells row by row (AND2, adder
    interleaved), adder row, outputs.  Symmetric, self-loops, mean-normalised, `batch` copies.
    Degree profile: 2n primary-input rows of n+1 entries (the high-degree class); AND2 rows of 4 entries;
    interior adder rows of 6 (3 fanins, 2 fanouts, itself): half as many nodes per multiplier bit as the AIG."""
    n = n_bits
    if n < 2 or n > 2048 or batch < 1:
        raise ValueError("bad cell graph parameters")
    a = np.arange(n)
    b = n + np.arange(n)
    cell0 = 2 * n
    i, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    and_id = cell0 + 2 * (i * n + j)
    fa_id = and_id + 1
    src, dst = [], []

    def edges(frm, to, mask=None):
        frm, to = np.broadcast_arrays(frm, to)
        if mask is not None:
            frm, to = frm[mask], to[mask]
        src.append(np.asarray(frm).ravel())
        dst.append(np.asarray(to).ravel())

    edges(a[j], and_id)
    edges(b[i], and_id)
    edges(and_id, fa_id)
    up = (i > 0) & (j + 1 < n)
    edges(np.where(up, fa_id - 2 * n + 2, 0), fa_id, up)               # sum of cell (i-1, j+1)
    edges(np.where(i > 0, fa_id - 2 * n, 0), fa_id, i > 0)             # carry of cell (i-1, j)
    add0 = cell0 + 2 * n * n
    k = np.arange(n)
    edges(np.where(k + 1 < n, fa_id[n - 1, np.minimum(k + 1, n - 1)], 0), add0 + k, k + 1 < n)
    edges(fa_id[n - 1, k], add0 + k)
    edges(np.where(k > 0, add0 + k - 1, 0), add0 + k, k > 0)
    po0 = add0 + n
    edges(fa_id[:, 0], po0 + np.arange(n))                              # low product bits leave the array's first column
    edges(add0 + k, po0 + n + k)
    n1 = po0 + 2 * n
    return _symmetric_mean_csr(src, dst, int(n1), batch)

"""Oracle aggregation: Y = A_hat X (eq. 1/3), its transpose, and the chunked form.

TEST INFRASTRUCTURE.  The loops live in agg_oracle.c (plain C, fp64, one row
summed sequentially in entry order); this file only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .graph import Graph, Sparse, plan_chunks

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "agg_oracle.c")
_LIB = os.path.join(_HERE, "libntp_oracle.so")
_lib = None


def build_native(force: bool = False) -> str:
    """Compile agg_oracle.c with gcc (OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_native())
        p = ctypes.c_void_p
        i64 = ctypes.c_int64
        lib.oracle_aggregate.argtypes = [i64, p, p, p, p, p, i64, i64, p, p, i64]
        lib.oracle_aggregate.restype = None
        lib.oracle_aggregate_transposed_scatter.argtypes = [i64, i64, p, p, p, p, i64, i64, p, i64]
        lib.oracle_aggregate_transposed_scatter.restype = None
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        lib.oracle_set_num_threads.restype = None
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """threads of the row loop from now on (results do not depend on it)"""
    _load().oracle_set_num_threads(int(n))


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else None


def aggregate(m: Sparse, X, rows=None, with_abs: bool = False):
    """fp64 result of sum_k val[k] * X[colidx[k], :] for every row of ``m`` (or
    only for ``rows``).  X: [n, f] any float dtype (converted to fp64).
    Returns Y [n_out, f] fp64, and with_abs also sum_k |val[k] * X[colidx[k], :]|."""
    X64 = np.ascontiguousarray(X, dtype=np.float64)
    if X64.ndim != 2:
        raise ValueError("X must be 2-D")
    f = X64.shape[1]
    rows_a = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    n_out = m.n if rows_a is None else rows_a.size
    Y = np.empty((n_out, f), dtype=np.float64)
    Ya = np.empty((n_out, f), dtype=np.float64) if with_abs else None
    rowptr = np.ascontiguousarray(m.rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(m.colidx, dtype=np.int32)
    val = np.ascontiguousarray(m.val, dtype=np.float32)
    if colidx.size and int(colidx.max()) >= X64.shape[0]:
        raise ValueError("column index beyond the rows of X")
    _load().oracle_aggregate(n_out, _ptr(rows_a), _ptr(rowptr), _ptr(colidx), _ptr(val),
                             _ptr(X64), f, f, _ptr(Y), _ptr(Ya), f)
    return (Y, Ya) if with_abs else Y


def aggregate_fwd(g: Graph, X, rows=None, with_abs=False):
    """Forward aggregation, eq. (1)/(3): row v sums its in-neighbours and itself."""
    return aggregate(g.csr, X, rows, with_abs)


def aggregate_bwd(g: Graph, G, rows=None, with_abs=False):
    """Backward aggregation (Section 4.2.1): a source vertex sums the gradients of the
    vertices it points to along its out-edges, i.e. A_hat^T G, through the
    by-source rows."""
    return aggregate(g.csc, G, rows, with_abs)


def aggregate_bwd_scatter(g: Graph, G):
    """A_hat^T G straight from the by-destination rows: entry (v, u, w) adds
    w * G[v] to output row u.  Does not use the CSC at all."""
    G64 = np.ascontiguousarray(G, dtype=np.float64)
    f = G64.shape[1]
    out = np.empty((g.n, f), dtype=np.float64)
    m = g.csr
    _load().oracle_aggregate_transposed_scatter(
        m.n, g.n, _ptr(np.ascontiguousarray(m.rowptr)), _ptr(np.ascontiguousarray(m.colidx)),
        _ptr(np.ascontiguousarray(m.val)), _ptr(G64), f, f, _ptr(out), f)
    return out


def chunked_aggregate(m: Sparse, X, chunk_edges: int):
    """Section 4.2.1: the rows are cut into contiguous chunks, each with all its
    entries, and aggregated one chunk after the other; the results are the row
    ranges of the full result laid end to end."""
    parts = []
    for r0, r1 in plan_chunks(m.rowptr, chunk_edges):
        parts.append(aggregate(m, X, rows=np.arange(r0, r1, dtype=np.int64)))
    return np.concatenate(parts, axis=0) if parts else np.empty((0, np.asarray(X).shape[1]))


def round_bf16(x) -> np.ndarray:
    """Round fp64/fp32 values to the nearest bfloat16 (ties to even) and return
    them as float32.  Goes through float32 first, as a device that accumulates in
    fp32 and stores bf16 does."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    u = x32.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(x32.shape)

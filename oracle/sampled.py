"""Oracle rows of A_hat computed one by one from an undirected edge list.

TEST INFRASTRUCTURE.  For graphs too large to sort on the host in a test, the rows
of the normalised adjacency that a test samples are built straight from the
definition (eq. 1, eq. 3, Section 4.1.3), without building the whole matrix:

    deg(v)  = 1 + number of distinct neighbours of v          (D + I)
    row v   = { (u, 1 / sqrt(deg(v) deg(u))) : u neighbour of v or u = v }

The edge list must hold every undirected edge once, without loops or repeats
(what the generators in ntp_inputs return); loops are rejected here, repeats are
the caller's contract.  Pinned against build_graph + aggregate on small graphs in
tests/test_oracle_pins.py.
"""
from __future__ import annotations

import numpy as np

from .graph import Sparse


def rows_from_undirected_edges(n: int, src, dst, rows) -> Sparse:
    """Rows `rows` (any order, distinct) of A_hat as a Sparse with len(rows) rows;
    column indices are vertex ids, ascending within a row."""
    src = np.asarray(src)
    dst = np.asarray(dst)
    rows = np.asarray(rows, dtype=np.int64)
    if np.any(src == dst):
        raise ValueError("edge list holds self loops")
    if np.unique(rows).size != rows.size:
        raise ValueError("sampled rows must be distinct")
    deg = (np.bincount(src, minlength=n) + np.bincount(dst, minlength=n) + 1).astype(np.float64)
    pos = np.full(n, -1, dtype=np.int64)          # vertex id -> position in `rows`
    pos[rows] = np.arange(rows.size)
    # every (row, neighbour) pair of the sampled rows, from both edge directions, plus the loop
    a = pos[dst] >= 0                              # edge u -> v with v sampled: neighbour u = src
    b = pos[src] >= 0                              # the mirrored direction: neighbour = dst
    r = np.concatenate([pos[dst[a]], pos[src[b]], np.arange(rows.size)])
    u = np.concatenate([src[a].astype(np.int64), dst[b].astype(np.int64), rows])
    order = np.lexsort((u, r))
    r, u = r[order], u[order]
    rowptr = np.zeros(rows.size + 1, dtype=np.int64)
    np.cumsum(np.bincount(r, minlength=rows.size), out=rowptr[1:])
    val = (1.0 / np.sqrt(deg[rows][r] * deg[u])).astype(np.float32)
    return Sparse(rowptr, u.astype(np.int32), val)

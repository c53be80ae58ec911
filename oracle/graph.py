"""Oracle graph build: edge list -> normalised CSR (by destination) and CSC (by source).

TEST INFRASTRUCTURE.  Written from the definitions in the paper, with numpy
sorting as the only library step; shares no code with the HIP library.

Definitions followed
  * eq. (1): a vertex aggregates over its in-neighbours and itself, so every
    vertex gets one self loop (A + I).
  * eq. (3): the weight of edge u -> v is 1 / sqrt(deg_in(v) * deg_out(u)).
  * Section 4.1.3: A_hat = D~^-1/2 (A + I) D~^-1/2 with D~ = D + I, i.e. the degrees
    in eq. (3) count the self loop.  For an undirected graph both readings agree.

Canonical edge sequence (the reading taken where the paper is silent):
  1. input edges (s, d, w) in input order;
  2. SYMMETRISE appends the reversed copies (d, s, w) in input order;
  3. DEDUP drops input self loops, then keeps the first of equal (s, d) pairs;
  4. ADD_SELF_LOOPS appends (v, v, 1) for v = 0..n-1;
  5. CSR = stable sort by (d, s): row d lists in-neighbours s ascending;
     CSC = stable sort by (s, d): row s lists out-neighbours d ascending;
  6. stored value = float32( w * (1 / sqrt(din(d) * dout(s))) ), the product, the
     square root and the reciprocal in fp64, for NORM_GCN_SYM (din/dout = CSR/CSC
     row lengths), else w itself; w = 1 when no edge weights are given.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SYMMETRISE = 1
DEDUP = 2
ADD_SELF_LOOPS = 4
NORM_GCN_SYM = 8
GCN_FLAGS = SYMMETRISE | DEDUP | ADD_SELF_LOOPS | NORM_GCN_SYM
DIRECTED_GCN_FLAGS = DEDUP | ADD_SELF_LOOPS | NORM_GCN_SYM


@dataclass
class Sparse:
    """Compressed rows: row r holds entries rowptr[r]..rowptr[r+1]."""
    rowptr: np.ndarray   # int64 [n+1]
    colidx: np.ndarray   # int32 [nnz]
    val: np.ndarray      # float32 [nnz]

    @property
    def n(self) -> int:
        return self.rowptr.size - 1

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


@dataclass
class Graph:
    n: int
    csr: Sparse          # by destination: forward aggregation
    csc: Sparse          # by source: backward aggregation (the transpose)
    d_in: np.ndarray     # int64 [n], CSR row lengths
    d_out: np.ndarray    # int64 [n], CSC row lengths

    @property
    def nnz(self) -> int:
        return self.csr.nnz

    @property
    def is_symmetric(self) -> bool:
        return (np.array_equal(self.csr.rowptr, self.csc.rowptr)
                and np.array_equal(self.csr.colidx, self.csc.colidx)
                and np.array_equal(self.csr.val.view(np.uint32), self.csc.val.view(np.uint32)))


def build_graph(n: int, src, dst, flags: int = GCN_FLAGS, edge_weight=None) -> Graph:
    s = np.asarray(src, dtype=np.int64)
    d = np.asarray(dst, dtype=np.int64)
    if s.shape != d.shape or s.ndim != 1:
        raise ValueError("src and dst must be 1-D arrays of equal length")
    if s.size and (s.min() < 0 or d.min() < 0 or s.max() >= n or d.max() >= n):
        raise ValueError("vertex id out of range")
    w = np.ones(s.size, dtype=np.float32) if edge_weight is None else np.asarray(edge_weight, dtype=np.float32)
    if flags & SYMMETRISE:
        s, d, w = np.concatenate([s, d]), np.concatenate([d, s]), np.concatenate([w, w])
    if flags & DEDUP:
        keep = s != d
        s, d, w = s[keep], d[keep], w[keep]
        key = d * n + s
        _, first = np.unique(key, return_index=True)   # index of first occurrence of each pair
        first.sort()
        s, d, w = s[first], d[first], w[first]
    if flags & ADD_SELF_LOOPS:
        loops = np.arange(n, dtype=np.int64)
        s, d, w = np.concatenate([s, loops]), np.concatenate([d, loops]), np.concatenate([w, np.ones(n, np.float32)])

    def compress(major, minor):
        order = np.argsort(major * n + minor, kind="stable")
        rowptr = np.zeros(n + 1, dtype=np.int64)
        np.cumsum(np.bincount(major, minlength=n), out=rowptr[1:])
        return order, rowptr

    o_r, rp_r = compress(d, s)
    o_c, rp_c = compress(s, d)
    d_in = np.diff(rp_r)
    d_out = np.diff(rp_c)
    if flags & NORM_GCN_SYM:
        scale = 1.0 / np.sqrt(d_in[d].astype(np.float64) * d_out[s].astype(np.float64))
        v = (w.astype(np.float64) * scale).astype(np.float32)
    else:
        v = w
    csr = Sparse(rp_r, s[o_r].astype(np.int32), v[o_r])
    csc = Sparse(rp_c, d[o_c].astype(np.int32), v[o_c])
    return Graph(n, csr, csc, d_in, d_out)


def plan_chunks(rowptr: np.ndarray, chunk_edges: int):
    """Chunk boundaries of Section 4.2.1: each chunk is a contiguous range of
    destination rows together with all their entries.  Greedy reading of "as
    large as possible": a chunk is extended row by row while it holds at most
    chunk_edges entries; a row that alone exceeds chunk_edges is a chunk of its
    own.  Returns the list of (row_begin, row_end)."""
    n = rowptr.size - 1
    out = []
    r = 0
    while r < n:
        limit = int(rowptr[r]) + int(chunk_edges)
        # last row boundary whose entry offset is still within the limit
        r1 = int(np.searchsorted(rowptr, limit, side="right")) - 1
        r1 = min(max(r1, r + 1), n)
        out.append((r, r1))
        r = r1
    return out


def edge_permutation(g: Graph) -> np.ndarray:
    """perm[k] = position in the by-destination form of the edge stored at position k of the
    by-source form.  The by-source form lists the sources u ascending and, for each, its edges in
    the order the by-destination form holds them (destinations ascending), so it is the
    by-destination entries stably sorted by their source."""
    return np.argsort(g.csr.colidx, kind="stable").astype(np.int64)


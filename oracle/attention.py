"""Oracle for GAT-style edge attention weights (TEST INFRASTRUCTURE).

Follows the AGG step of GAT in Section 2.1 of the paper: for every in-edge u -> v of a
vertex v (self loop included, as in eq. 1),

    e(u -> v)     = LeakyReLU( a^T [W h_u || W h_v] ) = LeakyReLU( p[u] + q[v] )
    alpha(u -> v) = exp(e(u -> v)) / sum_{u' in N_in(v)} exp(e(u' -> v))        (softmax over
                                                                                 the in-edges of v)

where p[u] = a_src . (W h_u) and q[v] = a_dst . (W h_v) are the two halves of the mapping
a^T [. || .]; they are per-vertex scalars and are inputs here (they come out of a dense
transform).  Section 4.1 computes these coefficients for all edges before the aggregation
starts and then aggregates with them as edge weights, which is what `weighted` does.

Plain numpy in fp64, one row at a time; no max-subtraction tricks beyond the textbook
shift by the row maximum (which does not change the value of a softmax).
"""
from __future__ import annotations

from dataclasses import replace

import numpy as np

from .graph import Graph, Sparse


def leaky_relu(x, negative_slope: float):
    x = np.asarray(x, dtype=np.float64)
    return np.where(x > 0, x, negative_slope * x)


def edge_softmax(g: Graph, p, q, negative_slope: float = 0.2):
    """Attention weights of every stored entry of g.

    Returns (alpha_in, alpha_out): float64 arrays in the entry order of g.csr (row v lists
    its in-neighbours u: alpha_in[k] = alpha(u_k -> v)) and of g.csc (row u lists its
    out-neighbours v: alpha_out[k] = alpha(u -> v_k), the same numbers transposed).
    """
    p = np.asarray(p, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    n = g.n
    csr, csc = g.csr, g.csc
    alpha_in = np.empty(csr.nnz, dtype=np.float64)
    row_max = np.zeros(n, dtype=np.float64)
    row_sum = np.ones(n, dtype=np.float64)
    for v in range(n):
        b, e = int(csr.rowptr[v]), int(csr.rowptr[v + 1])
        if e == b:
            continue
        s = leaky_relu(p[csr.colidx[b:e]] + q[v], negative_slope)
        m = s.max()
        w = np.exp(s - m)
        t = w.sum()
        alpha_in[b:e] = w / t
        row_max[v], row_sum[v] = m, t
    # the same coefficients in by-source order, from the definition (not by permuting alpha_in)
    alpha_out = np.empty(csc.nnz, dtype=np.float64)
    for u in range(n):
        b, e = int(csc.rowptr[u]), int(csc.rowptr[u + 1])
        if e == b:
            continue
        vs = csc.colidx[b:e]
        s = leaky_relu(p[u] + q[vs], negative_slope)
        alpha_out[b:e] = np.exp(s - row_max[vs]) / row_sum[vs]
    return alpha_in, alpha_out


def weighted(g: Graph, alpha_in, alpha_out) -> Graph:
    """g with its stored weights replaced by attention weights (float32, as the device holds them)."""
    return replace(g,
                   csr=Sparse(g.csr.rowptr, g.csr.colidx, np.asarray(alpha_in, dtype=np.float32)),
                   csc=Sparse(g.csc.rowptr, g.csc.colidx, np.asarray(alpha_out, dtype=np.float32)))


def edge_softmax_bwd(g: Graph, p, q, Z, dY, negative_slope: float = 0.2, gate=None):
    """Gradient of a scalar loss with respect to the scores p and q through the attention
    weights, when the loss depends on them only through Y = sum_u alpha(u -> v) Z[u]
    (AGG of GAT, Section 2.1) and dY = dLoss/dY is given.  Chain rule, step by step:

        dalpha(u -> v) = dY[v] . Z[u]
        t[v]           = sum_u alpha(u -> v) dalpha(u -> v)
        de(u -> v)     = alpha(u -> v) (dalpha(u -> v) - t[v])                (softmax over the in-edges of v)
        ds(u -> v)     = de(u -> v) * (1 if p[u] + q[v] > 0 else negative_slope)   (LeakyReLU)
        dq[v]          = sum over the in-edges of v of ds,   dp[u] = sum over the out-edges of u of ds

    gate (optional, boolean per entry of g.csr): the LeakyReLU branch of every edge (True: slope 1),
    given instead of taken from the sign of p[u] + q[v] (an epoch comparison resolves the edges whose
    sign is not determined in finite precision, see oracle.gat.resolve_gate).

    Returns (dp, dq, scale_p, scale_q) in float64; the scales are the sums of |alpha| (|dalpha| + |t|)
    over the same edges (what bounds the rounding error of any evaluation order).
    """
    p = np.asarray(p, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    Z = np.asarray(Z, dtype=np.float64)
    dY = np.asarray(dY, dtype=np.float64)
    alpha_in, _ = edge_softmax(g, p, q, negative_slope)
    n = g.n
    csr = g.csr
    dp = np.zeros(n)
    dq = np.zeros(n)
    sp = np.zeros(n)
    sq = np.zeros(n)
    for v in range(n):
        b, e = int(csr.rowptr[v]), int(csr.rowptr[v + 1])
        if e == b:
            continue
        us = csr.colidx[b:e]
        a = alpha_in[b:e]
        dalpha = Z[us] @ dY[v]
        t = float(np.dot(a, dalpha))
        de = a * (dalpha - t)
        branch = (p[us] + q[v] > 0) if gate is None else np.asarray(gate[b:e], dtype=bool)
        ds = de * np.where(branch, 1.0, negative_slope)
        mag = a * (np.abs(dalpha) + abs(t))
        dq[v] = ds.sum()
        sq[v] = mag.sum()
        np.add.at(dp, us, ds)
        np.add.at(sp, us, mag)
    return dp, dq, sp, sq


def edge_softmax_bwd_rows(m: Sparse, rows, p, q, Z, dY, negative_slope: float = 0.2):
    """The same quantities for selected destinations only, for graphs too large to walk whole:
    `m` holds the in-edge lists of the destinations `rows` (row i of m = in-neighbours of rows[i],
    self loop included; its weights are not used).  Per entry, in the order of m: alpha, dalpha,
    ds; per row: t and dq.  Returns dict(alpha, dalpha, ds, t, dq, scale) with `scale` the per-row
    sum of |alpha| (|dalpha| + |t|)."""
    p = np.asarray(p, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    nnz = int(m.rowptr[-1])
    alpha = np.zeros(nnz)
    dalpha = np.zeros(nnz)
    ds = np.zeros(nnz)
    t = np.zeros(rows.size)
    dq = np.zeros(rows.size)
    scale = np.zeros(rows.size)
    for i, v in enumerate(rows):
        b, e = int(m.rowptr[i]), int(m.rowptr[i + 1])
        if e == b:
            continue
        us = m.colidx[b:e]
        s = leaky_relu(p[us] + q[v], negative_slope)
        w = np.exp(s - s.max())
        a = w / w.sum()
        alpha[b:e] = a
        if Z is None:
            continue
        da = np.asarray(Z[us], dtype=np.float64) @ np.asarray(dY[v], dtype=np.float64)
        dalpha[b:e] = da
        t[i] = float(np.dot(a, da))
        de = a * (da - t[i])
        ds[b:e] = de * np.where(p[us] + q[v] > 0, 1.0, negative_slope)
        dq[i] = ds[b:e].sum()
        scale[i] = (a * (np.abs(da) + abs(t[i]))).sum()
    return dict(alpha=alpha, dalpha=dalpha, ds=ds, t=t, dq=dq, scale=scale)

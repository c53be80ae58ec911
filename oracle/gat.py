"""Oracle for a GAT epoch in the decoupled order (TEST INFRASTRUCTURE).

Section 4.1 of the paper extends decoupled training to GAT: the NN operations run first (an
MLP on the input features), the attention coefficient of every edge is computed before the
graph aggregation starts, and the aggregation rounds then use the coefficients as the edge
weights gamma of Z^k = gamma A Z^(k-1).  With the AGG of GAT from Section 2.1 this gives, for
one epoch (one attention head):

    Lhat  = MLP(X)                                       (transforms, ReLU between, none after the last)
    p     = Lhat a_src,   q = Lhat a_dst                 (the two halves of a^T [. || .])
    alpha = softmax over the in-edges of v of LeakyReLU(p[u] + q[v])
    Z^0   = Lhat,   Z^k[v] = sum_u alpha(u -> v) Z^(k-1)[u],   k = 1..rounds
    loss  = mean softmax cross-entropy of Z^rounds

Reading (the paper does not spell out the backward pass of the coefficients): the gradient is
the exact gradient of this composed function, i.e. it also flows through alpha into a_src, a_dst
and the MLP.  Every step below is the chain rule applied to one line of the forward pass; the
whole is pinned by finite differences of `loss` (tests/test_oracle_attention_pins.py).

fp64 throughout; numpy matmul and scipy's sparse-times-dense product are the library steps.
"""
from __future__ import annotations

import numpy as np
import scipy.sparse as sp

from .attention import edge_softmax, edge_softmax_bwd
from .gcn import ACT_NONE, ACT_RELU, _transform, nn_bwd, softmax_cross_entropy, threshold
from .graph import Graph


def attention_scores(Z, a_src, a_dst):
    """p[v] = Z[v,:] . a_src, q[v] = Z[v,:] . a_dst."""
    Z = np.asarray(Z, dtype=np.float64)
    return Z @ np.asarray(a_src, dtype=np.float64), Z @ np.asarray(a_dst, dtype=np.float64)


def attention_scores_bwd(Z, a_src, a_dst, dp, dq, dZ):
    """Chain rule through p = Z a_src, q = Z a_dst: returns (dZ + dp a_src^T + dq a_dst^T,
    Z^T dp, Z^T dq) -- the gradient arriving at Z with the scores' share added, and the
    gradients of the two attention vectors."""
    Z = np.asarray(Z, dtype=np.float64)
    dp = np.asarray(dp, dtype=np.float64)
    dq = np.asarray(dq, dtype=np.float64)
    out = np.asarray(dZ, dtype=np.float64) + np.outer(dp, a_src) + np.outer(dq, a_dst)
    return out, Z.T @ dp, Z.T @ dq


def resolve_gate(g: Graph, p, q, mag_p, mag_q, tol: float, device_gate=None):
    """LeakyReLU branch of every stored edge, in by-destination entry order: (gate, ambiguous).
    The branch is the sign of s = p[u] + q[v]; an evaluation in finite precision knows the two scores
    only up to rounding, which scales with the magnitude sums of their terms (mag_p = |Lhat| |a_src|,
    mag_q = |Lhat| |a_dst|), so where |s| <= tol * (mag_p[u] + mag_q[v]) the supplied decisions
    (`device_gate`: what the device decided) are taken, and only there (as oracle.gcn.resolve_relu)."""
    rows_of = np.repeat(np.arange(g.n), np.diff(g.csr.rowptr))
    cols = g.csr.colidx
    s = p[cols] + q[rows_of]
    own = s > 0
    mag = mag_p[cols] + mag_q[rows_of]
    amb = (np.abs(s) <= threshold(tol, mag)) & (mag > 0)
    if device_gate is None:
        return own, amb
    return np.where(amb, np.asarray(device_gate, dtype=bool), own), amb


def epoch_gat_decoupled(g: Graph, X, weights, a_src, a_dst, labels, rounds: int = 2,
                        negative_slope: float = 0.2, device_relu=None, device_gate=None, tol: float = 1e-5):
    """One forward + backward pass.  Returns dict(loss, logits, dW=[...], da_src, da_dst, p, q,
    alpha_in, alpha_out, Z=[Z^0..Z^rounds], G=[G^0..G^rounds] (G^k = dloss/dZ^k), dp, dq, dLhat),
    plus what a comparison in finite precision needs: relu_keep / relu_ambiguous per hidden layer,
    gate / gate_ambiguous per edge (by-destination order), dp_mag / dq_mag (sums of the magnitudes
    of the per-edge terms of dp, dq over all rounds).  device_relu / device_gate: the device's ReLU
    and LeakyReLU decisions, used only where the sign is ambiguous at `tol`."""
    L = len(weights)
    a_src = np.asarray(a_src, dtype=np.float64)
    a_dst = np.asarray(a_dst, dtype=np.float64)
    H = np.asarray(X, dtype=np.float64)
    ins, outs, keeps, ambs, mags, pre = [], [], [], [], [], []
    for l, W in enumerate(weights):
        ins.append(H)
        H, Zl, mag, keep, amb = _transform(H, W, l == L - 1, tol, None if device_relu is None or l == L - 1 else device_relu[l])
        outs.append(H)
        pre.append(Zl)
        mags.append(mag)
        if l < L - 1:
            keeps.append(keep)
            ambs.append(amb)
    Lhat = H
    p, q = attention_scores(Lhat, a_src, a_dst)
    gate, gate_amb = resolve_gate(g, p, q, np.abs(Lhat) @ np.abs(a_src), np.abs(Lhat) @ np.abs(a_dst), tol, device_gate)
    alpha_in, alpha_out = edge_softmax(g, p, q, negative_slope)
    n = g.n
    A = sp.csr_matrix((alpha_in, g.csr.colidx, g.csr.rowptr), shape=(n, n))      # rows = destinations
    At = sp.csr_matrix((alpha_out, g.csc.colidx, g.csc.rowptr), shape=(n, n))    # rows = sources
    Z = [Lhat]
    for _ in range(rounds):
        Z.append(A @ Z[-1])
    loss, dZ = softmax_cross_entropy(Z[-1], labels)
    G = [None] * (rounds + 1)
    G[rounds] = dZ
    dp = np.zeros(n)
    dq = np.zeros(n)
    dp_mag = np.zeros(n)
    dq_mag = np.zeros(n)
    for k in range(rounds, 0, -1):
        dpk, dqk, spk, sqk = edge_softmax_bwd(g, p, q, Z[k - 1], G[k], negative_slope, gate=gate)
        dp += dpk
        dq += dqk
        dp_mag += spk
        dq_mag += sqk
        G[k - 1] = At @ G[k]
    dLhat, da_src, da_dst = attention_scores_bwd(Lhat, a_src, a_dst, dp, dq, G[0])
    dH = dLhat
    dWs = [None] * L
    for l in range(L - 1, -1, -1):
        act = ACT_RELU if l < L - 1 else ACT_NONE
        dA, dW = nn_bwd(ins[l], weights[l], outs[l], dH, act, need_dA=(l > 0), relu_mask=keeps[l] if l < L - 1 else None)
        dWs[l] = dW
        dH = dA
    return dict(loss=loss, logits=Z[-1], dW=dWs, da_src=da_src, da_dst=da_dst, p=p, q=q,
                alpha_in=alpha_in, alpha_out=alpha_out, Z=Z, G=G, dp=dp, dq=dq, dLhat=dLhat,
                nn_in=ins, hidden=outs, preact=pre, preact_mag=mags, relu_keep=keeps, relu_ambiguous=ambs,
                gate=gate, gate_ambiguous=gate_amb, dp_mag=dp_mag, dq_mag=dq_mag)

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
from .gcn import ACT_NONE, ACT_RELU, nn_bwd, nn_fwd, softmax_cross_entropy
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


def epoch_gat_decoupled(g: Graph, X, weights, a_src, a_dst, labels, rounds: int = 2,
                        negative_slope: float = 0.2, relu_masks=None):
    """One forward + backward pass.  Returns dict(loss, logits, dW=[...], da_src, da_dst, p, q,
    alpha_in, alpha_out, Z=[Z^0..Z^rounds], G=[G^0..G^rounds] (G^k = dloss/dZ^k), dp, dq, dLhat)."""
    L = len(weights)
    mk = (lambda l: relu_masks[l] if relu_masks is not None and l < L - 1 else None)
    a_src = np.asarray(a_src, dtype=np.float64)
    a_dst = np.asarray(a_dst, dtype=np.float64)
    H = np.asarray(X, dtype=np.float64)
    ins, outs = [], []
    for l, W in enumerate(weights):
        ins.append(H)
        H = nn_fwd(H, W, ACT_RELU if l < L - 1 else ACT_NONE, mk(l))
        outs.append(H)
    Lhat = H
    p, q = attention_scores(Lhat, a_src, a_dst)
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
    for k in range(rounds, 0, -1):
        dpk, dqk, _, _ = edge_softmax_bwd(g, p, q, Z[k - 1], G[k], negative_slope)
        dp += dpk
        dq += dqk
        G[k - 1] = At @ G[k]
    dLhat, da_src, da_dst = attention_scores_bwd(Lhat, a_src, a_dst, dp, dq, G[0])
    dH = dLhat
    dWs = [None] * L
    for l in range(L - 1, -1, -1):
        act = ACT_RELU if l < L - 1 else ACT_NONE
        dA, dW = nn_bwd(ins[l], weights[l], outs[l], dH, act, need_dA=(l > 0), relu_mask=mk(l))
        dWs[l] = dW
        dH = dA
    return dict(loss=loss, logits=Z[-1], dW=dWs, da_src=da_src, da_dst=da_dst, p=p, q=q,
                alpha_in=alpha_in, alpha_out=alpha_out, Z=Z, G=G, dp=dp, dq=dq, dLhat=dLhat,
                nn_in=ins, hidden=outs)

"""Oracle dense transform (eq. 4) and GCN epochs (layer-wise and decoupled).

TEST INFRASTRUCTURE.  fp64 throughout; numpy's matmul is the only library step.
"""
from __future__ import annotations

import numpy as np

from .aggregate import aggregate_fwd, aggregate_bwd
from .graph import Graph

ACT_NONE = 0
ACT_RELU = 1


def nn_fwd(A, W, act: int = ACT_NONE, relu_mask=None) -> np.ndarray:
    """UPDATE of eq. (4): H = sigma(A W), sigma = ReLU or identity.  A: [n, K]
    (one aggregated row per vertex), W: [K, M].  Row-vector convention: the
    paper's W a_v for a column vector a_v is a_v^T W^T here, W stored [K, M].

    relu_mask (optional, boolean [n, M]): take the ReLU's keep/zero decision from
    the caller instead of from the sign of the fp64 pre-activation.  An epoch
    comparison passes the decisions the fp32 device took, so that both sides
    decide a pre-activation that is zero to rounding the same way; the values
    kept are still the fp64 ones."""
    H = np.asarray(A, dtype=np.float64) @ np.asarray(W, dtype=np.float64)
    if act == ACT_RELU:
        H = np.maximum(H, 0.0) if relu_mask is None else np.where(relu_mask, H, 0.0)
    return H


def nn_bwd(A, W, H, dH, act: int = ACT_NONE, need_dA: bool = True, relu_mask=None):
    """Gradients of nn_fwd.  dZ = dH * 1[H > 0] for ReLU (else dH);
    dW = A^T dZ [K, M]; dA = dZ W^T [n, K].  With relu_mask the kept entries are
    those the mask kept (see nn_fwd)."""
    A = np.asarray(A, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    dZ = np.asarray(dH, dtype=np.float64)
    if act == ACT_RELU:
        dZ = dZ * (np.asarray(relu_mask) if relu_mask is not None else np.asarray(H) > 0)
    dW = A.T @ dZ
    dA = dZ @ W.T if need_dA else None
    return dA, dW


def softmax_cross_entropy(Z, labels):
    """Mean over all vertices of -log softmax(Z)[label]; returns (loss, dZ) with
    dZ = (softmax(Z) - onehot) / n."""
    Z = np.asarray(Z, dtype=np.float64)
    n = Z.shape[0]
    zmax = Z.max(axis=1, keepdims=True)
    e = np.exp(Z - zmax)
    p = e / e.sum(axis=1, keepdims=True)
    idx = np.arange(n)
    loss = float(np.mean(-(Z[idx, labels] - zmax[:, 0] - np.log(e.sum(axis=1)))))
    dZ = p.copy()
    dZ[idx, labels] -= 1.0
    dZ /= n
    return loss, dZ


def epoch_layerwise(g: Graph, X, weights, labels, relu_masks=None):
    """One forward + backward pass of the layer-wise workflow of Section 3.1: per
    layer aggregate (eq. 3), then transform (eq. 4); ReLU between layers, none on
    the logits.  relu_masks: optional per-layer keep/zero decisions (see nn_fwd).  Returns dict(loss, logits, dW=[...], nn_in=[A_l], hidden=[H_l], dH=[...])."""
    L = len(weights)
    mk = (lambda l: relu_masks[l] if relu_masks is not None and l < L - 1 else None)
    H = np.asarray(X, dtype=np.float64)
    aggs, hid = [], []
    for l, W in enumerate(weights):
        A = aggregate_fwd(g, H)
        H = nn_fwd(A, W, ACT_RELU if l < L - 1 else ACT_NONE, mk(l))
        aggs.append(A)
        hid.append(H)
    loss, dH = softmax_cross_entropy(H, labels)
    dWs = [None] * L
    dHs = [None] * L          # gradient arriving at each layer's output (for error scales in tests)
    for l in range(L - 1, -1, -1):
        act = ACT_RELU if l < L - 1 else ACT_NONE
        dHs[l] = dH
        dA, dW = nn_bwd(aggs[l], weights[l], hid[l], dH, act, need_dA=(l > 0), relu_mask=mk(l))
        dWs[l] = dW
        if l > 0:
            dH = aggregate_bwd(g, dA)
    return dict(loss=loss, logits=hid[-1], dW=dWs, nn_in=aggs, hidden=hid, dH=dHs)


def epoch_decoupled(g: Graph, X, weights, labels, gamma: float = 1.0, relu_masks=None):
    """One forward + backward pass in the decoupled order of Section 4.1: all L
    transforms first (an MLP, ReLU between, none after the last), then L rounds
    of aggregation Z^k = gamma * A_hat Z^(k-1); backward runs the L transposed
    aggregations, then the MLP backward."""
    L = len(weights)
    mk = (lambda l: relu_masks[l] if relu_masks is not None and l < L - 1 else None)
    H = np.asarray(X, dtype=np.float64)
    ins, outs = [], []
    for l, W in enumerate(weights):
        ins.append(H)
        H = nn_fwd(H, W, ACT_RELU if l < L - 1 else ACT_NONE, mk(l))
        outs.append(H)
    Z = H
    for _ in range(L):
        Z = gamma * aggregate_fwd(g, Z)
    loss, dZ = softmax_cross_entropy(Z, labels)
    for _ in range(L):
        dZ = gamma * aggregate_bwd(g, dZ)
    dH = dZ
    dWs = [None] * L
    dHs = [None] * L
    for l in range(L - 1, -1, -1):
        act = ACT_RELU if l < L - 1 else ACT_NONE
        dHs[l] = dH
        dA, dW = nn_bwd(ins[l], weights[l], outs[l], dH, act, need_dA=(l > 0), relu_mask=mk(l))
        dWs[l] = dW
        dH = dA
    return dict(loss=loss, logits=Z, dW=dWs, nn_in=ins, hidden=outs, dH=dHs)

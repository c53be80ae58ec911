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

    relu_mask (optional, boolean [n, M]): the ReLU's keep/zero decisions, given
    instead of taken from the sign of the fp64 pre-activation (the epochs below
    pass the decisions resolved by `resolve_relu`); the values kept are the fp64 ones."""
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


# ---------------------------------------------------------------------------------------
# ReLU decisions a finite-precision evaluation cannot be held to.
#
# The activation of eq. (4) keeps or zeroes a pre-activation z = sum_k a_k w_k by its sign.
# An fp32 evaluation knows z only up to rounding, which scales with the magnitude sum of the
# terms, sum_k |a_k w_k|; where |z| is below that error the two sides may decide differently,
# and one such entry moves a weight gradient by far more than rounding.  The oracle therefore
# works out, from its own fp64 quantities, the set of entries whose sign is NOT determined at
# the comparison tolerance:
#
#     ambiguous(z)  :=  |z| <= tol * sum_k |a_k| |w_k|
#
# Outside that set the oracle's decision is final; inside it the caller may supply decisions
# (`device_relu`: what the device decided), and only there are they used.
def threshold(tol: float, mag):
    """tol * mag, with 0 where mag is 0 (also for an infinite tol)"""
    with np.errstate(invalid="ignore"):
        return np.where(mag > 0, tol * mag, 0.0)


def resolve_relu(z, mag, tol: float, device_relu=None):
    """(keep, ambiguous): keep = z > 0 outside the ambiguous set, the supplied decision inside it.
    mag: the magnitude sums |A| |W| of the pre-activations z = A W."""
    own = z > 0
    amb = (np.abs(z) <= threshold(tol, mag)) & (mag > 0)       # mag = 0: every term is zero, nothing to round
    if device_relu is None:
        return own, amb
    return np.where(amb, np.asarray(device_relu, dtype=bool), own), amb


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


def _transform(A, W, last: bool, tol: float, device_relu, mag=None):
    """one UPDATE of an epoch: (H, pre-activation, its magnitude sums (|A| |W| unless given), keep,
    ambiguous); no activation on the last layer"""
    Z = nn_fwd(A, W)
    if mag is None:
        mag = np.abs(np.asarray(A, dtype=np.float64)) @ np.abs(np.asarray(W, dtype=np.float64))
    if last:
        return Z, Z, mag, None, None
    keep, amb = resolve_relu(Z, mag, tol, device_relu)
    return np.where(keep, Z, 0.0), Z, mag, keep, amb


def epoch_layerwise(g: Graph, X, weights, labels, device_relu=None, tol: float = 1e-5, transform_first=None):
    """One forward + backward pass of the layer-wise workflow of Section 3.1: per
    layer aggregate (eq. 3), then transform (eq. 4); ReLU between layers, none on
    the logits.  device_relu: optional per-layer keep/zero decisions of the device,
    used only on pre-activations whose sign is ambiguous at `tol` (see resolve_relu).
    transform_first (optional, one flag per layer): the evaluation being compared forms that
    layer's pre-activation as A_hat (H W) instead of (A_hat H) W.  The value is the same; the
    magnitude sum of the terms of that evaluation is |A_hat| (|H| |W|), and the ambiguous set of
    the layer is taken against it.
    Returns dict(loss, logits, dW=[...], nn_in=[A_l], hidden=[H_l], dH=[...], preact=[A_l W_l],
    preact_mag=[|A_l| |W_l|], relu_keep=[...], relu_ambiguous=[...]) (the last two per hidden layer)."""
    L = len(weights)
    H = np.asarray(X, dtype=np.float64)
    aggs, hid, keeps, ambs, pre, mags = [], [], [], [], [], []
    for l, W in enumerate(weights):
        A = aggregate_fwd(g, H)
        mag_other = None
        if transform_first is not None and transform_first[l]:
            mag_other = aggregate_fwd(g, np.abs(H) @ np.abs(np.asarray(W, dtype=np.float64)), with_abs=True)[1]
        H, Z, mag, keep, amb = _transform(A, W, l == L - 1, tol, None if device_relu is None or l == L - 1 else device_relu[l], mag_other)
        aggs.append(A)
        hid.append(H)
        pre.append(Z)
        mags.append(mag)
        if l < L - 1:
            keeps.append(keep)
            ambs.append(amb)
    loss, dH = softmax_cross_entropy(H, labels)
    dWs = [None] * L
    dHs = [None] * L          # gradient arriving at each layer's output (for error scales in tests)
    for l in range(L - 1, -1, -1):
        act = ACT_RELU if l < L - 1 else ACT_NONE
        dHs[l] = dH
        dA, dW = nn_bwd(aggs[l], weights[l], hid[l], dH, act, need_dA=(l > 0), relu_mask=keeps[l] if l < L - 1 else None)
        dWs[l] = dW
        if l > 0:
            dH = aggregate_bwd(g, dA)
    return dict(loss=loss, logits=hid[-1], dW=dWs, nn_in=aggs, hidden=hid, dH=dHs,
                preact=pre, preact_mag=mags, relu_keep=keeps, relu_ambiguous=ambs)


def epoch_decoupled(g: Graph, X, weights, labels, gamma: float = 1.0, device_relu=None, tol: float = 1e-5):
    """One forward + backward pass in the decoupled order of Section 4.1: all L
    transforms first (an MLP, ReLU between, none after the last), then L rounds
    of aggregation Z^k = gamma * A_hat Z^(k-1); backward runs the L transposed
    aggregations, then the MLP backward.  Same outputs as epoch_layerwise."""
    L = len(weights)
    H = np.asarray(X, dtype=np.float64)
    ins, outs, keeps, ambs, pre, mags = [], [], [], [], [], []
    for l, W in enumerate(weights):
        ins.append(H)
        H, Zl, mag, keep, amb = _transform(H, W, l == L - 1, tol, None if device_relu is None or l == L - 1 else device_relu[l])
        outs.append(H)
        pre.append(Zl)
        mags.append(mag)
        if l < L - 1:
            keeps.append(keep)
            ambs.append(amb)
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
        dA, dW = nn_bwd(ins[l], weights[l], outs[l], dH, act, need_dA=(l > 0), relu_mask=keeps[l] if l < L - 1 else None)
        dWs[l] = dW
        dH = dA
    return dict(loss=loss, logits=Z, dW=dWs, nn_in=ins, hidden=outs, dH=dHs,
                preact=pre, preact_mag=mags, relu_keep=keeps, relu_ambiguous=ambs)

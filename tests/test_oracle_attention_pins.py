"""Pins for the attention-weight oracle (GAT AGG of Section 2.1), each against something
other than the oracle itself:

A1 every destination's weights sum to one and are positive;
A2 with negative slope 1 the LeakyReLU is the identity and the destination's score cancels:
   alpha(u -> v) = exp(p_u) / sum_u' exp(p_u'), written out with pure Python loops;
A3 equal scores give 1 / in-degree (self loop counted);
A4 a dense brute force (dictionary of edges, math.exp) on tiny directed graphs with the
   slope the GAT paper uses;
A5 the by-source order equals the transpose of the by-destination order (scipy.sparse);
A6 a worked example by hand: a star with scores chosen so that the exponentials are powers of two;
A7 a planted mistake (score of the wrong endpoint, softmax over the out-edges) fails A4.
"""
import math

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import ntp_inputs as gen


def _directed(n, m, seed):
    src, dst = gen.directed_random_edges(n, m, seed, hub=1, hub_in=min(n - 1, 12), hub_out=min(n - 1, 5))
    return oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)


def _scores(n, seed):
    rng = gen.stream_rng(seed, 31)
    return rng.normal(size=n) * 1.5, rng.normal(size=n) * 1.5


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_a1_rows_sum_to_one(seed):
    g = _directed(300, 2500, seed)
    p, q = _scores(g.n, seed)
    a_in, a_out = oracle.edge_softmax(g, p, q, 0.2)
    assert np.all(a_in > 0) and np.all(a_out > 0)
    sums = np.add.reduceat(a_in, g.csr.rowptr[:-1])
    assert np.allclose(sums, 1.0, rtol=0, atol=1e-14)
    # the same weights, summed per destination from the by-source order
    by_dst = np.bincount(g.csc.colidx, weights=a_out, minlength=g.n)
    assert np.allclose(by_dst, 1.0, rtol=0, atol=1e-13)


def test_a2_slope_one_closed_form():
    g = _directed(60, 300, 5)
    p, q = _scores(g.n, 5)
    a_in, _ = oracle.edge_softmax(g, p, q, 1.0)
    for v in range(g.n):
        b, e = int(g.csr.rowptr[v]), int(g.csr.rowptr[v + 1])
        us = [int(u) for u in g.csr.colidx[b:e]]
        den = sum(math.exp(p[u]) for u in us)
        for k, u in enumerate(us):
            assert abs(a_in[b + k] - math.exp(p[u]) / den) <= 1e-14


def test_a3_equal_scores_give_one_over_degree():
    g = _directed(200, 1500, 7)
    a_in, a_out = oracle.edge_softmax(g, np.full(g.n, 0.3), np.full(g.n, -1.1), 0.2)
    deg = np.diff(g.csr.rowptr)
    assert np.allclose(a_in, np.repeat(1.0 / deg, deg), rtol=1e-15, atol=0)
    assert np.allclose(a_out, 1.0 / deg[g.csc.colidx], rtol=1e-15, atol=0)


def _brute_force(n, src, dst, p, q, slope, score=None, over_out_edges=False):
    """alpha[(u, v)] from the definition, with Python dictionaries and math.exp"""
    edges = set()
    for s, d in zip(src, dst):
        if int(s) != int(d):
            edges.add((int(s), int(d)))
    for v in range(n):
        edges.add((v, v))
    if score is None:
        score = lambda u, v: p[u] + q[v]
    e = {}
    for (u, v) in edges:
        x = score(u, v)
        e[(u, v)] = x if x > 0 else slope * x
    alpha = {}
    for (u, v) in edges:
        if over_out_edges:
            den = sum(math.exp(e[(uu, vv)]) for (uu, vv) in edges if uu == u)
        else:
            den = sum(math.exp(e[(uu, vv)]) for (uu, vv) in edges if vv == v)
        alpha[(u, v)] = math.exp(e[(u, v)]) / den
    return alpha


@pytest.mark.parametrize("seed", [0, 3])
def test_a4_dense_brute_force(seed):
    n = 40
    src, dst = gen.directed_random_edges(n, 200, seed, hub=2, hub_in=15, hub_out=6)
    g = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    p, q = _scores(n, seed)
    a_in, a_out = oracle.edge_softmax(g, p, q, 0.2)
    want = _brute_force(n, src, dst, p, q, 0.2)
    assert len(want) == g.csr.nnz
    for v in range(n):
        for k in range(int(g.csr.rowptr[v]), int(g.csr.rowptr[v + 1])):
            assert abs(a_in[k] - want[(int(g.csr.colidx[k]), v)]) <= 1e-14
    for u in range(n):
        for k in range(int(g.csc.rowptr[u]), int(g.csc.rowptr[u + 1])):
            assert abs(a_out[k] - want[(u, int(g.csc.colidx[k]))]) <= 1e-14


def test_a5_by_source_order_is_the_transpose():
    g = _directed(500, 6000, 11)
    p, q = _scores(g.n, 11)
    a_in, a_out = oracle.edge_softmax(g, p, q, 0.2)
    M = sp.csr_matrix((a_in, g.csr.colidx, g.csr.rowptr), shape=(g.n, g.n))       # M[v, u]
    T = M.transpose().tocsr()                                                     # T[u, v]
    T.sort_indices()
    assert np.array_equal(T.indptr, g.csc.rowptr) and np.array_equal(T.indices, g.csc.colidx)
    assert np.allclose(T.data, a_out, rtol=1e-15, atol=0)


def test_a6_worked_star():
    """centre 0 with in-edges from 1, 2, 3 (one-way) and its self loop.  Scores chosen so that
    exp(e) are 1, 2, 4, 8: p = ln(1, 2, 4, 8), q = 0, all scores >= 0 (LeakyReLU inactive):
    alpha into the centre = (1, 2, 4, 8) / 15; the leaves have only their self loop: 1."""
    n = 4
    src = np.array([1, 2, 3], dtype=np.int32)
    dst = np.array([0, 0, 0], dtype=np.int32)
    g = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    p = np.log(np.array([1.0, 2.0, 4.0, 8.0]))
    a_in, a_out = oracle.edge_softmax(g, p, np.zeros(n), 0.2)
    assert g.csr.colidx[:4].tolist() == [0, 1, 2, 3]
    assert np.allclose(a_in[:4], np.array([1, 2, 4, 8]) / 15.0, rtol=1e-15)
    assert np.allclose(a_in[4:], 1.0)
    # by source: vertex 0 -> {0}; vertex k -> {0, k}
    assert np.allclose(a_out, [1 / 15, 2 / 15, 1.0, 4 / 15, 1.0, 8 / 15, 1.0], rtol=1e-15)
    # negative scores take the slope: p = -ln(1,2,4,8)/0.5 with slope 0.5 gives exp(e) = 1, 1/2, 1/4, 1/8
    a_in, _ = oracle.edge_softmax(g, -p / 0.5, np.zeros(n), 0.5)
    assert np.allclose(a_in[:4], np.array([8, 4, 2, 1]) / 15.0, rtol=1e-14)


def test_a7_planted_mistakes_are_caught():
    n = 30
    src, dst = gen.directed_random_edges(n, 150, 4, hub=2, hub_in=10, hub_out=4)
    g = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    p, q = _scores(n, 4)
    a_in, _ = oracle.edge_softmax(g, p, q, 0.2)

    def max_diff(want):
        return max(abs(a_in[k] - want[(int(g.csr.colidx[k]), v)])
                   for v in range(n) for k in range(int(g.csr.rowptr[v]), int(g.csr.rowptr[v + 1])))

    assert max_diff(_brute_force(n, src, dst, p, q, 0.2)) <= 1e-14
    assert max_diff(_brute_force(n, src, dst, p, q, 0.2, score=lambda u, v: p[v] + q[u])) > 1e-3     # endpoints swapped
    assert max_diff(_brute_force(n, src, dst, p, q, 0.2, over_out_edges=True)) > 1e-3               # wrong normalisation set
    assert max_diff(_brute_force(n, src, dst, p, q, 0.0)) > 1e-3                                    # slope dropped


# ---- gradient of the attention weights with respect to the scores -------------------------------
def _gat_loss(g, p, q, Z, dY, slope):
    """L = sum_v dY[v] . (sum_u alpha(u -> v) Z[u]), from the forward oracle and a dense matrix"""
    a_in, _ = oracle.edge_softmax(g, p, q, slope)
    M = sp.csr_matrix((a_in, g.csr.colidx, g.csr.rowptr), shape=(g.n, g.n))
    return float(np.sum(dY * (M @ Z)))


@pytest.mark.parametrize("slope", [0.2, 0.0, 1.0])
def test_a8_score_gradients_by_finite_differences(slope):
    n, m = 25, 6
    src, dst = gen.directed_random_edges(n, 120, 8, hub=3, hub_in=12, hub_out=5)
    g = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    p, q = _scores(n, 8)
    Z = gen.normal_features(n, m, 41).astype(np.float64)
    dY = gen.normal_features(n, m, 42).astype(np.float64)
    dp, dq, _, _ = oracle.edge_softmax_bwd(g, p, q, Z, dY, slope)
    eps = 1e-6
    for i in range(n):
        for arr, grad in ((p, dp), (q, dq)):
            save = arr[i]
            arr[i] = save + eps
            lp = _gat_loss(g, p, q, Z, dY, slope)
            arr[i] = save - eps
            lm = _gat_loss(g, p, q, Z, dY, slope)
            arr[i] = save
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad[i]) <= 1e-7 * max(1.0, abs(fd)), (i, fd, grad[i])


def test_a9_score_gradient_invariants():
    """with slope 1 the weights do not depend on q at all, and a common shift of p changes
    nothing: dq = 0 and sum(dp) = 0; in general the in-edge sums and the out-edge sums add up
    the same edge terms: sum(dp) = sum(dq)"""
    n, m = 200, 9
    g = _directed(n, 1500, 13)
    p, q = _scores(n, 13)
    Z = gen.normal_features(n, m, 43).astype(np.float64)
    dY = gen.normal_features(n, m, 44).astype(np.float64)
    dp, dq, sp_, sq_ = oracle.edge_softmax_bwd(g, p, q, Z, dY, 1.0)
    assert np.abs(dq).max() <= 1e-13 * sq_.max()
    assert abs(dp.sum()) <= 1e-12 * sp_.sum()
    dp, dq, sp_, sq_ = oracle.edge_softmax_bwd(g, p, q, Z, dY, 0.2)
    assert abs(dp.sum() - dq.sum()) <= 1e-12 * sp_.sum()
    # constant features: every dalpha of a row is the same number, so the softmax gradient vanishes
    dp, dq, _, _ = oracle.edge_softmax_bwd(g, p, q, np.ones((n, m)), dY, 0.2)
    assert np.abs(dp).max() <= 1e-12 and np.abs(dq).max() <= 1e-12


# ---- A10-A12: the decoupled GAT epoch (Section 4.1 with the AGG of GAT, Section 2.1) ---------------
def _tiny_gat(seed, directed, layers=2):
    n = 50
    if directed:
        src, dst = gen.directed_random_edges(n, 260, seed)
        g = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    else:
        src, dst = gen.erdos_renyi_edges(n, 170, seed)
        g = oracle.build_graph(n, src, dst)
    dims = (8, 6, 5)[3 - layers - 1:]
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(n, dims[0]))
    Ws = [rng.normal(size=(dims[i], dims[i + 1])) * 0.6 for i in range(layers)]
    a_src = rng.normal(size=dims[-1])
    a_dst = rng.normal(size=dims[-1])
    labels = rng.integers(0, dims[-1], size=n)
    return g, X, Ws, a_src, a_dst, labels


@pytest.mark.parametrize("directed", [False, True])
@pytest.mark.parametrize("rounds,slope", [(1, 0.2), (2, 0.2), (3, 0.0), (2, 1.0)])
def test_a10_gat_epoch_finite_differences(directed, rounds, slope):
    """every parameter gradient of the epoch against central differences of its loss"""
    g, X, Ws, a_s, a_d, labels = _tiny_gat(3, directed)
    fn = lambda Ws_, s_, d_: oracle.epoch_gat_decoupled(g, X, Ws_, s_, d_, labels, rounds, slope)["loss"]
    out = oracle.epoch_gat_decoupled(g, X, Ws, a_s, a_d, labels, rounds, slope)
    eps = 1e-6
    rng = np.random.default_rng(1)

    def close(fd, an):
        assert abs(fd - an) <= 2e-6 * max(1e-3, abs(fd)) + 1e-9, (fd, an)

    for l, W in enumerate(Ws):
        for _ in range(5):
            i, j = rng.integers(W.shape[0]), rng.integers(W.shape[1])
            Wp = [w.copy() for w in Ws]
            Wm = [w.copy() for w in Ws]
            Wp[l][i, j] += eps
            Wm[l][i, j] -= eps
            close((fn(Wp, a_s, a_d) - fn(Wm, a_s, a_d)) / (2 * eps), out["dW"][l][i, j])
    for j in range(len(a_s)):
        e = np.zeros_like(a_s)
        e[j] = eps
        close((fn(Ws, a_s + e, a_d) - fn(Ws, a_s - e, a_d)) / (2 * eps), out["da_src"][j])
        close((fn(Ws, a_s, a_d + e) - fn(Ws, a_s, a_d - e)) / (2 * eps), out["da_dst"][j])


def test_a11_gat_epoch_zero_attention_vectors_is_mean_aggregation():
    """a_src = a_dst = 0: every score is equal, alpha = 1 / in-degree, and the forward pass is the
    dense row-normalised (A + I)^rounds applied to the MLP output"""
    g, X, Ws, a_s, a_d, labels = _tiny_gat(5, True)
    out = oracle.epoch_gat_decoupled(g, X, Ws, 0 * a_s, 0 * a_d, labels, rounds=2)
    n = g.n
    M = np.zeros((n, n))
    for v in range(n):
        us = g.csr.colidx[g.csr.rowptr[v]:g.csr.rowptr[v + 1]]
        M[v, us] = 1.0 / len(us)
    H = np.maximum(X @ Ws[0], 0) @ Ws[1]
    want = M @ (M @ H)
    np.testing.assert_allclose(out["logits"], want, rtol=1e-12, atol=1e-14)
    loss, _ = oracle.softmax_cross_entropy(want, labels)
    assert abs(out["loss"] - loss) <= 1e-14
    # the MLP's gradient is then that of the fixed linear map M^2 (alpha's own gradient only moves a)
    dH = (M @ M).T @ oracle.softmax_cross_entropy(want, labels)[1]
    np.testing.assert_allclose(out["dLhat"], dH, rtol=1e-11, atol=1e-14)


def test_a12_gat_epoch_identity_graph_reduces_to_mlp():
    """no edges but the self loops: alpha = 1 on every self loop, Z^k = Lhat, zero attention gradient"""
    g, X, Ws, a_s, a_d, labels = _tiny_gat(7, True)
    n = g.n
    gi = oracle.build_graph(n, np.zeros(0, np.int32), np.zeros(0, np.int32), oracle.DIRECTED_GCN_FLAGS)
    out = oracle.epoch_gat_decoupled(gi, X, Ws, a_s, a_d, labels, rounds=3)
    H0 = X @ Ws[0]
    H = np.maximum(H0, 0) @ Ws[1]
    loss, dZ = oracle.softmax_cross_entropy(H, labels)
    assert abs(out["loss"] - loss) <= 1e-14
    np.testing.assert_allclose(out["alpha_in"], 1.0)
    np.testing.assert_allclose(out["da_src"], 0.0, atol=1e-15)
    np.testing.assert_allclose(out["da_dst"], 0.0, atol=1e-15)
    np.testing.assert_allclose(out["dW"][1], np.maximum(H0, 0).T @ dZ, rtol=1e-12, atol=1e-15)


def test_a12_attention_scores_bwd_is_the_adjoint():
    """<dp, Z a_src> + <dq, Z a_dst> seen from the other side: sum(dZ_added * Z') for a direction Z'
    equals the change of dp . p + dq . q; and the vector gradients are the matching contractions"""
    rng = np.random.default_rng(0)
    Z = rng.normal(size=(30, 7))
    a_s, a_d = rng.normal(size=7), rng.normal(size=7)
    dp, dq = rng.normal(size=30), rng.normal(size=30)
    out, da_s, da_d = oracle.attention_scores_bwd(Z, a_s, a_d, dp, dq, np.zeros_like(Z))
    Zd = rng.normal(size=Z.shape)
    pd, qd = oracle.attention_scores(Zd, a_s, a_d)
    assert abs(np.sum(out * Zd) - (dp @ pd + dq @ qd)) <= 1e-12
    ad = rng.normal(size=7)
    assert abs(da_s @ ad - dp @ (Z @ ad)) <= 1e-12 and abs(da_d @ ad - dq @ (Z @ ad)) <= 1e-12


def test_a13_row_restricted_score_gradient_matches_the_whole_graph_oracle():
    """edge_softmax_bwd_rows on rows built one by one from the edge list gives, for those rows, what
    the whole-graph functions (pinned above) give; dp of a vertex follows from the ds of its
    out-edges found in its neighbours' rows"""
    n = 400
    src, dst = gen.erdos_renyi_edges(n, 2500, 8)
    g = oracle.build_graph(n, src, dst)
    rng = np.random.default_rng(2)
    p, q = rng.normal(size=n), rng.normal(size=n)
    Z, dY = rng.normal(size=(n, 6)), rng.normal(size=(n, 6))
    a_in, _ = oracle.edge_softmax(g, p, q, 0.2)
    dp, dq, _, sq = oracle.edge_softmax_bwd(g, p, q, Z, dY, 0.2)
    rows = np.sort(rng.choice(n, size=60, replace=False))
    m = oracle.rows_from_undirected_edges(n, src, dst, rows)
    out = oracle.edge_softmax_bwd_rows(m, rows, p, q, Z, dY, 0.2)
    for i, v in enumerate(rows):
        b, e = g.csr.rowptr[v], g.csr.rowptr[v + 1]
        assert np.array_equal(m.colidx[m.rowptr[i]:m.rowptr[i + 1]], g.csr.colidx[b:e])
        np.testing.assert_allclose(out["alpha"][m.rowptr[i]:m.rowptr[i + 1]], a_in[b:e], rtol=1e-13)
    np.testing.assert_allclose(out["dq"], dq[rows], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(out["scale"], sq[rows], rtol=1e-12)
    # dp[u] for one vertex: every neighbour's row, the entry whose column is u
    u = int(rows[0])
    nb = g.csr.colidx[g.csr.rowptr[u]:g.csr.rowptr[u + 1]].astype(np.int64)       # symmetric graph: out-neighbours
    mu = oracle.rows_from_undirected_edges(n, src, dst, nb)
    ou = oracle.edge_softmax_bwd_rows(mu, nb, p, q, Z, dY, 0.2)
    total = 0.0
    for i in range(nb.size):
        cols = mu.colidx[mu.rowptr[i]:mu.rowptr[i + 1]]
        total += ou["ds"][mu.rowptr[i]:mu.rowptr[i + 1]][cols == u].sum()
    assert abs(total - dp[u]) <= 1e-12 * max(1.0, abs(dp[u]))


def test_a14_leaky_relu_branch_argument_and_ambiguous_edges():
    """edge_softmax_bwd with the branches given: the oracle's own branches change nothing; flipping one
    edge's branch changes dq of its destination and dp of its source by (1 - slope) x that edge's
    softmax term.  resolve_gate hands over exactly the edges whose score sum is zero at the tolerance."""
    n = 120
    src, dst = gen.directed_random_edges(n, 700, 5)
    g = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    rng = np.random.default_rng(4)
    p, q = rng.normal(size=n), rng.normal(size=n)
    Z, dY = rng.normal(size=(n, 5)), rng.normal(size=(n, 5))
    slope = 0.2
    rows_of = np.repeat(np.arange(n), np.diff(g.csr.rowptr))
    own = p[g.csr.colidx] + q[rows_of] > 0
    base = oracle.edge_softmax_bwd(g, p, q, Z, dY, slope)
    same = oracle.edge_softmax_bwd(g, p, q, Z, dY, slope, gate=own)
    for a, b in zip(base, same):
        np.testing.assert_array_equal(a, b)
    k = int(np.flatnonzero(own)[17])              # an edge on the slope-1 branch
    v, u = int(rows_of[k]), int(g.csr.colidx[k])
    flipped = own.copy()
    flipped[k] = False
    dp2, dq2, _, _ = oracle.edge_softmax_bwd(g, p, q, Z, dY, slope, gate=flipped)
    a_in, _ = oracle.edge_softmax(g, p, q, slope)
    b, e = g.csr.rowptr[v], g.csr.rowptr[v + 1]
    dalpha = Z[g.csr.colidx[b:e]] @ dY[v]
    de_k = a_in[k] * (dalpha[k - b] - a_in[b:e] @ dalpha)
    assert abs((base[1][v] - dq2[v]) - (1 - slope) * de_k) <= 1e-14
    assert abs((base[0][u] - dp2[u]) - (1 - slope) * de_k) <= 1e-14
    changed_q = np.flatnonzero(base[1] != dq2)
    changed_p = np.flatnonzero(base[0] != dp2)
    assert list(changed_q) == [v] and list(changed_p) == [u]
    # resolve_gate: plant one score sum of relative size 1e-9
    q2 = q.copy()
    mag_p, mag_q = np.abs(p) + 0.5, np.abs(q) + 0.5
    kk = int(g.csr.rowptr[40])                    # first in-edge of vertex 40
    q2[40] = -p[g.csr.colidx[kk]] + 1e-9
    gate, amb = oracle.resolve_gate(g, p, q2, mag_p, mag_q, 1e-5)
    assert amb[kk] and gate[kk]                   # tiny but positive: the oracle's own branch
    others = np.flatnonzero(amb)
    assert others.size >= 1 and np.all(np.abs(p[g.csr.colidx[others]] + q2[rows_of[others]]) <= 1e-5 * 20)
    dev = np.zeros(g.csr.nnz, dtype=bool)         # a device that puts every edge on the negative branch
    gate2, _ = oracle.resolve_gate(g, p, q2, mag_p, mag_q, 1e-5, device_gate=dev)
    assert not gate2[kk] and np.array_equal(gate2[~amb], gate[~amb])
    gate3, amb3 = oracle.resolve_gate(g, p, q2, mag_p, mag_q, 0.0, device_gate=dev)
    assert not amb3.any() and np.array_equal(gate3, p[g.csr.colidx] + q2[rows_of] > 0)


def test_a15_gat_epoch_device_decisions_count_only_where_ambiguous():
    """with tol = 0 arbitrary ReLU and LeakyReLU decisions handed to the epoch change nothing"""
    g, X, Ws, a_s, a_d, labels = _tiny_gat(9, True)
    a = oracle.epoch_gat_decoupled(g, X, Ws, a_s, a_d, labels, 2, 0.2)
    wrong_relu = [np.zeros_like(h, dtype=bool) for h in a["hidden"][:-1]]
    wrong_gate = np.ones(g.csr.nnz, dtype=bool)
    b = oracle.epoch_gat_decoupled(g, X, Ws, a_s, a_d, labels, 2, 0.2, device_relu=wrong_relu, device_gate=wrong_gate, tol=0.0)
    assert a["loss"] == b["loss"]
    for x, y in zip(a["dW"] + [a["da_src"], a["da_dst"]], b["dW"] + [b["da_src"], b["da_dst"]]):
        np.testing.assert_array_equal(x, y)
    c = oracle.epoch_gat_decoupled(g, X, Ws, a_s, a_d, labels, 2, 0.2, device_gate=wrong_gate, tol=np.inf)
    d = oracle.epoch_gat_decoupled(g, X, Ws, a_s, a_d, labels, 2, 1.0)      # every edge on the slope-1 branch = slope 1 ...
    # ... in the backward pass only: the forward still uses slope 0.2, so only check that the gradient moved
    assert c["loss"] == a["loss"] and not np.array_equal(c["da_src"], a["da_src"])
    assert d["loss"] != a["loss"]

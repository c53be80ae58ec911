"""Pins for the CPU oracle: each check ties it to something other than itself.

P1 brute-force dense A_hat built entry by entry from the definition;
P2 closed form of A_hat applied to the constant vector;
P3 fixed point A_hat sqrt(d) = sqrt(d), norm bound (Section 4.1.3);
P4 textbook graphs (empty, complete, star, ring);
P5 adjoint identity and explicit dense transpose on directed graphs;
P6 chunk and column-slice invariance (Sections 4.2.1 and 3.1);
P7 transform / epoch: finite differences, identity-adjacency reduction to an MLP;
P8 structure invariants of the compressed rows;
G  hand-derived fixture under tests/golden/.
"""
import os

import numpy as np
import pytest

import oracle
from oracle import gcn
import ntp_inputs as gen

HERE = os.path.dirname(os.path.abspath(__file__))


# ----------------------------------------------------------------------------
# an independent, dictionary-based construction of A_hat (pure Python loops)
def dense_ahat(n, src, dst, symmetrise=True):
    adj = [[0.0] * n for _ in range(n)]          # adj[v][u] = 1 if edge u -> v
    for s, d in zip(src, dst):
        s, d = int(s), int(d)
        if s == d:
            continue
        adj[d][s] = 1.0
        if symmetrise:
            adj[s][d] = 1.0
    for v in range(n):
        adj[v][v] = 1.0                           # A + I
    din = [sum(adj[v]) for v in range(n)]         # row sums: in-degree + 1
    dout = [sum(adj[v][u] for v in range(n)) for u in range(n)]
    A = np.zeros((n, n))
    for v in range(n):
        for u in range(n):
            if adj[v][u]:
                A[v, u] = 1.0 / np.sqrt(din[v] * dout[u])
    return A


def f32(a):
    """The stored weights are rounded to float32: compare against that."""
    return a.astype(np.float32).astype(np.float64)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_p1_dense_bruteforce_undirected(seed):
    n, m, f = 57, 160, 5
    src, dst = gen.erdos_renyi_edges(n, m, seed)
    g = oracle.build_graph(n, src, dst)
    A = f32(dense_ahat(n, src, dst, True))
    X = gen.normal_features(n, f, seed).astype(np.float64)
    np.testing.assert_allclose(oracle.aggregate_fwd(g, X), A @ X, rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.aggregate_bwd(g, X), A.T @ X, rtol=0, atol=1e-13)
    assert g.is_symmetric


@pytest.mark.parametrize("seed", [0, 3])
def test_p1_p5_dense_bruteforce_directed(seed):
    n, f = 41, 4
    src, dst = gen.directed_random_edges(n, 150, seed, hub=7, hub_in=25, hub_out=3)
    g = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    A = f32(dense_ahat(n, src, dst, False))
    assert not np.allclose(A, A.T)               # the test must be able to see a missing transpose
    X = gen.normal_features(n, f, seed).astype(np.float64)
    np.testing.assert_allclose(oracle.aggregate_fwd(g, X), A @ X, atol=1e-13)
    np.testing.assert_allclose(oracle.aggregate_bwd(g, X), A.T @ X, atol=1e-13)
    np.testing.assert_allclose(oracle.aggregate_bwd_scatter(g, X), A.T @ X, atol=1e-13)
    assert not g.is_symmetric


def test_p2_constant_vector_closed_form():
    n = 300
    src, dst = gen.rmat_edges(n, 1500, seed=4)
    g = oracle.build_graph(n, src, dst)
    # degrees recomputed independently from the raw edge list
    nbrs = [set([v]) for v in range(n)]
    for s, d in zip(src.tolist(), dst.tolist()):
        nbrs[s].add(d)
        nbrs[d].add(s)
    deg = np.array([len(x) for x in nbrs], dtype=np.float64)
    want = np.array([sum(1.0 / np.sqrt(deg[j]) for j in nbrs[i]) / np.sqrt(deg[i]) for i in range(n)])
    got = oracle.aggregate_fwd(g, np.ones((n, 1)))[:, 0]
    np.testing.assert_allclose(got, want, rtol=2e-7)   # float32 weights


def test_p3_fixed_point_and_norm_bound():
    n = 400
    src, dst = gen.rmat_edges(n, 2500, seed=5)
    g = oracle.build_graph(n, src, dst)
    sq = np.sqrt(g.d_in.astype(np.float64))[:, None]
    np.testing.assert_allclose(oracle.aggregate_fwd(g, sq), sq, rtol=3e-7)
    x = gen.normal_features(n, 3, 5).astype(np.float64)
    y = x
    for _ in range(6):
        y2 = oracle.aggregate_fwd(g, y)
        assert np.all(np.linalg.norm(y2, axis=0) <= np.linalg.norm(y, axis=0) * (1 + 1e-6))
        y = y2


def test_p4_textbook_graphs():
    n, f = 9, 3
    X = gen.normal_features(n, f, 6).astype(np.float64)
    empty = oracle.build_graph(n, np.zeros(0, np.int32), np.zeros(0, np.int32))
    np.testing.assert_array_equal(oracle.aggregate_fwd(empty, X), X)          # A_hat = I
    s, d = np.triu_indices(n, 1)
    complete = oracle.build_graph(n, s, d)
    np.testing.assert_allclose(oracle.aggregate_fwd(complete, X),
                               np.broadcast_to(X.mean(axis=0), (n, f)), rtol=1e-6)
    ring = oracle.build_graph(n, np.arange(n), (np.arange(n) + 1) % n)
    assert np.all(ring.csr.val == np.float32(1.0 / 3.0))
    np.testing.assert_allclose(oracle.aggregate_fwd(ring, X),
                               (X + np.roll(X, 1, 0) + np.roll(X, -1, 0)) / 3.0, rtol=1e-6)
    star = oracle.build_graph(n, np.zeros(n - 1, np.int64), np.arange(1, n))
    y = oracle.aggregate_fwd(star, X)
    np.testing.assert_allclose(y[0], X[0] / n + X[1:].sum(0) / np.sqrt(2.0 * n), rtol=1e-6)
    np.testing.assert_allclose(y[3], X[3] / 2 + X[0] / np.sqrt(2.0 * n), rtol=1e-6)


def test_p4_isolated_vertex_and_no_self_loops():
    # with self loops an isolated vertex keeps its own value
    g = oracle.build_graph(4, [0], [1])
    X = np.arange(8, dtype=np.float64).reshape(4, 2)
    np.testing.assert_array_equal(oracle.aggregate_fwd(g, X)[3], X[3])
    # without self loops an isolated vertex has an empty row and gets zero
    g2 = oracle.build_graph(4, [0], [1], oracle.SYMMETRISE | oracle.DEDUP | oracle.NORM_GCN_SYM)
    y = oracle.aggregate_fwd(g2, X)
    np.testing.assert_array_equal(y[3], 0)
    np.testing.assert_allclose(y[0], X[1])       # both degrees 1


@pytest.mark.parametrize("seed", [0, 1])
def test_p5_adjoint_identity(seed):
    n, f = 500, 3
    src, dst = gen.directed_random_edges(n, 4000, seed, hub=11, hub_in=300, hub_out=40)
    g = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    x = gen.normal_features(n, f, seed).astype(np.float64)
    y = gen.normal_features(n, f, seed + 100).astype(np.float64)
    lhs = np.sum(oracle.aggregate_fwd(g, x) * y)
    rhs = np.sum(x * oracle.aggregate_bwd(g, y))
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
    # gather form over by-source rows == scatter form over by-destination rows, bit for bit
    np.testing.assert_array_equal(oracle.aggregate_bwd(g, y), oracle.aggregate_bwd_scatter(g, y))


def test_p6_chunk_and_slice_invariance():
    n, f = 300, 12
    src, dst = gen.rmat_edges(n, 2000, seed=7)
    g = oracle.build_graph(n, src, dst)
    X = gen.normal_features(n, f, 7)
    full = oracle.aggregate_fwd(g, X)
    for ce in [1, 2, 7, 13, 101, 997, g.nnz // 3, g.nnz, 10 * g.nnz]:
        np.testing.assert_array_equal(oracle.chunked_aggregate(g.csr, X, ce), full)
        chunks = oracle.plan_chunks(g.csr.rowptr, ce)
        assert chunks[0][0] == 0 and chunks[-1][1] == n
        assert all(a[1] == b[0] for a, b in zip(chunks, chunks[1:]))
        for r0, r1 in chunks:                     # greedy and maximal
            e = g.csr.rowptr[r1] - g.csr.rowptr[r0]
            assert e <= ce or r1 == r0 + 1
            if r1 < n:
                assert g.csr.rowptr[r1 + 1] - g.csr.rowptr[r0] > ce
    for a, b in [(0, 3), (5, 12), (4, 5)]:
        np.testing.assert_array_equal(oracle.aggregate_fwd(g, X[:, a:b]), full[:, a:b])
    rows = np.array([5, 0, 299, 17], dtype=np.int64)
    np.testing.assert_array_equal(oracle.aggregate_fwd(g, X, rows=rows), full[rows])


def test_sampled_rows_match_full_build():
    """the row-by-row construction used for full-size samples equals the rows of the full build"""
    n = 900
    src, dst = gen.rmat_edges(n, 7000, seed=17)
    g = oracle.build_graph(n, src, dst)
    rows = np.array([17, 3, 899, 0, 450, int(np.argmax(g.d_in))], dtype=np.int64)
    m = oracle.rows_from_undirected_edges(n, src, dst, rows)
    for i, v in enumerate(rows):
        a, b = g.csr.rowptr[v], g.csr.rowptr[v + 1]
        np.testing.assert_array_equal(m.colidx[m.rowptr[i]:m.rowptr[i + 1]], g.csr.colidx[a:b])
        np.testing.assert_array_equal(m.val[m.rowptr[i]:m.rowptr[i + 1]].view(np.uint32), g.csr.val[a:b].view(np.uint32))
    X = gen.normal_features(n, 5, 17)
    np.testing.assert_array_equal(oracle.aggregate(m, X), oracle.aggregate_fwd(g, X, rows=rows))
    with pytest.raises(ValueError):
        oracle.rows_from_undirected_edges(n, [1, 2], [1, 3], rows)


def test_abs_sum_bounds_result():
    n = 200
    src, dst = gen.rmat_edges(n, 900, seed=8)
    g = oracle.build_graph(n, src, dst)
    X = gen.normal_features(n, 4, 8)
    y, ya = oracle.aggregate_fwd(g, X, with_abs=True)
    assert np.all(np.abs(y) <= ya * (1 + 1e-12))
    ypos, _ = oracle.aggregate_fwd(g, np.abs(X), with_abs=True)
    np.testing.assert_allclose(ya, ypos, rtol=1e-14)


def test_p7_transform_special_cases():
    A = gen.normal_features(30, 6, 9).astype(np.float64)
    np.testing.assert_array_equal(gcn.nn_fwd(A, np.eye(6)), A)
    np.testing.assert_array_equal(gcn.nn_fwd(A, np.eye(6), gcn.ACT_RELU), np.maximum(A, 0))
    w = np.arange(1, 7, dtype=np.float64)[:, None]
    np.testing.assert_allclose(gcn.nn_fwd(A, w)[:, 0], sum(A[:, k] * (k + 1) for k in range(6)), rtol=1e-14)
    # explicit triple loop on a tiny case (catches a transposed operand)
    A2, W2 = A[:4, :3], gen.normal_features(3, 5, 10).astype(np.float64)
    want = np.zeros((4, 5))
    for i in range(4):
        for j in range(5):
            for k in range(3):
                want[i, j] += A2[i, k] * W2[k, j]
    np.testing.assert_allclose(gcn.nn_fwd(A2, W2), want, rtol=1e-14)
    dH = gen.normal_features(4, 5, 11).astype(np.float64)
    H = gcn.nn_fwd(A2, W2, gcn.ACT_RELU)
    dA, dW = gcn.nn_bwd(A2, W2, H, dH, gcn.ACT_RELU)
    dZ = dH * (H > 0)
    wantW = np.zeros((3, 5))
    wantA = np.zeros((4, 3))
    for i in range(4):
        for j in range(5):
            for k in range(3):
                wantW[k, j] += A2[i, k] * dZ[i, j]
                wantA[i, k] += dZ[i, j] * W2[k, j]
    np.testing.assert_allclose(dW, wantW, rtol=1e-13)
    np.testing.assert_allclose(dA, wantA, rtol=1e-13)


def _tiny_model(seed, directed=False):
    n = 60
    if directed:
        src, dst = gen.directed_random_edges(n, 300, seed)
        g = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    else:
        src, dst = gen.erdos_renyi_edges(n, 200, seed)
        g = oracle.build_graph(n, src, dst)
    dims = (9, 7, 6, 4)
    X = gen.normal_features(n, dims[0], seed).astype(np.float64)
    Ws = [gen.glorot_weight(dims[i], dims[i + 1], seed, i).astype(np.float64) for i in range(3)]
    labels = gen.uniform_labels(n, dims[-1], seed)
    return g, X, Ws, labels


@pytest.mark.parametrize("epoch", ["layerwise", "decoupled"])
@pytest.mark.parametrize("directed", [False, True])
def test_p7_epoch_finite_differences(epoch, directed):
    fn = gcn.epoch_layerwise if epoch == "layerwise" else gcn.epoch_decoupled
    g, X, Ws, labels = _tiny_model(12, directed)
    out = fn(g, X, Ws, labels)
    eps = 1e-6
    rng = np.random.default_rng(0)
    for l, W in enumerate(Ws):
        for _ in range(4):
            i, j = rng.integers(W.shape[0]), rng.integers(W.shape[1])
            Wp = [w.copy() for w in Ws]
            Wm = [w.copy() for w in Ws]
            Wp[l][i, j] += eps
            Wm[l][i, j] -= eps
            fd = (fn(g, X, Wp, labels)["loss"] - fn(g, X, Wm, labels)["loss"]) / (2 * eps)
            assert abs(fd - out["dW"][l][i, j]) <= 1e-6 * max(1e-3, abs(fd)) + 1e-9


def test_p7_identity_adjacency_reduces_to_mlp():
    n = 25
    g = oracle.build_graph(n, np.zeros(0, np.int32), np.zeros(0, np.int32))
    X = gen.normal_features(n, 5, 13).astype(np.float64)
    Ws = [gen.glorot_weight(5, 4, 13, 0).astype(np.float64), gen.glorot_weight(4, 3, 13, 1).astype(np.float64)]
    labels = gen.uniform_labels(n, 3, 13)
    a = gcn.epoch_layerwise(g, X, Ws, labels)
    b = gcn.epoch_decoupled(g, X, Ws, labels)
    Z = np.maximum(X @ Ws[0], 0) @ Ws[1]
    np.testing.assert_allclose(a["logits"], Z, rtol=1e-13)
    np.testing.assert_allclose(b["logits"], Z, rtol=1e-13)
    # loss against the textbook log-sum-exp form
    lse = np.log(np.exp(Z).sum(1))
    assert abs(a["loss"] - np.mean(lse - Z[np.arange(n), labels])) < 1e-12
    for x, y in zip(a["dW"], b["dW"]):
        np.testing.assert_allclose(x, y, rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("epoch", ["layerwise", "decoupled"])
def test_p7_device_relu_decisions_count_only_where_the_sign_is_ambiguous(epoch):
    """Decisions handed to the epoch are used only on pre-activations that are zero at the given
    tolerance: with tol = 0 nothing but exact zeros is ambiguous and arbitrary decisions change
    nothing; with an infinite tolerance every entry is ambiguous and the decisions are the activation;
    a planted near-zero pre-activation is the one entry a small tolerance hands over"""
    fn = gcn.epoch_layerwise if epoch == "layerwise" else gcn.epoch_decoupled
    g, X, Ws, labels = _tiny_model(16)
    a = fn(g, X, Ws, labels)
    assert all(not amb.any() for amb in fn(g, X, Ws, labels, tol=0.0)["relu_ambiguous"])
    for k, keep in enumerate(a["relu_keep"]):
        np.testing.assert_array_equal(keep, a["preact"][k] > 0)
    wrong = [np.ones_like(h, dtype=bool) for h in a["hidden"][:-1]]
    b = fn(g, X, Ws, labels, device_relu=wrong, tol=0.0)
    assert a["loss"] == b["loss"]
    for x, y in zip(a["dW"], b["dW"]):
        np.testing.assert_array_equal(x, y)
    c = fn(g, X, Ws, labels, device_relu=wrong, tol=np.inf)          # identity activation everywhere
    np.testing.assert_allclose(c["hidden"][0], c["nn_in"][0] @ Ws[0], rtol=1e-14)
    assert all(amb.all() for amb in c["relu_ambiguous"]) and c["loss"] != a["loss"]
    # plant a pre-activation of relative size 1e-9 in layer 0: shift one weight column so that
    # entry (v, j) of the first pre-activation becomes 1e-9 of its magnitude sum
    v, j = 7, 3
    A0 = a["nn_in"][0]
    W0 = Ws[0].copy()
    k = int(np.argmax(np.abs(A0[v])))
    target = 1e-9 * (np.abs(A0[v]) @ np.abs(W0[:, j]))
    W0[k, j] -= (a["preact"][0][v, j] - target) / A0[v, k]
    Wp = [W0] + Ws[1:]
    base = fn(g, X, Wp, labels)
    amb0 = base["relu_ambiguous"][0]
    assert amb0[v, j] and amb0.sum() == 1 and base["relu_keep"][0][v, j]            # tiny but positive: kept
    flip = [np.ones_like(h, dtype=bool) for h in base["hidden"][:-1]]
    flip[0][v, j] = False
    d = fn(g, X, Wp, labels, device_relu=flip)
    assert not d["relu_keep"][0][v, j] and (d["relu_keep"][0] != base["relu_keep"][0]).sum() == 1
    assert d["hidden"][0][v, j] == 0.0
    # the gradient of W0[:, j] loses exactly that entry's term A0[v, :] * dZ[v, j] (first layer: nothing upstream changes;
    # downstream the forward value moved by 1e-9 of its scale only)
    dZ_vj = base["dH"][0][v, j]
    np.testing.assert_allclose(base["dW"][0][:, j] - d["dW"][0][:, j], base["nn_in"][0][v] * dZ_vj, rtol=1e-5, atol=1e-12)


def test_p7_transform_first_changes_only_the_magnitude_sums():
    """naming the other evaluation order of a layer changes no value; its magnitude sums
    |A_hat| (|H| |W|) are never below those of the aggregate-first order, |A_hat H| |W|"""
    g, X, Ws, labels = _tiny_model(19, directed=True)
    a = gcn.epoch_layerwise(g, X, Ws, labels)
    b = gcn.epoch_layerwise(g, X, Ws, labels, transform_first=[True, False, True])
    assert a["loss"] == b["loss"]
    for x, y in zip(a["dW"], b["dW"]):
        np.testing.assert_array_equal(x, y)
    np.testing.assert_array_equal(a["preact_mag"][1], b["preact_mag"][1])
    for l in (0, 2):
        assert np.all(b["preact_mag"][l] >= a["preact_mag"][l] * (1 - 1e-14))
    assert (b["preact_mag"][0] > a["preact_mag"][0] * 1.01).any()       # signed inputs cancel in A_hat H
    # dense check of the other order's magnitude sums on layer 0
    n = g.n
    D = np.zeros((n, n))
    for v in range(n):
        for k in range(g.csr.rowptr[v], g.csr.rowptr[v + 1]):
            D[v, g.csr.colidx[k]] += abs(float(g.csr.val[k]))
    np.testing.assert_allclose(b["preact_mag"][0], D @ (np.abs(X) @ np.abs(Ws[0])), rtol=1e-12)


def test_p7_decoupled_is_power_of_ahat():
    g, X, Ws, labels = _tiny_model(14)
    out = gcn.epoch_decoupled(g, X, Ws, labels)
    H = X
    for l, W in enumerate(Ws):
        H = H @ W
        if l < 2:
            H = np.maximum(H, 0)
    # dense A_hat^3 from the stored weights
    A = np.zeros((g.n, g.n))
    for v in range(g.n):
        for k in range(g.csr.rowptr[v], g.csr.rowptr[v + 1]):
            A[v, g.csr.colidx[k]] += g.csr.val[k]
    np.testing.assert_allclose(out["logits"], np.linalg.matrix_power(A, 3) @ H, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("directed", [False, True])
def test_p8_structure_invariants(directed):
    n = 700
    if directed:
        src, dst = gen.directed_random_edges(n, 6000, 15, hub=3, hub_in=500, hub_out=20)
        g = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    else:
        src, dst = gen.rmat_edges(n, 5000, seed=15)
        g = oracle.build_graph(n, src, dst)
    for m in (g.csr, g.csc):
        assert m.rowptr[0] == 0 and m.rowptr[-1] == m.colidx.size == m.val.size
        assert np.all(np.diff(m.rowptr) >= 1)                      # the self loop
        for r in range(n):
            cols = m.colidx[m.rowptr[r]:m.rowptr[r + 1]]
            assert np.all(np.diff(cols) > 0)                       # strictly ascending
            assert np.count_nonzero(cols == r) == 1                # exactly one diagonal entry
    assert g.d_in.sum() == g.d_out.sum() == g.nnz
    # the by-source rows are exactly the transpose pattern, with the same stored value
    rows = np.repeat(np.arange(n), np.diff(g.csr.rowptr))
    a = sorted(zip(g.csr.colidx.tolist(), rows.tolist(), g.csr.val.view(np.uint32).tolist()))
    rows_c = np.repeat(np.arange(n), np.diff(g.csc.rowptr))
    b = sorted(zip(rows_c.tolist(), g.csc.colidx.tolist(), g.csc.val.view(np.uint32).tolist()))
    assert a == b
    # the edge set equals the deduplicated input plus loops
    want = set((int(s), int(d)) for s, d in zip(src, dst) if s != d)
    if not directed:
        want |= set((d, s) for s, d in want)
    want |= set((v, v) for v in range(n))
    assert set(zip(g.csr.colidx.tolist(), rows.tolist())) == want


def test_build_flags_and_weights():
    # no DEDUP: parallel edges and input loops stay, in input order; custom weights pass through
    src = np.array([0, 0, 2, 1, 0], dtype=np.int32)
    dst = np.array([1, 1, 2, 0, 1], dtype=np.int32)
    w = np.array([0.5, 0.25, 2.0, 3.0, 0.125], dtype=np.float32)
    g = oracle.build_graph(3, src, dst, 0, w)
    assert g.csr.rowptr.tolist() == [0, 1, 4, 5]
    assert g.csr.colidx.tolist() == [1, 0, 0, 0, 2]
    assert g.csr.val.tolist() == [3.0, 0.5, 0.25, 0.125, 2.0]
    # DEDUP keeps the first weight; symmetrised copies come after all originals
    g = oracle.build_graph(3, src, dst, oracle.DEDUP | oracle.SYMMETRISE, w)
    assert g.csr.colidx.tolist() == [1, 0]
    assert g.csr.val.tolist() == [3.0, 0.5]      # edge 1->0 was given (3.0) before the mirrored 0->1
    g = oracle.build_graph(3, src, dst, oracle.DEDUP | oracle.ADD_SELF_LOOPS | oracle.NORM_GCN_SYM, w)
    # din = (2, 2, 1), dout = (2, 2, 1); entry (v=1,u=0) = 0.5 / sqrt(2*2)
    assert g.csr.colidx.tolist() == [0, 1, 0, 1, 2]
    np.testing.assert_array_equal(g.csr.val, np.array([0.5, 1.5, 0.25, 0.5, 1.0], np.float32))


def test_round_bf16():
    x = np.array([1.0, 1.00390625, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -2.5, 3.140625, 1e-40, 65504.0], np.float32)
    r = oracle.round_bf16(x)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: even mantissa wins (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 and r[3] == np.float32(1.0 + 2 ** -6)
    assert r[4] == -2.5 and r[5] == 3.140625
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    np.testing.assert_array_equal(r, gen.bf16_bits_to_f32(gen.to_bf16_bits(x)))


def _read_golden(path):
    cases, cur = {}, None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *rest = line.split()
        if key == "case":
            cur = cases.setdefault(rest[0], {})
        elif key in ("undirected", "directed"):
            cur["kind"] = key
            cur["edges"] = [int(t) for t in rest]
        elif key == "n":
            cur["n"] = int(rest[0])
        else:
            cur[key] = [float(t) for t in rest]
    return cases


def test_golden_worked_examples():
    cases = _read_golden(os.path.join(HERE, "golden", "star_and_directed_triangle.txt"))
    assert set(cases) == {"star", "dtri"}
    for name, c in cases.items():
        e = np.array(c["edges"]).reshape(-1, 2)
        flags = oracle.GCN_FLAGS if c["kind"] == "undirected" else oracle.DIRECTED_GCN_FLAGS
        g = oracle.build_graph(c["n"], e[:, 0], e[:, 1], flags)
        x = np.array(c["x"])[:, None]
        np.testing.assert_allclose(oracle.aggregate_fwd(g, x)[:, 0], c["fwd"], rtol=2e-7, err_msg=name)
        np.testing.assert_allclose(oracle.aggregate_bwd(g, x)[:, 0], c["bwd"], rtol=2e-7, err_msg=name)


def test_p7_softmax_cross_entropy_direct():
    """the loss of the downstream task on its own: equal logits give log(classes) and the
    gradient (1/c - onehot)/n; gradient rows sum to zero; finite differences on single logits"""
    n, c = 9, 5
    labels = np.array([0, 1, 2, 3, 4, 0, 2, 4, 1])
    loss, dZ = gcn.softmax_cross_entropy(np.full((n, c), 3.7), labels)
    assert abs(loss - np.log(c)) < 1e-14
    want = np.full((n, c), 1.0 / c)
    want[np.arange(n), labels] -= 1.0
    np.testing.assert_allclose(dZ, want / n, rtol=1e-14)
    Z = gen.normal_features(n, c, 21).astype(np.float64) * 4.0
    loss, dZ = gcn.softmax_cross_entropy(Z, labels)
    np.testing.assert_allclose(dZ.sum(axis=1), 0.0, atol=1e-16)
    eps = 1e-6
    for (i, j) in ((0, 0), (3, 1), (8, 4), (5, 2)):
        Zp, Zm = Z.copy(), Z.copy()
        Zp[i, j] += eps
        Zm[i, j] -= eps
        fd = (gcn.softmax_cross_entropy(Zp, labels)[0] - gcn.softmax_cross_entropy(Zm, labels)[0]) / (2 * eps)
        assert abs(fd - dZ[i, j]) <= 1e-8
    # shift invariance and no overflow on large logits
    big, dB = gcn.softmax_cross_entropy(Z + 800.0, labels)
    assert abs(big - loss) < 1e-10 and np.allclose(dB, dZ, atol=1e-12)

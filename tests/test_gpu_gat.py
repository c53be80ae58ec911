"""GPU parity of the per-vertex attention scores (ntp_attention_scores_fwd / _bwd) and of a whole
decoupled GAT epoch composed from the library calls (Section 4.1 with the GAT aggregation of
Section 2.1) against the oracle."""
import sys

import numpy as np
import pytest

import oracle
import ntp_inputs as gen
import paper_2412_20379_amd as ntp
from helpers import check_activation_decisions, TOL_F32

pytestmark = pytest.mark.gpu
TOL = 1e-5


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.mark.parametrize("n,m,ldz,lddz", [(1, 1, 1, 1), (1000, 8, 8, 8), (3001, 16, 20, 16), (5000, 47, 47, 64),
                                          (777, 64, 64, 64), (20000, 128, 128, 160), (4099, 300, 304, 300),
                                          (2500, 1024, 1024, 1024), (150000, 40, 40, 40)])
def test_attention_scores_forward_and_backward(n, m, ldz, lddz):
    import torch
    from gpu_util import dev_f32
    rng = gen.stream_rng(n + m, 5)
    Z = rng.normal(size=(n, m)).astype(np.float32)
    a_s = rng.normal(size=m).astype(np.float32)
    a_d = rng.normal(size=m).astype(np.float32)
    dp = rng.normal(size=n).astype(np.float32)
    dq = rng.normal(size=n).astype(np.float32)
    dZ0 = rng.normal(size=(n, m)).astype(np.float32)
    say("   scores n=%d m=%d ldz=%d lddz=%d" % (n, m, ldz, lddz))
    Zd = torch.full((n, ldz), float("nan"), device="cuda:0")
    Zd[:, :m] = dev_f32(Z)
    p = torch.full((n,), float("nan"), device="cuda:0")
    q = torch.full((n,), float("nan"), device="cuda:0")
    ntp.ntp_attention_scores_fwd(Zd, dev_f32(a_s), dev_f32(a_d), p, q, n, m, ldz)
    torch.cuda.synchronize()
    rp, rq = oracle.attention_scores(Z, a_s, a_d)
    Za = np.abs(Z.astype(np.float64))
    sp_, sq_ = Za @ np.abs(a_s), Za @ np.abs(a_d)
    assert (np.abs(p.cpu().numpy() - rp) / sp_).max() <= TOL
    assert (np.abs(q.cpu().numpy() - rq) / sq_).max() <= TOL
    # backward
    dZd = torch.full((n, lddz), 3.5, device="cuda:0")
    dZd[:, :m] = dev_f32(dZ0)
    da_s = torch.full((m,), float("nan"), device="cuda:0")
    da_d = torch.full((m,), float("nan"), device="cuda:0")
    nb = ntp.ntp_attention_scores_bwd_scratch_bytes(n, m)
    assert 0 < nb <= 4 << 20
    scratch = torch.full((nb // 4,), float("nan"), device="cuda:0")
    ntp.ntp_attention_scores_bwd(Zd, dev_f32(a_s), dev_f32(a_d), dev_f32(dp), dev_f32(dq), dZd, da_s, da_d,
                                 n, m, ldz, lddz, scratch, nb)
    torch.cuda.synchronize()
    r_dZ, r_das, r_dad = oracle.attention_scores_bwd(Z, a_s, a_d, dp, dq, dZ0)
    got = dZd.cpu().numpy().astype(np.float64)
    scale = np.abs(dZ0) + np.outer(np.abs(dp), np.abs(a_s)) + np.outer(np.abs(dq), np.abs(a_d))
    assert (np.abs(got[:, :m] - r_dZ) / scale).max() <= TOL
    assert np.all(got[:, m:] == 3.5)                       # padding columns untouched
    for gotv, ref, g in ((da_s, r_das, dp), (da_d, r_dad, dq)):
        s = Za.T @ np.abs(g)
        err = (np.abs(gotv.cpu().numpy() - ref) / s).max()
        say("      column sums: error vs sum of |terms| %.2e" % err)
        assert err <= TOL
    # deterministic: a second call on the same inputs gives the same bits
    dZd2 = torch.full((n, lddz), 3.5, device="cuda:0")
    dZd2[:, :m] = dev_f32(dZ0)
    da_s2 = torch.empty_like(da_s)
    da_d2 = torch.empty_like(da_d)
    ntp.ntp_attention_scores_bwd(Zd, dev_f32(a_s), dev_f32(a_d), dev_f32(dp), dev_f32(dq), dZd2, da_s2, da_d2,
                                 n, m, ldz, lddz, scratch, nb)
    torch.cuda.synchronize()
    assert torch.equal(da_s, da_s2) and torch.equal(da_d, da_d2) and torch.equal(dZd, dZd2)


def test_attention_scores_argument_errors():
    import torch
    z = torch.zeros(10, 8, device="cuda:0")
    a = torch.zeros(8, device="cuda:0")
    v = torch.zeros(10, device="cuda:0")
    s = torch.zeros(1024, device="cuda:0")
    with pytest.raises(ntp.NtpError):
        ntp.ntp_attention_scores_fwd(z, a, a, v, v, 10, 0, 8)
    with pytest.raises(ntp.NtpError):
        ntp.ntp_attention_scores_fwd(z, a, a, v, v, 10, 8, 4)
    with pytest.raises(ntp.NtpError):
        ntp.ntp_attention_scores_fwd(z, a, a, v, v, 10, 1025, 1025)
    with pytest.raises(ntp.NtpError):
        ntp.ntp_attention_scores_fwd(z, None, a, v, v, 10, 8, 8)
    with pytest.raises(ntp.NtpError):          # scratch too small
        ntp.ntp_attention_scores_bwd(z, a, a, v, v, z.clone(), a.clone(), a.clone(), 10, 8, 8, 8, s, 8)
    with pytest.raises(ntp.NtpError):
        ntp.ntp_attention_scores_bwd(z, a, a, v, v, z.clone(), a.clone(), a.clone(), 10, 8, 8, 4, s, 4096)
    ntp.ntp_attention_scores_fwd(z, a, a, v, v, 0, 8, 8)       # nothing to do


def _gat_epoch(n, src, dst, flags, dims, rounds, slope, seed, what, chunk_edges=None, extra_flags=0, scale_floor=0.0, grad_tol=1e-5):
    """one decoupled GAT epoch on the device against the oracle: decisions, loss, logits, weights, every gradient"""
    import torch
    from paper_2412_20379_amd.gat import GatEpoch
    from gpu_util import dev_f32
    og = oracle.build_graph(n, src, dst, flags)
    kw = dict(chunk_edges=chunk_edges) if chunk_edges else {}
    g = ntp.ntp_graph_build(n, src, dst, flags=flags | extra_flags, **kw)
    rng = gen.stream_rng(seed, 3)
    X = rng.normal(size=(n, dims[0])).astype(np.float32)
    Ws = [gen.glorot_weight(dims[i], dims[i + 1], seed, i) for i in range(len(dims) - 1)]
    c = dims[-1]
    a_s = (rng.normal(size=c) * 0.7).astype(np.float32)
    a_d = (rng.normal(size=c) * 0.7).astype(np.float32)
    labels = gen.uniform_labels(n, c, seed)
    say("   GAT epoch: %s n=%d nnz=%d dims=%s rounds=%d slope=%g" % (what, n, og.csr.nnz, dims, rounds, slope))
    ep = GatEpoch(g, n, og.csr.nnz, dims, rounds=rounds, negative_slope=slope)
    loss = ep.run(dev_f32(X), [dev_f32(w) for w in Ws], dev_f32(a_s), dev_f32(a_d),
                  torch.from_numpy(labels.astype(np.int64)).to("cuda:0"))
    torch.cuda.synchronize()
    # ReLU and LeakyReLU decisions: the oracle works out from its own fp64 values which pre-activations
    # and which edge scores are zero at 1e-5 of the magnitude sums of their terms, and takes the
    # device's decision there and only there; everywhere else the device must have decided as the
    # oracle does.  The device's LeakyReLU branch of an edge is the sign of the fp32 sum of its two
    # fp32 scores, recomputed here from the scores the device wrote.
    hid_dev = [h.cpu().numpy() for h in ep.hid[:-1]]
    rows_of = np.repeat(np.arange(n), np.diff(og.csr.rowptr))
    p_dev, q_dev = ep.p.cpu().numpy(), ep.q.cpu().numpy()
    gate_dev = (p_dev[og.csr.colidx] + q_dev[rows_of]) > np.float32(0)
    ref = oracle.epoch_gat_decoupled(og, X, Ws, a_s, a_d, labels, rounds, slope,
                                     device_relu=[h > 0 for h in hid_dev], device_gate=gate_dev)
    check_activation_decisions(hid_dev, ref, what, say, calls_per_layer=1, scale_floor=scale_floor)
    own_gate = (ref["p"][og.csr.colidx] + ref["q"][rows_of]) > 0
    amb = ref["gate_ambiguous"]
    say("      %d of %d edge scores ambiguous at 1e-5 of their magnitude sums, %d device branches differ"
        % (int(amb.sum()), amb.size, int((gate_dev != own_gate).sum())))
    if slope != 1.0:
        assert not ((gate_dev != own_gate) & ~amb).any(), "LeakyReLU branches differ outside the ambiguous set"
    assert amb.mean() <= 1e-3
    say("      loss %.7f oracle %.7f" % (float(loss), ref["loss"]))
    assert abs(float(loss) - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    Z = ep.logits.cpu().numpy().astype(np.float64)
    assert np.abs(Z - ref["logits"]).max() <= 2e-5 * np.abs(ref["logits"]).max()
    a_in = ep.alpha_in.cpu().numpy().astype(np.float64)
    assert (np.abs(a_in - ref["alpha_in"]) / ref["alpha_in"]).max() <= 5e-5
    # gradients: error against the sum of the magnitudes of the terms each one adds up; an epoch
    # chains about a dozen fp32 calls; measured errors stay below 5e-6, so the per-call 1e-5 is kept.
    # The terms of dp[u], dq[v] are the per-edge alpha (dalpha - t) of all rounds, whose magnitudes
    # the oracle sums up (dp_mag, dq_mag); da_src = Lhat^T dp inherits them through |Lhat|.
    Lh = np.abs(ref["Z"][0])
    tiny = np.finfo(np.float64).tiny
    for name, got, want, mag in (("dp", ep.dp, ref["dp"], ref["dp_mag"]), ("dq", ep.dq, ref["dq"], ref["dq_mag"])):
        err = (np.abs(got.cpu().numpy() - want) / np.maximum(mag, tiny)).max()
        say("      %s error vs sum of |terms| per vertex %.2e" % (name, err))
        assert err <= grad_tol, name
    for name, got, want, mag in (("da_src", ep.da_src, ref["da_src"], ref["dp_mag"]), ("da_dst", ep.da_dst, ref["da_dst"], ref["dq_mag"])):
        err = (np.abs(got.cpu().numpy() - want) / np.maximum(Lh.T @ mag, tiny)).max()
        say("      %s error vs sum of |terms| %.2e" % (name, err))
        assert err <= grad_tol, name
    L = len(Ws)
    dH = ref["dLhat"]
    for l in range(L - 1, -1, -1):
        got = ep.dW[l].cpu().numpy().astype(np.float64)
        dZl = dH * ref["relu_keep"][l] if l < L - 1 else dH
        scale_l = np.abs(ref["nn_in"][l]).T @ np.abs(dZl)
        # scale_floor: entries whose terms are small against the largest entry's are measured against
        # that fraction of it (their inputs carry the rounding of the calls before)
        scale_l = np.maximum(np.maximum(scale_l, scale_floor * scale_l.max()), np.finfo(np.float64).tiny)
        err = (np.abs(got - ref["dW"][l]) / scale_l).max()
        nerr = np.abs(got - ref["dW"][l]).max() / max(np.abs(ref["dW"][l]).max(), np.finfo(np.float64).tiny)
        say("      dW[%d] error vs sum of |terms| %.2e, vs max|dW| %.2e" % (l, err, nerr))
        assert err <= TOL_F32, "dW[%d]" % l
        dH = dZl @ Ws[l].astype(np.float64).T
    g.close()


@pytest.mark.parametrize("rounds,slope", [(1, 0.2), (2, 0.2), (3, 0.0)])
def test_gat_epoch_directed_hub_graph(rounds, slope):
    n = 3000
    src, dst = gen.directed_random_edges(n, 40000, 21, hub=5, hub_in=2600, hub_out=900)
    _gat_epoch(n, src, dst, oracle.DIRECTED_GCN_FLAGS, (24, 16, 8), rounds, slope, 4, "hub graph")


def test_gat_epoch_chunked_resident():
    n = 3000
    src, dst = gen.directed_random_edges(n, 40000, 21, hub=5, hub_in=2600, hub_out=900)
    _gat_epoch(n, src, dst, oracle.DIRECTED_GCN_FLAGS, (24, 8), 2, 0.2, 6, "chunks of 700 edges", chunk_edges=700)


def test_gat_epoch_configs():
    for cfg, scale, dims in ((1, 1, (64, 16, 7)), (2, 4, (128, 32, 40))):
        n, src, dst = gen.make_graph(cfg, seed=0, scale_down=scale)
        _gat_epoch(n, src, dst, oracle.GCN_FLAGS, dims, 2, 0.2, cfg, "config %d / %d" % (cfg, scale))


def test_gat_epoch_with_edge_permutation():
    n = 3000
    src, dst = gen.directed_random_edges(n, 40000, 21, hub=5, hub_in=2600, hub_out=900)
    _gat_epoch(n, src, dst, oracle.DIRECTED_GCN_FLAGS, (24, 16, 8), 3, 0.2, 4, "hub graph, edge permutation",
               extra_flags=ntp.NTP_EDGE_PERM)
    _gat_epoch(n, src, dst, oracle.DIRECTED_GCN_FLAGS, (24, 8), 2, 0.2, 6, "chunks of 700 edges, edge permutation",
               chunk_edges=700, extra_flags=ntp.NTP_EDGE_PERM)
    n, src, dst = gen.make_graph(2, seed=0, scale_down=4)
    _gat_epoch(n, src, dst, oracle.GCN_FLAGS, (128, 32, 40), 2, 0.2, 2, "config 2 / 4, edge permutation",
               extra_flags=ntp.NTP_EDGE_PERM)



def test_gat_epoch_captured_in_a_hip_graph_replays_identically():
    """every library call of the GAT epoch is capturable once its scratch exists (no allocation
    after the first call, fill kernels instead of memset nodes): replays with eager work between
    them give the bits of the eager run, with and without the edge permutation"""
    import torch
    from paper_2412_20379_amd.gat import GatEpoch
    from gpu_util import dev_f32
    n = 3000
    src, dst = gen.directed_random_edges(n, 40000, 21, hub=5, hub_in=2600, hub_out=900)
    dims = (24, 16, 7)
    rng = gen.stream_rng(8, 3)
    X = dev_f32(rng.normal(size=(n, dims[0])))
    Ws = [dev_f32(gen.glorot_weight(dims[i], dims[i + 1], 8, i)) for i in range(2)]
    a_s, a_d = dev_f32(rng.normal(size=dims[-1])), dev_f32(rng.normal(size=dims[-1]))
    labels = torch.from_numpy(gen.uniform_labels(n, dims[-1], 8).astype(np.int64)).to("cuda:0")
    for extra in (0, ntp.NTP_EDGE_PERM):
        g = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS | extra)
        nnz = ntp.ntp_graph_info(g)["nnz"]
        ep = GatEpoch(g, n, nnz, dims, rounds=2)
        ep.run(X, Ws, a_s, a_d, labels)                 # scratch is allocated here
        torch.cuda.synchronize()
        want = [float(ep.loss)] + [t.clone() for t in (ep.dW[0], ep.dW[1], ep.da_src, ep.da_dst)]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            ep.run(X, Ws, a_s, a_d, labels)
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ep.run(X, Ws, a_s, a_d, labels)
        for r in range(3):
            for t in (ep.dW_buf[0], ep.dW_buf[1], ep.da_buf, ep.dp, ep.dq):
                t.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert float(ep.loss) == want[0], "replay %d" % r
            for a, b in zip((ep.dW[0], ep.dW[1], ep.da_src, ep.da_dst), want[1:]):
                assert torch.equal(a, b), "replay %d" % r
            _ = float((X * 2).sum())                    # eager work between the replays
        del graph, ep
        g.close()

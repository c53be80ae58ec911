"""Seeded random sweep: graphs, flags, widths, strides, dtypes, chunkings and call variants drawn
at random (fixed seeds), each compared with the oracle.  Complements the hand-picked cases."""
import os
import sys

import numpy as np
import pytest

import oracle
import ntp_inputs as gen
import paper_2412_20379_amd as ntp

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def seeds(count):
    """0..count-1, or the range "first:last" of NTP_SWEEP_SEEDS for a wider sweep"""
    v = os.environ.get("NTP_SWEEP_SEEDS")
    if v:
        a, b = v.split(":")
        return list(range(int(a), int(b)))
    return list(range(count))


@pytest.mark.parametrize("seed", seeds(24))
def test_random_aggregation_case(seed):
    from gpu_util import check_agg
    rng = gen.stream_rng(seed, 99)
    n = int(rng.integers(1, 4000))
    m = int(rng.integers(0, 12 * n + 1))
    hub_in = int(rng.integers(0, max(1, n - 1)))
    src, dst = gen.directed_random_edges(n, m, seed, hub=int(rng.integers(0, n)), hub_in=hub_in,
                                         hub_out=int(rng.integers(0, max(1, n // 3))))
    flags = int(rng.choice([oracle.GCN_FLAGS, oracle.DIRECTED_GCN_FLAGS, oracle.DEDUP | oracle.ADD_SELF_LOOPS,
                            oracle.SYMMETRISE | oracle.DEDUP | oracle.NORM_GCN_SYM, oracle.DEDUP]))
    weighted = bool(rng.integers(0, 2))
    w = (rng.random(src.size).astype(np.float32) + 0.25) if weighted else None
    og = oracle.build_graph(n, src, dst, flags, w)
    mode = str(rng.choice(["resident", "chunked", "stream", "scatter"]))
    kw = {}
    dev_flags = flags
    if mode == "chunked":
        kw = dict(chunk_edges=int(rng.integers(1, max(2, og.csr.nnz))))
    elif mode == "stream":
        kw = dict(chunk_edges=int(rng.integers(64, max(65, og.csr.nnz))))
        dev_flags |= ntp.NTP_FORCE_STREAM
    elif mode == "scatter":
        dev_flags |= ntp.NTP_SCATTER_BWD
    g = ntp.ntp_graph_build(n, src, dst, w, flags=dev_flags, **kw)
    rp, ci, va = ntp.ntp_graph_export(g, ntp.NTP_CSR)
    assert np.array_equal(rp, og.csr.rowptr) and np.array_equal(ci, og.csr.colidx)
    assert np.array_equal(va.view(np.uint32), og.csr.val.view(np.uint32))
    for _ in range(3):
        f = int(rng.choice([1, 2, 3, 5, 8, 16, 17, 31, 32, 33, 64, 76, 100, 128, 130, 256, 300]))
        dtype = "bf16" if (mode != "scatter" and rng.integers(0, 3) == 0) else "f32"
        pad_in, pad_out = int(rng.choice([0, 0, 1, 4, 28])), int(rng.choice([0, 0, 3, 4, 60]))
        direction = str(rng.choice(["fwd", "bwd"]))
        if dtype == "bf16" and direction == "bwd" and mode == "scatter":
            dtype = "f32"
        x = gen.normal_features(n, f, seed=seed * 7 + f)
        say("  seed %d: n=%d nnz=%d flags=%d %s f=%d %s %s ld=(%d,%d)" % (seed, n, og.csr.nnz, flags, mode, f, dtype, direction, f + pad_in, f + pad_out))
        check_agg(g, og, x, direction, dtype, "random seed %d" % seed, chunked=mode in ("chunked", "stream"),
                  ld_in=f + pad_in, ld_out=f + pad_out)
    g.close()


@pytest.mark.parametrize("seed", seeds(12))
def test_random_transform_case(seed):
    import torch
    from gpu_util import dev_f32
    from helpers import assert_close, TOL_F32
    from oracle import gcn as ogcn
    rng = gen.stream_rng(seed, 98)
    n = int(rng.integers(1, 6000))
    k = int(rng.choice([1, 3, 16, 40, 64, 100, 128, 160, 192, 256, 300, 602]))
    m = int(rng.choice([1, 2, 7, 16, 40, 47, 64, 65, 128, 130, 256]))
    act = int(rng.integers(0, 2))
    say("  seed %d: n=%d k=%d m=%d act=%d" % (seed, n, k, m, act))
    A = gen.normal_features(n, k, seed=seed)
    W = gen.glorot_weight(k, m, seed=seed)
    dH = gen.normal_features(n, m, seed=seed, stream=6)
    H = torch.full((n, m), float("nan"), device="cuda:0")
    ntp.ntp_nn_fwd(dev_f32(A), dev_f32(W), H, n, k, m, act)
    torch.cuda.synchronize()
    sc = np.abs(A).astype(np.float64) @ np.abs(W).astype(np.float64)
    assert_close(H.cpu().numpy(), ogcn.nn_fwd(A, W, act), sc, TOL_F32, "fwd")
    Href = ogcn.nn_fwd(A, W, act).astype(np.float32)
    dA_ref, dW_ref = ogcn.nn_bwd(A, W, Href, dH, act, need_dA=True)
    dZ = dH * (Href > 0) if act else dH
    dA = torch.full((n, k), float("nan"), device="cuda:0")
    dW = torch.full((k, m), float("nan"), device="cuda:0")
    wsb = ntp.ntp_nn_bwd_workspace_bytes(n, k, m)
    ws = torch.empty(max(wsb, 4), dtype=torch.uint8, device="cuda:0")
    # dW and dA in one call, then each alone: same bits
    ntp.ntp_nn_bwd(dev_f32(A), dev_f32(W), dev_f32(Href), dev_f32(dH), dA, dW, n, k, m, act, ntp.NTP_F32, ws, wsb)
    torch.cuda.synchronize()
    assert_close(dW.cpu().numpy(), dW_ref, np.abs(A.T).astype(np.float64) @ np.abs(dZ).astype(np.float64), TOL_F32, "dW")
    assert_close(dA.cpu().numpy(), dA_ref, np.abs(dZ).astype(np.float64) @ np.abs(W.T).astype(np.float64), TOL_F32, "dA")
    dA2 = torch.full((n, k), float("nan"), device="cuda:0")
    dW2 = torch.full((k, m), float("nan"), device="cuda:0")
    ntp.ntp_nn_bwd(dev_f32(A), dev_f32(W), dev_f32(Href), dev_f32(dH), dA2, None, n, k, m, act, ntp.NTP_F32, None, 0)
    ntp.ntp_nn_bwd(dev_f32(A), dev_f32(W), dev_f32(Href), dev_f32(dH), None, dW2, n, k, m, act, ntp.NTP_F32, ws, wsb)
    torch.cuda.synchronize()
    assert torch.equal(dA, dA2) and torch.equal(dW, dW2)


@pytest.mark.parametrize("seed", seeds(16))
def test_random_attention_case(seed):
    """attention weights in both orders and the gradient of the scores on a random graph: flags,
    chunking, edge permutation, width, strides and slope drawn at random"""
    from test_gpu_attention import _scores, _device_alpha, _check_alpha, _score_grad_case
    rng = gen.stream_rng(seed, 97)
    n = int(rng.integers(1, 3000))
    m_edges = int(rng.integers(0, 10 * n + 1))
    src, dst = gen.directed_random_edges(n, m_edges, seed, hub=int(rng.integers(0, n)),
                                         hub_in=int(rng.integers(0, max(1, n - 1))), hub_out=int(rng.integers(0, max(1, n // 2))))
    flags = int(rng.choice([oracle.GCN_FLAGS, oracle.DIRECTED_GCN_FLAGS, oracle.DEDUP | oracle.ADD_SELF_LOOPS, oracle.DEDUP]))
    og = oracle.build_graph(n, src, dst, flags)
    dev_flags = flags | (ntp.NTP_EDGE_PERM if rng.integers(0, 2) else 0)
    kw = dict(chunk_edges=int(rng.integers(1, max(2, og.csr.nnz)))) if rng.integers(0, 3) == 0 else {}
    slope = float(rng.choice([0.2, 0.0, 1.0, 0.01]))
    m = int(rng.choice([1, 2, 4, 7, 8, 16, 24, 32, 40, 47, 64, 76, 128, 172, 256, 600]))
    pad_z, pad_dy = int(rng.choice([0, 0, 1, 4, 8, 32])), int(rng.choice([0, 0, 3, 4, 16]))
    if m > 256:          # wider than 256 columns needs 16-byte aligned rows (documented limit)
        pad_z, pad_dy = pad_z // 4 * 4, pad_dy // 4 * 4
    say("  seed %d: n=%d nnz=%d flags=%d dev_flags=%d %s slope=%g m=%d ld=(%d,%d)" % (seed, n, og.csr.nnz, flags, dev_flags, kw, slope, m, m + pad_z, m + pad_dy))
    g = ntp.ntp_graph_build(n, src, dst, flags=dev_flags, **kw)
    p, q = _scores(n, seed, scale=float(rng.choice([0.5, 1.5, 6.0])))
    if og.csr.nnz > 0:
        a_in, a_out = _device_alpha(g, og.csr.nnz, p, q, slope)
        _check_alpha(og, a_in, a_out, p, q, slope, "random seed %d" % seed)
        _score_grad_case(g, og, m, slope, seed, "random seed %d" % seed, ldz=m + pad_z, lddy=m + pad_dy)
    g.close()


@pytest.mark.parametrize("seed", seeds(12))
def test_random_epoch_case(seed):
    """a whole GCN epoch on a random graph: depth, widths, order, flags and chunking drawn at random"""
    from test_gpu_epoch import run_epoch_case
    rng = gen.stream_rng(seed, 96)
    n = int(rng.integers(50, 3000))
    src, dst = gen.directed_random_edges(n, int(rng.integers(n, 10 * n)), seed, hub=int(rng.integers(0, n)),
                                         hub_in=int(rng.integers(0, n - 1)), hub_out=int(rng.integers(0, n // 2)))
    flags = int(rng.choice([oracle.GCN_FLAGS, oracle.DIRECTED_GCN_FLAGS]))
    depth = int(rng.integers(1, 5))
    dims = [int(rng.choice([3, 8, 16, 32, 40, 64, 100, 128, 130, 256, 300]))]
    dims += [int(rng.choice([4, 16, 32, 64, 128, 256])) for _ in range(depth - 1)]
    dims += [int(rng.choice([2, 7, 16, 40, 41, 47, 64, 172]))]
    order = str(rng.choice(["layerwise", "decoupled", "reordered", "auto"]))
    chunked = bool(rng.integers(0, 3) == 0)
    kw = dict(chunk_edges=int(rng.integers(500, 20000))) if chunked else {}
    overlap = bool(order in ("layerwise", "auto") and not chunked and rng.integers(0, 2))
    say("  seed %d: n=%d flags=%d dims=%s order=%s chunked=%s %s overlap_dw=%s" % (seed, n, flags, dims, order, chunked, kw, overlap))
    X = gen.normal_features(n, dims[0], seed=seed)
    run_epoch_case(n, src, dst, flags, X, dims, order, chunked=chunked, overlap_dw=overlap, build_kw=kw, what="random seed %d" % seed, seed=seed, scale_floor=1e-2)


@pytest.mark.parametrize("seed", seeds(8))
def test_random_gat_epoch_case(seed):
    """a whole decoupled GAT epoch on a random graph: depth, widths, rounds, slope, flags, chunking
    and the edge permutation drawn at random"""
    from test_gpu_gat import _gat_epoch
    rng = gen.stream_rng(seed, 95)
    n = int(rng.integers(200, 3000))
    src, dst = gen.directed_random_edges(n, int(rng.integers(n, 10 * n)), seed, hub=int(rng.integers(0, n)),
                                         hub_in=int(rng.integers(0, n - 1)), hub_out=int(rng.integers(0, n // 2)))
    flags = int(rng.choice([oracle.GCN_FLAGS, oracle.DIRECTED_GCN_FLAGS]))
    depth = int(rng.integers(1, 4))
    dims = [int(rng.choice([8, 16, 32, 64, 100, 128, 256]))]
    dims += [int(rng.choice([16, 32, 64, 128])) for _ in range(depth - 1)]
    dims += [int(rng.choice([2, 7, 16, 40, 41, 47, 64, 172]))]
    rounds = int(rng.integers(1, 4))
    slope = float(rng.choice([0.2, 0.0, 0.05]))
    chunk_edges = int(rng.integers(500, 20000)) if rng.integers(0, 3) == 0 else None
    extra = ntp.NTP_EDGE_PERM if rng.integers(0, 2) else 0
    _gat_epoch(n, src, dst, flags, dims, rounds, slope, seed, "random seed %d, chunk_edges %s, extra flags %d" % (seed, chunk_edges, extra),
               chunk_edges=chunk_edges, extra_flags=extra, scale_floor=1e-2)

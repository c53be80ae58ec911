"""GPU parity of the scatter-add backward aggregation (graphs built with NTP_SCATTER_BWD:
only the by-destination form is stored and the transposed product is accumulated with
fp32 atomics along the in-edges, Section 4.2.1) against the CPU oracle's by-source form."""
import sys

import numpy as np
import pytest

import oracle
import ntp_inputs as gen
import paper_2412_20379_amd as ntp

pytestmark = pytest.mark.gpu

FLAGS = ntp.NTP_DIRECTED_GCN_FLAGS | ntp.NTP_SCATTER_BWD


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def hub():
    n = 3000
    src, dst = gen.directed_random_edges(n, 40000, 21, hub=5, hub_in=2600, hub_out=900)
    og = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    g = ntp.ntp_graph_build(n, src, dst, flags=FLAGS)
    yield n, src, dst, g, og
    g.close()


def test_build_keeps_one_form(hub):
    n, src, dst, g, og = hub
    both = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS)
    # the by-destination form (weights use the out-degrees of the form that is not stored)
    rp, ci, va = ntp.ntp_graph_export(g, ntp.NTP_CSR)
    assert np.array_equal(rp, og.csr.rowptr) and np.array_equal(ci, og.csr.colidx)
    assert np.array_equal(va.view(np.uint32), og.csr.val.view(np.uint32))
    with pytest.raises(ntp.NtpError):
        ntp.ntp_graph_export(g, ntp.NTP_CSC)
    with pytest.raises(ntp.NtpError):
        ntp.ntp_graph_chunks(g, ntp.NTP_CSC)
    assert ntp.ntp_graph_info(g)["is_symmetric"] == 0
    b1, b2 = ntp.ntp_graph_device_bytes(g), ntp.ntp_graph_device_bytes(both)
    say("device bytes: one form", b1, "two forms", b2)
    assert b1 < 0.6 * b2
    both.close()


@pytest.mark.parametrize("f", [1, 2, 3, 7, 13, 16, 32, 33, 64, 76, 100, 128, 129, 200, 256, 257, 602])
def test_widths(hub, f):
    from gpu_util import check_agg
    n, src, dst, g, og = hub
    say("scatter bwd f", f)
    x = gen.normal_features(n, f, seed=f)
    check_agg(g, og, x, "bwd", "f32", "scatter bwd f=%d" % f)


@pytest.mark.parametrize("f,ld_in,ld_out", [(32, 40, 32), (32, 32, 48), (76, 602, 80), (13, 100, 13), (16, 17, 19), (257, 264, 260)])
def test_strided(hub, f, ld_in, ld_out):
    from gpu_util import check_agg
    n, src, dst, g, og = hub
    say("scatter bwd strided", f, ld_in, ld_out)
    x = gen.normal_features(n, f, seed=9)
    check_agg(g, og, x, "bwd", "f32", "scatter strided", ld_in=ld_in, ld_out=ld_out)   # also checks the padding is untouched


def test_forward_unchanged_and_bf16_rejected(hub):
    import torch
    from gpu_util import run_agg, dev_bf16_bits
    n, src, dst, g, og = hub
    both = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS)
    x = gen.normal_features(n, 48, seed=3)
    assert np.array_equal(run_agg(g, x, "fwd"), run_agg(both, x, "fwd"))
    bits, _ = dev_bf16_bits(x)
    out = torch.zeros_like(bits)
    with pytest.raises(ntp.NtpError):
        ntp.ntp_aggregate_bwd(g, bits, out, 48, 48, 48, ntp.NTP_BF16)
    ntp.ntp_aggregate_fwd(g, bits, out, 48, 48, 48, ntp.NTP_BF16)      # the gather direction still takes bf16
    torch.cuda.synchronize()
    both.close()


def test_degree_edge_cases():
    """rows with the entry counts around every bin and split boundary, scattered"""
    from gpu_util import check_agg
    degs = [1, 2, 3, 4, 5, 8, 9, 16, 17, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257,
            511, 512, 513, 1023, 1024, 1025, 2047, 2048, 2049, 5000]
    n = 6000
    rng = gen.stream_rng(5, 1)
    src, dst = [], []
    for v, d in enumerate(degs):
        others = rng.choice(np.setdiff1d(np.arange(n), [v]), size=d - 1, replace=False)
        src.append(others)
        dst.append(np.full(d - 1, v))
    src = np.concatenate(src).astype(np.int32)
    dst = np.concatenate(dst).astype(np.int32)
    og = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    g = ntp.ntp_graph_build(n, src, dst, flags=FLAGS)
    for f in (4, 16, 32, 76, 128, 256):
        say("scatter degree_edge_cases f", f)
        check_agg(g, og, gen.normal_features(n, f, seed=f), "bwd", "f32", "scatter degrees f=%d" % f)
    g.close()


@pytest.mark.parametrize("chunk_edges,mode", [(101, "stream"), (5003, "stream"), (5003, "partial"), (20000, "resident")])
def test_chunked(hub, chunk_edges, mode):
    """streamed, partly resident and resident chunks, among them pieces of the hub's row"""
    import torch
    from gpu_util import check_agg, dev_f32
    from helpers import assert_close, TOL_F32
    n, src, dst, _, og = hub
    flags = FLAGS | (ntp.NTP_FORCE_STREAM if mode == "stream" else 0)
    budget = 400_000 if mode == "partial" else 0
    g = ntp.ntp_graph_build(n, src, dst, flags=flags, device_budget_bytes=budget, chunk_edges=chunk_edges)
    res = ntp.ntp_graph_chunks(g, ntp.NTP_CSR)["resident"]
    say("scatter chunked", chunk_edges, mode, "chunks", len(res), "resident", int(np.sum(res)))
    if mode == "partial":
        assert 0 < np.sum(res) < len(res)
    for f in (24, 76):
        x = gen.normal_features(n, f, seed=60 + f)
        check_agg(g, og, x, "bwd", "f32", "scatter chunked f=%d" % f, chunked=True)
        check_agg(g, og, x, "fwd", "f32", "fwd of a one-form graph f=%d" % f, chunked=True)
    # several right-hand sides per chunk visit
    f, k = 24, 3
    xs_np = [gen.normal_features(n, f, seed=70 + i) for i in range(k)]
    xs = [dev_f32(x) for x in xs_np]
    ys = [torch.full((n, f), float("nan"), device="cuda:0") for _ in range(k)]
    cs, cp = torch.cuda.Stream(), torch.cuda.Stream()
    ntp.ntp_chunked_aggregate_multi(g, ntp.NTP_BWD, xs, ys, f, f, f, ntp.NTP_F32, cs, cp)
    torch.cuda.synchronize()
    for i in range(k):
        ref, ref_abs = oracle.aggregate(og.csc, xs_np[i], with_abs=True)
        assert_close(ys[i].cpu().numpy(), ref, ref_abs, TOL_F32, "scatter multi rhs %d" % i)
    g.close()


def test_flag_is_a_no_op_on_a_symmetric_graph():
    from gpu_util import run_agg
    n, src, dst = gen.make_graph(1, seed=2)
    a = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_GCN_FLAGS)
    b = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_GCN_FLAGS | ntp.NTP_SCATTER_BWD)
    assert ntp.ntp_graph_info(b)["is_symmetric"] == 1
    x = gen.normal_features(n, 40, seed=4)
    assert np.array_equal(run_agg(a, x, "bwd"), run_agg(b, x, "bwd"))
    rp, ci, va = ntp.ntp_graph_export(b, ntp.NTP_CSC)
    rp0, ci0, va0 = ntp.ntp_graph_export(a, ntp.NTP_CSC)
    assert np.array_equal(rp, rp0) and np.array_equal(ci, ci0) and np.array_equal(va, va0)
    a.close()
    b.close()


def test_scaled_config3_scatter_matches_gather():
    """a power-law graph with one-way edges: scatter against the library's own gather form"""
    from gpu_util import run_agg, check_agg
    n, src, dst = gen.make_graph(3, seed=1, scale_down=64)
    og = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    g = ntp.ntp_graph_build(n, src, dst, flags=FLAGS)
    x = gen.normal_features(n, 32, seed=8)
    check_agg(g, og, x, "bwd", "f32", "cfg3/64 scatter")
    g.close()

"""The aggregation with the most gathered columns' feature rows in an LDS table (hub table, an
opt-in kernel variant: graphs built with NTP_AGG_HUB=1): the same bits as the plain kernel,
whatever the shape, and parity with the oracle."""
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


def build(n, src, dst, flags, hub, min_count=1, **kw):
    """graph with (hub=True: every column gathered at least min_count times may get a slot) or
    without hub tables; the environment is read by the build only"""
    old = {k: os.environ.get(k) for k in ("NTP_AGG_HUB", "NTP_AGG_HUB_MIN_COUNT")}
    try:
        if hub:
            os.environ["NTP_AGG_HUB"] = "1"
            os.environ["NTP_AGG_HUB_MIN_COUNT"] = str(min_count)
        else:
            os.environ.pop("NTP_AGG_HUB", None)
        return ntp.ntp_graph_build(n, src, dst, flags=flags, **kw)
    finally:
        for k, v in old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v


@pytest.fixture(scope="module")
def graphs():
    n = 6000
    src, dst = gen.directed_random_edges(n, 90000, 31, hub=11, hub_in=5000, hub_out=2500)
    og = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    plain = build(n, src, dst, ntp.NTP_DIRECTED_GCN_FLAGS, hub=False)
    hub = build(n, src, dst, ntp.NTP_DIRECTED_GCN_FLAGS, hub=True)
    few = build(n, src, dst, ntp.NTP_DIRECTED_GCN_FLAGS, hub=True, min_count=40)      # a handful of hubs only
    chunked = build(n, src, dst, ntp.NTP_DIRECTED_GCN_FLAGS, hub=True, chunk_edges=9000)
    nnz = og.csr.nnz
    assert ntp.ntp_graph_device_bytes(hub) >= ntp.ntp_graph_device_bytes(plain) + 2 * 4 * nnz       # 4 bytes per entry and form
    yield n, og, plain, hub, few, chunked
    for g in (plain, hub, few, chunked):
        g.close()


@pytest.mark.parametrize("f,ld,dtype", [(32, 32, "f32"), (16, 16, "f32"), (13, 16, "f32"), (24, 24, "f32"), (76, 96, "f32"),
                                         (256, 256, "f32"), (5, 8, "f32"), (64, 64, "bf16"), (76, 128, "bf16"), (30, 32, "bf16"),
                                         (33, 33, "f32"), (100, 100, "f32")])
def test_hub_table_gives_the_bits_of_the_plain_kernel(graphs, f, ld, dtype):
    """forward and backward, line-wide and half-line rows, column passes, ragged widths; widths
    whose rows are not read in 16-byte vectors fall back to the plain kernel on both sides"""
    from gpu_util import run_agg
    from helpers import assert_close, TOL_F32, TOL_BF16
    n, og, plain, hub, few, chunked = graphs
    x = gen.normal_features(n, f, seed=f)
    for direction in ("fwd", "bwd"):
        want = run_agg(plain, x, direction, dtype, ld_in=ld, ld_out=ld)
        for name, g in (("every column a hub", hub), ("few hubs", few), ("chunks", chunked)):
            say("hub table:", name, direction, "f", f, "ld", ld, dtype)
            got = run_agg(g, x, direction, dtype, ld_in=ld, ld_out=ld, chunked=name == "chunks")
            if name == "chunks":        # other pieces of the long rows: equal to rounding
                assert np.abs(got - want).max() <= (1e-5 if dtype == "f32" else 2e-2) * np.abs(want).max()
            else:
                assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), "%s %s: bits differ" % (name, direction)
        x_used = x if dtype == "f32" else gen.bf16_bits_to_f32(gen.to_bf16_bits(x))
        ref, ref_abs = oracle.aggregate(og.csr if direction == "fwd" else og.csc, x_used, with_abs=True)
        if dtype == "bf16":
            ref = oracle.round_bf16(ref).astype(np.float64)
        assert_close(got, ref, ref_abs, TOL_F32 if dtype == "f32" else TOL_BF16, "hub table, chunks, %s" % direction)


def test_hub_table_with_caller_weights(graphs):
    """ntp_aggregate_weighted takes the hub path too (the weights keep their entry order)"""
    import torch
    from gpu_util import dev_f32
    n, og, plain, hub, few, chunked = graphs
    f = 32
    x = dev_f32(gen.normal_features(n, f, seed=3))
    for direction, m in ((ntp.NTP_FWD, og.csr), (ntp.NTP_BWD, og.csc)):
        w = dev_f32(gen.stream_rng(4, 77).random(m.nnz).astype(np.float32))
        y0, y1 = torch.empty_like(x), torch.empty_like(x)
        ntp.ntp_aggregate_weighted(plain, direction, w, x, y0, f, f, f)
        ntp.ntp_aggregate_weighted(hub, direction, w, x, y1, f, f, f)
        torch.cuda.synchronize()
        assert torch.equal(y0, y1)


def test_hub_table_on_a_power_law_graph():
    """config 2 at a quarter of its size with the default bound (columns gathered 256 times or more):
    same bits as without, at the widths of its model"""
    import torch
    from gpu_util import dev_f32
    n, src, dst = gen.make_graph(2, seed=0, scale_down=4)
    plain = build(n, src, dst, ntp.NTP_GCN_FLAGS, hub=False)
    hub = build(n, src, dst, ntp.NTP_GCN_FLAGS, hub=True, min_count=256)
    extra = ntp.ntp_graph_device_bytes(hub) - ntp.ntp_graph_device_bytes(plain)
    say("config 2 / 4: hub table takes %d bytes more" % extra)
    assert extra > 4 * ntp.ntp_graph_info(hub)["nnz"]
    for f in (128, 256, 40):
        x = dev_f32(gen.normal_features(n, f, seed=0))
        y0, y1 = torch.empty_like(x), torch.empty_like(x)
        ntp.ntp_aggregate_fwd(plain, x, y0, f, f, f)
        ntp.ntp_aggregate_fwd(hub, x, y1, f, f, f)
        torch.cuda.synchronize()
        assert torch.equal(y0, y1), f
    plain.close()
    hub.close()


def test_streamed_graphs_have_no_hub_table():
    n = 3000
    src, dst = gen.directed_random_edges(n, 30000, 5)
    a = build(n, src, dst, ntp.NTP_DIRECTED_GCN_FLAGS | ntp.NTP_FORCE_STREAM, hub=True, chunk_edges=5000)
    b = build(n, src, dst, ntp.NTP_DIRECTED_GCN_FLAGS | ntp.NTP_FORCE_STREAM, hub=False, chunk_edges=5000)
    assert ntp.ntp_graph_device_bytes(a) == ntp.ntp_graph_device_bytes(b)
    a.close()
    b.close()

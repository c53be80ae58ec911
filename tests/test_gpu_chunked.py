"""GPU parity of ntp_chunked_aggregate (chunk scheduling of Section 4.2.1): the chunked
result equals the in-memory result and the oracle, whatever the chunk size and however
many chunks are resident."""
import sys

import numpy as np
import pytest

import oracle
import ntp_inputs as gen
import paper_2412_20379_amd as ntp

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def inputs():
    n = 4000
    src, dst = gen.directed_random_edges(n, 60000, 41, hub=17, hub_in=3500, hub_out=1200)
    og = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    return n, src, dst, og


@pytest.mark.parametrize("chunk_edges", [1, 7, 101, 997, 5003, 20000, 10 ** 7])
@pytest.mark.parametrize("mode", ["resident", "stream", "partial"])
def test_chunked_equals_oracle(inputs, chunk_edges, mode):
    from gpu_util import check_agg, run_agg
    n, src, dst, og = inputs
    if chunk_edges < 100 and mode != "resident":
        pytest.skip("thousands of tiny copies: covered by the resident case")
    flags = ntp.NTP_DIRECTED_GCN_FLAGS
    budget = 0
    if mode == "stream":
        flags |= ntp.NTP_FORCE_STREAM
    elif mode == "partial":
        budget = 700_000          # holds the staging buffers and some of the chunks
    say("chunked", chunk_edges, mode)
    try:
        g = ntp.ntp_graph_build(n, src, dst, flags=flags, device_budget_bytes=budget, chunk_edges=chunk_edges)
    except ntp.NtpError as e:
        assert mode == "partial" and e.code == ntp.NTP_EBUDGET     # staging alone exceeds the budget
        return
    ch = ntp.ntp_graph_chunks(g, ntp.NTP_CSR)
    if mode == "stream":
        assert ch["resident"].sum() == 0
    if mode == "resident":
        assert ch["resident"].all()
    x = gen.normal_features(n, 32, seed=5)
    for direction in ("fwd", "bwd"):
        got = check_agg(g, og, x, direction, "f32", "chunked %d %s %s" % (chunk_edges, mode, direction), chunked=True)
        if mode == "resident":
            again = run_agg(g, x, direction, "f32")
            # same per-row kernel path when the plan is the same: identical bits
            assert np.array_equal(got.view(np.uint32), again.view(np.uint32))
        else:
            with pytest.raises(ntp.NtpError) as e:
                run_agg(g, x, direction, "f32")
            assert e.value.code == ntp.NTP_EBUDGET
    # repeated calls reuse the staging buffers safely
    a = run_agg(g, x, "fwd", "f32", chunked=True)
    b = run_agg(g, x, "fwd", "f32", chunked=True)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    check_agg(g, og, x, "fwd", "bf16", "chunked bf16", chunked=True)
    g.close()


def test_chunked_same_stream_rejected_when_streaming(inputs):
    import torch
    n, src, dst, og = inputs
    g = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS | ntp.NTP_FORCE_STREAM, chunk_edges=20000)
    x = torch.zeros(n, 8, device="cuda:0")
    y = torch.zeros(n, 8, device="cuda:0")
    s = torch.cuda.Stream()
    with pytest.raises(ntp.NtpError) as e:
        ntp.ntp_chunked_aggregate(g, ntp.NTP_FWD, x, y, 8, 8, 8, ntp.NTP_F32, s, s)
    assert e.value.code == ntp.NTP_EINVAL
    g.close()


def test_chunked_config2_budget():
    """config 2 under a budget that keeps about half of the topology resident"""
    from gpu_util import check_agg
    n, src, dst = gen.make_graph(2, seed=0)
    og = oracle.build_graph(n, src, dst)
    g = ntp.ntp_graph_build(n, src, dst, device_budget_bytes=16 << 20, chunk_edges=300_000)
    ch = ntp.ntp_graph_chunks(g, ntp.NTP_CSR)
    say("config 2 chunks", len(ch["resident"]), "resident", int(ch["resident"].sum()))
    assert 0 < ch["resident"].sum() < len(ch["resident"])
    assert ntp.ntp_graph_device_bytes(g) <= (16 << 20) + 4 * og.n * 128   # topology within budget (+ scratch)
    x = gen.normal_features(n, 128, 0)
    check_agg(g, og, x, "fwd", "f32", "cfg2 chunked", chunked=True)
    check_agg(g, og, x, "bwd", "f32", "cfg2 chunked bwd", chunked=True)
    g.close()


@pytest.mark.parametrize("chunk_edges,mode", [(101, "stream"), (5003, "stream"), (5003, "partial"), (20000, "resident")])
@pytest.mark.parametrize("direction", ["fwd", "bwd"])
def test_multi_rhs_equals_separate_calls(inputs, chunk_edges, mode, direction):
    """several right-hand sides per chunk visit: same bits as one call per right-hand side"""
    import torch
    from gpu_util import dev_f32
    from helpers import assert_close, TOL_F32
    n, src, dst, og = inputs
    flags = ntp.NTP_DIRECTED_GCN_FLAGS | (ntp.NTP_FORCE_STREAM if mode == "stream" else 0)
    budget = 700_000 if mode == "partial" else 0
    g = ntp.ntp_graph_build(n, src, dst, flags=flags, device_budget_bytes=budget, chunk_edges=chunk_edges)
    f, k = 24, 3
    d = ntp.NTP_FWD if direction == "fwd" else ntp.NTP_BWD
    xs_np = [gen.normal_features(n, f, seed=50 + i) for i in range(k)]
    xs = [dev_f32(x) for x in xs_np]
    ys = [torch.full((n, f), float("nan"), device="cuda:0") for _ in range(k)]
    cs, cp = torch.cuda.Stream(), torch.cuda.Stream()
    ntp.ntp_chunked_aggregate_multi(g, d, xs, ys, f, f, f, ntp.NTP_F32, cs, cp)
    torch.cuda.synchronize()
    m = og.csr if direction == "fwd" else og.csc
    for i in range(k):
        one = torch.empty(n, f, device="cuda:0")
        ntp.ntp_chunked_aggregate(g, d, xs[i], one, f, f, f, ntp.NTP_F32, cs, cp)
        torch.cuda.synchronize()
        assert torch.equal(one, ys[i]), "right-hand side %d differs from its separate call" % i
        ref, ref_abs = oracle.aggregate(m, xs_np[i], with_abs=True)
        assert_close(ys[i].cpu().numpy(), ref, ref_abs, TOL_F32, "multi rhs %d" % i)
    with pytest.raises(ntp.NtpError):            # an output that is also an input
        ntp.ntp_chunked_aggregate_multi(g, d, xs, [ys[0], xs[1], ys[2]], f, f, f, ntp.NTP_F32, cs, cp)
    with pytest.raises(ntp.NtpError):            # two outputs alias
        ntp.ntp_chunked_aggregate_multi(g, d, xs, [ys[0], ys[0], ys[2]], f, f, f, ntp.NTP_F32, cs, cp)
    g.close()


@pytest.mark.parametrize("case", ["gcn directed", "gcn symmetric", "no normalisation", "caller weights", "gcn scatter backward"])
def test_streamed_weights_rebuilt_on_the_device_are_the_stored_ones(inputs, case):
    """A streamed chunk travels without its weights when they follow from the structure (GCN
    normalisation of unit weights, or all ones): the values rebuilt on the device must be the
    stored ones bit for bit, so streamed and resident results are identical; with caller weights
    the stored values travel as before."""
    from gpu_util import run_agg
    n, src, dst, og = inputs
    w = None
    if case == "gcn directed":
        flags = ntp.NTP_DIRECTED_GCN_FLAGS
    elif case == "gcn symmetric":
        flags = ntp.NTP_GCN_FLAGS
    elif case == "no normalisation":
        flags = ntp.NTP_DEDUP | ntp.NTP_ADD_SELF_LOOPS
    elif case == "caller weights":
        flags = ntp.NTP_DIRECTED_GCN_FLAGS
        w = (gen.stream_rng(3, 8).random(src.size) + 0.5).astype(np.float32)
    else:
        flags = ntp.NTP_DIRECTED_GCN_FLAGS | ntp.NTP_SCATTER_BWD
    x = gen.normal_features(n, 24, seed=6)
    resident = ntp.ntp_graph_build(n, src, dst, w, flags=flags, chunk_edges=3001)
    streamed = ntp.ntp_graph_build(n, src, dst, w, flags=flags | ntp.NTP_FORCE_STREAM, chunk_edges=3001)
    nnz = ntp.ntp_graph_info(streamed)["nnz"]
    assert ntp.ntp_graph_stream_bytes(resident) == 0
    per_entry = 8 if case == "caller weights" else 4
    got = ntp.ntp_graph_stream_bytes(streamed)
    assert per_entry * nnz < got < per_entry * nnz + 40 * n + 64 * ntp.ntp_graph_info(streamed)["n_chunks"] + 4096
    for direction in ("fwd", "bwd"):
        a = run_agg(resident, x, direction, "f32", chunked=True)
        b = run_agg(streamed, x, direction, "f32", chunked=True)
        if case == "gcn scatter backward" and direction == "bwd":      # atomics: order of additions not fixed
            assert np.abs(a - b).max() <= 1e-5 * np.abs(a).max()
        else:
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), "%s %s" % (case, direction)
    resident.close()
    streamed.close()


def test_config5_shape_streams_under_a_budget():
    """Config 5's shape at one eighth of its size (13.9 M vertices, 0.42 B stored entries, one
    worker's 16-column slice, chunks of 32 Mi entries = the config's 256 Mi scaled) under a device
    budget that leaves more than half of the chunks streamed from pinned host memory on every
    call: forward and backward through ntp_chunked_aggregate give, bit for bit, what the same
    chunking gives with every chunk resident, and 21,000 sampled rows (20,000 uniform + the 1,000
    with most entries) match oracle rows built one by one from the edge list."""
    import time
    import torch
    from gpu_util import dev_f32
    from helpers import assert_close, TOL_F32
    scale, f = 8, 16
    t0 = time.time()
    n, src, dst = gen.make_graph(5, seed=0, scale_down=scale)
    ce = gen.CONFIGS[5].chunk_edges // scale
    say("config 5 / %d: n %d, undirected edges %d, chunk_edges %d (generated in %.0fs)" % (scale, n, src.size, ce, time.time() - t0))
    x_np = gen.normal_features(n, f, 0)
    x = dev_f32(x_np)
    cs, xs = torch.cuda.Stream(), torch.cuda.Stream()

    def both_directions(g):
        out = []
        for direction in (ntp.NTP_FWD, ntp.NTP_BWD):
            y = torch.full((n, f), float("nan"), device="cuda:0")
            torch.cuda.synchronize()
            ntp.ntp_chunked_aggregate(g, direction, x, y, f, f, f, ntp.NTP_F32, cs, xs)
            torch.cuda.synchronize()
            out.append(y)
        return out

    t0 = time.time()
    g = ntp.ntp_graph_build(n, src, dst, chunk_edges=ce)
    info = ntp.ntp_graph_info(g)
    nnz = info["nnz"]
    say("  all-resident graph built in %.0fs: nnz %d, %d chunks, longest row %d" % (time.time() - t0, nnz, info["n_chunks"], info["max_degree"]))
    assert ntp.ntp_graph_chunks(g)["resident"].all() and info["n_chunks"] >= 12
    want_fwd, want_bwd = both_directions(g)
    rowptr = np.empty(n + 1, dtype=np.int64)
    ntp.binding._check(ntp.lib().ntp_graph_export(g.handle, ntp.NTP_CSR, ntp.binding._ptr(rowptr), None, None))
    g.close()
    t0 = time.time()
    g = ntp.ntp_graph_build(n, src, dst, device_budget_bytes=int(0.45 * (8 * nnz + 12 * n)), chunk_edges=ce)
    res = ntp.ntp_graph_chunks(g)["resident"]
    say("  budgeted graph built in %.0fs: %d of %d chunks resident, %d bytes streamed per pass"
        % (time.time() - t0, int(res.sum()), res.size, ntp.ntp_graph_stream_bytes(g)))
    assert 2 * int(res.sum()) <= res.size and res.sum() >= 1
    for rep in range(2):                    # the second call finds the staging buffers in use
        got_fwd, got_bwd = both_directions(g)
        assert torch.equal(got_fwd, want_fwd) and torch.equal(got_bwd, want_bwd), "streamed and resident results differ"
    assert torch.equal(got_fwd, got_bwd)    # the adjacency is symmetric
    g.close()
    deg = np.diff(rowptr)
    assert int(rowptr[-1]) == nnz == 2 * src.size + n
    top = np.argsort(deg)[-1000:]
    uni = gen.stream_rng(0, 98).choice(np.setdiff1d(np.arange(n), top), size=20000, replace=False)
    rows = np.concatenate([top, uni]).astype(np.int64)
    t0 = time.time()
    m = oracle.rows_from_undirected_edges(n, src, dst, rows)
    assert np.array_equal(np.diff(m.rowptr), deg[rows])
    ref, ref_abs = oracle.aggregate(m, x_np, with_abs=True)
    say("  oracle rows in %.0fs (%d entries)" % (time.time() - t0, m.nnz))
    got = got_fwd[torch.from_numpy(rows).to("cuda:0")].cpu().numpy()
    assert_close(got, ref, ref_abs, TOL_F32, "config 5 / 8 sampled rows")

"""ntp_aggregate_fwd_noalloc (static device scratch, no allocation) against ntp_aggregate_fwd.

Collected last on purpose (file name): the full test run stops at the first failure."""
import sys

import numpy as np
import pytest

import oracle
import ntp_inputs as gen
import paper_2412_20379_amd as ntp
from helpers import assert_close, TOL_F32

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def _hub_graph(n, m, seed, hub_in):
    return gen.directed_random_edges(n, m, seed, hub=n // 3, hub_in=hub_in, hub_out=hub_in // 4)


def _both(g, og, x_np, f, ld, what):
    """the two entry points on the same input: equal bits, and equal to the oracle to tolerance"""
    import torch
    from gpu_util import dev_f32
    n = x_np.shape[0]
    x = torch.full((n, ld), 3.5, dtype=torch.float32, device="cuda:0")
    x[:, :f] = dev_f32(x_np)
    y_ref = torch.full((n, ld), -1.0, dtype=torch.float32, device="cuda:0")
    y_new = torch.full((n, ld), -2.0, dtype=torch.float32, device="cuda:0")
    torch.cuda.synchronize()
    say("no-alloc case:", what, "n", n, "f", f, "ld", ld)
    ntp.ntp_aggregate_fwd(g, x, y_ref, f, ld, ld, ntp.NTP_F32)
    ntp.ntp_aggregate_fwd_noalloc(g, x, y_new, f, ld, ld, ntp.NTP_F32)
    torch.cuda.synchronize()
    assert torch.equal(y_ref[:, :f], y_new[:, :f]), what + ": the two entry points differ"
    if ld > f:
        assert bool((y_new[:, f:] == -2.0).all()), what + ": columns outside the slice were written"
    ref, ref_abs = oracle.aggregate(og.csr, x_np, with_abs=True)
    assert_close(y_new[:, :f].cpu().numpy(), ref, ref_abs, TOL_F32, what)


def test_two_calls_in_a_row_second_smaller():
    """first a graph whose hub is cut into many pieces at a wide slice, then a smaller graph at a
    narrow slice: the second call finds the first one's partial sums in the shared scratch and must
    not be disturbed by them; then the first again"""
    big = _hub_graph(20000, 150000, 11, hub_in=9000)
    small = _hub_graph(3000, 20000, 12, hub_in=1500)
    og_big = oracle.build_graph(20000, *big, oracle.DIRECTED_GCN_FLAGS)
    og_small = oracle.build_graph(3000, *small, oracle.DIRECTED_GCN_FLAGS)
    assert np.diff(og_big.csr.rowptr).max() > 4096 and np.diff(og_small.csr.rowptr).max() > 600      # both have split rows
    g_big = ntp.ntp_graph_build(20000, *big, flags=ntp.NTP_DIRECTED_GCN_FLAGS)
    g_small = ntp.ntp_graph_build(3000, *small, flags=ntp.NTP_DIRECTED_GCN_FLAGS)
    x_big = gen.normal_features(20000, 96, 5)
    x_small = gen.normal_features(3000, 20, 6)
    _both(g_big, og_big, x_big, 96, 96, "large graph, 96 columns")
    _both(g_small, og_small, x_small, 20, 24, "small graph after the large one, 20 columns in rows of 24")
    _both(g_big, og_big, x_big[:, :33], 33, 36, "large graph again, 33 columns")
    g_big.close()
    g_small.close()


def test_chunked_plan_and_bf16_share_the_scratch():
    """a resident graph cut into several chunks (one reduce launch for all) and the bf16 variant"""
    import torch
    from gpu_util import dev_bf16_bits
    n = 12000
    src, dst = _hub_graph(n, 90000, 13, hub_in=7000)
    g = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS, chunk_edges=20000)
    assert ntp.ntp_graph_info(g)["n_chunks"] > 2
    og = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    _both(g, og, gen.normal_features(n, 64, 7), 64, 64, "five resident chunks")
    bits, _ = dev_bf16_bits(gen.normal_features(n, 40, 8))
    y0 = torch.zeros_like(bits)
    y1 = torch.ones_like(bits)
    ntp.ntp_aggregate_fwd(g, bits, y0, 40, 40, 40, ntp.NTP_BF16)
    ntp.ntp_aggregate_fwd_noalloc(g, bits, y1, 40, 40, 40, ntp.NTP_BF16)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    g.close()


def test_sizes_beyond_the_static_scratch_are_refused():
    """a row of 150,001 entries is 586 pieces: at 4096 columns their partial sums need 9.6 MB, more
    than the 8 MiB array, at 2048 columns they fit"""
    import torch
    n = 150000
    src = np.arange(n, dtype=np.int32)
    dst = np.full(n, 7, dtype=np.int32)
    g = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS)
    x = torch.randn(n, 4096, device="cuda:0")
    y = torch.zeros_like(x)
    with pytest.raises(ntp.NtpError) as e:
        ntp.ntp_aggregate_fwd_noalloc(g, x, y, 4096, 4096, 4096, ntp.NTP_F32)
    assert e.value.code == ntp.NTP_EUNSUPPORTED and "static scratch" in str(e.value)
    assert not bool(y.any()), "a refused call must not have run"
    y2 = torch.zeros_like(x)
    ntp.ntp_aggregate_fwd(g, x, y, 2048, 4096, 4096, ntp.NTP_F32)
    ntp.ntp_aggregate_fwd_noalloc(g, x, y2, 2048, 4096, 4096, ntp.NTP_F32)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    g.close()


def test_static_scratch_needs_no_device_memory_from_the_handle():
    """the handle's device bytes do not grow over a no-alloc call, whatever the width (the allocating
    call grows them once a slice is wider than the 256 columns its scratch was sized for at build)"""
    import torch
    src, dst = _hub_graph(5000, 30000, 14, hub_in=3000)
    g = ntp.ntp_graph_build(5000, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS)
    x = torch.randn(5000, 512, device="cuda:0")
    y = torch.empty_like(x)
    before = ntp.ntp_graph_device_bytes(g)
    ntp.ntp_aggregate_fwd_noalloc(g, x, y, 512, 512, 512, ntp.NTP_F32)
    assert ntp.ntp_graph_device_bytes(g) == before
    ntp.ntp_aggregate_fwd(g, x, y, 256, 512, 512, ntp.NTP_F32)
    assert ntp.ntp_graph_device_bytes(g) == before
    y2 = torch.empty_like(x)
    ntp.ntp_aggregate_fwd(g, x, y2, 512, 512, 512, ntp.NTP_F32)
    assert ntp.ntp_graph_device_bytes(g) > before
    ntp.ntp_aggregate_fwd_noalloc(g, x, y, 512, 512, 512, ntp.NTP_F32)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    g.close()


def test_captured_in_a_hip_graph_at_a_width_the_handle_has_no_scratch_for():
    """what the entry point is for: a caller under HIP graph capture, at a slice width (512) for which the
    allocating call would have to hipMalloc.  Captured once, replayed four times with eager work and
    synchronisations between the replays; every replay gives the bits of the eager call."""
    import torch
    src, dst = _hub_graph(6000, 40000, 15, hub_in=3500)
    g = ntp.ntp_graph_build(6000, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS)
    x = torch.randn(6000, 512, device="cuda:0")
    want = torch.empty_like(x)
    before = ntp.ntp_graph_device_bytes(g)
    ntp.ntp_aggregate_fwd_noalloc(g, x, want, 512, 512, 512, ntp.NTP_F32)
    torch.cuda.synchronize()
    y = torch.zeros_like(x)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):              # warm-up on the capture stream's kind, as torch asks for
        ntp.ntp_aggregate_fwd_noalloc(g, x, y, 512, 512, 512, ntp.NTP_F32, torch.cuda.current_stream())
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ntp.ntp_aggregate_fwd_noalloc(g, x, y, 512, 512, 512, ntp.NTP_F32, torch.cuda.current_stream())
    for r in range(4):
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want), "replay %d" % r
        _ = float((x * 2).sum())               # eager work between the replays
    assert ntp.ntp_graph_device_bytes(g) == before
    del graph
    g.close()

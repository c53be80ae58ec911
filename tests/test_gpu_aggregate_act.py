"""ntp_aggregate_act: the aggregation with the activation of eq. (4) applied on the way out,
against the oracle's aggregation followed by the definition of the ReLU and of its mask."""
import sys

import numpy as np
import pytest

import oracle
import ntp_inputs as gen
import paper_2412_20379_amd as ntp
from helpers import TOL_F32, TOL_BF16

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def graph():
    n = 5000
    src, dst = gen.directed_random_edges(n, 70000, 51, hub=9, hub_in=4200, hub_out=1500)
    og = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    resident = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS)
    streamed = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS | ntp.NTP_FORCE_STREAM, chunk_edges=6000)
    yield n, og, resident, streamed
    resident.close()
    streamed.close()


def _compare(got, ref, ref_abs, keep, tol, what):
    """kept elements: the aggregation's value to tolerance; dropped ones: exactly zero.  An element
    whose own sign decides (ReLU) and whose value is zero to rounding may fall either way."""
    got = np.asarray(got, dtype=np.float64)
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - np.where(keep, ref, 0.0))
    bound = tol * np.maximum(ref_abs, np.abs(ref).max() * 1e-30)
    bad = err > bound
    assert not bad.any(), "%s: %d elements off, worst %.3e of the magnitude sum" % (what, int(bad.sum()), (err / np.maximum(ref_abs, 1e-300)).max())


@pytest.mark.parametrize("f,ld,dtype", [(32, 32, "f32"), (20, 24, "f32"), (7, 7, "f32"), (100, 128, "f32"), (256, 256, "f32"),
                                         (64, 64, "bf16"), (40, 48, "bf16")])
@pytest.mark.parametrize("which", ["resident", "streamed"])
def test_relu_on_the_way_out_and_backward_mask(graph, f, ld, dtype, which):
    import torch
    from gpu_util import dev_f32, dev_bf16_bits, host_bf16
    n, og, resident, streamed = graph
    g = resident if which == "resident" else streamed
    bf = dtype == "bf16"
    code = ntp.NTP_BF16 if bf else ntp.NTP_F32
    tol = TOL_BF16 if bf else TOL_F32
    x_np = gen.normal_features(n, f, seed=f)
    m_np = gen.normal_features(n, f, seed=f + 1000)
    m_np[::7] = 0.0                               # zeros in the mask drop the element
    if bf:
        xb, x_used = dev_bf16_bits(x_np)
        mb, m_used = dev_bf16_bits(m_np)
        X = torch.full((n, ld), 0x4000, dtype=torch.int16, device="cuda:0")
        M = torch.full((n, ld), 0x4000, dtype=torch.int16, device="cuda:0")
        X[:, :f] = xb
        M[:, :f] = mb
        fill = 0x4150
    else:
        x_used, m_used = x_np, m_np
        X = torch.full((n, ld), 2.5, device="cuda:0")
        M = torch.full((n, ld), 2.5, device="cuda:0")
        X[:, :f] = dev_f32(x_np)
        M[:, :f] = dev_f32(m_np)
        fill = -3.25
    cs, xs = torch.cuda.Stream(), torch.cuda.Stream()

    def run(direction, mask):
        Y = torch.full((n, ld), fill, dtype=X.dtype, device="cuda:0")
        torch.cuda.synchronize()
        ntp.ntp_aggregate_act(g, direction, X, Y, f, ld, ld, code, ntp.NTP_ACT_RELU, mask, ld, cs, xs)
        torch.cuda.synchronize()
        if ld > f:
            assert bool((Y[:, f:] == fill).all()), "columns outside the slice were written"
        out = Y[:, :f].contiguous()
        return host_bf16(out) if bf else out.cpu().numpy()

    say("aggregate_act", which, f, ld, dtype)
    # forward: Y = max(A_hat X, 0)
    ref, ref_abs = oracle.aggregate(og.csr, x_used, with_abs=True)
    got = run(ntp.NTP_FWD, None)
    sure = np.abs(ref) > tol * ref_abs            # sign determined at the tolerance
    keep = ref > 0
    if bf:
        ref_r = oracle.round_bf16(ref).astype(np.float64)
    else:
        ref_r = ref
    _compare(np.where(sure, got, 0), np.where(sure, ref_r, 0), ref_abs, keep, tol, "forward relu")
    amb = ~sure
    assert np.all(np.abs(got[amb]) <= 2 * tol * ref_abs[amb] + 1e-30)
    assert np.all(got >= 0)
    # backward: Y = (A_hat^T X) * 1[M > 0]
    ref, ref_abs = oracle.aggregate(og.csc, x_used, with_abs=True)
    ref_r = oracle.round_bf16(ref).astype(np.float64) if bf else ref
    got = run(ntp.NTP_BWD, M)
    keep = m_used > 0
    _compare(got, ref_r, ref_abs, keep, tol, "backward mask")
    assert np.all(got[~keep] == 0)
    # against the plain aggregation followed by the mask: the same bits
    Y0 = torch.empty_like(X)
    ntp.ntp_chunked_aggregate(g, ntp.NTP_BWD, X, Y0, f, ld, ld, code, cs, xs)
    torch.cuda.synchronize()
    plain = Y0[:, :f].contiguous()
    plain = host_bf16(plain) if bf else plain.cpu().numpy()
    assert np.array_equal(np.where(keep, plain, 0).view(np.uint32), got.view(np.uint32))


def test_act_none_is_the_plain_aggregation_and_errors(graph):
    import torch
    n, og, resident, streamed = graph
    x = torch.randn(n, 16, device="cuda:0")
    y0, y1 = torch.empty_like(x), torch.empty_like(x)
    ntp.ntp_aggregate_fwd(resident, x, y0, 16, 16, 16)
    ntp.ntp_aggregate_act(resident, ntp.NTP_FWD, x, y1, 16, 16, 16, ntp.NTP_F32, ntp.NTP_ACT_NONE)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    with pytest.raises(ntp.NtpError):
        ntp.ntp_aggregate_act(resident, ntp.NTP_FWD, x, y1, 16, 16, 16, ntp.NTP_F32, 7)
    with pytest.raises(ntp.NtpError):          # the mask overlaps the output
        ntp.ntp_aggregate_act(resident, ntp.NTP_BWD, x, y1, 16, 16, 16, ntp.NTP_F32, ntp.NTP_ACT_RELU, y1, 16)
    with pytest.raises(ntp.NtpError):          # mask rows shorter than the slice
        ntp.ntp_aggregate_act(resident, ntp.NTP_BWD, x, y1, 16, 16, 16, ntp.NTP_F32, ntp.NTP_ACT_RELU, y0, 8)
    src, dst = gen.directed_random_edges(300, 2000, 3)
    gs = ntp.ntp_graph_build(300, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS | ntp.NTP_SCATTER_BWD)
    xs_, ys_, ms_ = (torch.randn(300, 8, device="cuda:0") for _ in range(3))
    with pytest.raises(ntp.NtpError) as e:
        ntp.ntp_aggregate_act(gs, ntp.NTP_BWD, xs_, ys_, 8, 8, 8, ntp.NTP_F32, ntp.NTP_ACT_RELU, ms_, 8)
    assert e.value.code == ntp.NTP_EUNSUPPORTED
    ntp.ntp_aggregate_act(gs, ntp.NTP_FWD, xs_, ys_, 8, 8, 8, ntp.NTP_F32, ntp.NTP_ACT_RELU)      # forward is a gather: fine
    torch.cuda.synchronize()
    assert bool((ys_ >= 0).all())
    gs.close()

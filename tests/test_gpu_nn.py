"""GPU parity of ntp_nn_fwd / ntp_nn_bwd (dense transform of eq. 4) against the oracle."""
import sys

import numpy as np
import pytest

import oracle
from oracle import gcn as ogcn
import ntp_inputs as gen
import paper_2412_20379_amd as ntp
from helpers import assert_close, TOL_F32, TOL_BF16

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def _abs_scale(A, B):
    return np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64)


SHAPES = [(1, 1, 1), (5, 3, 2), (300, 16, 7), (257, 33, 65), (1000, 128, 256), (2708, 1433, 16),
          (4097, 256, 256), (3000, 256, 40), (2050, 100, 47), (1500, 602, 128), (999, 128, 41), (70000, 64, 32),
          # tall matrices (several rounds of blocks on the chip): ragged last tile, partial last contraction
          # step, odd and narrow outputs, more than one column tile
          (20001, 128, 256), (17000, 256, 40), (16500, 100, 47), (18000, 72, 300), (33000, 64, 64)]


@pytest.mark.parametrize("n,k,m", SHAPES)
@pytest.mark.parametrize("act", [ntp.NTP_ACT_NONE, ntp.NTP_ACT_RELU])
def test_nn_fwd_fp32(n, k, m, act):
    import torch
    from gpu_util import dev_f32
    say("nn_fwd", n, k, m, act)
    A = gen.normal_features(n, k, seed=n + k)
    W = gen.glorot_weight(k, m, seed=m)
    H = torch.full((n, m), float("nan"), device="cuda:0")
    ntp.ntp_nn_fwd(dev_f32(A), dev_f32(W), H, n, k, m, act)
    torch.cuda.synchronize()
    ref = ogcn.nn_fwd(A, W, act)
    assert_close(H.cpu().numpy(), ref, _abs_scale(A, W), TOL_F32, "nn_fwd %s" % ((n, k, m),))


@pytest.mark.parametrize("n,k,m", SHAPES)
@pytest.mark.parametrize("act", [ntp.NTP_ACT_NONE, ntp.NTP_ACT_RELU])
@pytest.mark.parametrize("need_dA", [True, False])
def test_nn_bwd_fp32(n, k, m, act, need_dA):
    import torch
    from gpu_util import dev_f32
    say("nn_bwd", n, k, m, act, need_dA)
    A = gen.normal_features(n, k, seed=n + k)
    W = gen.glorot_weight(k, m, seed=m)
    dH = gen.normal_features(n, m, seed=7, stream=6)
    Href = ogcn.nn_fwd(A, W, act).astype(np.float32)      # the H the backward call is given
    dA_ref, dW_ref = ogcn.nn_bwd(A, W, Href, dH, act, need_dA=True)
    dZ = dH * (Href > 0) if act == ntp.NTP_ACT_RELU else dH
    dA = torch.full((n, k), float("nan"), device="cuda:0") if need_dA else None
    dW = torch.full((k, m), float("nan"), device="cuda:0")
    wsb = ntp.ntp_nn_bwd_workspace_bytes(n, k, m)
    ws = torch.empty(max(wsb, 4), dtype=torch.uint8, device="cuda:0")
    ntp.ntp_nn_bwd(dev_f32(A), dev_f32(W), dev_f32(Href), dev_f32(dH), dA, dW, n, k, m, act, ntp.NTP_F32, ws, wsb)
    torch.cuda.synchronize()
    assert_close(dW.cpu().numpy(), dW_ref, _abs_scale(A.T, dZ), TOL_F32, "dW %s" % ((n, k, m),))
    if need_dA:
        assert_close(dA.cpu().numpy(), dA_ref, _abs_scale(dZ, W.T), TOL_F32, "dA %s" % ((n, k, m),))


@pytest.mark.parametrize("n,k,m", [(300, 16, 8), (1000, 128, 256), (2049, 100, 48), (1500, 604, 128)])
def test_nn_bf16(n, k, m):
    import torch
    from gpu_util import dev_bf16_bits, host_bf16, dev_f32
    say("nn_bf16", n, k, m)
    A = gen.normal_features(n, k, seed=n)
    W = gen.glorot_weight(k, m, seed=m)
    dH = gen.normal_features(n, m, seed=8, stream=6)
    Ab, Av = dev_bf16_bits(A)
    Wb, Wv = dev_bf16_bits(W)
    Hb = torch.zeros((n, m), dtype=torch.int16, device="cuda:0")
    ntp.ntp_nn_fwd(Ab, Wb, Hb, n, k, m, ntp.NTP_ACT_RELU, ntp.NTP_BF16)
    torch.cuda.synchronize()
    ref = oracle.round_bf16(ogcn.nn_fwd(Av, Wv, ntp.NTP_ACT_RELU)).astype(np.float64)
    got = host_bf16(Hb)
    assert_close(got, ref, _abs_scale(Av, Wv), TOL_BF16, "bf16 fwd")
    # backward with the H the device produced
    dHb, dHv = dev_bf16_bits(dH)
    dAb = torch.zeros((n, k), dtype=torch.int16, device="cuda:0")
    dW = torch.zeros((k, m), device="cuda:0")
    wsb = ntp.ntp_nn_bwd_workspace_bytes(n, k, m)
    ws = torch.empty(max(wsb, 4), dtype=torch.uint8, device="cuda:0")
    ntp.ntp_nn_bwd(Ab, Wb, Hb, dHb, dAb, dW, n, k, m, ntp.NTP_ACT_RELU, ntp.NTP_BF16, ws, wsb)
    torch.cuda.synchronize()
    dA_ref, dW_ref = ogcn.nn_bwd(Av, Wv, got, dHv, ntp.NTP_ACT_RELU)
    dZ = dHv * (got > 0)
    assert_close(dW.cpu().numpy(), dW_ref, _abs_scale(Av.T, dZ), TOL_F32 * 2, "bf16 dW")
    assert_close(host_bf16(dAb), oracle.round_bf16(dA_ref).astype(np.float64), _abs_scale(dZ, Wv.T), TOL_BF16, "bf16 dA")


def test_nn_deterministic():
    import torch
    from gpu_util import dev_f32
    n, k, m = 20000, 128, 256
    A, W = dev_f32(gen.normal_features(n, k, 1)), dev_f32(gen.glorot_weight(k, m, 1))
    dH = dev_f32(gen.normal_features(n, m, 2))
    H = torch.empty((n, m), device="cuda:0")
    ntp.ntp_nn_fwd(A, W, H, n, k, m, ntp.NTP_ACT_RELU)
    wsb = ntp.ntp_nn_bwd_workspace_bytes(n, k, m)
    ws = torch.empty(max(wsb, 4), dtype=torch.uint8, device="cuda:0")
    outs = []
    for _ in range(2):
        dW = torch.empty((k, m), device="cuda:0")
        ntp.ntp_nn_bwd(A, W, H, dH, None, dW, n, k, m, ntp.NTP_ACT_RELU, ntp.NTP_F32, ws, wsb)
        torch.cuda.synchronize()
        outs.append(dW.cpu().numpy())
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32))


@pytest.mark.parametrize("n,f,ld", [(1, 1, 1), (1000, 7, 7), (777, 40, 48), (5000, 128, 128)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_relu_alone(n, f, ld, dtype):
    """ntp_relu_fwd / ntp_relu_bwd against max(x, 0) and the 1[h > 0] mask; exact"""
    import torch
    from gpu_util import dev_f32, dev_bf16_bits, host_bf16
    h = gen.normal_features(n, ld, seed=n)
    h[::7, 0] = 0.0                                   # exact zeros are not kept
    dh = gen.normal_features(n, ld, seed=n + 1, stream=6)
    if dtype == "f32":
        H, dH = dev_f32(h), dev_f32(dh)
        code, hv, dhv = ntp.NTP_F32, h, dh
        back = lambda t: t.cpu().numpy()
    else:
        (H, hv), (dH, dhv) = dev_bf16_bits(h), dev_bf16_bits(dh)
        code = ntp.NTP_BF16
        back = host_bf16
    dZ = torch.zeros_like(dH)
    ntp.ntp_relu_bwd(dH, H, dZ, n, f, ld, code)
    ntp.ntp_relu_fwd(H, n, f, ld, code)
    torch.cuda.synchronize()
    want_h = hv.copy()
    want_h[:, :f] = np.maximum(hv[:, :f], 0)          # columns beyond f untouched
    assert np.array_equal(back(H), want_h)
    want_dz = np.zeros_like(dhv)
    want_dz[:, :f] = np.where(hv[:, :f] > 0, dhv[:, :f], 0)
    assert np.array_equal(back(dZ), want_dz)


@pytest.mark.parametrize("n,k,m", [(2048, 1024, 256), (1111, 160, 130), (3000, 130, 256), (5000, 512, 192), (20000, 256, 256)])
def test_wide_dynamic_range_keeps_fp32_accuracy(n, k, m):
    """Operands whose magnitudes span six decades: the transform (whose default core forms
    fp32 products from bf16 pieces) must stay at fp32-class accuracy, far inside the
    tolerance: every piece product that matters at 2^-23 has to be there."""
    import torch
    from gpu_util import dev_f32
    from helpers import rel_errors
    say("nn dynamic range", n, k, m)
    rng = gen.stream_rng(n + k + m, 77)
    A = (gen.normal_features(n, k, seed=k) * 10.0 ** rng.uniform(-3, 3, size=(n, k))).astype(np.float32)
    W = (gen.glorot_weight(k, m, seed=m) * 10.0 ** rng.uniform(-3, 3, size=(k, m))).astype(np.float32)
    dH = (gen.normal_features(n, m, seed=9, stream=6) * 10.0 ** rng.uniform(-3, 3, size=(n, m))).astype(np.float32)
    H = torch.full((n, m), float("nan"), device="cuda:0")
    ntp.ntp_nn_fwd(dev_f32(A), dev_f32(W), H, n, k, m, ntp.NTP_ACT_NONE)
    dA = torch.full((n, k), float("nan"), device="cuda:0")
    dW = torch.full((k, m), float("nan"), device="cuda:0")
    wsb = ntp.ntp_nn_bwd_workspace_bytes(n, k, m)
    ws = torch.empty(max(wsb, 4), dtype=torch.uint8, device="cuda:0")
    ntp.ntp_nn_bwd(dev_f32(A), dev_f32(W), H, dev_f32(dH), dA, dW, n, k, m, ntp.NTP_ACT_NONE, ntp.NTP_F32, ws, wsb)
    torch.cuda.synchronize()
    A64, W64, dH64 = A.astype(np.float64), W.astype(np.float64), dH.astype(np.float64)
    for name, got, ref, scale in (("H", H, A64 @ W64, _abs_scale(A, W)),
                                  ("dA", dA, dH64 @ W64.T, _abs_scale(dH, W.T)),
                                  ("dW", dW, A64.T @ dH64, _abs_scale(A.T, dH))):
        norm, comp, _ = rel_errors(got.cpu().numpy(), ref, scale)
        say("   %s: normwise %.2e componentwise %.2e" % (name, norm, comp))
        assert comp <= 2e-6 and norm <= 2e-6, name


@pytest.mark.parametrize("n,c", [(1, 1), (7, 3), (1000, 7), (2708, 16), (5000, 40), (3001, 47), (999, 172), (70000, 41), (4099, 300),
                                 # more than 16384 block sums (1024 partial sums in between); a row that does not
                                 # fit eight classes per lane; exactly eight per lane
                                 (600000, 10), (3000, 600), (2000, 512), (2000, 64), (2000, 65)])
def test_softmax_cross_entropy(n, c):
    """loss of the downstream task and its gradient against the oracle; strided logits,
    large logits (no overflow), determinism"""
    import torch
    from gpu_util import dev_f32
    say("softmax_xent", n, c)
    Z = (gen.normal_features(n, c, seed=n + c) * 6.0).astype(np.float32)
    Z[::7] += 300.0                                  # rows of large logits
    labels = gen.uniform_labels(n, c, n)
    ld = c + 3
    Zd = torch.full((n, ld), 1e30, device="cuda:0")
    Zd[:, :c] = dev_f32(Z)
    dZ = torch.full((n, c), float("nan"), device="cuda:0")
    loss = torch.full((1,), float("nan"), device="cuda:0")
    lab = torch.from_numpy(labels.astype(np.int64)).to("cuda:0")
    nb = ntp.ntp_softmax_xent_scratch_bytes(n)
    scratch = torch.empty(nb // 4, device="cuda:0")
    ntp.ntp_softmax_xent(Zd, lab, dZ, loss, scratch, nb, n, c, ld, c)
    torch.cuda.synchronize()
    want_loss, want_dZ = ogcn.softmax_cross_entropy(Z, labels)
    got = dZ.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    assert abs(float(loss) - want_loss) <= 1e-5 * max(abs(want_loss), 1e-3), (float(loss), want_loss)
    assert np.abs(got - want_dZ).max() <= 1e-5 / n                 # every entry of dZ is a probability / n
    first = (float(loss), dZ.clone())
    ntp.ntp_softmax_xent(Zd, lab, dZ, loss, scratch, nb, n, c, ld, c)
    torch.cuda.synchronize()
    assert float(loss) == first[0] and torch.equal(dZ, first[1])
    with pytest.raises(ntp.NtpError):
        ntp.ntp_softmax_xent(Zd, lab, dZ, loss, scratch, nb - 4, n, c, ld, c)


def test_matrices_beyond_4_gib():
    """4.4 M rows x 256 columns of fp32 are 4.5 GB: element offsets of A, H, dH and dA pass 2^32 bytes (the
    share of one worker on the largest config is of that size).  Forward and dA on sampled rows (the first,
    the last, a thousand in between) against the oracle's rows; dW, which contracts over all rows, against the
    oracle's sum taken over row blocks."""
    import torch
    n, k, m = 4_400_000, 256, 256
    assert n * k * 4 > (1 << 32)
    say("nn beyond 4 GiB", n, k, m)
    dev = "cuda:0"
    gen_t = torch.Generator(device=dev)
    gen_t.manual_seed(11)
    A = torch.randn(n, k, device=dev, generator=gen_t)
    dH = torch.randn(n, m, device=dev, generator=gen_t)
    W = torch.from_numpy(gen.glorot_weight(k, m, seed=3)).to(dev)
    H = torch.empty(n, m, device=dev)
    dA = torch.empty(n, k, device=dev)
    dW = torch.empty(k, m, device=dev)
    wsb = ntp.ntp_nn_bwd_workspace_bytes(n, k, m)
    ws = torch.empty(max(wsb, 4), dtype=torch.uint8, device=dev)
    ntp.ntp_nn_fwd(A, W, H, n, k, m, ntp.NTP_ACT_RELU)
    ntp.ntp_nn_bwd(A, W, H, dH, dA, dW, n, k, m, ntp.NTP_ACT_RELU, ntp.NTP_F32, ws, wsb)
    torch.cuda.synchronize()
    rng = gen.stream_rng(5, 77)
    rows = np.unique(np.concatenate([np.arange(300), np.arange(n - 1000, n), rng.integers(0, n, 1000)]))
    idx = torch.from_numpy(rows).to(dev)
    Wn = W.cpu().numpy()
    A_s, dH_s, H_s, dA_s = (t[idx].cpu().numpy() for t in (A, dH, H, dA))
    ref_H = ogcn.nn_fwd(A_s, Wn, ntp.NTP_ACT_RELU)
    assert_close(H_s, ref_H, _abs_scale(A_s, Wn), TOL_F32, "nn_fwd rows beyond 4 GiB")
    # the backward call is given the device's H (as in test_nn_bwd_fp32 it is given the oracle's): same mask on both sides
    ref_dA, _ = ogcn.nn_bwd(A_s, Wn, H_s, dH_s, ntp.NTP_ACT_RELU)
    dZ_s = dH_s * (H_s > 0)
    assert_close(dA_s, ref_dA, _abs_scale(dZ_s, Wn.T), TOL_F32, "dA rows beyond 4 GiB")
    ref_dW = np.zeros((k, m))
    mag_dW = np.zeros((k, m))
    step = 200_000
    for r0 in range(0, n, step):
        a = A[r0:r0 + step].cpu().numpy()
        h = H[r0:r0 + step].cpu().numpy()
        d = dH[r0:r0 + step].cpu().numpy()
        _, part = ogcn.nn_bwd(a, Wn, h, d, ntp.NTP_ACT_RELU, need_dA=False)
        ref_dW += part
        mag_dW += np.abs(a).astype(np.float64).T @ np.abs(d * (h > 0)).astype(np.float64)
    assert_close(dW.cpu().numpy(), ref_dW, mag_dW, TOL_F32, "dW over 4.4 M rows")


def test_softmax_cross_entropy_beyond_4_gib():
    """6.4 M vertices x 172 classes are 4.4 GB of logits: row offsets pass 2^32 bytes.  The loss against the
    oracle's mean taken over row blocks, the gradient on sampled rows (first, last, a thousand between)."""
    import torch
    n, c = 6_400_000, 172
    assert n * c * 4 > (1 << 32)
    say("softmax_xent beyond 4 GiB", n, c)
    dev = "cuda:0"
    gen_t = torch.Generator(device=dev)
    gen_t.manual_seed(13)
    Z = torch.randn(n, c, device=dev, generator=gen_t) * 4.0
    lab = torch.randint(0, c, (n,), device=dev, generator=gen_t, dtype=torch.int64)
    dZ = torch.empty(n, c, device=dev)
    loss = torch.full((1,), float("nan"), device=dev)
    nb = ntp.ntp_softmax_xent_scratch_bytes(n)
    scratch = torch.empty(nb // 4, device=dev)
    ntp.ntp_softmax_xent(Z, lab, dZ, loss, scratch, nb, n, c, c, c)
    torch.cuda.synchronize()
    total, step = 0.0, 400_000
    for r0 in range(0, n, step):
        l, _ = ogcn.softmax_cross_entropy(Z[r0:r0 + step].cpu().numpy(), lab[r0:r0 + step].cpu().numpy())
        total += l * min(step, n - r0)
    want_loss = total / n
    assert abs(float(loss) - want_loss) <= 1e-5 * abs(want_loss), (float(loss), want_loss)
    rng = gen.stream_rng(6, 78)
    rows = np.unique(np.concatenate([np.arange(300), np.arange(n - 1000, n), rng.integers(0, n, 1000)]))
    idx = torch.from_numpy(rows).to(dev)
    _, want = ogcn.softmax_cross_entropy(Z[idx].cpu().numpy(), lab[idx].cpu().numpy())
    # the oracle divides by the rows it is given; the device by all n
    got = dZ[idx].cpu().numpy().astype(np.float64) * n
    assert np.abs(got - want * rows.size).max() <= 1e-5

"""GPU parity of whole GCN epochs (forward + backward) composed from the library calls."""
import sys

import numpy as np
import pytest

import oracle
from oracle import gcn as ogcn
import ntp_inputs as gen
import paper_2412_20379_amd as ntp
from helpers import check_activation_decisions, TOL_F32

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def _run(cfg, order, scale=1, chunked=False, directed=False, scatter=False, overlap_dw=False, dims=None, workers=0, build_kw=None):
    spec = gen.CONFIGS[cfg]
    n, src, dst = gen.make_graph(cfg, seed=0, scale_down=scale)
    flags = oracle.GCN_FLAGS
    if directed:                       # keep the edges one-way so the transpose matters
        flags = oracle.DIRECTED_GCN_FLAGS
    dims = dims or spec.layers
    X = gen.make_features(cfg, dims[0], seed=0, scale_down=scale)
    kw = build_kw or (dict(device_budget_bytes=8 << 20, chunk_edges=200_000) if chunked else {})
    run_epoch_case(n, src, dst, flags, X, dims, order, chunked=chunked, scatter=scatter, overlap_dw=overlap_dw, build_kw=kw,
                   what="config %d / %d" % (cfg, scale), workers=workers)


def run_epoch_case(n, src, dst, flags, X, dims, order, chunked=False, scatter=False, overlap_dw=False, build_kw=None, what="", seed=0,
                   scale_floor=0.0, workers=0, dw_tol=TOL_F32):
    """one epoch on the device against the oracle: loss, logits, every dW.  scale_floor: entries of dW whose
    sum of |terms| is below this fraction of the largest one are measured against that fraction (the inputs of
    the product carry the rounding of the calls before it, which is relative to THEIR sums of magnitudes and can
    exceed a cancelled entry's own)"""
    import torch
    from paper_2412_20379_amd.gcn import GcnEpoch
    from gpu_util import dev_f32
    og = oracle.build_graph(n, src, dst, flags)
    g = ntp.ntp_graph_build(n, src, dst, flags=flags | (ntp.NTP_SCATTER_BWD if scatter else 0), **(build_kw or {}))
    Ws = [gen.glorot_weight(dims[i], dims[i + 1], seed, i) for i in range(len(dims) - 1)]
    labels = gen.uniform_labels(n, dims[-1], seed)
    if workers:      # the same epoch cut into the calls of `workers` tensor-parallel workers (layer-wise order)
        from paper_2412_20379_amd.tp import TensorParallelEpoch
        assert order == "layerwise"
        ep = TensorParallelEpoch(g, n, dims, workers=workers, chunked=chunked, overlap_dw=overlap_dw)
        ep.transform_first = [False] * (len(dims) - 1)
    else:
        ep = GcnEpoch(g, n, dims, order=order, chunked=chunked, overlap_dw=overlap_dw)
    loss = ep.run(dev_f32(X), [dev_f32(w) for w in Ws], torch.from_numpy(labels.astype(np.int64)).to("cuda:0"))
    torch.cuda.synchronize()
    fn = ogcn.epoch_decoupled if order == "decoupled" else ogcn.epoch_layerwise
    # The ReLU keeps or zeroes a pre-activation by its sign.  Where the pre-activation is zero to
    # rounding, fp32 and fp64 may decide differently, and one such entry on a hub vertex moves dW by
    # far more than rounding.  The oracle works out from its own fp64 values which entries those are
    # (|z| <= 1e-5 of the magnitude sum of z's terms) and takes the device's decision there and only
    # there; everywhere else the device must have decided as the oracle does.
    hid_dev = [h.cpu().numpy() for h in ep.hid[:-1]]
    kw = {} if order == "decoupled" else dict(transform_first=ep.transform_first)
    ref = fn(og, X, Ws, labels, device_relu=[h > 0 for h in hid_dev], **kw)
    check_activation_decisions(hid_dev, ref, what, say, calls_per_layer=1 if order == "decoupled" else 2, scale_floor=scale_floor)
    say(what, order, "loss", float(loss), "oracle", ref["loss"])
    assert abs(float(loss) - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    Z = ep.logits.cpu().numpy().astype(np.float64)
    zs = np.abs(ref["logits"]).max()
    assert np.abs(Z - ref["logits"]).max() <= 2e-5 * zs
    # dW_l sums n products of mixed sign: its rounding error scales with the sum of
    # absolute products |A_l|^T |dZ_l|, not with the (much smaller) result.  The fixed cases
    # hold the per-call 1e-5 against that scale (measured: at most 2e-6); the random sweeps, whose
    # graphs produce columns of dW that cancel almost completely, pass scale_floor and a wider dw_tol.
    L = len(Ws)
    for l, dW in enumerate(ep.dW):
        got = dW.cpu().numpy().astype(np.float64)
        dZ = ref["dH"][l] * ref["relu_keep"][l] if l < L - 1 else ref["dH"][l]
        scale_l = np.abs(ref["nn_in"][l]).T @ np.abs(dZ)
        scale_l = np.maximum(scale_l, scale_floor * scale_l.max())
        err = (np.abs(got - ref["dW"][l]) / np.maximum(scale_l, np.finfo(np.float64).tiny)).max()
        nerr = np.abs(got - ref["dW"][l]).max() / max(np.abs(ref["dW"][l]).max(), np.finfo(np.float64).tiny)   # a dead layer has dW = 0
        say("  dW[%d] error vs sum of |terms| %.2e, vs max|dW| %.2e" % (l, err, nerr))
        assert err <= dw_tol, "dW[%d]" % l
    g.close()


@pytest.mark.parametrize("order", ["layerwise", "decoupled"])
def test_epoch_config1(order):
    _run(1, order)


def test_epoch_config1_directed():
    _run(1, "auto", directed=True)
    _run(1, "reordered", directed=True)
    _run(1, "layerwise", directed=True)
    _run(1, "decoupled", directed=True)


def test_epoch_config1_directed_scatter_backward():
    """same epoch with the by-source form left out: gradients flow back by scatter-add"""
    _run(1, "layerwise", directed=True, scatter=True)
    _run(1, "decoupled", directed=True, scatter=True)
    _run(1, "auto", directed=True, scatter=True, chunked=True)


@pytest.mark.parametrize("order", ["layerwise", "decoupled", "reordered", "auto"])
def test_epoch_config2(order):
    _run(2, order)


@pytest.mark.parametrize("order", ["layerwise", "auto"])
def test_epoch_config2_dw_on_a_second_stream(order):
    """dW of a layer issued beside dA and the backward aggregation: same gradients"""
    _run(2, order, overlap_dw=True)
    _run(1, order, overlap_dw=True, directed=True)


# The model shapes of the power-law configs on scaled-down instances of their graphs: config 3
# (100 -> 256 -> 256 -> 47), config 4 (602 -> 128 -> 41), config 5 (128 -> 128 -> 128 -> 172, the
# hidden width the paper's Table 1 gives for that shape).
MODEL_SHAPES = [(3, 64), (4, 8), (5, 512)]


@pytest.mark.parametrize("cfg,scale", MODEL_SHAPES)
@pytest.mark.parametrize("order", ["layerwise", "auto"])
def test_epoch_model_shapes_of_configs_3_4_5(cfg, scale, order):
    _run(cfg, order, scale=scale)


@pytest.mark.parametrize("cfg,scale", MODEL_SHAPES)
def test_worker_share_epoch_equals_full_model(cfg, scale):
    """Section 3.1: eight workers, each aggregating its column slice over the full graph and
    transforming its row share at full width, together compute the layer-wise epoch of the full
    model: the calls the benchmark times as one worker's share on configs 3 and 4, all eight of
    them, against the oracle.  Config 5's shape runs under a device budget that streams about half
    of its chunks (its chunk size scaled with the graph)."""
    if cfg == 5:
        ce = (256 << 20) // scale
        _run(cfg, "layerwise", scale=scale, workers=8, chunked=True, build_kw=dict(device_budget_bytes=8 * (ce * 8 + (1 << 20)), chunk_edges=ce))
    else:
        _run(cfg, "layerwise", scale=scale, workers=8)
        _run(cfg, "layerwise", scale=scale, workers=8, overlap_dw=True)


def test_epoch_class_count_padded_to_whole_lines():
    """41 classes: the harness appends zero columns to the last transform up to 64 and tells only
    the loss the real count; logits and gradients are those of the 41-class model"""
    for order in ("layerwise", "decoupled", "auto"):
        _run(1, order, dims=(1433, 32, 41))
    _run(1, "layerwise", directed=True, dims=(1433, 48, 35))


def test_epoch_auto_order_mixed_widths():
    """widths that go down, up and down again: both evaluation orders inside one model"""
    import torch
    from paper_2412_20379_amd.gcn import GcnEpoch
    from gpu_util import dev_f32
    n, src, dst = gen.make_graph(2, seed=1, scale_down=8)
    og = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    g = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS)
    dims = (48, 24, 64, 10)
    X = gen.normal_features(n, dims[0], 1)
    Ws = [gen.glorot_weight(dims[i], dims[i + 1], 1, i) for i in range(3)]
    labels = gen.uniform_labels(n, dims[-1], 1)
    ep = GcnEpoch(g, n, dims, order="auto")
    assert ep.transform_first == [True, False, True]
    loss = ep.run(dev_f32(X), [dev_f32(w) for w in Ws], torch.from_numpy(labels.astype(np.int64)).to("cuda:0"))
    torch.cuda.synchronize()
    hid_dev = [h.cpu().numpy() for h in ep.hid[:-1]]
    ref = ogcn.epoch_layerwise(og, X, Ws, labels, device_relu=[h > 0 for h in hid_dev], transform_first=ep.transform_first)
    check_activation_decisions(hid_dev, ref, "mixed widths", say)
    assert abs(float(loss) - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    for l in range(3):
        got = ep.dW[l].cpu().numpy().astype(np.float64)
        dZ = ref["dH"][l] * ref["relu_keep"][l] if l < 2 else ref["dH"][l]
        scale = np.abs(ref["nn_in"][l]).T @ np.abs(dZ)
        assert (np.abs(got - ref["dW"][l]) / scale).max() <= TOL_F32, "dW[%d]" % l
    g.close()


def test_epoch_config2_chunked():
    _run(2, "layerwise", chunked=True)


def test_column_slices_equal_full_width():
    """Section 3.1: a worker's slice result equals the same columns of the full result"""
    import torch
    from gpu_util import dev_f32
    n, src, dst = gen.make_graph(2, seed=0, scale_down=4)
    g = ntp.ntp_graph_build(n, src, dst)
    x = dev_f32(gen.normal_features(n, 256, 0))
    full = torch.empty_like(x)
    ntp.ntp_aggregate_fwd(g, x, full, 256, 256, 256)
    parts = torch.zeros_like(x)
    for w in range(8):                      # eight workers' column windows of the same matrix
        xs = x[:, 32 * w:]
        ys = parts[:, 32 * w:]
        ntp.ntp_aggregate_fwd(g, xs, ys, 32, 256, 256)
    torch.cuda.synchronize()
    a, b = full.cpu().numpy(), parts.cpu().numpy()
    # different lane mapping per width: equal to rounding, not bit-equal
    assert np.abs(a - b).max() <= 1e-5 * np.abs(a).max()
    g.close()


def test_epoch_captured_in_a_hip_graph_replays_identically():
    """The library calls of an epoch are capturable (no allocation after the first call, no
    memset nodes): several replays, with eager work and synchronisations between them, give
    the bits of the eager run."""
    import torch
    from paper_2412_20379_amd.gcn import GcnEpoch
    from gpu_util import dev_f32
    cfg = 1
    n, src, dst = gen.make_graph(cfg, seed=0)
    dims = gen.CONFIGS[cfg].layers
    g = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_GCN_FLAGS)
    X = dev_f32(gen.make_features(cfg, dims[0], seed=0))
    Ws = [dev_f32(gen.glorot_weight(dims[i], dims[i + 1], 0, i)) for i in range(len(dims) - 1)]
    labels = torch.from_numpy(gen.uniform_labels(n, dims[-1], 0).astype(np.int64)).to("cuda:0")
    for order in ("layerwise", "decoupled", "auto"):
        ep = GcnEpoch(g, n, dims, order=order)
        ep.run(X, Ws, labels)                      # first call: scratch is allocated here
        torch.cuda.synchronize()
        want_loss = float(ep.loss)
        want_dW = [w.clone() for w in ep.dW]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            ep.run(X, Ws, labels)
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ep.run(X, Ws, labels)
        for r in range(4):
            for w in ep.dW:
                w.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert float(ep.loss) == want_loss, "%s replay %d" % (order, r)
            for a, b in zip(ep.dW, want_dW):
                assert torch.equal(a, b), "%s replay %d" % (order, r)
            _ = float((X * 2).sum())               # eager work between the replays
    g.close()

"""The layer-wise epoch of Section 3.1 cut the way W tensor-parallel workers run it, on one GPU.

Worker w of W holds the whole graph and, per layer, a column slice of the vertex features
(width ceil(d / W), the last slice the remainder): it aggregates ITS slice over the full graph
(forward and backward), and applies the dense transform to ITS share of the vertices
(ceil(n / W) rows) at full width.  Between the two the paper's `gather` / `split` exchange
re-cuts the matrix from column slices to row shares and back (Section 3.1; an all-to-all between
the workers).  This harness keeps the buffers of all W workers on the one GPU, runs the workers'
library calls one after the other, and stands in for the exchange with strided device copies
(data movement only, no arithmetic); the sum of the workers' weight gradients (the all-reduce
that closes an epoch) is one torch add per layer.  Every aggregation, transform, activation and
the loss run in libntp's kernels.

Running all W workers gives the full model's epoch (checked against the oracle's layer-wise epoch
in tests/test_gpu_epoch.py); running the calls of one worker (`run_worker`) is one worker's share,
which is what the benchmark times on configs 3 and 4.
"""
from __future__ import annotations

import torch

from . import binding as ntp


def line_padded_ld(f: int, elem: int = 4) -> int:
    """row stride (elements) of a compact slice of width f: rows of at least one 128-byte line
    start on line boundaries, narrower ones on 16-byte vectors"""
    per_line, per_vec = 128 // elem, 16 // elem
    return -(-f // per_line) * per_line if f >= per_line else -(-f // per_vec) * per_vec


class TensorParallelEpoch:
    def __init__(self, graph: ntp.Graph, n: int, dims, workers: int = 8, device="cuda:0", chunked=False, overlap_dw=False):
        self.g, self.n, self.dims, self.W = graph, n, tuple(dims), workers
        self.chunked = chunked
        # overlap_dw: the weight gradient of a layer (matrix cores, needed by nobody downstream) runs on a
        # second stream beside the layer's dA and the backward aggregation that follows it (memory system)
        self.overlap_dw = overlap_dw
        self.dw_stream = torch.cuda.Stream(device=device) if overlap_dw else None
        L = self.L = len(dims) - 1
        f32 = dict(dtype=torch.float32, device=device)
        W = workers
        self.n_share = -(-n // W)
        self.rows = [(min(n, w * self.n_share), min(n, (w + 1) * self.n_share)) for w in range(W)]
        # column slices of every layer's input width
        self.s = [-(-dims[l] // W) for l in range(L)]
        self.cols = [[(min(dims[l], w * self.s[l]), min(dims[l], (w + 1) * self.s[l])) for w in range(W)] for l in range(L)]
        self.ld = [line_padded_ld(self.s[l]) for l in range(L)]
        # per layer and worker: the slice it aggregates (S), the aggregated slice (T); backward: the
        # gradient slice it aggregates (dS) and the result (dT).  Padding columns stay zero.
        self.S = [[torch.zeros(n, self.ld[l], **f32) for _ in range(W)] for l in range(L)]
        self.T = [[torch.zeros(n, self.ld[l], **f32) for _ in range(W)] for l in range(L)]
        self.dS = [[torch.zeros(n, self.ld[l], **f32) for _ in range(W)] if l > 0 else None for l in range(L)]
        self.dT = [[torch.zeros(n, self.ld[l], **f32) for _ in range(W)] if l > 0 else None for l in range(L)]
        # full-width matrices, cut by rows between the workers: transform input, output, gradients
        self.A = [torch.empty(n, dims[l], **f32) for l in range(L)]
        self.H = [torch.empty(n, dims[l + 1], **f32) for l in range(L)]
        self.dH = [torch.empty(n, dims[l + 1], **f32) for l in range(L)]
        self.dA = [torch.empty(n, dims[l], **f32) if l > 0 else None for l in range(L)]
        self.dW_part = [torch.empty(W, dims[l], dims[l + 1], **f32) for l in range(L)]
        self.dW = [torch.empty(dims[l], dims[l + 1], **f32) for l in range(L)]
        self.ws_bytes = max(ntp.ntp_nn_bwd_workspace_bytes(self.n_share, dims[l], dims[l + 1]) for l in range(L))
        self.ws = torch.empty(max(self.ws_bytes, 4), dtype=torch.uint8, device=device)
        self.ws2 = torch.empty(max(self.ws_bytes, 4), dtype=torch.uint8, device=device) if overlap_dw else None
        self.loss_buf = torch.zeros(1, **f32)
        self.loss_scratch = torch.empty(ntp.ntp_softmax_xent_scratch_bytes(n) // 4, **f32)
        self.copy_stream = torch.cuda.Stream(device=device) if chunked else None
        self.weights = None
        self.labels = None
        self.loss = None
        self.logits = self.H[-1]
        self.hid = self.H
        self.events = None      # set to a list to collect (tag, start, end) HIP events per library call

    # ---- library calls of one worker --------------------------------------------------------
    def _timed(self, tag, fn, *a):
        if self.events is None:
            return fn(*a)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        fn(*a)
        e1.record()
        self.events.append((tag, e0, e1))

    def _agg(self, direction, src, dst, f, ld, mask=None):
        st = torch.cuda.current_stream()
        tag = "agg_%s f=%d" % ("fwd" if direction == ntp.NTP_FWD else "bwd", f)
        if mask is not None:
            # the gradient flows back into a ReLU layer: its mask rides on the aggregation's way out
            self._timed(tag, ntp.ntp_aggregate_act, self.g, direction, src, dst, f, ld, ld, ntp.NTP_F32, ntp.NTP_ACT_RELU,
                        mask, ld, st, self.copy_stream)
        elif self.chunked:
            self._timed(tag, ntp.ntp_chunked_aggregate, self.g, direction, src, dst, f, ld, ld, ntp.NTP_F32, st, self.copy_stream)
        elif direction == ntp.NTP_FWD:
            self._timed(tag, ntp.ntp_aggregate_fwd, self.g, src, dst, f, ld, ld, ntp.NTP_F32, st)
        else:
            self._timed(tag, ntp.ntp_aggregate_bwd, self.g, src, dst, f, ld, ld, ntp.NTP_F32, st)

    def agg_fwd(self, l, w):
        c0, c1 = self.cols[l][w]
        if c1 > c0:
            self._agg(ntp.NTP_FWD, self.S[l][w], self.T[l][w], c1 - c0, self.ld[l])

    def agg_bwd(self, l, w):
        c0, c1 = self.cols[l][w]
        if c1 > c0:
            # the result is the gradient at H_{l-1}, whose slice this worker holds as the input of
            # its forward aggregation: masked by its sign, it is dZ of layer l-1 already
            self._agg(ntp.NTP_BWD, self.dS[l][w], self.dT[l][w], c1 - c0, self.ld[l], mask=self.S[l][w])

    def nn_fwd(self, l, w):
        r0, r1 = self.rows[w]
        if r1 > r0:
            d = self.dims
            act = ntp.NTP_ACT_RELU if l < self.L - 1 else ntp.NTP_ACT_NONE
            self._timed("nn_fwd %dx%d" % (d[l], d[l + 1]), ntp.ntp_nn_fwd, self.A[l][r0:r1], self.weights[l], self.H[l][r0:r1],
                        r1 - r0, d[l], d[l + 1], act, ntp.NTP_F32, torch.cuda.current_stream())

    def nn_bwd(self, l, w):
        r0, r1 = self.rows[w]
        d = self.dims
        if r1 <= r0:
            self.dW_part[l][w].zero_()
            return
        # no activation here: the gradient of a hidden layer arrives masked (agg_bwd), the last layer has none
        st = torch.cuda.current_stream()
        args = (self.A[l][r0:r1], self.weights[l], self.H[l][r0:r1], self.dH[l][r0:r1])
        shape = (r1 - r0, d[l], d[l + 1], ntp.NTP_ACT_NONE, ntp.NTP_F32)
        if self.overlap_dw and l > 0:
            ready = torch.cuda.Event()
            ready.record(st)
            self.dw_stream.wait_event(ready)
            ntp.ntp_nn_bwd(*args, None, self.dW_part[l][w], *shape, self.ws2, self.ws_bytes, self.dw_stream)
            self._timed("nn_bwd %dx%d dA only" % (d[l], d[l + 1]), ntp.ntp_nn_bwd, *args, self.dA[l][r0:r1], None, *shape, None, 0, st)
        else:
            self._timed("nn_bwd %dx%d%s" % (d[l], d[l + 1], " +dA" if l > 0 else ""), ntp.ntp_nn_bwd, *args,
                        self.dA[l][r0:r1] if l > 0 else None, self.dW_part[l][w], *shape, self.ws, self.ws_bytes, st)

    def _join_dw(self):
        """the main stream waits for the weight gradients issued on the side stream"""
        if self.overlap_dw:
            done = torch.cuda.Event()
            done.record(self.dw_stream)
            torch.cuda.current_stream().wait_event(done)

    # ---- stand-ins for the exchange between the workers (device copies) ---------------------
    def _split(self, full, slices, l):
        """column slices of a full-width matrix, one per worker"""
        for w, (c0, c1) in enumerate(self.cols[l]):
            if c1 > c0:
                slices[w][:, : c1 - c0].copy_(full[:, c0:c1])

    def _gather(self, slices, full, l):
        """the full-width matrix from the workers' column slices"""
        for w, (c0, c1) in enumerate(self.cols[l]):
            if c1 > c0:
                full[:, c0:c1].copy_(slices[w][:, : c1 - c0])

    # ---- the epoch ----------------------------------------------------------------------------
    def run(self, X, weights, labels):
        """all W workers, one after the other: the full model's forward + backward pass"""
        self.weights, self.labels = list(weights), labels
        L, W = self.L, self.W
        full = X
        for l in range(L):
            self._split(full, self.S[l], l)
            for w in range(W):
                self.agg_fwd(l, w)
            self._gather(self.T[l], self.A[l], l)
            for w in range(W):
                self.nn_fwd(l, w)
            full = self.H[l]
        # loss over all vertices in one call (a worker's part is its rows; the mean needs all of them)
        c = self.dims[-1]
        self._timed("softmax_xent %d" % c, ntp.ntp_softmax_xent, self.H[-1], labels, self.dH[-1], self.loss_buf, self.loss_scratch,
                    self.loss_scratch.numel() * 4, self.n, c, c, c, torch.cuda.current_stream())
        self.loss = self.loss_buf[0]
        for l in range(L - 1, -1, -1):
            for w in range(W):
                self.nn_bwd(l, w)
            self._join_dw()
            torch.sum(self.dW_part[l], dim=0, out=self.dW[l])       # stands in for the all-reduce of the weight gradients
            if l > 0:
                self._split(self.dA[l], self.dS[l], l)
                for w in range(W):
                    self.agg_bwd(l, w)
                self._gather(self.dT[l], self.dH[l - 1], l)
        return self.loss

    def run_worker(self, w: int = 0):
        """only worker w's library calls, on the buffers a full run left behind (one worker's share
        of the epoch's kernel work; the exchange with the other workers is not part of it)"""
        L = self.L
        for l in range(L):
            self.agg_fwd(l, w)
            self.nn_fwd(l, w)
        for l in range(L - 1, -1, -1):
            self.nn_bwd(l, w)
            if l > 0:
                self.agg_bwd(l, w)
        self._join_dw()

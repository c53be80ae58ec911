"""Layer-wise and decoupled GCN epochs composed from the library calls.

Harness code: it owns the device buffers (torch tensors) and the order of the calls;
all arithmetic of an epoch runs inside libntp: aggregation, transform, activation and
the softmax cross-entropy of the downstream task that closes the forward pass of Alg. 1.
"""
from __future__ import annotations

import torch

from . import binding as ntp


def padded_width(c: int) -> int:
    """whole 128-byte lines of floats, or whole 16-byte vectors below one line"""
    return -(-c // 32) * 32 if c >= 32 else -(-c // 4) * 4


class GcnEpoch:
    """One forward + backward pass of an L-layer GCN on one GPU (no optimiser step).

    layer-wise (Section 3.1):  A_l = A_hat H_{l-1};  H_l = relu(A_l W_l), logits = A_L W_L
    decoupled (Section 4.1):   H = MLP(X);  Z = A_hat^L H
    reordered:                 layer-wise, but the last layer (no activation) is evaluated as
                               A_hat (H_{L-1} W_L) when that is the narrower side, so its forward
                               and backward aggregations run at the output width; same function
                               and gradients as layer-wise, fewer edge-feature products.
    auto:                      every layer whose output is narrower than its input is evaluated
                               as sigma(A_hat (H W)) (ntp_relu_fwd / ntp_relu_bwd supply the
                               activation); the others stay aggregate-first.
    """

    def __init__(self, graph: ntp.Graph, n: int, dims, device="cuda:0", order="layerwise", chunked=False,
                 overlap_dw=False, pad_classes=True, fuse_activation=True):
        # fuse_activation: activations that directly follow an aggregation ride on its way out
        # (ntp_aggregate_act) instead of taking a pass of their own (ntp_relu_fwd / ntp_relu_bwd, or
        # the mask reads of ntp_nn_bwd)
        # A class count that is not a multiple of four floats makes every row of the logits (and of
        # whatever is aggregated at that width) start off a 16-byte boundary.  The last transform
        # then gets zero columns appended up to whole 128-byte lines (16-byte vectors below 32
        # classes): logits and gradients carry zero padding columns that change no sum, and only
        # the loss is told the real count.
        self.classes = dims[-1]
        if pad_classes and dims[-1] % 4:
            dims = tuple(dims[:-1]) + (padded_width(dims[-1]),)
        self.g, self.n, self.dims, self.order, self.chunked = graph, n, tuple(dims), order, chunked
        # overlap_dw: in the layer-wise backward, dW of a layer runs on a second stream beside
        # dA and the backward aggregation that follows it (matrix cores beside the memory system)
        self.overlap_dw = overlap_dw
        L = len(dims) - 1
        f32 = dict(dtype=torch.float32, device=device)
        # per layer: evaluate as sigma(A_hat (H W)) instead of sigma((A_hat H) W)?
        narrower = [dims[l + 1] < dims[l] for l in range(L)]
        if order == "auto":
            self.transform_first = narrower
        elif order == "reordered":
            self.transform_first = [False] * (L - 1) + [narrower[-1]]
        else:
            self.transform_first = [False] * L
        lw = order in ("layerwise", "reordered", "auto")
        self.aggs = [None if self.transform_first[l] else torch.empty(n, dims[l], **f32) for l in range(L)] if lw else []
        self.tbuf = [torch.empty(n, dims[l + 1], **f32) if self.transform_first[l] else None for l in range(L)] if lw else []
        self.hid = [torch.empty(n, dims[l + 1], **f32) for l in range(L)]
        self.dW_buf = [torch.empty(dims[l], dims[l + 1], **f32) for l in range(L)]
        self.dW = self.dW_buf[:-1] + [self.dW_buf[-1][:, :self.classes]]      # views without the padding columns
        self.w_last = torch.zeros(dims[-2], dims[-1], **f32) if dims[-1] != self.classes else None
        wmax = max(dims)
        self.tmp = [torch.empty(n, wmax, **f32) for _ in range(3 if overlap_dw else 2)]
        self.logits_buf = torch.empty(n, dims[-1], **f32) if order == "decoupled" else None
        ws = max(ntp.ntp_nn_bwd_workspace_bytes(n, dims[l], dims[l + 1]) for l in range(L))
        self.ws_bytes = ws
        self.ws = torch.empty(max(ws, 4), dtype=torch.uint8, device=device)
        self.dlogits = torch.zeros(n, dims[-1], **f32)       # padding columns stay zero
        self.loss_buf = torch.zeros(1, **f32)
        self.loss_scratch = torch.empty(ntp.ntp_softmax_xent_scratch_bytes(n) // 4, **f32)
        self.copy_stream = torch.cuda.Stream(device=device) if chunked else None
        self.dw_stream = torch.cuda.Stream(device=device) if overlap_dw else None
        self.ws2 = torch.empty(max(ws, 4), dtype=torch.uint8, device=device) if overlap_dw else None
        self.loss = None
        self.logits = None
        self.fuse_activation = fuse_activation
        self.events = None      # set to a list to collect (tag, start, end) HIP events per library call

    def _timed(self, tag, fn, *a):
        if self.events is None:
            return fn(*a)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        fn(*a)
        e1.record()
        self.events.append((tag, e0, e1))

    def _nn_fwd(self, *a):
        self._timed("nn_fwd %dx%d" % (a[4], a[5]), ntp.ntp_nn_fwd, *a)

    def _nn_bwd(self, *a):
        tag = "nn_bwd %dx%d%s" % (a[7], a[8], "" if a[4] is None else (" +dA" if a[5] is not None else " dA only"))
        self._timed(tag, ntp.ntp_nn_bwd, *a)

    def _agg(self, direction, src, dst, f, relu=False, mask=None):
        """aggregate; relu / mask: with the activation applied on the way out (ntp_aggregate_act):
        forward ReLU of a transform-first layer, or the backward mask 1[mask > 0] of the ReLU layer
        below.  Returns False when the activation could not ride along (scatter-add backward) and
        the plain aggregation ran instead."""
        tag = "agg_%s f=%d" % ("fwd" if direction == ntp.NTP_FWD else "bwd", f)
        if (relu or mask is not None) and self.fuse_activation:
            try:
                self._timed(tag, ntp.ntp_aggregate_act, self.g, direction, src, dst, f, f, f, ntp.NTP_F32, ntp.NTP_ACT_RELU,
                            mask, f, torch.cuda.current_stream(), self.copy_stream)
                return True
            except ntp.NtpError as e:
                if e.code != ntp.NTP_EUNSUPPORTED:
                    raise
                self.fuse_activation = False
        self._timed(tag, self._agg_call, direction, src, dst, f)
        return False

    def _agg_call(self, direction, src, dst, f):
        st = torch.cuda.current_stream()
        if self.chunked:
            ntp.ntp_chunked_aggregate(self.g, direction, src, dst, f, f, f, ntp.NTP_F32, st, self.copy_stream)
        elif direction == ntp.NTP_FWD:
            ntp.ntp_aggregate_fwd(self.g, src, dst, f, f, f, ntp.NTP_F32, st)
        else:
            ntp.ntp_aggregate_bwd(self.g, src, dst, f, f, f, ntp.NTP_F32, st)

    def _view(self, i, f):
        return self.tmp[i].view(-1)[: self.n * f].view(self.n, f)

    def _loss_grad(self, Z, labels):
        c, ld = self.classes, self.dims[-1]
        self._timed("softmax_xent %d" % c, ntp.ntp_softmax_xent, Z, labels, self.dlogits, self.loss_buf, self.loss_scratch,
                    self.loss_scratch.numel() * 4, self.n, c, ld, ld, torch.cuda.current_stream())
        self.loss = self.loss_buf[0]
        return self.dlogits

    def run(self, X, weights, labels):
        if self.w_last is not None:
            self.w_last[:, :self.classes].copy_(weights[-1])
            weights = list(weights[:-1]) + [self.w_last]
        if self.order in ("layerwise", "reordered", "auto"):
            loss = self._layerwise(X, weights, labels)
        else:
            loss = self._decoupled(X, weights, labels)
        self.logits = self.logits[:, :self.classes]
        return loss

    def _other_view(self, t, f):
        """a scratch view of width f that does not share memory with tensor t"""
        i = 1 if (t is not None and t.data_ptr() == self.tmp[0].data_ptr()) else 0
        return self._view(i, f)

    def _layerwise(self, X, Ws, labels):
        n, d = self.n, self.dims
        L = len(Ws)
        st = torch.cuda.current_stream()
        tf = self.transform_first
        ins = []
        H = X
        for l in range(L):
            ins.append(H)
            last = l == L - 1
            if tf[l]:
                # sigma(A_hat (H W)): transform first, aggregate at the output width, then activate
                self._nn_fwd(H, Ws[l], self.tbuf[l], n, d[l], d[l + 1], ntp.NTP_ACT_NONE, ntp.NTP_F32, st)
                if not self._agg(ntp.NTP_FWD, self.tbuf[l], self.hid[l], d[l + 1], relu=not last) and not last:
                    self._timed("relu_fwd %d" % d[l + 1], ntp.ntp_relu_fwd, self.hid[l], n, d[l + 1], d[l + 1], ntp.NTP_F32, st)
            else:
                self._agg(ntp.NTP_FWD, H, self.aggs[l], d[l])
                act = ntp.NTP_ACT_NONE if last else ntp.NTP_ACT_RELU
                self._nn_fwd(self.aggs[l], Ws[l], self.hid[l], n, d[l], d[l + 1], act, ntp.NTP_F32, st)
            H = self.hid[l]
        self.logits = H
        dH = self._loss_grad(H, labels)
        pending = None      # event of the last dW issued on the side stream
        masked = False      # dH already carries the mask of this layer's ReLU (applied by the aggregation that produced it)
        for l in range(L - 1, -1, -1):
            last = l == L - 1
            was_masked, masked = masked, False
            if tf[l]:
                if pending is not None:
                    st.wait_event(pending)
                    pending = None
                if not last and not was_masked:       # dZ = dH * 1[H > 0], in place
                    self._timed("relu_bwd %d" % d[l + 1], ntp.ntp_relu_bwd, dH, self.hid[l], dH, n, d[l + 1], d[l + 1], ntp.NTP_F32, st)
                dT = self.tbuf[l]  # dT = A_hat^T dZ at the output width; then dW = H_in^T dT, dH_in = dT W^T
                self._agg(ntp.NTP_BWD, dH, dT, d[l + 1])
                dHin = self._view(0, d[l]) if l > 0 else None
                self._nn_bwd(ins[l], Ws[l], self.hid[l], dT, dHin, self.dW_buf[l], n, d[l], d[l + 1],
                             ntp.NTP_ACT_NONE, ntp.NTP_F32, self.ws, self.ws_bytes, st)
                dH = dHin
            elif self.overlap_dw and l > 0:
                act = ntp.NTP_ACT_NONE if (last or was_masked) else ntp.NTP_ACT_RELU
                # dW beside dA + aggregation: the side stream reads dH, which therefore must not
                # be overwritten before its event; three scratch buffers rotate
                ready = torch.cuda.Event()
                ready.record(st)
                self.dw_stream.wait_event(ready)
                ntp.ntp_nn_bwd(self.aggs[l], Ws[l], self.hid[l], dH, None, self.dW_buf[l], n, d[l], d[l + 1], act,
                               ntp.NTP_F32, self.ws2, self.ws_bytes, self.dw_stream)
                done = torch.cuda.Event()
                done.record(self.dw_stream)
                used = {dH.data_ptr()} if any(dH.data_ptr() == t.data_ptr() for t in self.tmp) else set()
                ia = next(i for i in range(3) if self.tmp[i].data_ptr() not in used)
                dA = self._view(ia, d[l])
                if pending is not None:        # the buffer of the previous layer's dH may be written now
                    st.wait_event(pending)
                self._nn_bwd(self.aggs[l], Ws[l], self.hid[l], dH, dA, None, n, d[l], d[l + 1], act,
                             ntp.NTP_F32, None, 0, st)
                used.add(dA.data_ptr())
                io = next(i for i in range(3) if self.tmp[i].data_ptr() not in used)
                out = self._view(io, d[l])
                masked = self._agg(ntp.NTP_BWD, dA, out, d[l], mask=self.hid[l - 1])
                dH = out
                pending = done
            else:
                act = ntp.NTP_ACT_NONE if (last or was_masked) else ntp.NTP_ACT_RELU
                dA = self._other_view(dH, d[l]) if l > 0 else None
                if pending is not None:
                    st.wait_event(pending)
                    pending = None
                self._nn_bwd(self.aggs[l], Ws[l], self.hid[l], dH, dA, self.dW_buf[l], n, d[l], d[l + 1], act,
                             ntp.NTP_F32, self.ws, self.ws_bytes, st)
                if l > 0:
                    dH = self._other_view(dA, d[l])
                    masked = self._agg(ntp.NTP_BWD, dA, dH, d[l], mask=self.hid[l - 1])
        if pending is not None:
            st.wait_event(pending)
        return self.loss

    def _decoupled(self, X, Ws, labels):
        n, d = self.n, self.dims
        L = len(Ws)
        st = torch.cuda.current_stream()
        ins = [X]
        H = X
        for l in range(L):
            act = ntp.NTP_ACT_RELU if l < L - 1 else ntp.NTP_ACT_NONE
            self._nn_fwd(H, Ws[l], self.hid[l], n, d[l], d[l + 1], act, ntp.NTP_F32, st)
            H = self.hid[l]
            ins.append(H)
        c = d[-1]
        Z = H
        for k in range(L):          # L rounds of aggregation at the output width, no intermediates kept
            out = self._view(k % 2, c) if k < L - 1 else self.logits_buf
            self._agg(ntp.NTP_FWD, Z, out, c)
            Z = out
        self.logits = Z
        dZ = self._loss_grad(Z, labels)
        for k in range(L):
            out = self._view(k % 2, c)
            self._agg(ntp.NTP_BWD, dZ, out, c)
            dZ = out
        dH = dZ
        for l in range(L - 1, -1, -1):
            act = ntp.NTP_ACT_RELU if l < L - 1 else ntp.NTP_ACT_NONE
            dA = None
            if l > 0:
                # the two scratch views are free again except the one holding dH
                dA = self._view(0 if dH.data_ptr() != self.tmp[0].data_ptr() else 1, d[l])
            self._nn_bwd(ins[l], Ws[l], self.hid[l], dH, dA, self.dW_buf[l], n, d[l], d[l + 1], act,
                         ntp.NTP_F32, self.ws, self.ws_bytes, st)
            dH = dA
        return self.loss

"""A decoupled GAT epoch composed from the library calls (one attention head).

Section 4.1's decoupled order with the attention of Section 2.1 as the edge weights:
    Lhat = MLP(X);  p = Lhat a_src, q = Lhat a_dst;  alpha = edge softmax of LeakyReLU(p[u] + q[v]);
    Z^0 = Lhat, Z^k = sum_u alpha(u -> v) Z^(k-1)[u] for k = 1..rounds;  loss = softmax cross-entropy(Z^rounds)
and the exact backward pass of that function (the weights' own gradient included).

Harness code: it owns the device buffers (torch tensors) and the order of the calls; all
arithmetic runs inside libntp.

The class width c is padded to a row of whole 128-byte lines (16-byte vectors below 32 classes):
the last transform gets zero columns appended, so Lhat, every Z^k and every gradient carry zero
padding columns that change no sum; only the loss is told the real c.  Gathered rows then start
on line boundaries and every kernel takes its vector-load path.
"""
from __future__ import annotations

import torch

from . import binding as ntp


def padded_width(c: int) -> int:
    return -(-c // 32) * 32 if c >= 32 else -(-c // 4) * 4


class GatEpoch:
    def __init__(self, graph: ntp.Graph, n: int, nnz: int, dims, rounds: int = 2, negative_slope: float = 0.2,
                 device="cuda:0", padded_classes=None):
        self.g, self.n, self.nnz, self.dims, self.rounds, self.slope = graph, n, nnz, tuple(dims), rounds, negative_slope
        L = len(dims) - 1
        c = dims[-1]
        cp = self.cp = padded_classes or padded_width(c)
        assert cp >= c
        self.pdims = tuple(dims[:-1]) + (cp,)
        f32 = dict(dtype=torch.float32, device=device)
        self.hid = [torch.empty(n, self.pdims[l + 1], **f32) for l in range(L)]      # hid[-1] = Lhat = Z^0
        self.Z = [self.hid[-1]] + [torch.empty(n, cp, **f32) for _ in range(rounds)]
        self.G = [torch.empty(n, cp, **f32) for _ in range(2)]                       # G^k below the logits' gradient
        self.dlogits = torch.zeros(n, cp, **f32)                                     # padding columns stay zero
        self.p, self.q = torch.empty(n, **f32), torch.empty(n, **f32)
        self.dp, self.dq = torch.empty(n, **f32), torch.empty(n, **f32)
        self.alpha_in, self.alpha_out = torch.empty(nnz, **f32), torch.empty(nnz, **f32)
        self.w_last = torch.zeros(dims[-2], cp, **f32)                               # last transform, zero columns appended
        self.a_pad = torch.zeros(2, cp, **f32)
        self.dW_buf = [torch.empty(self.pdims[l], self.pdims[l + 1], **f32) for l in range(L)]
        self.dW = self.dW_buf[:-1] + [self.dW_buf[-1][:, :c]]
        self.da_buf = torch.empty(2, cp, **f32)
        self.da_src, self.da_dst = self.da_buf[0, :c], self.da_buf[1, :c]
        self.tmp = [torch.empty(n, max(self.pdims), **f32) for _ in range(2)]
        self.ws_bytes = max(ntp.ntp_nn_bwd_workspace_bytes(n, self.pdims[l], self.pdims[l + 1]) for l in range(L))
        self.ws = torch.empty(max(self.ws_bytes, 4), dtype=torch.uint8, device=device)
        self.sc_bytes = ntp.ntp_attention_scores_bwd_scratch_bytes(n, cp)
        self.sc = torch.empty(max(self.sc_bytes, 4), dtype=torch.uint8, device=device)
        self.loss_buf = torch.zeros(1, **f32)
        self.loss_scratch = torch.empty(ntp.ntp_softmax_xent_scratch_bytes(n) // 4, **f32)
        self.loss = None
        self.logits = None

    def _view(self, i, f):
        return self.tmp[i].view(-1)[: self.n * f].view(self.n, f)

    def run(self, X, weights, a_src, a_dst, labels):
        n, d, R, g = self.n, self.pdims, self.rounds, self.g
        L = len(weights)
        c, cp = self.dims[-1], self.cp
        st = torch.cuda.current_stream()
        self.w_last[:, :c].copy_(weights[-1])
        self.a_pad[0, :c].copy_(a_src)
        self.a_pad[1, :c].copy_(a_dst)
        weights = list(weights[:-1]) + [self.w_last]
        a_src, a_dst = self.a_pad[0], self.a_pad[1]
        ins = [X]
        H = X
        for l in range(L):
            act = ntp.NTP_ACT_RELU if l < L - 1 else ntp.NTP_ACT_NONE
            ntp.ntp_nn_fwd(H, weights[l], self.hid[l], n, d[l], d[l + 1], act, ntp.NTP_F32, st)
            H = self.hid[l]
            ins.append(H)
        ntp.ntp_attention_scores_fwd(H, a_src, a_dst, self.p, self.q, n, cp, cp, st)
        ntp.ntp_edge_softmax(g, self.p, self.q, self.slope, self.alpha_in, self.alpha_out, st)
        for k in range(1, R + 1):
            ntp.ntp_aggregate_weighted(g, ntp.NTP_FWD, self.alpha_in, self.Z[k - 1], self.Z[k], cp, cp, cp, ntp.NTP_F32, st)
        self.logits = self.Z[R][:, :c]
        ntp.ntp_softmax_xent(self.Z[R], labels, self.dlogits, self.loss_buf, self.loss_scratch,
                             self.loss_scratch.numel() * 4, n, c, cp, cp, st)
        self.loss = self.loss_buf[0]
        # backward: G^k = dloss/dZ^k; every round adds its share of the scores' gradient
        Gk = self.dlogits
        for k in range(R, 0, -1):
            ntp.ntp_edge_softmax_bwd(g, self.p, self.q, self.slope, self.alpha_in, self.alpha_out, self.Z[k - 1], Gk,
                                     cp, cp, cp, self.dp, self.dq, k != R, st)
            out = self.G[k % 2]
            ntp.ntp_aggregate_weighted(g, ntp.NTP_BWD, self.alpha_out, Gk, out, cp, cp, cp, ntp.NTP_F32, st)
            Gk = out
        # Gk = G^0; the scores' share makes it the gradient of Lhat
        ntp.ntp_attention_scores_bwd(self.hid[-1], a_src, a_dst, self.dp, self.dq, Gk, self.da_buf[0], self.da_buf[1],
                                     n, cp, cp, cp, self.sc, self.sc_bytes, st)
        dH = Gk
        for l in range(L - 1, -1, -1):
            act = ntp.NTP_ACT_RELU if l < L - 1 else ntp.NTP_ACT_NONE
            dA = self._view(l % 2, d[l]) if l > 0 else None
            ntp.ntp_nn_bwd(ins[l], weights[l], self.hid[l], dH, dA, self.dW_buf[l], n, d[l], d[l + 1], act,
                           ntp.NTP_F32, self.ws, self.ws_bytes, st)
            dH = dA
        return self.loss

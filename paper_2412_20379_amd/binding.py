"""ctypes binding of libntp.so: same names as include/ntp.h, argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))

NTP_OK, NTP_EINVAL, NTP_ENOMEM, NTP_EHIP, NTP_EBUDGET, NTP_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
NTP_SYMMETRISE, NTP_DEDUP, NTP_ADD_SELF_LOOPS, NTP_NORM_GCN_SYM, NTP_HOST_ONLY, NTP_FORCE_STREAM = 1, 2, 4, 8, 16, 32
NTP_SCATTER_BWD = 64
NTP_EDGE_PERM = 128
NTP_GCN_FLAGS = NTP_SYMMETRISE | NTP_DEDUP | NTP_ADD_SELF_LOOPS | NTP_NORM_GCN_SYM
NTP_DIRECTED_GCN_FLAGS = NTP_DEDUP | NTP_ADD_SELF_LOOPS | NTP_NORM_GCN_SYM
NTP_CSR, NTP_CSC = 0, 1
NTP_F32, NTP_BF16 = 0, 1
NTP_FWD, NTP_BWD = 0, 1
NTP_ACT_NONE, NTP_ACT_RELU = 0, 1

EXPORTED_SYMBOLS = [
    "ntp_graph_build", "ntp_graph_info", "ntp_graph_export", "ntp_graph_export_perm", "ntp_graph_chunks", "ntp_graph_stream_bytes",
    "ntp_graph_device_bytes", "ntp_aggregate_fwd", "ntp_aggregate_fwd_noalloc", "ntp_aggregate_bwd", "ntp_chunked_aggregate",
    "ntp_chunked_aggregate_multi", "ntp_aggregate_act", "ntp_edge_softmax", "ntp_edge_softmax_bwd", "ntp_aggregate_weighted",
    "ntp_attention_scores_fwd", "ntp_attention_scores_bwd", "ntp_attention_scores_bwd_scratch_bytes",
    "ntp_nn_fwd", "ntp_nn_bwd", "ntp_nn_bwd_workspace_bytes", "ntp_softmax_xent", "ntp_softmax_xent_scratch_bytes", "ntp_relu_fwd", "ntp_relu_bwd",
    "ntp_graph_free", "ntp_last_error",
]


class NtpError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("libntp error %d: %s" % (code, text))
        self.code = code


def lib_path() -> str:
    return os.path.join(_PKG, "libntp.so")


_lib = None


def lib():
    """Load libntp.so, building it first only when no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build()
    L = ctypes.CDLL(path)
    vp, i64, i32, u32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32
    L.ntp_graph_build.argtypes = [i64, i64, vp, vp, vp, u32, i64, i64, ctypes.POINTER(vp)]
    L.ntp_graph_info.argtypes = [vp, vp, vp, vp, vp, vp]
    L.ntp_graph_export.argtypes = [vp, ctypes.c_int, vp, vp, vp]
    L.ntp_graph_export_perm.argtypes = [vp, vp]
    L.ntp_graph_stream_bytes.argtypes = [vp, ctypes.c_int, vp]
    L.ntp_graph_chunks.argtypes = [vp, ctypes.c_int, vp, vp, vp, vp, vp, vp]
    L.ntp_graph_device_bytes.argtypes = [vp, vp]
    L.ntp_aggregate_fwd.argtypes = [vp, vp, vp, i64, i64, i64, ctypes.c_int, vp]
    L.ntp_aggregate_bwd.argtypes = [vp, vp, vp, i64, i64, i64, ctypes.c_int, vp]
    L.ntp_aggregate_fwd_noalloc.argtypes = [vp, vp, vp, i64, i64, i64, ctypes.c_int, vp]
    L.ntp_chunked_aggregate.argtypes = [vp, ctypes.c_int, vp, vp, i64, i64, i64, ctypes.c_int, vp, vp]
    L.ntp_chunked_aggregate_multi.argtypes = [vp, ctypes.c_int, i32, vp, vp, i64, i64, i64, ctypes.c_int, vp, vp]
    L.ntp_aggregate_act.argtypes = [vp, ctypes.c_int, vp, vp, i64, i64, i64, ctypes.c_int, ctypes.c_int, vp, i64, vp, vp]
    L.ntp_edge_softmax.argtypes = [vp, vp, vp, ctypes.c_float, vp, vp, vp]
    L.ntp_edge_softmax_bwd.argtypes = [vp, vp, vp, ctypes.c_float, vp, vp, vp, vp, i64, i64, i64, vp, vp, ctypes.c_int, vp]
    L.ntp_attention_scores_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp]
    L.ntp_attention_scores_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, vp, i64, vp]
    L.ntp_attention_scores_bwd_scratch_bytes.argtypes = [i64, i64]
    L.ntp_attention_scores_bwd_scratch_bytes.restype = i64
    L.ntp_aggregate_weighted.argtypes = [vp, ctypes.c_int, vp, vp, vp, i64, i64, i64, ctypes.c_int, vp]
    L.ntp_nn_fwd.argtypes = [vp, vp, vp, i64, i64, i64, ctypes.c_int, ctypes.c_int, vp]
    L.ntp_nn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, ctypes.c_int, ctypes.c_int, vp, i64, vp]
    L.ntp_relu_fwd.argtypes = [vp, i64, i64, i64, ctypes.c_int, vp]
    L.ntp_relu_bwd.argtypes = [vp, vp, vp, i64, i64, i64, ctypes.c_int, vp]
    L.ntp_nn_bwd_workspace_bytes.argtypes = [i64, i64, i64]
    L.ntp_nn_bwd_workspace_bytes.restype = i64
    L.ntp_softmax_xent.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, vp]
    L.ntp_softmax_xent_scratch_bytes.argtypes = [i64]
    L.ntp_softmax_xent_scratch_bytes.restype = i64
    L.ntp_graph_free.argtypes = [vp]
    L.ntp_graph_free.restype = None
    L.ntp_last_error.restype = ctypes.c_char_p
    for name in EXPORTED_SYMBOLS:
        fn = getattr(L, name)
        if name not in ("ntp_graph_free", "ntp_last_error", "ntp_nn_bwd_workspace_bytes", "ntp_softmax_xent_scratch_bytes",
                        "ntp_attention_scores_bwd_scratch_bytes"):
            fn.restype = ctypes.c_int
    _lib = L
    return L


def ntp_last_error() -> str:
    return lib().ntp_last_error().decode()


def _check(rc: int):
    if rc != NTP_OK:
        raise NtpError(rc, ntp_last_error())


def _ptr(x):
    """Device or host address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return ctypes.c_void_p(x)
    if isinstance(x, np.ndarray):
        return ctypes.c_void_p(x.ctypes.data)
    return ctypes.c_void_p(x.data_ptr())          # torch tensor


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return ctypes.c_void_p(s)
    return ctypes.c_void_p(s.cuda_stream)          # torch.cuda.Stream


class Graph:
    """Owner of an ntp_graph_t*; frees it on close() or garbage collection."""

    def __init__(self, handle):
        self.handle = handle

    def close(self):
        if self.handle:
            lib().ntp_graph_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def ntp_graph_build(n_vertices, src, dst, edge_weight=None, flags=NTP_GCN_FLAGS,
                    device_budget_bytes=0, chunk_edges=0) -> Graph:
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    if src.shape != dst.shape or src.ndim != 1:
        raise ValueError("src and dst must be 1-D arrays of equal length")
    w = None if edge_weight is None else np.ascontiguousarray(edge_weight, dtype=np.float32)
    if w is not None and w.shape != src.shape:
        raise ValueError("edge_weight must match the edge list")
    out = ctypes.c_void_p()
    _check(lib().ntp_graph_build(int(n_vertices), int(src.size), _ptr(src), _ptr(dst), _ptr(w),
                                 int(flags), int(device_budget_bytes), int(chunk_edges), ctypes.byref(out)))
    return Graph(out)


def ntp_graph_info(g: Graph) -> dict:
    n, nnz, md = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    nc, sym = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().ntp_graph_info(g.handle, ctypes.byref(n), ctypes.byref(nnz), ctypes.byref(nc),
                                ctypes.byref(sym), ctypes.byref(md)))
    return dict(n_vertices=n.value, nnz=nnz.value, n_chunks=nc.value, is_symmetric=bool(sym.value),
                max_degree=md.value)


def ntp_graph_export(g: Graph, which=NTP_CSR):
    info = ntp_graph_info(g)
    n = info["n_vertices"]
    rowptr = np.empty(n + 1, dtype=np.int64)
    _check(lib().ntp_graph_export(g.handle, which, _ptr(rowptr), None, None))
    nnz = int(rowptr[-1])
    colidx = np.empty(nnz, dtype=np.int32)
    val = np.empty(nnz, dtype=np.float32)
    _check(lib().ntp_graph_export(g.handle, which, None, _ptr(colidx), _ptr(val)))
    return rowptr, colidx, val


def ntp_graph_stream_bytes(g: Graph, which=NTP_CSR) -> int:
    """host-to-device bytes of one chunked pass over the form (0 when every chunk is resident)"""
    b = ctypes.c_int64()
    _check(lib().ntp_graph_stream_bytes(g.handle, int(which), ctypes.byref(b)))
    return int(b.value)


def ntp_graph_export_perm(g: Graph) -> np.ndarray:
    """by-source entry -> by-destination entry of a graph built with NTP_EDGE_PERM"""
    perm = np.empty(ntp_graph_info(g)["nnz"], dtype=np.int32)
    _check(lib().ntp_graph_export_perm(g.handle, _ptr(perm)))
    return perm


def ntp_graph_chunks(g: Graph, which=NTP_CSR) -> dict:
    nc = ctypes.c_int32()
    _check(lib().ntp_graph_chunks(g.handle, which, ctypes.byref(nc), None, None, None, None, None))
    k = nc.value
    rb, re, eb, ee = (np.empty(k, dtype=np.int64) for _ in range(4))
    res = np.empty(k, dtype=np.int32)
    _check(lib().ntp_graph_chunks(g.handle, which, ctypes.byref(nc), _ptr(rb), _ptr(re), _ptr(eb), _ptr(ee), _ptr(res)))
    return dict(row_begin=rb, row_end=re, entry_begin=eb, entry_end=ee, resident=res)


def ntp_graph_device_bytes(g: Graph) -> int:
    b = ctypes.c_int64()
    _check(lib().ntp_graph_device_bytes(g.handle, ctypes.byref(b)))
    return b.value


def ntp_graph_free(g: Graph):
    g.close()


def ntp_aggregate_fwd(g: Graph, X, Y, f_slice, ldx, ldy, dtype=NTP_F32, stream=None):
    _check(lib().ntp_aggregate_fwd(g.handle, _ptr(X), _ptr(Y), int(f_slice), int(ldx), int(ldy), int(dtype), _stream(stream)))


NTP_NOALLOC_SCRATCH_BYTES = 8 << 20


def ntp_aggregate_fwd_noalloc(g: Graph, X, Y, f_slice, ldx, ldy, dtype=NTP_F32, stream=None):
    _check(lib().ntp_aggregate_fwd_noalloc(g.handle, _ptr(X), _ptr(Y), int(f_slice), int(ldx), int(ldy), int(dtype), _stream(stream)))


def ntp_aggregate_bwd(g: Graph, Gout, Gin, f_slice, ldg_out, ldg_in, dtype=NTP_F32, stream=None):
    _check(lib().ntp_aggregate_bwd(g.handle, _ptr(Gout), _ptr(Gin), int(f_slice), int(ldg_out), int(ldg_in), int(dtype), _stream(stream)))


def ntp_edge_softmax(g: Graph, p, q, negative_slope, alpha_in, alpha_out=None, stream=None):
    _check(lib().ntp_edge_softmax(g.handle, _ptr(p), _ptr(q), float(negative_slope), _ptr(alpha_in), _ptr(alpha_out),
                                  _stream(stream)))


def ntp_edge_softmax_bwd(g: Graph, p, q, negative_slope, alpha_in, alpha_out, Z, dY, m, ldz, lddy, dp, dq, accumulate=False,
                         stream=None):
    _check(lib().ntp_edge_softmax_bwd(g.handle, _ptr(p), _ptr(q), float(negative_slope), _ptr(alpha_in), _ptr(alpha_out),
                                      _ptr(Z), _ptr(dY), int(m), int(ldz), int(lddy), _ptr(dp), _ptr(dq), int(bool(accumulate)),
                                      _stream(stream)))


def ntp_attention_scores_fwd(Z, a_src, a_dst, p, q, n, m, ldz, stream=None):
    _check(lib().ntp_attention_scores_fwd(_ptr(Z), _ptr(a_src), _ptr(a_dst), _ptr(p), _ptr(q), int(n), int(m), int(ldz),
                                          _stream(stream)))


def ntp_attention_scores_bwd_scratch_bytes(n, m) -> int:
    return int(lib().ntp_attention_scores_bwd_scratch_bytes(int(n), int(m)))


def ntp_attention_scores_bwd(Z, a_src, a_dst, dp, dq, dZ, da_src, da_dst, n, m, ldz, lddz, scratch, scratch_bytes, stream=None):
    _check(lib().ntp_attention_scores_bwd(_ptr(Z), _ptr(a_src), _ptr(a_dst), _ptr(dp), _ptr(dq), _ptr(dZ), _ptr(da_src),
                                          _ptr(da_dst), int(n), int(m), int(ldz), int(lddz), _ptr(scratch), int(scratch_bytes),
                                          _stream(stream)))


def ntp_aggregate_weighted(g: Graph, direction, weights, X, Y, f_slice, ldx, ldy, dtype=NTP_F32, stream=None):
    _check(lib().ntp_aggregate_weighted(g.handle, int(direction), _ptr(weights), _ptr(X), _ptr(Y), int(f_slice),
                                        int(ldx), int(ldy), int(dtype), _stream(stream)))


def ntp_chunked_aggregate(g: Graph, direction, X, Y, f_slice, ldx, ldy, dtype=NTP_F32,
                          compute_stream=None, copy_stream=None):
    _check(lib().ntp_chunked_aggregate(g.handle, int(direction), _ptr(X), _ptr(Y), int(f_slice), int(ldx), int(ldy),
                                       int(dtype), _stream(compute_stream), _stream(copy_stream)))


def ntp_aggregate_act(g: Graph, direction, X, Y, f_slice, ldx, ldy, dtype=NTP_F32, act=NTP_ACT_RELU, M=None, ldm=0,
                      compute_stream=None, copy_stream=None):
    _check(lib().ntp_aggregate_act(g.handle, int(direction), _ptr(X), _ptr(Y), int(f_slice), int(ldx), int(ldy), int(dtype),
                                   int(act), _ptr(M), int(ldm), _stream(compute_stream), _stream(copy_stream)))


def ntp_chunked_aggregate_multi(g: Graph, direction, Xs, Ys, f_slice, ldx, ldy, dtype=NTP_F32,
                                compute_stream=None, copy_stream=None):
    if len(Xs) != len(Ys) or not Xs:
        raise ValueError("Xs and Ys must be non-empty lists of equal length")
    k = len(Xs)
    xa = (ctypes.c_void_p * k)(*[_ptr(x) for x in Xs])
    ya = (ctypes.c_void_p * k)(*[_ptr(y) for y in Ys])
    _check(lib().ntp_chunked_aggregate_multi(g.handle, int(direction), k, xa, ya, int(f_slice), int(ldx), int(ldy),
                                             int(dtype), _stream(compute_stream), _stream(copy_stream)))


def ntp_nn_fwd(A, W, H, n, k, m, act=NTP_ACT_NONE, dtype=NTP_F32, stream=None):
    _check(lib().ntp_nn_fwd(_ptr(A), _ptr(W), _ptr(H), int(n), int(k), int(m), int(act), int(dtype), _stream(stream)))


def ntp_nn_bwd_workspace_bytes(n, k, m) -> int:
    return int(lib().ntp_nn_bwd_workspace_bytes(int(n), int(k), int(m)))


def ntp_nn_bwd(A, W, H, dH, dA, dW, n, k, m, act=NTP_ACT_NONE, dtype=NTP_F32,
               workspace=None, workspace_bytes=0, stream=None):
    _check(lib().ntp_nn_bwd(_ptr(A), _ptr(W), _ptr(H), _ptr(dH), _ptr(dA), _ptr(dW), int(n), int(k), int(m),
                            int(act), int(dtype), _ptr(workspace), int(workspace_bytes), _stream(stream)))


def ntp_softmax_xent_scratch_bytes(n) -> int:
    return int(lib().ntp_softmax_xent_scratch_bytes(int(n)))


def ntp_softmax_xent(Z, labels, dZ, loss, scratch, scratch_bytes, n, c, ldz, lddz, stream=None):
    _check(lib().ntp_softmax_xent(_ptr(Z), _ptr(labels), _ptr(dZ), _ptr(loss), _ptr(scratch), int(scratch_bytes),
                                  int(n), int(c), int(ldz), int(lddz), _stream(stream)))


def ntp_relu_fwd(H, n, f, ld, dtype=NTP_F32, stream=None):
    _check(lib().ntp_relu_fwd(_ptr(H), int(n), int(f), int(ld), int(dtype), _stream(stream)))


def ntp_relu_bwd(dH, H, dZ, n, f, ld, dtype=NTP_F32, stream=None):
    _check(lib().ntp_relu_bwd(_ptr(dH), _ptr(H), _ptr(dZ), int(n), int(f), int(ld), int(dtype), _stream(stream)))

"""MI355X-native aggregation hot path of feature-dimension tensor-parallel full-graph
GNN training: a thin ctypes binding over libntp.so (hand-written HIP for gfx950).

The binding only marshals arguments; every step runs in the library's kernels.  There
is no CPU fallback: if the library is missing or cannot be loaded, importing the binding
functions raises.
"""
from .binding import (  # noqa: F401
    NtpError, Graph, lib, lib_path,
    ntp_graph_build, ntp_graph_info, ntp_graph_export, ntp_graph_export_perm, ntp_graph_chunks, ntp_graph_stream_bytes, ntp_graph_device_bytes,
    ntp_graph_free, ntp_aggregate_fwd, ntp_aggregate_fwd_noalloc, NTP_NOALLOC_SCRATCH_BYTES, ntp_aggregate_bwd, ntp_chunked_aggregate, ntp_chunked_aggregate_multi, ntp_aggregate_act, ntp_edge_softmax, ntp_edge_softmax_bwd, ntp_aggregate_weighted,
    ntp_attention_scores_fwd, ntp_attention_scores_bwd, ntp_attention_scores_bwd_scratch_bytes,
    ntp_nn_fwd, ntp_nn_bwd, ntp_nn_bwd_workspace_bytes, ntp_softmax_xent, ntp_softmax_xent_scratch_bytes, ntp_relu_fwd, ntp_relu_bwd, ntp_last_error,
    NTP_SYMMETRISE, NTP_DEDUP, NTP_ADD_SELF_LOOPS, NTP_NORM_GCN_SYM, NTP_HOST_ONLY, NTP_FORCE_STREAM, NTP_SCATTER_BWD, NTP_EDGE_PERM,
    NTP_GCN_FLAGS, NTP_DIRECTED_GCN_FLAGS, NTP_CSR, NTP_CSC, NTP_F32, NTP_BF16, NTP_FWD, NTP_BWD,
    NTP_ACT_NONE, NTP_ACT_RELU, NTP_OK, NTP_EINVAL, NTP_ENOMEM, NTP_EHIP, NTP_EBUDGET, NTP_EUNSUPPORTED,
    EXPORTED_SYMBOLS,
)

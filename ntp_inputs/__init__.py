"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU harness.

This package only draws random graphs, features, labels and weights.  It holds
none of the method's arithmetic: no normalisation, no CSR construction, no
aggregation.  Both the oracle side and the HIP side of a parity test call the
same generator with the same seed and then go their separate ways.
"""
from .generators import (  # noqa: F401
    stream_rng,
    erdos_renyi_edges,
    rmat_edges,
    zipf_configuration_edges,
    directed_random_edges,
    normal_features,
    bernoulli_features,
    uniform_labels,
    glorot_weight,
    to_bf16_bits,
    bf16_bits_to_f32,
)
from .configs import CONFIGS, make_graph, make_features, WorkloadSpec  # noqa: F401

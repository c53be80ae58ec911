"""CPU oracle for the aggregation hot path (TEST INFRASTRUCTURE).

A plain, slow, fp64 implementation of what the HIP library computes, written
from the paper's definitions: graph normalisation, forward and transposed
neighbour aggregation, chunked aggregation, the dense transform and a GCN
epoch.  Only tests, the smoke check and the benchmark's cpu_baseline leg may
import it; the product never does, and it imports nothing from the product.

Pins (tests/test_oracle_pins.py): dense brute force on tiny graphs, the
constant-vector closed form, the sqrt-degree fixed point, textbook graphs
(empty, complete, star, ring), the adjoint identity on directed graphs,
chunk/slice invariance, finite-difference gradients of the epoch loss, a
hand-derived fixture under tests/golden/, and for the attention weights: rows
summing to one, the slope-1 closed form, equal scores giving 1/degree, a dense
brute force, and the transposed order against scipy's transpose; the gradient
of the attention scores and the whole GAT epoch by finite differences and by
the reductions to a mean aggregation and to an MLP.  No function here is unpinned.
"""
from .graph import (  # noqa: F401
    Graph, Sparse, build_graph, plan_chunks, edge_permutation,
    SYMMETRISE, DEDUP, ADD_SELF_LOOPS, NORM_GCN_SYM, GCN_FLAGS, DIRECTED_GCN_FLAGS,
)
from .aggregate import (  # noqa: F401
    aggregate, aggregate_fwd, aggregate_bwd, aggregate_bwd_scatter,
    chunked_aggregate, round_bf16, num_threads, set_num_threads, build_native,
)
from .sampled import rows_from_undirected_edges  # noqa: F401
from .attention import edge_softmax, edge_softmax_bwd, edge_softmax_bwd_rows, leaky_relu, weighted  # noqa: F401
from .gat import attention_scores, attention_scores_bwd, epoch_gat_decoupled, resolve_gate  # noqa: F401
from .gcn import (  # noqa: F401
    nn_fwd, nn_bwd, softmax_cross_entropy, epoch_layerwise, epoch_decoupled, resolve_relu,
)

"""The five synthetic workloads (graph recipe + model shape).

Each one is a stand-in with the vertex count, edge count, degree structure and
feature widths of a workload class; none of them is a public dataset.  The
``scale_down`` argument divides the vertex and edge counts so the CPU oracle
can check a whole instance in seconds.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import generators as g


@dataclass
class WorkloadSpec:
    name: str
    n_vertices: int
    n_undirected: int            # distinct undirected edges drawn (each stored once)
    graph: str                   # "er" | "rmat" | "zipf"
    layers: tuple                # full layer widths, e.g. (128, 256, 256, 40)
    agg_slices: tuple            # aggregation widths timed on one worker's share
    n_workers: int = 1           # feature-dimension shares this GPU stands for one of
    exact_edges: bool = False
    feature_kind: str = "normal"
    bernoulli_p: float = 0.0
    device_budget_bytes: int = 0
    chunk_edges: int = 0
    dtypes: tuple = ("f32",)
    notes: str = ""
    extra: dict = field(default_factory=dict)


CONFIGS = {
    1: WorkloadSpec("cfg1-tiny-er", 2708, 5278, "er", (1433, 16, 7), (1433, 16), 1,
                    exact_edges=True, feature_kind="bernoulli", bernoulli_p=0.0127),
    2: WorkloadSpec("cfg2-rmat-169k", 169343, 1166243, "rmat", (128, 256, 256, 40), (128, 256), 1,
                    exact_edges=True),
    3: WorkloadSpec("cfg3-rmat-2.4m", 2449029, 61860000, "rmat", (100, 256, 256, 47), (32, 13), 8),
    4: WorkloadSpec("cfg4-zipf-233k", 232965, 57300000, "zipf", (602, 128, 41), (76, 16), 8,
                    dtypes=("f32", "bf16")),
    5: WorkloadSpec("cfg5-rmat-111m", 111059956, 1600000000, "rmat", (128, 128, 128, 172), (16,), 8,
                    device_budget_bytes=64 << 30, chunk_edges=256 << 20),
}


def make_graph(cfg: int, seed: int = 0, scale_down: int = 1, permute: bool = True):
    """Undirected edge list (each edge once) for config ``cfg``.

    permute = False keeps the generator's own vertex numbering (R-MAT: low ids
    are the hubs; Zipf: ids sorted by degree) instead of relabelling the vertices
    at random: the best case for locality, not what the configs ask for.

    Returns (n_vertices, src, dst).  With scale_down = k the vertex and edge
    counts are divided by k (same generator, same parameters); the dense
    Zipf graph divides its edge count by k^2 instead.
    """
    spec = CONFIGS[cfg]
    n = max(8, spec.n_vertices // scale_down)
    m = max(8, spec.n_undirected // scale_down)
    if spec.graph == "zipf":
        # the dense graph keeps its density (edges / vertices^2), not its average
        # degree, which would exceed the degree cap on a small vertex set
        m = max(8, spec.n_undirected // (scale_down * scale_down))
    if spec.graph == "er":
        src, dst = g.erdos_renyi_edges(n, m, seed)
    elif spec.graph == "rmat":
        # exact configs keep the first m distinct edges; the others keep every
        # distinct edge of the batches drawn (a little above m; callers print it)
        src, dst = g.rmat_edges(n, m, seed, exact=spec.exact_edges, permute=permute)
    elif spec.graph == "zipf":
        src, dst = g.zipf_configuration_edges(n, 2 * m, seed, s=1.1, cap=max(1, n // 8), permute=permute)
    else:
        raise ValueError(spec.graph)
    return n, src, dst


def make_features(cfg: int, width: int, seed: int = 0, scale_down: int = 1) -> np.ndarray:
    spec = CONFIGS[cfg]
    n = max(8, spec.n_vertices // scale_down)
    if spec.feature_kind == "bernoulli":
        return g.bernoulli_features(n, width, spec.bernoulli_p, seed)
    return g.normal_features(n, width, seed)

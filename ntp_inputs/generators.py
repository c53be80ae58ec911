"""Counter-based seeded generators for graphs, features, labels and weights.

Every generator takes ``(seed, stream)`` and builds a Philox generator keyed by
that pair, so any input can be regenerated independently, in any order, by the
oracle side and by the GPU side of a test.  All edge lists are returned as two
int32 arrays ``(src, dst)`` meaning a directed edge ``src -> dst``; undirected
generators return each edge ONCE (the graph build symmetrises it).
"""
from __future__ import annotations

import numpy as np

# stream ids: one per kind of input, so that changing the feature width does
# not change the graph drawn from the same seed.
STREAM_GRAPH = 1
STREAM_PERM = 2
STREAM_FEAT = 3
STREAM_LABEL = 4
STREAM_WEIGHT = 5
STREAM_GRAD = 6
STREAM_TOPUP = 7


def stream_rng(seed: int, stream: int, sub: int = 0) -> np.random.Generator:
    """Philox generator keyed by (seed, stream, sub)."""
    key = (int(seed) & 0xFFFFFFFF) | ((int(stream) & 0xFFFF) << 32) | ((int(sub) & 0xFFFF) << 48)
    return np.random.Generator(np.random.Philox(key=key))


def _first_unique(keys: np.ndarray, m: int | None) -> np.ndarray:
    """Unique keys in order of first appearance, truncated to the first m."""
    _, first = np.unique(keys, return_index=True)
    first.sort()
    if m is not None:
        first = first[:m]
    return keys[first]


def _permute_ids(n: int, src: np.ndarray, dst: np.ndarray, seed: int):
    perm = stream_rng(seed, STREAM_PERM).permutation(n).astype(np.int32)
    return perm[src], perm[dst]


def erdos_renyi_edges(n: int, m: int, seed: int = 0):
    """G(n, m): exactly m distinct undirected edges without loops, each once."""
    if m > n * (n - 1) // 2:
        raise ValueError("more edges than vertex pairs")
    rng = stream_rng(seed, STREAM_GRAPH)
    keys = np.empty(0, dtype=np.int64)
    while keys.size < m:
        k = max(1024, int((m - keys.size) * 1.2) + 16)
        a = rng.integers(0, n, size=k, dtype=np.int64)
        b = rng.integers(0, n, size=k, dtype=np.int64)
        ok = a != b
        lo = np.minimum(a[ok], b[ok])
        hi = np.maximum(a[ok], b[ok])
        keys = _first_unique(np.concatenate([keys, lo * n + hi]), m)
    return (keys // n).astype(np.int32), (keys % n).astype(np.int32)


def _rmat_batch(seed: int, batch_id: int, k: int, n: int, scale: int, a: float, b: float, c: float):
    """k R-MAT draws from the sub-stream of batch ``batch_id``; returns the
    canonical keys lo * n + hi of the accepted ones, in draw order."""
    rng = stream_rng(seed, STREAM_GRAPH, batch_id)
    u = np.zeros(k, dtype=np.int64)
    v = np.zeros(k, dtype=np.int64)
    ab = a + b
    abc = a + b + c
    for _ in range(scale):
        r = rng.random(k, dtype=np.float32)
        ubit = r >= ab                      # quadrants c, d: lower half of rows
        vbit = ((r >= a) & (r < ab)) | (r >= abc)  # quadrants b, d: right half
        u = (u << 1) | ubit
        v = (v << 1) | vbit
    ok = (u < n) & (v < n) & (u != v)
    u, v = u[ok], v[ok]
    return np.minimum(u, v) * n + np.maximum(u, v)


_RMAT_BATCH = 1 << 22


def _rmat_draw(seed: int, first_batch: int, n_batches: int, n: int, scale: int, abc, bsz: int):
    """Batches first_batch .. first_batch + n_batches - 1, each from its own
    sub-stream, so the result does not depend on how many threads ran them."""
    from concurrent.futures import ThreadPoolExecutor
    import os
    ids = range(first_batch, first_batch + n_batches)
    if n_batches == 1:
        return [_rmat_batch(seed, first_batch, bsz, n, scale, *abc)]
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        return list(ex.map(lambda b: _rmat_batch(seed, b, bsz, n, scale, *abc), ids))


def _bucket_unique(parts, n: int, n_buckets: int = 256):
    """Distinct keys of the concatenation of `parts` (int64 keys lo * n + hi), found
    bucket by bucket: keys are first grouped by an 8-bit multiplicative hash (a counting
    sort on one byte), then each bucket is made unique on its own thread.  Same set as
    np.unique of the concatenation, without one global sort; the order is by bucket, then
    ascending, and does not depend on the number of threads."""
    from concurrent.futures import ThreadPoolExecutor
    import os
    if not parts:
        return np.empty(0, dtype=np.int64)
    total = sum(p.size for p in parts)
    if total < (1 << 22):
        return np.unique(np.concatenate(parts))
    mult = np.uint64(0x9E3779B97F4A7C15)

    def split(p):
        b = ((p.view(np.uint64) * mult) >> np.uint64(56)).astype(np.uint8)
        order = np.argsort(b, kind="stable")        # radix sort on one byte
        counts = np.bincount(b, minlength=n_buckets)
        return p[order], counts

    workers = min(16, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=workers) as ex:
        grouped = list(ex.map(split, parts))

        def uniq(k):
            segs = []
            for p, counts in grouped:
                off = int(counts[:k].sum())
                segs.append(p[off:off + int(counts[k])])
            return np.unique(np.concatenate(segs)) if segs else np.empty(0, np.int64)

        out = list(ex.map(uniq, range(n_buckets)))
    return np.concatenate(out)


def rmat_edges(n: int, m: int, seed: int = 0, abcd=(0.57, 0.19, 0.19, 0.05),
               exact: bool = True, permute: bool = True):
    """R-MAT undirected edges on n vertices.

    Recursion depth ceil(log2 n); an edge with an endpoint >= n or with equal
    endpoints is rejected; (u, v) and (v, u) are the same edge.  Draws come in
    batches of min(2^22, max(2^12, 2^ceil(log2 m))), batch b from sub-stream b.
    Batches are added until at least m distinct edges exist.  With ``exact`` the
    first m distinct edges in draw order are kept; otherwise all distinct edges
    of the batches drawn are kept (a little more than m), in hash-bucket order.
    Vertex ids are then relabelled by a seeded random permutation unless
    ``permute`` is False.
    """
    a, b, c, _ = abcd
    scale = max(1, int(np.ceil(np.log2(n))))
    drawn = []            # per-batch keys in draw order
    n_unique = 0
    keys = None
    next_batch = 0
    bsz = min(_RMAT_BATCH, max(1 << 12, 1 << int(np.ceil(np.log2(max(2, m))))))
    while n_unique < m:
        deficit = m - n_unique
        # first round: as many draws as edges wanted; later rounds oversample the deficit
        nb = max(1, int(np.ceil(deficit * (1.0 if next_batch == 0 else 1.2) / bsz)))
        drawn.extend(_rmat_draw(seed, next_batch, nb, n, scale, (a, b, c), bsz))
        next_batch += nb
        keys = _bucket_unique(drawn, n)
        n_unique = keys.size
    if exact:
        keys = _first_unique(np.concatenate(drawn), m)
    del drawn
    src = (keys // n).astype(np.int32)
    dst = (keys % n).astype(np.int32)
    del keys
    if permute:
        src, dst = _permute_ids(n, src, dst, seed)
    return src, dst


def zipf_degree_sequence(n: int, total_degree: int, s: float = 1.1, cap: int | None = None):
    """d_r = clamp(round(C * r^-s), 1, cap), C found by bisection so that the
    sum is as close to total_degree as the rounding allows."""
    cap = cap if cap is not None else max(1, n // 8)
    r = np.arange(1, n + 1, dtype=np.float64) ** (-s)
    lo, hi = 0.0, float(total_degree) * 4.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        d = np.clip(np.rint(mid * r), 1, cap)
        if d.sum() < total_degree:
            lo = mid
        else:
            hi = mid
    return np.clip(np.rint(hi * r), 1, cap).astype(np.int64)


def zipf_configuration_edges(n: int, total_degree: int, seed: int = 0, s: float = 1.1,
                             cap: int | None = None, topup_frac: float = 0.98,
                             permute: bool = True):
    """Erased configuration model on a capped Zipf degree sequence.

    Stubs are shuffled and paired; loops and repeated pairs are erased.  While
    the number of distinct undirected edges is below topup_frac * total/2,
    further pairs are drawn with probability proportional to the degree
    sequence and merged in.  Returns each undirected edge once.
    """
    deg = zipf_degree_sequence(n, total_degree, s, cap)
    if deg.sum() % 2:
        deg[-1] += 1
    rng = stream_rng(seed, STREAM_GRAPH)
    stubs = np.repeat(np.arange(n, dtype=np.int32), deg)
    rng.shuffle(stubs)
    a = stubs[0::2].astype(np.int64)
    b = stubs[1::2].astype(np.int64)
    del stubs
    ok = a != b
    keys = np.unique(np.minimum(a[ok], b[ok]) * n + np.maximum(a[ok], b[ok]))
    del a, b, ok
    want = int(topup_frac * (total_degree // 2))
    trng = stream_rng(seed, STREAM_TOPUP)
    cdf = np.cumsum(deg, dtype=np.float64)
    cdf /= cdf[-1]
    rounds = 0
    while keys.size < want and rounds < 64:
        k = int((want - keys.size) * 1.5) + 1024
        a = np.searchsorted(cdf, trng.random(k), side="right").astype(np.int64)
        b = np.searchsorted(cdf, trng.random(k), side="right").astype(np.int64)
        a = np.minimum(a, n - 1)
        b = np.minimum(b, n - 1)
        ok = a != b
        new = np.minimum(a[ok], b[ok]) * n + np.maximum(a[ok], b[ok])
        keys = np.unique(np.concatenate([keys, new]))
        rounds += 1
    src = (keys // n).astype(np.int32)
    dst = (keys % n).astype(np.int32)
    if permute:
        src, dst = _permute_ids(n, src, dst, seed)
    return src, dst


def directed_random_edges(n: int, m: int, seed: int = 0, hub: int | None = None,
                          hub_in: int = 0, hub_out: int = 0):
    """m random DIRECTED edges (duplicates and loops possible, on purpose: the
    graph build has to remove them), plus optionally a hub vertex with hub_in
    extra in-edges and hub_out extra out-edges.  For transposed-path tests."""
    rng = stream_rng(seed, STREAM_GRAPH)
    src = rng.integers(0, n, size=m, dtype=np.int64)
    dst = rng.integers(0, n, size=m, dtype=np.int64)
    if hub is not None:
        hs = rng.integers(0, n, size=hub_in, dtype=np.int64)
        hd = rng.integers(0, n, size=hub_out, dtype=np.int64)
        src = np.concatenate([src, hs, np.full(hub_out, hub, dtype=np.int64)])
        dst = np.concatenate([dst, np.full(hub_in, hub, dtype=np.int64), hd])
    return src.astype(np.int32), dst.astype(np.int32)


def normal_features(n: int, f: int, seed: int = 0, stream: int = STREAM_FEAT) -> np.ndarray:
    """[n, f] float32 standard normal, row-major."""
    return stream_rng(seed, stream).standard_normal((n, f), dtype=np.float32)


def bernoulli_features(n: int, f: int, p: float, seed: int = 0) -> np.ndarray:
    """[n, f] float32 in {0, 1} with P(1) = p."""
    return (stream_rng(seed, STREAM_FEAT).random((n, f), dtype=np.float32) < p).astype(np.float32)


def uniform_labels(n: int, n_classes: int, seed: int = 0) -> np.ndarray:
    return stream_rng(seed, STREAM_LABEL).integers(0, n_classes, size=n, dtype=np.int32)


def glorot_weight(fan_in: int, fan_out: int, seed: int = 0, layer: int = 0) -> np.ndarray:
    """[fan_in, fan_out] float32 uniform(-a, a), a = sqrt(6 / (fan_in + fan_out))."""
    a = np.sqrt(6.0 / (fan_in + fan_out))
    w = stream_rng(seed, STREAM_WEIGHT, layer).random((fan_in, fan_out), dtype=np.float64)
    return ((2.0 * w - 1.0) * a).astype(np.float32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even.
    A storage-format conversion for preparing inputs; NaN is kept quiet."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    out = rounded.astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> the float32 values they denote."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)

"""Host-side tests of the C boundary (no GPU): exported symbols, bit-exact graph
construction against the oracle, chunk planning, argument checking."""
import os
import re

import numpy as np
import pytest

import oracle
import ntp_inputs as gen
import paper_2412_20379_amd as ntp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST = ntp.NTP_HOST_ONLY


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "ntp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(ntp_[a-z_]+)\s*\(", text)))
    assert declared, "no declarations found"
    L = ntp.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert sorted(ntp.EXPORTED_SYMBOLS) == declared


def _assert_same(g, og):
    for which, m in ((ntp.NTP_CSR, og.csr), (ntp.NTP_CSC, og.csc)):
        rowptr, colidx, val = ntp.ntp_graph_export(g, which)
        np.testing.assert_array_equal(rowptr, m.rowptr)
        np.testing.assert_array_equal(colidx, m.colidx)
        np.testing.assert_array_equal(val.view(np.uint32), m.val.view(np.uint32))
    info = ntp.ntp_graph_info(g)
    assert info["nnz"] == og.nnz and info["n_vertices"] == og.n
    assert info["is_symmetric"] == og.is_symmetric
    assert info["max_degree"] == int(og.d_in.max()) if og.n else True


@pytest.mark.parametrize("cfg", [1, 2])
def test_graph_build_bit_exact_configs(cfg):
    n, src, dst = gen.make_graph(cfg, seed=0)
    g = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_GCN_FLAGS | HOST)
    og = oracle.build_graph(n, src, dst)
    _assert_same(g, og)
    spec = gen.CONFIGS[cfg]
    assert og.nnz == 2 * spec.n_undirected + n


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_graph_build_bit_exact_directed(seed):
    n = 3000
    src, dst = gen.directed_random_edges(n, 40000, seed, hub=5, hub_in=2500, hub_out=700)
    g = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS | HOST)
    og = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    assert not og.is_symmetric
    _assert_same(g, og)


@pytest.mark.parametrize("flags", [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15])
@pytest.mark.parametrize("weighted", [False, True])
def test_graph_build_every_flag_combination(flags, weighted):
    n = 200
    src, dst = gen.directed_random_edges(n, 1500, seed=flags, hub=0, hub_in=100, hub_out=50)
    # make sure loops and repeated pairs are present
    src = np.concatenate([src, src[:50], np.arange(20, dtype=np.int32)])
    dst = np.concatenate([dst, dst[:50], np.arange(20, dtype=np.int32)])
    w = gen.stream_rng(flags, 9).random(src.size).astype(np.float32) + 0.5 if weighted else None
    g = ntp.ntp_graph_build(n, src, dst, w, flags=flags | HOST)
    og = oracle.build_graph(n, src, dst, flags, w)
    _assert_same(g, og)


@pytest.mark.parametrize("flags", [0, 2, 4, 8, 14])
@pytest.mark.parametrize("weighted", [False, True])
def test_graph_build_without_by_source_form(flags, weighted):
    """NTP_SCATTER_BWD: the by-destination form is unchanged (its weights still use the
    out-degrees), the by-source form is refused"""
    n = 300
    src, dst = gen.directed_random_edges(n, 2500, seed=40 + flags, hub=3, hub_in=150, hub_out=80)
    w = gen.stream_rng(flags, 11).random(src.size).astype(np.float32) + 0.5 if weighted else None
    g = ntp.ntp_graph_build(n, src, dst, w, flags=flags | HOST | ntp.NTP_SCATTER_BWD)
    og = oracle.build_graph(n, src, dst, flags, w)
    rowptr, colidx, val = ntp.ntp_graph_export(g, ntp.NTP_CSR)
    assert np.array_equal(rowptr, og.csr.rowptr) and np.array_equal(colidx, og.csr.colidx)
    assert np.array_equal(val.view(np.uint32), og.csr.val.view(np.uint32))
    assert not ntp.ntp_graph_info(g)["is_symmetric"]
    with pytest.raises(ntp.NtpError) as e:
        ntp.ntp_graph_export(g, ntp.NTP_CSC)
    assert e.value.code == ntp.NTP_EUNSUPPORTED
    with pytest.raises(ntp.NtpError):
        ntp.ntp_graph_chunks(g, ntp.NTP_CSC)
    # with SYMMETRISE and unit weights the flag changes nothing
    gs = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_GCN_FLAGS | HOST | ntp.NTP_SCATTER_BWD)
    assert ntp.ntp_graph_info(gs)["is_symmetric"]
    _assert_same(gs, oracle.build_graph(n, src, dst, oracle.GCN_FLAGS))


@pytest.mark.parametrize("flags", [0, 1, 2, 3, 4, 6, 7, 14, 15])
@pytest.mark.parametrize("weighted", [False, True])
def test_edge_permutation_bit_exact(flags, weighted):
    """NTP_EDGE_PERM: by-source entry -> by-destination entry, equal to the oracle's; both forms
    unchanged by the flag; the permuted by-destination entries are the by-source entries"""
    n = 250
    src, dst = gen.directed_random_edges(n, 2000, seed=70 + flags, hub=2, hub_in=120, hub_out=60)
    src = np.concatenate([src, src[:40], np.arange(15, dtype=np.int32)])      # repeated pairs and loops
    dst = np.concatenate([dst, dst[:40], np.arange(15, dtype=np.int32)])
    w = gen.stream_rng(flags, 13).random(src.size).astype(np.float32) + 0.5 if weighted else None
    g = ntp.ntp_graph_build(n, src, dst, w, flags=flags | HOST | ntp.NTP_EDGE_PERM)
    og = oracle.build_graph(n, src, dst, flags, w)
    _assert_same(g, og)
    perm = ntp.ntp_graph_export_perm(g)
    want = oracle.edge_permutation(og)
    # parallel copies of one edge (no DEDUP) may be matched in any order: compare what is unique
    rows = np.repeat(np.arange(n), np.diff(og.csr.rowptr))
    assert np.array_equal(np.sort(perm), np.arange(og.csr.nnz))
    assert np.array_equal(rows[perm], og.csc.colidx) and np.array_equal(og.csr.colidx[perm], np.repeat(np.arange(n), np.diff(og.csc.rowptr)))
    if flags & 2:
        assert np.array_equal(perm, want)


def test_edge_permutation_pins_of_the_oracle():
    """the oracle's permutation against scipy's transpose of an entry-numbered matrix, and on a
    three-vertex example written out by hand"""
    import scipy.sparse as sp
    n = 300
    src, dst = gen.directed_random_edges(n, 3000, 21, hub=5, hub_in=200, hub_out=90)
    og = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    ids = sp.csr_matrix((np.arange(1, og.csr.nnz + 1, dtype=np.float64), og.csr.colidx, og.csr.rowptr), shape=(n, n))
    t = ids.transpose().tocsr()
    t.sort_indices()
    assert np.array_equal(oracle.edge_permutation(og), t.data.astype(np.int64) - 1)
    # edges 0 -> 1, 0 -> 2, 2 -> 1, no self loops.  By destination: row 1 = [0, 2], row 2 = [0], i.e.
    # entries (0->1), (2->1), (0->2) at positions 0, 1, 2.  By source: row 0 = [1, 2], row 2 = [1], i.e.
    # (0->1), (0->2), (2->1): positions 0, 2, 1 of the by-destination form.
    g3 = oracle.build_graph(3, np.array([0, 0, 2], np.int32), np.array([1, 2, 1], np.int32), oracle.DEDUP)
    assert g3.csr.colidx.tolist() == [0, 2, 0] and g3.csc.colidx.tolist() == [1, 2, 1]
    assert oracle.edge_permutation(g3).tolist() == [0, 2, 1]


def test_edge_permutation_errors():
    n = 50
    src, dst = gen.directed_random_edges(n, 200, 1)
    with pytest.raises(ntp.NtpError) as e:
        ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS | HOST | ntp.NTP_EDGE_PERM | ntp.NTP_SCATTER_BWD)
    assert e.value.code == ntp.NTP_EINVAL
    g = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS | HOST)
    with pytest.raises(ntp.NtpError) as e:
        ntp.ntp_graph_export_perm(g)
    assert e.value.code == ntp.NTP_EUNSUPPORTED
    g0 = ntp.ntp_graph_build(0, [], [], flags=ntp.NTP_GCN_FLAGS | HOST | ntp.NTP_EDGE_PERM)
    assert ntp.ntp_graph_export_perm(g0).size == 0


def test_symmetric_input_without_symmetrise_flag_is_detected():
    n = 500
    s, d = gen.erdos_renyi_edges(n, 2000, 3)
    src, dst = np.concatenate([s, d]), np.concatenate([d, s])
    g = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS | HOST)
    assert ntp.ntp_graph_info(g)["is_symmetric"]
    _assert_same(g, oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS))


def test_empty_and_edgeless_graphs():
    g = ntp.ntp_graph_build(0, [], [], flags=ntp.NTP_GCN_FLAGS | HOST)
    assert ntp.ntp_graph_info(g)["nnz"] == 0
    g = ntp.ntp_graph_build(5, [], [], flags=ntp.NTP_GCN_FLAGS | HOST)
    rowptr, colidx, val = ntp.ntp_graph_export(g)
    assert rowptr.tolist() == [0, 1, 2, 3, 4, 5] and colidx.tolist() == [0, 1, 2, 3, 4]
    assert np.all(val == 1.0)


@pytest.mark.parametrize("chunk_edges", [1, 3, 17, 100, 1009, 50000, 10 ** 9])
def test_chunk_plan_matches_greedy_rule(chunk_edges):
    n = 2000
    src, dst = gen.directed_random_edges(n, 20000, 4, hub=9, hub_in=1500, hub_out=10)
    g = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_DIRECTED_GCN_FLAGS | HOST, chunk_edges=chunk_edges)
    og = oracle.build_graph(n, src, dst, oracle.DIRECTED_GCN_FLAGS)
    for which, m in ((ntp.NTP_CSR, og.csr), (ntp.NTP_CSC, og.csc)):
        ch = ntp.ntp_graph_chunks(g, which)
        # entries are covered once, in order
        assert ch["entry_begin"][0] == 0 and ch["entry_end"][-1] == m.nnz
        np.testing.assert_array_equal(ch["entry_begin"][1:], ch["entry_end"][:-1])
        assert np.all(ch["entry_end"] - ch["entry_begin"] <= max(chunk_edges, 1))
        # whole-row chunks follow the greedy rule; a row above the limit is cut by entry range
        want = oracle.plan_chunks(m.rowptr, chunk_edges)
        rows = sorted(set(zip(ch["row_begin"].tolist(), ch["row_end"].tolist())))
        assert rows == want
        for (r0, r1) in want:
            sel = (ch["row_begin"] == r0) & (ch["row_end"] == r1)
            assert ch["entry_begin"][sel].min() == m.rowptr[r0] and ch["entry_end"][sel].max() == m.rowptr[r1]
            if sel.sum() > 1:
                assert r1 == r0 + 1 and m.rowptr[r1] - m.rowptr[r0] > chunk_edges


def test_argument_errors():
    L = ntp.lib()
    with pytest.raises(ntp.NtpError) as e:
        ntp.ntp_graph_build(3, [0, 5], [1, 2], flags=HOST)
    assert e.value.code == ntp.NTP_EINVAL and "outside" in str(e.value)
    with pytest.raises(ntp.NtpError) as e:
        ntp.ntp_graph_build(3, [0], [1], flags=HOST | 1024)
    assert e.value.code == ntp.NTP_EINVAL
    with pytest.raises(ntp.NtpError) as e:
        ntp.ntp_graph_build(-1, [], [], flags=HOST)
    assert e.value.code == ntp.NTP_EINVAL
    g = ntp.ntp_graph_build(3, [0], [1], flags=ntp.NTP_GCN_FLAGS | HOST)
    x = np.zeros((3, 4), np.float32)
    y = np.zeros((3, 4), np.float32)
    with pytest.raises(ntp.NtpError) as e:      # host-only graph: nothing on the device
        ntp.ntp_aggregate_fwd(g, x, y, 4, 4, 4)
    assert e.value.code == ntp.NTP_EBUDGET
    assert L.ntp_graph_info(None, None, None, None, None, None) == ntp.NTP_EINVAL
    assert "NULL" in ntp.ntp_last_error()
    assert L.ntp_graph_export(g.handle, 7, None, None, None) == ntp.NTP_EINVAL
    # transform argument checks happen before any device work
    with pytest.raises(ntp.NtpError):
        ntp.ntp_nn_fwd(x, x, y, 3, 0, 4)
    with pytest.raises(ntp.NtpError):
        ntp.ntp_nn_fwd(x, x, y, 3, 4, 4, act=9)
    with pytest.raises(ntp.NtpError):
        ntp.ntp_nn_bwd(x, x, y, y, None, None, 3, 4, 4)
    assert ntp.ntp_nn_bwd_workspace_bytes(100000, 256, 256) > 0
    L.ntp_graph_free(None)                       # NULL is allowed


def test_overlapping_strided_views_are_refused():
    """Input and output of an aggregation call must not share a byte, also when both are column
    windows of one wider matrix (a worker's slices of a full-width buffer).  The check runs before
    anything touches the device, so a host-only handle shows it: overlapping windows give
    NTP_EINVAL, disjoint ones pass the check and end at the host-only handle's NTP_EBUDGET."""
    n = 1000
    g = ntp.ntp_graph_build(n, [0, 1], [1, 2], flags=ntp.NTP_GCN_FLAGS | HOST)
    base = 1 << 30                     # addresses only: nothing is dereferenced on a host-only handle

    def code(x, y, f, ldx, ldy, dtype=ntp.NTP_F32):
        with pytest.raises(ntp.NtpError) as e:
            ntp.ntp_aggregate_fwd(g, x, y, f, ldx, ldy, dtype)
        return e.value.code

    ld = 256
    # Y = X + 16 columns inside rows of 256: the 32-column windows share 16 columns of every row
    assert code(base, base + 16 * 4, 32, ld, ld) == ntp.NTP_EINVAL
    assert code(base + 16 * 4, base, 32, ld, ld) == ntp.NTP_EINVAL
    # neighbouring windows of the same rows do not overlap
    assert code(base, base + 32 * 4, 32, ld, ld) == ntp.NTP_EBUDGET
    assert code(base + 32 * 4, base, 32, ld, ld) == ntp.NTP_EBUDGET
    # the last window of a row against the first window: disjoint although the address distance wraps
    assert code(base, base + 224 * 4, 32, ld, ld) == ntp.NTP_EBUDGET
    assert code(base, base + 225 * 4, 32, ld, ld) == ntp.NTP_EINVAL        # 225 + 32 > 256: runs into the next row's first window
    # a window that starts some rows further down still overlaps if its columns do
    assert code(base, base + (5 * ld + 8) * 4, 32, ld, ld) == ntp.NTP_EINVAL
    assert code(base, base + (5 * ld + 40) * 4, 32, ld, ld) == ntp.NTP_EBUDGET
    # compact matrices: equal, shifted by half a matrix, back to back
    assert code(base, base, 32, 32, 32) == ntp.NTP_EINVAL
    assert code(base, base + n * 16 * 4, 32, 32, 32) == ntp.NTP_EINVAL
    assert code(base, base + n * 32 * 4, 32, 32, 32) == ntp.NTP_EBUDGET
    # bf16 elements are two bytes wide
    assert code(base, base + 32 * 2, 32, ld, ld, ntp.NTP_BF16) == ntp.NTP_EBUDGET
    assert code(base, base + 31 * 2, 32, ld, ld, ntp.NTP_BF16) == ntp.NTP_EINVAL
    # different strides inside one span cannot be told apart cheaply: refused
    assert code(base, base + 64, 32, 256, 128) == ntp.NTP_EINVAL
    assert code(base, base + n * 256 * 4, 32, 256, 128) == ntp.NTP_EBUDGET
    # row strides of 2^30 elements or more are refused (row addresses are id x stride-in-bytes in 32 x 32 -> 64 bits)
    assert code(base, base + (1 << 40), 32, 1 << 30, 32) == ntp.NTP_EINVAL
    assert code(base, base + (1 << 40), 32, 32, 1 << 30) == ntp.NTP_EINVAL
    # several right-hand sides: every output against every input and every other output
    L = ntp.lib()
    import ctypes

    def multi(xs, ys):
        xa = (ctypes.c_void_p * len(xs))(*xs)
        ya = (ctypes.c_void_p * len(ys))(*ys)
        return L.ntp_chunked_aggregate_multi(g.handle, ntp.NTP_FWD, len(xs), xa, ya, 32, ld, ld, ntp.NTP_F32, None, None)

    far = base + n * ld * 4
    assert multi([base, base + 128], [far, far + 128]) == ntp.NTP_EBUDGET
    assert multi([base, base + 512], [far, base + 64]) == ntp.NTP_EINVAL and "overlaps an input" in ntp.ntp_last_error()
    assert multi([base, base + 128], [far, far + 64]) == ntp.NTP_EINVAL and "two outputs" in ntp.ntp_last_error()
    g.close()


def test_inputs_are_reproducible():
    a = gen.make_graph(2, seed=0, scale_down=16)
    b = gen.make_graph(2, seed=0, scale_down=16)
    c = gen.make_graph(2, seed=1, scale_down=16)
    np.testing.assert_array_equal(a[1], b[1])
    np.testing.assert_array_equal(a[2], b[2])
    assert not np.array_equal(a[1], c[1])
    n, s, d = gen.make_graph(4, seed=0, scale_down=8)
    deg = np.bincount(np.concatenate([s, d]), minlength=n)
    assert deg.max() > 5 * deg.mean() and deg.min() >= 1             # heavy head, no isolated vertex
    n, s, d = gen.make_graph(3, seed=0, scale_down=64)
    deg = np.bincount(np.concatenate([s, d]), minlength=n)
    assert deg.max() > 50 * deg.mean()                              # power-law hubs


def test_bench_refuses_more_than_one_gpu():
    """the benchmark is a one-GPU program: asking for more ends with a message, not a run"""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)

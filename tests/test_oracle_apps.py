"""Pins for the oracle's application definitions (CPU only): closed forms,
library routines that compute the same thing by other means (numpy fancy
indexing / bincount / fsum, scipy's graph search), special cases, and
invariants of the result."""
import math

import numpy as np
import pytest
import scipy.sparse as sp
from scipy.sparse.csgraph import shortest_path

import oracle
from paper_2411_05309_amd import inputs


# ---------------------------------------------------------------- gather

def test_gather_closed_form_and_library():
    n = 1000
    host = np.arange(n, dtype=np.uint32) * 3 + 1
    idx = np.array([0, 999, 5, 5, 17, 0], np.uint32)
    out, s = oracle.gather(host, idx)
    assert out.tolist() == [1, 2998, 16, 16, 52, 1]
    assert s == 1 + 2998 + 16 + 16 + 52 + 1
    rng = np.random.default_rng(0)
    host = rng.integers(0, 1 << 32, 5000, dtype=np.uint64).astype(np.uint32)
    idx = rng.integers(0, 5000, 20000).astype(np.uint32)
    out, s = oracle.gather(host, idx)
    assert np.array_equal(out, host[idx])
    assert s == sum(int(v) for v in host[idx])


def test_gather_sum_needs_64_bits_and_empty():
    host = np.full(4, 0xFFFFFFFF, np.uint32)
    out, s = oracle.gather(host, np.zeros(10, np.uint32))
    assert s == 10 * 0xFFFFFFFF                       # > 2^32
    out, s = oracle.gather(host, np.zeros(0, np.uint32))
    assert out.size == 0 and s == 0


# ---------------------------------------------------------------- stream

def test_stream_reduce_closed_forms():
    # x[i] = i / 2^10, i < 2^12: exact in fp32; block sums are arithmetic series
    n, blk = 4096, 1000
    x = (np.arange(n) / 1024.0).astype(np.float32)
    s = oracle.stream_reduce(x, blk, 3)
    assert s.shape == (3, 5)
    for b in range(5):
        lo, hi = b * blk, min(n, (b + 1) * blk)
        assert s[0, b] == (hi * (hi - 1) // 2 - lo * (lo - 1) // 2) / 1024.0
    assert np.array_equal(s[0], s[1]) and np.array_equal(s[0], s[2])


def test_stream_reduce_against_exact_summation():
    x = inputs.f32_uniform(7, 0, 10000)
    assert x.min() >= -1.0 and x.max() < 1.0
    s = oracle.stream_reduce(x, 1024, 1)[0]
    a = oracle.stream_abs(x, 1024)
    for b in range(10):
        blk = x[b * 1024:(b + 1) * 1024].astype(np.float64)
        assert abs(s[b] - math.fsum(blk)) <= 1e-12 * math.fsum(np.abs(blk))
        assert abs(a[b] - math.fsum(np.abs(blk))) <= 1e-12 * a[b]
    # sign symmetry: a dropped or doubled element would break one of these
    assert np.allclose(oracle.stream_reduce(-x, 1024, 1)[0], -s, rtol=0, atol=0)


# ---------------------------------------------------------------- BFS

def _csr(nv, edges):
    src = np.array([e[0] for e in edges], np.int64)
    dst = np.array([e[1] for e in edges], np.int64)
    order = np.argsort(src, kind="stable")
    row_ptr = np.zeros(nv + 1, np.int64)
    np.cumsum(np.bincount(src, minlength=nv), out=row_ptr[1:])
    return row_ptr, dst[order].astype(np.int32)


def test_bfs_special_graphs():
    n = 50
    rp, ci = _csr(n, [(i, i + 1) for i in range(n - 1)])           # directed path
    assert oracle.bfs(rp, ci, 0).tolist() == list(range(n))
    assert oracle.bfs(rp, ci, 10).tolist() == [-1] * 10 + list(range(n - 10))
    rp, ci = _csr(n, [(0, i) for i in range(1, n)])                 # star
    assert oracle.bfs(rp, ci, 0).tolist() == [0] + [1] * (n - 1)
    assert oracle.bfs(rp, ci, 3).tolist() == [-1] * 3 + [0] + [-1] * (n - 4)
    rp, ci = _csr(63, [(v, 2 * v + 1) for v in range(31)] + [(v, 2 * v + 2) for v in range(31)])
    assert oracle.bfs(rp, ci, 0).tolist() == [int(math.log2(v + 1)) for v in range(63)]
    rp, ci = _csr(4, [(0, 0), (0, 1), (0, 1), (1, 0), (2, 3)])      # loops, duplicates
    assert oracle.bfs(rp, ci, 0).tolist() == [0, 1, -1, -1]


def test_bfs_against_scipy_on_rmat():
    scale = 10
    rp, ci = inputs.rmat_csr(3, scale, edge_factor=8)
    nv = 1 << scale
    assert rp[-1] == ci.size == 8 << scale
    level = oracle.bfs(rp, ci, 0)
    m = sp.csr_matrix((np.ones(ci.size, np.int8), ci.copy(), rp.copy()), shape=(nv, nv))
    m.sum_duplicates()
    d = shortest_path(m, method="D", directed=True, unweighted=True, indices=0)
    want = np.where(np.isinf(d), -1, d).astype(np.int32)
    assert np.array_equal(level, want)
    # structural invariants of any BFS labelling
    assert level[0] == 0
    src = np.repeat(np.arange(nv), np.diff(rp))
    reach = level[src] >= 0
    assert np.all(level[ci[reach]] >= 0)
    assert np.all(level[ci[reach]] <= level[src[reach]] + 1)
    has_parent = np.zeros(nv, bool)
    par = reach & (level[ci] == level[src] + 1)
    has_parent[ci[par]] = True
    assert np.all(has_parent[level > 0])


# ---------------------------------------------------------------- embedding bag

def test_embedding_bag_closed_form():
    rows, dim = 100, 8
    table = (np.arange(rows)[:, None] * np.ones(dim)[None, :]).astype(np.float32)
    table += np.arange(dim, dtype=np.float32)[None, :] * 1000
    ids = np.array([[1, 2, 3, 4], [7, 7, 7, 7], [99, 0, 0, 99]], np.int32)
    want = ids.sum(1)[:, None] + 4000.0 * np.arange(dim)[None, :]
    assert np.array_equal(oracle.embedding_bag(table, ids), want)
    assert np.array_equal(oracle.embedding_bag_f32(table, ids), want.astype(np.float32))
    assert np.array_equal(oracle.embedding_bag_abs(table, ids), want)


def test_embedding_bag_against_numpy_and_ordered_fp32():
    rng = np.random.default_rng(4)
    table = inputs.f32_uniform(11, 0, 300 * 16).reshape(300, 16)
    ids = inputs.bag_row_ids(5, 0, 50 * 32, 300, scramble=False).reshape(50, 32)
    assert ids.min() >= 0 and ids.max() < 300
    ref = table.astype(np.float64)[ids].sum(axis=1)
    got = oracle.embedding_bag(table, ids)
    assert np.max(np.abs(got - ref)) <= 1e-13 * 32
    # fp32 variant: one rounding per addition, rows in listed order
    f32 = oracle.embedding_bag_f32(table, ids)
    acc = np.zeros((50, 16), np.float32)
    for j in range(32):
        acc = (acc + table[ids[:, j]]).astype(np.float32)
    assert np.array_equal(f32, acc)
    scale = oracle.embedding_bag_abs(table, ids)
    assert np.all(np.abs(f32 - ref) <= 1e-5 * scale)
    # order matters in fp32, not in the definition: reversed bags
    assert np.allclose(oracle.embedding_bag(table, ids[:, ::-1].copy()), got, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- scatter

def test_scatter_increment_is_a_histogram():
    idx = inputs.scatter_indices(3, 0, 100000, 1 << 12)
    assert idx.max() < 1 << 12
    host = np.zeros(1 << 12, np.uint64)
    oracle.scatter_increment(host, idx)
    assert np.array_equal(host, np.bincount(idx, minlength=1 << 12).astype(np.uint64))
    assert int(host.sum()) == 100000
    oracle.scatter_increment(host, idx[:10])                     # accumulates
    assert int(host.sum()) == 100010


# ---------------------------------------------------------------- input generators

def test_generators_are_counter_based_and_shaped():
    a = inputs.u32_values(1, 0, 1000)
    b = np.concatenate([inputs.u32_values(1, 0, 300), inputs.u32_values(1, 300, 700)])
    assert np.array_equal(a, b) and len(set(a.tolist())) > 990
    i = inputs.u32_indices(2, 0, 100000, 1 << 24)
    assert i.max() < 1 << 24 and abs(i.mean() / (1 << 23) - 1) < 0.02
    x = inputs.f32_uniform(3, 0, 200000)
    assert abs(x.mean()) < 0.01 and abs(x.var() - 1 / 3) < 0.01
    r = inputs.zipf_ranks(4, 0, 200000, 10 ** 6, 1.05)
    assert r.min() >= 1 and r.max() <= 10 ** 6
    assert np.mean(r <= 10) > 0.2                              # heavy head
    ids = inputs.bag_row_ids(4, 0, 1000, 5 * 10 ** 7)
    assert ids.min() >= 0 and ids.max() < 5 * 10 ** 7
    rp, ci = inputs.rmat_csr(1, 8)
    deg = np.diff(rp)
    assert deg.argmax() == 0 and deg.max() > 20 * deg.mean()   # vertex 0 is the hub


def test_torch_twins_match_numpy():
    import torch
    assert np.array_equal(inputs.t_u32_values(5, 100, 999, "cpu").numpy().view(np.uint32),
                          inputs.u32_values(5, 100, 999))
    assert np.array_equal(inputs.t_u32_indices(6, 7, 999, 1 << 24, "cpu").numpy().view(np.uint32),
                          inputs.u32_indices(6, 7, 999, 1 << 24))
    assert np.array_equal(inputs.t_f32_uniform(7, 50, 999, "cpu").numpy(),
                          inputs.f32_uniform(7, 50, 999))
    rp, ci = inputs.rmat_csr(2, 9)
    trp, tci = inputs.t_rmat_csr(2, 9, "cpu", chunk=1000)
    assert np.array_equal(trp.numpy(), rp) and np.array_equal(tci.numpy(), ci)


# ---------------------------------------------------------------- CC and SSSP

def test_cc_against_scipy_and_special_cases():
    from scipy.sparse.csgraph import connected_components
    rp, ci = _csr(7, [(0, 1), (2, 1), (3, 4), (5, 5)])          # {0,1,2} {3,4} {5} {6}
    assert oracle.cc(rp, ci).tolist() == [0, 0, 0, 3, 3, 5, 6]
    rp, ci = _csr(6, [(5, 4), (4, 3), (3, 2), (2, 1), (1, 0)])  # a path against the sweep direction
    assert oracle.cc(rp, ci).tolist() == [0] * 6
    for scale, ef in ((9, 1), (10, 2), (11, 8)):
        rp, ci = inputs.rmat_csr(7, scale, edge_factor=ef)
        nv = 1 << scale
        label = oracle.cc(rp, ci)
        m = sp.csr_matrix((np.ones(ci.size, np.int8), ci.copy(), rp.copy()), shape=(nv, nv))
        ncomp, comp = connected_components(m, directed=True, connection="weak")
        assert len(np.unique(label)) == ncomp
        # same partition, and the label is the smallest member
        first = np.full(ncomp, nv, np.int64)
        np.minimum.at(first, comp, np.arange(nv))
        assert np.array_equal(label, first[comp].astype(np.int32))


def test_sssp_against_scipy_and_special_cases():
    from scipy.sparse.csgraph import dijkstra
    INF = 0xFFFFFFFF
    rp, ci = _csr(5, [(0, 1), (0, 2), (1, 2), (2, 3)])
    w = np.array([10, 1, 1, 5], np.uint32)                       # edges sorted by source: 0->1, 0->2, 1->2, 2->3
    assert oracle.sssp(rp, ci, w, 0).tolist() == [0, 10, 1, 6, INF]
    assert oracle.sssp(rp, ci, w, 1).tolist() == [INF, 0, 1, 6, INF]
    # unit weights: SSSP is BFS
    rp, ci = inputs.rmat_csr(3, 10, edge_factor=8)
    lv = oracle.bfs(rp, ci, 0)
    d = oracle.sssp(rp, ci, np.ones(ci.size, np.uint32), 0)
    assert np.array_equal(np.where(d == INF, -1, d).astype(np.int32), lv)
    # random weights against scipy (duplicate edges: scipy needs the lightest one)
    w = inputs.edge_weights(9, 0, ci.size)
    assert w.min() >= 1 and w.max() <= 64
    nv = rp.size - 1
    src = np.repeat(np.arange(nv), np.diff(rp))
    key = src.astype(np.int64) * nv + ci
    order = np.lexsort((w, key))
    keep = np.ones(ci.size, bool)
    keep[1:] = key[order][1:] != key[order][:-1]
    sel = order[keep]
    m = sp.csr_matrix((w[sel].astype(np.float64), (src[sel], ci[sel])), shape=(nv, nv))
    ref = dijkstra(m, directed=True, indices=0)
    want = np.where(np.isinf(ref), INF, ref).astype(np.uint32)
    assert np.array_equal(oracle.sssp(rp, ci, w, 0), want)


# ---------------------------------------------------------------- column-order product, filter-then-gather

def test_matvec_t_against_numpy_and_closed_form():
    A = np.arange(12, dtype=np.float32).reshape(4, 3)            # columns 0 3 6 9 / 1 4 7 10 / 2 5 8 11
    x = np.array([1, 10, 100, 1000], np.float32)
    y, yabs = oracle.matvec_t(A, x)
    assert y.tolist() == [9630.0, 10741.0, 11852.0] and yabs.tolist() == y.tolist()
    A = inputs.f32_uniform(3, 0, 300 * 70).reshape(300, 70)
    x = inputs.f32_uniform(4, 0, 300)
    y, yabs = oracle.matvec_t(A, x)
    ref = A.astype(np.float64).T @ x.astype(np.float64)
    assert np.max(np.abs(y - ref)) <= 1e-12
    assert np.all(yabs >= np.abs(y)) and np.allclose(yabs, np.abs(A.astype(np.float64) * x[:, None]).sum(0), rtol=1e-12)
    yt, _ = oracle.matvec_t(np.ascontiguousarray(A.T), inputs.f32_uniform(4, 0, 70))   # not symmetric in rows/cols
    assert yt.shape == (300,)


def test_matvec_against_numpy_closed_form_and_its_transpose():
    A = np.arange(12, dtype=np.float32).reshape(4, 3)            # rows 0 1 2 / 3 4 5 / 6 7 8 / 9 10 11
    x = np.array([1, 10, 100], np.float32)
    y, yabs = oracle.matvec(A, x)
    assert y.tolist() == [210.0, 543.0, 876.0, 1209.0] and yabs.tolist() == y.tolist()
    A = inputs.f32_uniform(3, 0, 300 * 70).reshape(300, 70)
    x = inputs.f32_uniform(4, 0, 70)
    y, yabs = oracle.matvec(A, x)
    ref = A.astype(np.float64) @ x.astype(np.float64)
    assert np.max(np.abs(y - ref)) <= 1e-12
    assert np.all(yabs >= np.abs(y)) and np.allclose(yabs, np.abs(A.astype(np.float64) * x[None, :]).sum(1), rtol=1e-12)
    # A x is (A^T)^T x: the two products pin each other through an explicit transpose
    yt, _ = oracle.matvec_t(np.ascontiguousarray(A.T), x)
    assert np.max(np.abs(y - yt)) <= 1e-12
    # a sign pattern that a dropped or transposed term would break: row i of the identity picks x[i]
    assert oracle.matvec(np.eye(5, dtype=np.float32), np.arange(5, dtype=np.float32))[0].tolist() == [0, 1, 2, 3, 4]
    # terms that cancel: the scale keeps what the sum loses
    y, yabs = oracle.matvec(np.array([[1, -1]], np.float32), np.array([3, 3], np.float32))
    assert y.tolist() == [0.0] and yabs.tolist() == [6.0]


def test_filter_sum_against_numpy():
    key = inputs.u32_values(5, 0, 100000)
    val = inputs.u32_values(6, 0, 100000)
    thr = 0xFFFFFFFF - int(0.0008 * 2 ** 32)
    c, s = oracle.filter_sum(key, val, thr)
    m = key > thr
    assert c == int(m.sum()) and 40 < c < 130                     # ~0.08 % of the rows
    assert s == int(val[m].astype(np.uint64).sum())
    assert oracle.filter_sum(key, val, 0xFFFFFFFF) == (0, 0)
    assert oracle.filter_sum(key[:0], val[:0], 5) == (0, 0)
    assert oracle.filter_sum(np.array([6, 5, 7], np.uint32), np.array([1, 2, 4], np.uint32), 5) == (2, 5)


def test_vector_add_is_ieee_fp32_addition():
    a = inputs.f32_uniform(1, 0, 10001)
    b = inputs.f32_uniform(2, 0, 10001) * np.float32(1e-3)
    c = oracle.vector_add(a, b)
    assert c.dtype == np.float32 and np.array_equal(c, a + b)            # numpy's fp32 add
    exact = a.astype(np.float64) + b.astype(np.float64)
    assert np.all(np.abs(c - exact) <= np.abs(exact) * 2.0 ** -24 + 1e-45)  # correctly rounded
    assert oracle.vector_add(np.array([1.0, -2.5], np.float32), np.array([2.0, 2.5], np.float32)).tolist() == [3.0, 0.0]


# ---------------------------------------------------------------- the all-cores build of the same loops

def test_parallel_for_leg_equals_the_sequential_oracle():
    """oracle/gpuvm_oracle_par.c is timed by the benchmark's cpu_baseline leg only;
    it must return what the sequential definitions return."""
    assert oracle.par_threads() >= 1
    data = inputs.u32_values(1, 0, 1 << 16)
    idx = inputs.u32_indices(2, 0, 30011, 1 << 16)
    a, b = oracle.gather(data, idx), oracle.par_gather(data, idx)
    assert np.array_equal(a[0], b[0]) and a[1] == b[1]
    x = inputs.f32_uniform(7, 0, (1 << 18) + 333)
    assert np.array_equal(oracle.stream_reduce(x, 4096, 2), oracle.par_stream_reduce(x, 4096, 2))   # same order inside a block
    rp, ci = inputs.rmat_csr(5, 13)
    for src in (0, 77):
        assert np.array_equal(oracle.bfs(rp, ci, src), oracle.par_bfs(rp, ci, src))
    table = inputs.f32_uniform(11, 0, 512 * 64).reshape(512, 64)
    ids = inputs.u32_indices(3, 0, 200 * 9, 512).astype(np.int32).reshape(200, 9)
    assert np.array_equal(oracle.embedding_bag_f32(table, ids), oracle.par_embedding_bag_f32(table, ids))
    sidx = inputs.scatter_indices(3, 0, 100000, 1 << 12)
    h1, h2 = np.zeros(1 << 12, np.uint64), np.zeros(1 << 12, np.uint64)
    assert np.array_equal(oracle.scatter_increment(h1, sidx), oracle.par_scatter_increment(h2, sidx))

"""Streaming reduce, BFS, embedding bag and scatter-increment through the paged
view vs the oracle, at sizes the oracle finishes in seconds but that span many
pages, a ragged tail and an oversubscribed pool."""
import numpy as np
import pytest
import torch

import oracle
import paper_2411_05309_amd as gv
from paper_2411_05309_amd import inputs

from gpu_util import Backing, check_invariants, dev, host

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------- streaming read-reduce

@pytest.mark.parametrize("n_floats,page,frames,block_pages", [
    (1 << 22, 65536, 64, 16),            # 256 pages, 64 frames, 1 MiB blocks
    ((1 << 20) + 12345, 4096, 16, 4),    # short last page (not a multiple of 16 bytes), ragged last block
    (1 << 18, 16384, 64, 1),             # fits the pool
])
def test_stream_reduce(gpu, n_floats, page, frames, block_pages):
    x = inputs.f32_uniform(7, 0, n_floats)
    block_elems = block_pages * page // 4
    passes = 3
    want = oracle.stream_reduce(x, block_elems, passes)
    scale = oracle.stream_abs(x, block_elems)
    nblocks = want.shape[1]
    with Backing(x, page, frames * page) as b:
        d_s = torch.full((nblocks,), -1.0, dtype=torch.float64, device="cuda")
        got = np.empty_like(want)
        for p in range(passes):
            gv.gpuvm_run_stream_reduce(b.vm, block_elems, d_s)
            gv.gpuvm_check(b.vm)
            got[p] = d_s.cpu().numpy()
        # |gpu - ref| <= 1e-5 * sum|x| per block (the stated fp32-sum tolerance;
        # fp64 accumulation keeps the real error near 1e-13)
        assert np.all(np.abs(got - want) <= 1e-5 * scale[None, :])
        assert np.all(np.abs(got - want) <= 1e-11 * scale[None, :])
        st, *_ = check_invariants(b, read_only=True, pristine=x)
        n_pages = b.n_pages
        if n_pages <= frames:
            assert st["faults"] == n_pages
        else:
            # cyclic scan over more pages than frames: (almost) every access faults
            assert st["faults"] >= passes * n_pages - 2 * frames
            assert st["faults"] <= passes * n_pages


# ---------------------------------------------------------------- BFS

def _bfs_case(rp, ci, src, page, frames, policy=gv.POLICY_CLOCK, balanced=False):
    nv = rp.size - 1
    want = oracle.bfs(rp, ci, src)
    run = gv.gpuvm_run_bfs_balanced if balanced else gv.gpuvm_run_bfs
    with Backing(ci, page, frames * page, policy) as b:
        d_rp = dev(rp)
        d_level = torch.zeros(nv, dtype=torch.int32, device="cuda")
        levels = run(b.vm, d_rp, nv, src, d_level)
        got = d_level.cpu().numpy()
        assert np.array_equal(got, want)
        assert levels == want.max() + 1
        st, *_ = check_invariants(b, read_only=True, pristine=ci)
    return st


@pytest.mark.parametrize("balanced", [False, True])
@pytest.mark.parametrize("scale,page,frames", [(14, 4096, 16), (16, 65536, 16), (12, 4096, 512), (17, 4096, 64)])
def test_bfs_rmat(gpu, scale, page, frames, balanced):
    rp, ci = inputs.rmat_csr(5, scale)
    st = _bfs_case(rp, ci, 0, page, frames, balanced=balanced)
    assert st["faults"] > 0
    if balanced:
        assert st["loading_waits"] == 0          # a page belongs to one wave per level


@pytest.mark.parametrize("balanced", [False, True])
def test_bfs_special_graphs(gpu, balanced):
    n = 5000                                                       # long path: many levels
    src = np.arange(n - 1)
    rp = np.concatenate([np.arange(n), [n - 1]]).astype(np.int64)
    ci = (src + 1).astype(np.int32)
    _bfs_case(rp[:n + 1], ci, 0, 4096, 8, balanced=balanced)
    nv = 3000                                                      # star with a huge hub + unreachable tail
    rp = np.zeros(nv + 1, np.int64)
    rp[1:] = 2500
    ci = np.arange(1, 2501, dtype=np.int32)
    _bfs_case(rp, ci, 0, 4096, 8, balanced=balanced)
    _bfs_case(rp, ci, 7, 4096, 8, balanced=balanced)               # source without edges
    # many empty rows before, between and after the only rows that have edges
    nv = 100000
    rp = np.zeros(nv + 1, np.int64)
    rp[50001:] = 3000
    rp[90001:] = 3010
    ci = np.concatenate([np.arange(60000, 63000), np.full(10, 50000)]).astype(np.int32)
    _bfs_case(rp, ci, 50000, 4096, 8, balanced=balanced)
    _bfs_case(rp, ci, 90000, 4096, 8, balanced=balanced)


# ---------------------------------------------------------------- embedding bag

@pytest.mark.parametrize("dim,rows,page,frames,bags,bag_len", [
    (128, 20000, 65536, 32, 3000, 32),      # 157 pages over 32 frames
    (64, 5000, 4096, 16, 1001, 7),
    (256, 3000, 65536, 8, 500, 70),         # bag longer than a wavefront
])
def test_embedding_bag(gpu, dim, rows, page, frames, bags, bag_len):
    table = inputs.f32_uniform(11, 0, rows * dim).reshape(rows, dim)
    ids = inputs.bag_row_ids(5, 0, bags * bag_len, rows, scramble=(np.gcd(2654435761, rows) == 1)).reshape(bags, bag_len)
    ids[0, 0], ids[-1, -1] = 0, rows - 1
    want32 = oracle.embedding_bag_f32(table, ids)
    want64 = oracle.embedding_bag(table, ids)
    scale = oracle.embedding_bag_abs(table, ids)
    with Backing(table, page, frames * page) as b:
        d_ids = dev(ids)
        d_out = torch.full((bags, dim), -7.0, dtype=torch.float32, device="cuda")
        for _ in range(2):                                           # second batch on the warm pool
            gv.gpuvm_run_embedding_bag(b.vm, dim, d_ids, bags, bag_len, d_out)
            gv.gpuvm_check(b.vm)
            got = d_out.cpu().numpy()
            assert np.array_equal(got, want32)                        # same order, same precision
            assert np.all(np.abs(got - want64) <= 1e-5 * scale)
        check_invariants(b, read_only=True, pristine=table)


# ---------------------------------------------------------------- scatter-increment

@pytest.mark.parametrize("wb_mode", [gv.WB_OVERLAPPED, gv.WB_SERIAL])
@pytest.mark.parametrize("policy", [gv.POLICY_CLOCK, gv.POLICY_FIFO, gv.POLICY_FIFO_WAIT, gv.POLICY_CLOCK_WRITE_AWARE, gv.POLICY_GCLOCK])
@pytest.mark.parametrize("n_elems,page,frames,n_upd", [
    (1 << 17, 4096, 32, 200000),            # 256 pages over 32 frames: dirty evictions
    ((1 << 15) + 77, 4096, 16, 50001),      # short last page
    (1 << 14, 65536, 8, 30000),             # fits: only the flush writes back
    (1 << 17, 65536, 8, 20000),             # 64 KiB pages, dirty evictions
])
def test_scatter_increment(gpu, policy, n_elems, page, frames, n_upd, wb_mode):
    idx = inputs.scatter_indices(3, 0, n_upd, n_elems)
    # spread the hot head so that evictions really are dirty and re-faulted
    idx = ((idx.astype(np.uint64) * 40503) % n_elems).astype(np.uint32)
    idx[-1] = n_elems - 1
    want = np.zeros(n_elems, np.uint64)
    oracle.scatter_increment(want, idx)
    with Backing(np.zeros(n_elems, np.uint64), page, frames * page, policy) as b:
        gv.gpuvm_set_writeback_mode(b.vm, wb_mode)
        d_idx = dev(idx)
        half = n_upd // 2
        gv.gpuvm_run_scatter_increment(b.vm, d_idx, half)
        gv.gpuvm_run_scatter_increment(b.vm, d_idx[half:], n_upd - half)     # second launch, mappings persist
        gv.gpuvm_check(b.vm)
        st, f, *_ = check_invariants(b, read_only=False)
        if b.n_pages > frames:
            assert st["writebacks_evict"] > 0
        gv.gpuvm_flush(b.vm)
        st2, f2, *_ = check_invariants(b, read_only=False)
        assert not np.any(f2["dirty"])
        assert st2["writebacks_flush"] == int(np.count_nonzero(f["dirty"]))
        assert np.array_equal(b.arr, want)
        assert int(b.arr.sum()) == n_upd
        gv.gpuvm_flush(b.vm)                                                    # nothing left to do
        assert gv.gpuvm_stats(b.vm)["writebacks_flush"] == st2["writebacks_flush"]
        # reset = flush + cold start; host memory stays authoritative
        gv.gpuvm_run_scatter_increment(b.vm, d_idx, 1000)
        gv.gpuvm_reset(b.vm)
        oracle.scatter_increment(want, idx[:1000])
        assert np.array_equal(b.arr, want)
        pte, owner, hand = gv.gpuvm_dump_tables(b.vm)
        assert not pte.any() and np.all(owner == gv.NO_PAGE) and hand == 0


def test_store_then_load_roundtrip_through_eviction(gpu):
    """Dirty pages written back at eviction are re-read correctly by later faults
    (write-back ordering against the re-fault's reads)."""
    n_elems, page, frames = 1 << 16, 4096, 8
    rounds = 6
    idx = (inputs.u32_indices(9, 0, 40000, 1 << 30) % n_elems).astype(np.uint32)
    want = np.zeros(n_elems, np.uint64)
    with Backing(np.zeros(n_elems, np.uint64), page, frames * page) as b:
        d_idx = dev(idx)
        for r in range(rounds):
            gv.gpuvm_run_scatter_increment(b.vm, d_idx, idx.size)
            oracle.scatter_increment(want, idx)
        gv.gpuvm_flush(b.vm)
        assert np.array_equal(b.arr, want)
        st = gv.gpuvm_stats(b.vm)
        assert st["writebacks_evict"] > 10 * frames


# ---------------------------------------------------------------- CC and SSSP (edge-balanced)

@pytest.mark.parametrize("scale,ef,page,frames", [(14, 16, 4096, 16), (16, 2, 65536, 8), (12, 1, 4096, 256),
                                                  (14, 16, 4096, 64), (16, 16, 4096, 1024)])
def test_cc_balanced(gpu, scale, ef, page, frames):
    rp, ci = inputs.rmat_csr(7, scale, edge_factor=ef)
    nv = 1 << scale
    want = oracle.cc(rp, ci)
    with Backing(ci, page, frames * page) as b:
        d_label = torch.zeros(nv, dtype=torch.int32, device="cuda")
        rounds = gv.gpuvm_run_cc_balanced(b.vm, dev(rp), nv, d_label)
        assert rounds >= 2
        assert np.array_equal(d_label.cpu().numpy(), want)
        st, *_ = check_invariants(b, read_only=True, pristine=ci)
        if b.n_pages > frames:                                   # every round re-reads every page
            assert st["faults"] >= (rounds - 1) * (b.n_pages - frames)
            if frames >= 64:
                # ... and starts with what the round before left in the pool, before its own
                # faults can evict it (a quarter of the pool at the very least)
                assert st["faults"] <= rounds * b.n_pages - (rounds - 1) * (frames // 4)


@pytest.mark.parametrize("scale,page,frames,src", [(14, 4096, 16, 0), (16, 65536, 8, 5), (12, 4096, 256, 0)])
def test_sssp_balanced(gpu, scale, page, frames, src):
    rp, ci = inputs.rmat_csr(9, scale)
    w = inputs.edge_weights(4, 0, ci.size)
    nv = 1 << scale
    want = oracle.sssp(rp, ci, w, src)
    with Backing(ci, page, frames * page) as b, Backing(w, page, frames * page) as bw:
        d_dist = torch.zeros(nv, dtype=torch.int32, device="cuda")
        rounds = gv.gpuvm_run_sssp_balanced(b.vm, bw.vm, dev(rp), nv, src, d_dist)
        assert rounds >= 2
        assert np.array_equal(host(d_dist, np.uint32), want)
        st, *_ = check_invariants(b, read_only=True, pristine=ci)
        stw, *_ = check_invariants(bw, read_only=True, pristine=w)
        # the two arrays are walked in lock step, each in a pool of its own (victim choice may differ by timing)
        assert abs(st["faults"] - stw["faults"]) <= max(2, st["faults"] // 20)
        with pytest.raises(gv.GpuvmError):                         # mismatched second array
            gv.gpuvm_run_sssp_balanced(b.vm, b.vm, dev(rp), nv, src, d_dist)


def test_sssp_pools_of_different_size(gpu):
    """The two paged arrays of SSSP need not have pools of the same size: a round's
    pages are ordered by what the pool of col_idx holds, the weights follow."""
    rp, ci = inputs.rmat_csr(9, 14)
    w = inputs.edge_weights(4, 0, ci.size)
    nv = 1 << 14
    want = oracle.sssp(rp, ci, w, 3)
    with Backing(ci, 4096, 64 * 4096) as b, Backing(w, 4096, 24 * 4096) as bw:
        d_dist = torch.zeros(nv, dtype=torch.int32, device="cuda")
        rounds = gv.gpuvm_run_sssp_balanced(b.vm, bw.vm, dev(rp), nv, 3, d_dist)
        assert rounds >= 2
        assert np.array_equal(host(d_dist, np.uint32), want)
        st, *_ = check_invariants(b, read_only=True, pristine=ci)
        stw, *_ = check_invariants(bw, read_only=True, pristine=w)
        assert stw["faults"] >= st["faults"]                       # the smaller pool keeps less from round to round


# ---------------------------------------------------------------- column-order access, sparse filter

@pytest.mark.parametrize("rows,cols,page,frames", [
    (512, 4096, 4096, 64),            # a row = 4 pages; 2048 pages over 64 frames
    (300, 1000, 4096, 16),            # ragged: columns not a multiple of 64, short last page
    (64, 16384, 65536, 8),
    # sliding window and fault-ahead helpers on (every column block has a wave of its
    # own and the pool holds 256 rows), 5 working waves in a grid rounded up to 8:
    # the idle ones must not count as the slowest wave
    (2048, 320, 4096, 80),
    (1024, 1000, 4096, 128),          # the same with 16 working waves, ragged columns
])
def test_matvec_t_column_order(gpu, rows, cols, page, frames):
    A = inputs.f32_uniform(3, 0, rows * cols).reshape(rows, cols)
    x = inputs.f32_uniform(4, 0, rows)
    want, scale = oracle.matvec_t(A, x)
    with Backing(A, page, frames * page) as b:
        d_y = torch.full((cols,), -1.0, dtype=torch.float64, device="cuda")
        gv.gpuvm_run_matvec_t(b.vm, rows, cols, dev(x), d_y)
        gv.gpuvm_check(b.vm)
        got = d_y.cpu().numpy()
        assert np.all(np.abs(got - want) <= 1e-5 * scale)          # stated bar
        assert np.all(np.abs(got - want) <= 1e-12 * scale + 1e-300)  # same order, fp64: essentially exact
        check_invariants(b, read_only=True, pristine=A)
        with pytest.raises(gv.GpuvmError):
            gv.gpuvm_run_matvec_t(b.vm, rows + 1, cols, dev(x), d_y)


@pytest.mark.parametrize("rows,cols,page,frames", [
    (512, 4096, 4096, 512),           # a row = 4 pages; 2048 pages over 512 frames, the rows in flight fit
    (300, 1000, 4096, 16),            # ragged rows, short last page, far more rows in flight than frames
    (200, 16384, 65536, 64),          # a row = one 64 KiB page
])
def test_matvec_row_per_thread(gpu, rows, cols, page, frames):
    A = inputs.f32_uniform(3, 0, rows * cols).reshape(rows, cols)
    x = inputs.f32_uniform(4, 0, cols)
    want, scale = oracle.matvec(A, x)
    with Backing(A, page, frames * page) as b:
        d_y = torch.full((rows,), -1.0, dtype=torch.float64, device="cuda")
        gv.gpuvm_run_matvec(b.vm, rows, cols, dev(x), d_y)
        gv.gpuvm_check(b.vm)
        got = d_y.cpu().numpy()
        assert np.all(np.abs(got - want) <= 1e-5 * scale)          # stated bar
        assert np.array_equal(got, want)                             # same order, fp64, no contraction: exact
        st, *_ = check_invariants(b, read_only=True, pristine=A)
        assert st["faults"] >= b.n_pages
        for bad_rows, bad_cols in ((rows + 1, cols), (rows * 2, cols // 2 + 1)):
            with pytest.raises(gv.GpuvmError):
                gv.gpuvm_run_matvec(b.vm, bad_rows, bad_cols, dev(x), d_y)


@pytest.mark.parametrize("n,page,frames,sel", [
    (1 << 20, 4096, 32, 0.0008),      # the paper's 0.08 % selectivity, 4 KiB pages
    ((1 << 18) + 333, 4096, 16, 0.02),
    (1 << 16, 65536, 8, 0.5),
])
def test_filter_sum(gpu, n, page, frames, sel):
    key = inputs.u32_values(5, 0, n)
    val = inputs.u32_values(6, 0, n)
    thr = 0xFFFFFFFF - int(sel * 2 ** 32)
    want = oracle.filter_sum(key, val, thr)
    with Backing(key, page, frames * page) as bk, Backing(val, page, frames * page) as bv:
        d_c = torch.zeros(1, dtype=torch.int64, device="cuda")
        d_s = torch.zeros(1, dtype=torch.int64, device="cuda")
        for _ in range(2):
            gv.gpuvm_run_filter_sum(bk.vm, bv.vm, thr, d_c, d_s)
            gv.gpuvm_check(bk.vm)
            gv.gpuvm_check(bv.vm)
            assert (int(host(d_c, np.uint64)[0]), int(host(d_s, np.uint64)[0])) == want
        stk, *_ = check_invariants(bk, read_only=True, pristine=key)
        stv, *_ = check_invariants(bv, read_only=True, pristine=val)
        touched = len(np.unique(np.nonzero(key > thr)[0] * 4 // page))
        assert stv["faults"] >= touched                              # only pages with a matching row are fetched
        if sel < 0.001:
            assert stv["faults"] < 2 * bv.n_pages * 0.8             # well below two full scans


# ---------------------------------------------------------------- the paper's vector addition (stores)

@pytest.mark.parametrize("n,page,frames", [(1 << 20, 65536, 16), ((1 << 18) + 777, 4096, 16), (5000, 4096, 8)])
def test_vector_add_through_three_paged_vectors(gpu, n, page, frames):
    a = inputs.f32_uniform(1, 0, n)
    b = inputs.f32_uniform(2, 0, n)
    want = oracle.vector_add(a, b)
    with Backing(a, page, frames * page) as ba, Backing(b, page, frames * page) as bb, \
            Backing(np.full(n, -9.0, np.float32), page, frames * page) as bc:
        gv.gpuvm_run_vector_add(ba.vm, bb.vm, bc.vm, n)
        for x in (ba, bb, bc):
            gv.gpuvm_check(x.vm)
        check_invariants(ba, read_only=True, pristine=a)
        check_invariants(bb, read_only=True, pristine=b)
        stc, fc, *_ = check_invariants(bc, read_only=False)
        if bc.n_pages > frames:
            assert stc["writebacks_evict"] > 0
        gv.gpuvm_flush(bc.vm)
        assert np.array_equal(bc.arr, want)                              # bit-exact fp32
        # in place: A += A (A and B the same handle), result in C
        gv.gpuvm_run_vector_add(ba.vm, ba.vm, bc.vm, n)
        gv.gpuvm_flush(bc.vm)
        assert np.array_equal(bc.arr, oracle.vector_add(a, a))
        with pytest.raises(gv.GpuvmError):
            gv.gpuvm_run_vector_add(ba.vm, bb.vm, ba.vm, n)


@pytest.mark.parametrize("n,page,frames", [(1 << 20, 65536, 16), ((1 << 18) + 777, 4096, 16), (5000, 4096, 8)])
def test_vector_add_overwrite_installs_without_fetching(gpu, n, page, frames):
    a = inputs.f32_uniform(1, 0, n)
    b = inputs.f32_uniform(2, 0, n)
    want = oracle.vector_add(a, b)
    with Backing(a, page, frames * page) as ba, Backing(b, page, frames * page) as bb, \
            Backing(np.full(n, -9.0, np.float32), page, frames * page) as bc:
        gv.gpuvm_run_vector_add_overwrite(ba.vm, bb.vm, bc.vm, n)
        for x in (ba, bb, bc):
            gv.gpuvm_check(x.vm)
        check_invariants(ba, read_only=True, pristine=a)
        check_invariants(bb, read_only=True, pristine=b)
        stc, *_ = check_invariants(bc, read_only=False)
        assert stc["faults"] == bc.n_pages and stc["faults_no_fetch"] == bc.n_pages and stc["bytes_in"] == 0
        gv.gpuvm_flush(bc.vm)
        assert np.array_equal(bc.arr, want)                              # bit-exact fp32
        # second run over the pages still resident (hits) and the evicted ones (misses again)
        gv.gpuvm_run_vector_add_overwrite(ba.vm, ba.vm, bc.vm, n)
        gv.gpuvm_flush(bc.vm)
        assert np.array_equal(bc.arr, oracle.vector_add(a, a))
        assert gv.gpuvm_stats(bc.vm)["bytes_in"] == 0
        # a prefix that ends on a page boundary leaves the rest of C alone ...
        part = (n * 4 // page // 2) * (page // 4)
        if part:
            gv.gpuvm_run_vector_add_overwrite(ba.vm, bb.vm, bc.vm, part)
            gv.gpuvm_flush(bc.vm)
            assert np.array_equal(bc.arr[:part], want[:part])
            assert np.array_equal(bc.arr[part:], oracle.vector_add(a, a)[part:])
        # ... and one that ends inside a page is refused (the page would need its old content)
        with pytest.raises(gv.GpuvmError):
            gv.gpuvm_run_vector_add_overwrite(ba.vm, bb.vm, bc.vm, n - 3 if (n - 3) * 4 % page else n - 5)
        with pytest.raises(gv.GpuvmError):
            gv.gpuvm_run_vector_add_overwrite(ba.vm, bb.vm, ba.vm, n)


def test_graph_launchers_report_bad_neighbour_ids(gpu):
    """A neighbour id outside [0, nv) - too large, or negative - is reported as
    GPUVM_ERANGE by every graph launcher instead of becoming a stray write."""
    nv = 2000
    rp, ci = inputs.rmat_csr(6, 11)
    rp, ci = rp[:nv + 1].copy(), ci[:int(rp[nv])].copy() % nv
    w = inputs.edge_weights(4, 0, ci.size)
    first = int(rp[0])                                               # an edge of the source vertex: always visited
    assert rp[1] > rp[0]
    for bad in (nv, nv + 12345, -1, -(1 << 31)):
        c2 = ci.copy()
        c2[first] = bad
        for name in ("bfs", "bfs_balanced", "cc", "sssp"):
            with Backing(c2, 4096, 8 * 4096) as b, Backing(w, 4096, 8 * 4096) as bw:
                d_out = torch.zeros(nv, dtype=torch.int32, device="cuda")
                with pytest.raises(gv.GpuvmError) as e:
                    if name == "bfs":
                        gv.gpuvm_run_bfs(b.vm, dev(rp), nv, 0, d_out)
                    elif name == "bfs_balanced":
                        gv.gpuvm_run_bfs_balanced(b.vm, dev(rp), nv, 0, d_out)
                    elif name == "cc":
                        gv.gpuvm_run_cc_balanced(b.vm, dev(rp), nv, d_out)
                    else:
                        gv.gpuvm_run_sssp_balanced(b.vm, bw.vm, dev(rp), nv, 0, d_out)
                assert e.value.code == gv.ERANGE, (name, bad)


def test_bfs_zero_copy_baseline_matches_the_oracle(gpu):
    rp, ci = inputs.rmat_csr(9, 14)
    want = oracle.bfs(rp, ci, 0)
    with Backing(ci, 4096, 16 * 4096) as b:
        d_level = torch.zeros(1 << 14, dtype=torch.int32, device="cuda")
        levels = gv.gpuvm_bench_bfs_zero_copy(b.vm, dev(rp), 1 << 14, 0, d_level)
        assert levels >= 2 and np.array_equal(host(d_level, np.int32), want)
        st = gv.gpuvm_stats(b.vm)
        assert st["faults"] == 0                                   # nothing was paged
        # the same with pages in the pool (a paged run first): every page is still read in
        # place, whatever is resident
        gv.gpuvm_run_bfs_balanced(b.vm, dev(rp), 1 << 14, 0, d_level)
        paged = gv.gpuvm_stats(b.vm)["faults"]
        assert paged > 0
        d_level.fill_(7)
        gv.gpuvm_bench_bfs_zero_copy(b.vm, dev(rp), 1 << 14, 0, d_level)
        assert np.array_equal(host(d_level, np.int32), want)
        assert gv.gpuvm_stats(b.vm)["faults"] == paged


@pytest.mark.parametrize("dim", [64, 128, 256])
def test_embedding_zero_copy_baseline_matches_the_oracle(gpu, dim):
    rows, bags, bag_len, page = 3000, 500, 7, 65536
    rows -= rows % (page // (dim * 4))                              # whole pages of rows
    table = inputs.f32_uniform(11, 0, rows * dim).reshape(rows, dim)
    ids = inputs.bag_row_ids(5, 0, bags * bag_len, rows - 1 if np.gcd(2654435761, rows) != 1 else rows, 1.05).reshape(bags, bag_len)
    ids = np.ascontiguousarray(ids % rows).astype(np.int32)
    with Backing(table, page, 8 * page) as b:
        d_out = torch.zeros((bags, dim), dtype=torch.float32, device="cuda")
        gv.gpuvm_bench_embedding_bag_zero_copy(b.vm, dim, dev(ids), bags, bag_len, d_out)
        gv.gpuvm_check(b.vm)
        assert np.array_equal(d_out.cpu().numpy(), oracle.embedding_bag_f32(table, ids))
        assert gv.gpuvm_stats(b.vm)["faults"] == 0


def test_plain_scatter_microbenchmark_in_hbm_and_in_host_memory(gpu):
    n64, n = 1 << 16, 50000
    idx = inputs.scatter_indices(3, 0, n, n64)
    want = np.zeros(n64, np.uint64)
    oracle.scatter_increment(want, idx)
    d = torch.zeros(n64, dtype=torch.int64, device="cuda")
    gv.gpuvm_bench_scatter_plain(d, dev(idx), n)
    torch.cuda.synchronize()
    assert np.array_equal(host(d, np.uint64), want)
    h = gv.pinned_array((n64,), np.uint64)
    try:
        h[:] = 0
        gv.gpuvm_bench_scatter_plain(h, dev(idx), n)                  # atomics executed over the link
        torch.cuda.synchronize()
        assert np.array_equal(h, want)
    finally:
        gv.free_pinned(h)


@pytest.mark.parametrize("nbytes,chunk,waves", [
    ((1 << 20) + 4096 + 48, 4096, 64),       # last chunk 48 bytes
    ((1 << 21) + 16, 65536, 16),             # eight 8 KiB rounds per chunk, last chunk 16 bytes
    (5 * 20480 + 1040, 20480, 8),            # a chunk that is not a multiple of 8 KiB: two full rounds and half a one
])
def test_copy_microbenchmarks_move_every_byte(gpu, nbytes, chunk, waves):
    """The two forms of the wavefront mover as microbenchmarks (staged through
    registers, staged through LDS): host to device and back, byte for byte."""
    src = inputs.u32_values(0x51, 0, (nbytes + 3) // 4).view(np.uint8)[:nbytes]
    h = gv.pinned_array((nbytes,), np.uint8)
    back = gv.pinned_array((nbytes,), np.uint8)
    try:
        for fn in (gv.gpuvm_bench_copy, gv.gpuvm_bench_copy_lds):
            h[:] = src
            back[:] = 0
            d = torch.zeros(nbytes + 64, dtype=torch.uint8, device="cuda")     # 64 guard bytes behind the data
            fn(d, h, nbytes, chunk, waves)
            torch.cuda.synchronize()
            got = d.cpu().numpy()
            assert np.array_equal(got[:nbytes], src), fn.__name__
            assert not got[nbytes:].any(), fn.__name__
            fn(back, d, nbytes, chunk, waves)
            torch.cuda.synchronize()
            assert np.array_equal(back, src), fn.__name__
        with pytest.raises(gv.GpuvmError):
            gv.gpuvm_bench_copy_lds(d, h, nbytes - 8, chunk, waves)              # not a multiple of 16
    finally:
        gv.free_pinned(h)
        gv.free_pinned(back)

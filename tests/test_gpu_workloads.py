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

@pytest.mark.parametrize("policy", [gv.POLICY_CLOCK, gv.POLICY_FIFO])
@pytest.mark.parametrize("n_elems,page,frames,n_upd", [
    (1 << 17, 4096, 32, 200000),            # 256 pages over 32 frames: dirty evictions
    ((1 << 15) + 77, 4096, 16, 50001),      # short last page
    (1 << 14, 65536, 8, 30000),             # fits: only the flush writes back
])
def test_scatter_increment(gpu, policy, n_elems, page, frames, n_upd):
    idx = inputs.scatter_indices(3, 0, n_upd, n_elems)
    # spread the hot head so that evictions really are dirty and re-faulted
    idx = ((idx.astype(np.uint64) * 40503) % n_elems).astype(np.uint32)
    idx[-1] = n_elems - 1
    want = np.zeros(n_elems, np.uint64)
    oracle.scatter_increment(want, idx)
    with Backing(np.zeros(n_elems, np.uint64), page, frames * page, policy) as b:
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

"""Remote-first reads (gpuvm_set_remote_first): a read that misses is served in
place over the link until the page's reads in place have cost what a migration
costs; then the page migrates.  Results must not change, only the traffic."""
import numpy as np
import pytest
import torch

import oracle
import paper_2411_05309_amd as gv
from paper_2411_05309_amd import inputs

from gpu_util import Backing, check_invariants, dev, host

pytestmark = pytest.mark.gpu


def _gather(b, idx):
    d_out = torch.zeros(idx.size, dtype=torch.int32, device="cuda")
    d_sum = torch.zeros(1, dtype=torch.int64, device="cuda")
    gv.gpuvm_configure(b.vm, 0, True)
    gv.gpuvm_run_gather(b.vm, dev(idx), idx.size, d_out, d_sum)
    gv.gpuvm_check(b.vm)
    return host(d_out, np.uint32), int(host(d_sum, np.uint64)[0])


@pytest.mark.parametrize("policy", [gv.POLICY_CLOCK, gv.POLICY_FIFO_WAIT, gv.POLICY_GCLOCK])
@pytest.mark.parametrize("n_elems,page,frames,n_idx,per_touch", [
    ((1 << 18) + 5, 4096, 16, 40000, 4),       # 32 reads in place buy a 4 KiB page
    (1 << 18, 4096, 16, 40000, 1024),          # 4
    (1 << 20, 65536, 8, 150000, 4),            # 512 for a 64 KiB page
])
def test_gather_results_do_not_change(gpu, policy, n_elems, page, frames, n_idx, per_touch):
    data = inputs.u32_values(31, 0, n_elems)
    # half of the reads go to a few hot pages (they migrate), the rest is spread thin (served in place)
    hot = inputs.u32_indices(32, 0, n_idx, 1 << 30) % np.uint32(4 * page // 4)
    cold = inputs.u32_indices(33, 0, n_idx, 1 << 30) % np.uint32(n_elems)
    idx = np.where(inputs.u32_indices(34, 0, n_idx, 2) == 0, hot, cold).astype(np.uint32)
    idx[-1] = n_elems - 1
    want, want_sum = oracle.gather(data, idx)
    with Backing(data, page, frames * page, policy) as b:
        got, got_sum = _gather(b, idx)
        plain = gv.gpuvm_stats(b.vm)
        assert np.array_equal(got, want) and got_sum == want_sum and plain["remote_reads"] == 0
        gv.gpuvm_reset(b.vm)
        gv.gpuvm_set_remote_first(b.vm, per_touch)
        got, got_sum = _gather(b, idx)
        assert np.array_equal(got, want) and got_sum == want_sum
        st, f, *_ = check_invariants(b, read_only=True, pristine=data, remote_first=True)
        limit = page // max(per_touch, 128)
        assert st["remote_reads"] > 0 and 0 < st["faults"] < plain["faults"]  # the hot pages were bought, the rest rented
        assert np.all(f["frame"][f["state"] == gv.ST_INVALID] < limit)        # nobody rents beyond the price
        # every page group was served one way or another
        assert st["hits"] + st["faults"] + st["remote_reads"] == st["wave_page_groups"]
        # off again: back to the paper's behaviour
        gv.gpuvm_set_remote_first(b.vm, 0)
        gv.gpuvm_stats_clear(b.vm)
        got, _ = _gather(b, idx)
        assert np.array_equal(got, want) and gv.gpuvm_stats(b.vm)["remote_reads"] == 0


def test_thinly_spread_reads_never_migrate(gpu):
    n_elems, page = 1 << 20, 4096                                            # 1024 pages
    data = inputs.u32_values(35, 0, n_elems)
    idx = (np.arange(1024 * 8, dtype=np.uint32) % 1024) * 1024 + 7           # every page 8 times: below the price of 32
    with Backing(data, page, 16 * page) as b:
        gv.gpuvm_set_remote_first(b.vm, 4)
        got, _ = _gather(b, idx)
        assert np.array_equal(got, oracle.gather(data, idx)[0])
        st = gv.gpuvm_stats(b.vm)
        assert st["faults"] == 0 and st["bytes_in"] == 0 and st["remote_reads"] > 0


def test_reads_in_place_see_what_was_written_back(gpu):
    n64, page, frames = 1 << 16, 4096, 8
    idx_w = ((inputs.zipf_ranks(36, 0, 50000, n64, 0.9) - 1) * 40503 % n64).astype(np.uint32)
    model = np.zeros(n64, np.uint64)
    oracle.scatter_increment(model, idx_w)
    idx_r = (inputs.u32_indices(37, 0, 30000, 1 << 30) % np.uint32(2 * n64)).astype(np.uint32)
    with Backing(np.zeros(n64, np.uint64), page, frames * page) as b:
        gv.gpuvm_set_remote_first(b.vm, 4)
        gv.gpuvm_run_scatter_increment(b.vm, dev(idx_w), idx_w.size)          # writes always migrate; dirty pages get evicted
        got, _ = _gather(b, idx_r)                                            # resident pages from frames, the rest in place
        assert np.array_equal(got, oracle.gather(model.view(np.uint32), idx_r)[0])
        st = gv.gpuvm_stats(b.vm)
        assert st["writebacks_evict"] > 0 and st["remote_reads"] > 0


@pytest.mark.parametrize("dim", [64, 128])
def test_embedding_bag_results_do_not_change(gpu, dim):
    rows, bags, bag_len, page = 6000, 4000, 16, 65536
    rows -= rows % (page // (dim * 4))
    table = inputs.f32_uniform(11, 0, rows * dim).reshape(rows, dim)
    ids = inputs.bag_row_ids(5, 0, bags * bag_len, rows - 1 if np.gcd(2654435761, rows) != 1 else rows, 1.05).reshape(bags, bag_len)
    ids = np.ascontiguousarray(ids % rows).astype(np.int32)
    want = oracle.embedding_bag_f32(table, ids)
    with Backing(table, page, 8 * page) as b:
        d_out = torch.zeros((bags, dim), dtype=torch.float32, device="cuda")
        gv.gpuvm_run_embedding_bag(b.vm, dim, dev(ids), bags, bag_len, d_out)
        gv.gpuvm_check(b.vm)
        plain = gv.gpuvm_stats(b.vm)
        assert np.array_equal(d_out.cpu().numpy(), want)
        gv.gpuvm_reset(b.vm)
        gv.gpuvm_set_remote_first(b.vm, dim * 4)
        d_out.zero_()
        gv.gpuvm_run_embedding_bag(b.vm, dim, dev(ids), bags, bag_len, d_out)
        gv.gpuvm_check(b.vm)
        assert np.array_equal(d_out.cpu().numpy(), want)                      # bit-exact, as before
        st, *_ = check_invariants(b, read_only=True, pristine=table, remote_first=True)
        assert st["remote_reads"] > 0 and st["faults"] < plain["faults"]


@pytest.mark.parametrize("scale,page,frames,src", [(14, 4096, 16, 0), (16, 65536, 8, 5), (13, 4096, 8, 77)])
def test_bfs_reads_sparse_pages_in_place(gpu, scale, page, frames, src):
    rp, ci = inputs.rmat_csr(9, scale)
    nv = 1 << scale
    want = oracle.bfs(rp, ci, src)
    with Backing(ci, page, frames * page) as b:
        d_level = torch.zeros(nv, dtype=torch.int32, device="cuda")
        gv.gpuvm_run_bfs_balanced(b.vm, dev(rp), nv, src, d_level)
        gv.gpuvm_check(b.vm)
        plain = gv.gpuvm_stats(b.vm)
        assert np.array_equal(host(d_level, np.int32), want)
        gv.gpuvm_reset(b.vm)
        gv.gpuvm_set_remote_first(b.vm, 4)
        d_level.zero_()
        levels = gv.gpuvm_run_bfs_balanced(b.vm, dev(rp), nv, src, d_level)
        gv.gpuvm_check(b.vm)
        assert levels >= 2 and np.array_equal(host(d_level, np.int32), want)
        st, *_ = check_invariants(b, read_only=True, pristine=ci, remote_first=True)
        assert st["remote_reads"] > 0 and st["faults"] <= plain["faults"]
        # connected components walk every edge in every round: nothing is sparse, results as before
        d_label = torch.zeros(nv, dtype=torch.int32, device="cuda")
        gv.gpuvm_run_cc_balanced(b.vm, dev(rp), nv, d_label)
        gv.gpuvm_check(b.vm)
        assert np.array_equal(host(d_label, np.int32), oracle.cc(rp, ci))


@pytest.mark.parametrize("scale,page,frames,src", [(14, 4096, 16, 0), (16, 65536, 8, 5)])
def test_sssp_reads_sparse_pages_of_both_arrays_in_place(gpu, scale, page, frames, src):
    rp, ci = inputs.rmat_csr(9, scale)
    w = inputs.edge_weights(4, 0, ci.size)
    nv = 1 << scale
    want = oracle.sssp(rp, ci, w, src)
    with Backing(ci, page, frames * page) as b, Backing(w, page, frames * page) as bw:
        gv.gpuvm_set_remote_first(b.vm, 4)
        d_dist = torch.zeros(nv, dtype=torch.int32, device="cuda")
        rounds = gv.gpuvm_run_sssp_balanced(b.vm, bw.vm, dev(rp), nv, src, d_dist)
        assert rounds >= 2 and np.array_equal(host(d_dist, np.uint32), want)
        st, *_ = check_invariants(b, read_only=True, pristine=ci, remote_first=True)
        check_invariants(bw, read_only=True, pristine=w)
        assert st["remote_reads"] > 0

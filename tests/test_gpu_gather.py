"""Random gather through the paged view vs the oracle (bit-exact), plus the
quiesced-state invariants.  Sizes span many tiles, ragged tails, a short last
page, heavy and light oversubscription, both policies."""
import numpy as np
import pytest
import torch

import oracle
import paper_2411_05309_amd as gv
from paper_2411_05309_amd import inputs

from gpu_util import Backing, check_invariants, dev, host

pytestmark = pytest.mark.gpu


def run_gather(b, idx, access_stats=False):
    d_idx = dev(idx)
    d_out = torch.zeros(max(idx.size, 1), dtype=torch.int32, device="cuda")
    d_sum = torch.zeros(1, dtype=torch.int64, device="cuda")
    gv.gpuvm_configure(b.vm, 0, access_stats)
    gv.gpuvm_run_gather(b.vm, d_idx, idx.size, d_out, d_sum)
    gv.gpuvm_check(b.vm)
    return host(d_out, np.uint32)[:idx.size], int(host(d_sum, np.uint64)[0])


@pytest.mark.parametrize("policy", [gv.POLICY_CLOCK, gv.POLICY_FIFO, gv.POLICY_FIFO_WAIT, gv.POLICY_GCLOCK])
@pytest.mark.parametrize("n_elems,page,frames,n_idx", [
    (1 << 18, 4096, 64, 1 << 15),          # 256 pages over 64 frames
    ((1 << 18) + 1000, 4096, 16, 10007),   # short last page, ragged index count
    (1 << 16, 4096, 64, 4096),             # everything fits: compulsory misses only
    (1 << 20, 65536, 8, 70001),            # 64 KiB pages, tiny pool
    (1 << 23, 1 << 20, 8, 20011),          # the largest page size (1 MiB), the smallest pool
])
def test_gather_matches_oracle(gpu, policy, n_elems, page, frames, n_idx):
    data = inputs.u32_values(1, 0, n_elems)
    idx = (inputs.u32_indices(2, 0, n_idx, 1 << 30) % n_elems).astype(np.uint32)
    idx[-1] = n_elems - 1                                   # touch the very last element
    want, want_sum = oracle.gather(data, idx)
    with Backing(data, page, frames * page, policy) as b:
        got, got_sum = run_gather(b, idx, access_stats=True)
        assert np.array_equal(got, want)
        assert got_sum == want_sum
        st, f, owner, hand = check_invariants(b, read_only=True, pristine=data)
        distinct = len(np.unique(idx.astype(np.int64) * 4 // page))
        assert st["faults"] >= distinct
        if distinct <= frames:
            assert st["faults"] == distinct and st["evictions"] == 0
        if policy == gv.POLICY_FIFO_WAIT:
            assert st["alloc_skips"] == 0 and st["alloc_sweeps"] == 0   # frames are taken strictly in ring order
        # dedup bookkeeping: every lane is either a group of its own or rides on one
        assert st["wave_page_groups"] + st["lanes_coalesced"] == n_idx
        # every group either found its page resident (at once or after waiting) or faulted
        assert st["hits"] + st["faults"] == st["wave_page_groups"]
        # a second run on the warm pool gives the same answer
        got2, _ = run_gather(b, idx)
        assert np.array_equal(got2, want)
        check_invariants(b, read_only=True, pristine=data)


def test_gather_degenerate_patterns(gpu):
    n_elems, page = 1 << 16, 4096
    data = inputs.u32_values(3, 0, n_elems)
    with Backing(data, page, 8 * page) as b:
        for name, idx in {
            "all lanes same element": np.full(1000, 12345, np.uint32),
            "all lanes same page": (np.arange(5000) % 1024 + 2048).astype(np.uint32),
            "every lane a different page": ((np.arange(4096) * 1024 + np.arange(4096) % 7) % n_elems).astype(np.uint32),
            "single access": np.array([n_elems - 1], np.uint32),
            "partial wavefront": np.arange(37, dtype=np.uint32) * 999 % n_elems,
        }.items():
            want, want_sum = oracle.gather(data, idx)
            got, got_sum = run_gather(b, idx)
            assert np.array_equal(got, want), name
            assert got_sum == want_sum, name
        check_invariants(b, read_only=True, pristine=data)
        gv.gpuvm_run_gather(b.vm, None, 0, None, None)           # empty input is a no-op


def test_gather_full_size_config(gpu):
    """The headline configuration: 64 MiB uint32 array, 4 KiB pages, 16 MiB pool
    (4x oversubscribed), 2^20 uniform indices - in the launch shape bench.py times."""
    n_elems, n_idx, page, pool = 1 << 24, 1 << 20, 4096, 16 << 20
    data = inputs.u32_values(0x9E3779B9, 0, n_elems)
    idx = inputs.u32_indices(1, 0, n_idx, n_elems)
    want, want_sum = oracle.gather(data, idx)
    with Backing(data, page, pool) as b:
        assert gv.gpuvm_max_waves(b.vm) <= (pool // page) // 2
        got, got_sum = run_gather(b, idx)
        assert np.array_equal(got, want)
        assert got_sum == want_sum
        st, *_ = check_invariants(b, read_only=True, pristine=data)
        # independent-reference model: steady hit ratio ~ frames/pages = 1/4
        assert 0.4 * n_idx < st["faults"] <= n_idx   # sanity band: ~3/4 miss minus in-flight coalescing across waves
        gv.gpuvm_reset(b.vm)
        st0 = gv.gpuvm_stats(b.vm)
        assert st0["faults"] == 0
        got, got_sum = run_gather(b, idx)
        assert np.array_equal(got, want) and got_sum == want_sum


def test_errors_are_reported_not_fatal(gpu):
    data = inputs.u32_values(5, 0, 1 << 14)
    with pytest.raises(gv.GpuvmError) as e:                     # plain numpy memory is not pinned
        gv.gpuvm_create(data.ctypes.data, data.nbytes, 4096, 8 * 4096, gv.POLICY_CLOCK)
    assert e.value.code == gv.EPIN
    with Backing(data, 4096, 8 * 4096) as b:
        for bad in [dict(page_bytes=3000), dict(page_bytes=2048), dict(frame_pool_bytes=4096), dict(policy=7)]:
            kw = dict(page_bytes=4096, frame_pool_bytes=8 * 4096, policy=gv.POLICY_CLOCK)
            kw.update(bad)
            with pytest.raises(gv.GpuvmError) as e:
                gv.gpuvm_create(b.arr.ctypes.data, b.arr.nbytes, kw["page_bytes"], kw["frame_pool_bytes"], kw["policy"])
            assert e.value.code == gv.EINVAL
        idx = np.array([1, 2, 1 << 14, 3], np.uint32)            # one index out of range
        d_idx, d_out = dev(idx), torch.zeros(4, dtype=torch.int32, device="cuda")
        gv.gpuvm_run_gather(b.vm, d_idx, 4, d_out, None)
        with pytest.raises(gv.GpuvmError) as e:
            gv.gpuvm_check(b.vm)
        assert e.value.code == gv.ERANGE
        gv.gpuvm_reset(b.vm)                                     # clears the recorded error
        gv.gpuvm_check(b.vm)
    with Backing(data, 4096, 2 * 4096) as b:                     # 2 frames: no wave may run
        d_idx, d_out = dev(idx[:2]), torch.zeros(2, dtype=torch.int32, device="cuda")
        with pytest.raises(gv.GpuvmError) as e:
            gv.gpuvm_run_gather(b.vm, d_idx, 2, d_out, None)
        assert e.value.code == gv.EDEADLK


def test_bounded_waits_drain_and_report(gpu):
    """Failure handling forced from the host: with a spin limit of 1 a wave that
    has to wait for another wave's fault gives up at once, records
    GPUVM_EDEADLK and every kernel still runs to its end; after a reset the
    handle works again."""
    n_elems, page = 1 << 18, 4096
    data = inputs.u32_values(8, 0, n_elems)
    # many waves, few pages, small pool: pages are constantly LOADING / EVICTING
    idx = ((np.arange(1 << 16) * 1024) % n_elems).astype(np.uint32)
    want, _ = oracle.gather(data, idx)
    with Backing(data, page, 16 * page) as b:
        gv.gpuvm_configure(b.vm, 1, True)
        d_idx, d_out = dev(idx), torch.zeros(idx.size, dtype=torch.int32, device="cuda")
        gv.gpuvm_run_gather(b.vm, d_idx, idx.size, d_out, None)
        torch.cuda.synchronize()                                  # the kernel drained
        st_err = None
        try:
            gv.gpuvm_check(b.vm)
        except gv.GpuvmError as e:
            st_err = e.code
        assert st_err in (None, gv.EDEADLK)
        if st_err is None:                                        # nobody had to wait: result must be right
            assert np.array_equal(host(d_out, np.uint32), want)
        gv.gpuvm_reset(b.vm)
        gv.gpuvm_configure(b.vm, 0, False)
        got, _ = run_gather(b, idx)
        assert np.array_equal(got, want)
        check_invariants(b, read_only=True, pristine=data)


def test_prefetch_makes_a_range_resident(gpu):
    n_elems, page, frames = 1 << 18, 4096, 64
    data = inputs.u32_values(5, 0, n_elems)
    with Backing(data, page, frames * page) as b:
        gv.gpuvm_run_prefetch(b.vm, 100, 40)
        gv.gpuvm_check(b.vm)
        st, f, *_ = check_invariants(b, read_only=True, pristine=data)
        assert st["faults"] == 40 and st["evictions"] == 0
        assert np.all(f["state"][100:140] == gv.ST_RESIDENT)
        assert np.count_nonzero(f["state"] == gv.ST_RESIDENT) == 40
        # a gather inside the range finds everything in place
        idx = (100 * 1024 + inputs.u32_indices(6, 0, 5000, 1 << 20) % (40 * 1024)).astype(np.uint32)
        want, want_sum = oracle.gather(data, idx)
        got, got_sum = run_gather(b, idx)
        assert np.array_equal(got, want) and got_sum == want_sum
        assert gv.gpuvm_stats(b.vm)["faults"] == 40
        # prefetching it again moves nothing; a range beyond the pool turns the pool over
        gv.gpuvm_run_prefetch(b.vm, 100, 40)
        gv.gpuvm_check(b.vm)
        assert gv.gpuvm_stats(b.vm)["faults"] == 40
        gv.gpuvm_run_prefetch(b.vm, 0, b.n_pages)
        gv.gpuvm_check(b.vm)
        st, f, *_ = check_invariants(b, read_only=True, pristine=data)
        assert np.count_nonzero(f["state"] == gv.ST_RESIDENT) == frames
        gv.gpuvm_run_prefetch(b.vm, b.n_pages, 0)                       # empty range at the end: fine
        for first, count in ((b.n_pages, 1), (0, b.n_pages + 1), (b.n_pages + 1, 0)):
            with pytest.raises(gv.GpuvmError) as e:
                gv.gpuvm_run_prefetch(b.vm, first, count)
            assert e.value.code == gv.ERANGE

"""The accessors under divergence: only the lanes whose mask byte is set enter
gpuvm_load / gpuvm_atomic_add, so faults are taken and pages are moved by
whatever lanes are active, down to a single one, and the last wave of a launch
is partial.  Data sets end in a page whose length is not a multiple of 16
bytes, which a wave with few active lanes has to copy completely too."""
import numpy as np
import pytest
import torch

import oracle
import paper_2411_05309_amd as gv
from paper_2411_05309_amd import inputs

from gpu_util import Backing, check_invariants, dev, host

pytestmark = pytest.mark.gpu


def _masks(n, seed):
    u = inputs.u32_indices(seed, 0, n, 1 << 16)
    k = np.arange(n)
    return {
        "one lane in a hundred": (u % 100 == 0),
        "half of the lanes": (u % 2 == 0),
        "all lanes": np.ones(n, bool),
        "lane 5 of every wave": (k % 64 == 5),
        "first lanes of every fourth wave": ((k % 256) < 3),
        "nobody": np.zeros(n, bool),
    }


@pytest.mark.parametrize("policy", [gv.POLICY_CLOCK, gv.POLICY_FIFO_WAIT])
@pytest.mark.parametrize("n_elems,page,frames,n_idx", [
    ((1 << 16) + 1, 4096, 16, 20011),      # last page: 4 bytes
    ((1 << 17) + 3, 65536, 8, 9001),       # last page: 12 bytes, 64 KiB pages
])
def test_masked_gather(gpu, policy, n_elems, page, frames, n_idx):
    data = inputs.u32_values(21, 0, n_elems)
    idx = (inputs.u32_indices(22, 0, n_idx, 1 << 30) % n_elems).astype(np.uint32)
    for name, m in _masks(n_idx, 23).items():
        idx2 = idx.copy()
        if m.any():
            idx2[np.nonzero(m)[0][-1]] = n_elems - 1                 # the element in the odd tail of the last page
        with Backing(data, page, frames * page, policy) as b:
            d_out = torch.full((n_idx,), -7, dtype=torch.int32, device="cuda")
            gv.gpuvm_run_gather_masked(b.vm, dev(idx2), dev(m.astype(np.uint8)), n_idx, d_out)
            gv.gpuvm_check(b.vm)
            got = host(d_out, np.uint32)
            want, _ = oracle.gather(data, np.ascontiguousarray(idx2[m]))
            assert np.array_equal(got[m], want), name
            assert np.all(got[~m] == np.uint32(0xFFFFFFF9)), name       # untouched
            st, *_ = check_invariants(b, read_only=True, pristine=data)
            assert (st["faults"] > 0) == bool(m.any())


@pytest.mark.parametrize("policy", [gv.POLICY_CLOCK, gv.POLICY_FIFO, gv.POLICY_CLOCK_WRITE_AWARE])
@pytest.mark.parametrize("n64,page,frames,n_upd", [
    ((1 << 15) + 1, 4096, 16, 30011),      # last page: 8 bytes; dirty evictions
    ((1 << 16) + 1, 65536, 8, 12001),
])
def test_masked_increment(gpu, policy, n64, page, frames, n_upd):
    idx = ((inputs.zipf_ranks(24, 0, n_upd, n64, 0.9) - 1) * 40503 % n64).astype(np.uint32)
    for name, m in _masks(n_upd, 25).items():
        idx2 = idx.copy()
        if m.any():
            idx2[np.nonzero(m)[0][0]] = n64 - 1
        want = np.zeros(n64, np.uint64)
        oracle.scatter_increment(want, np.ascontiguousarray(idx2[m]))
        with Backing(np.zeros(n64, np.uint64), page, frames * page, policy) as b:
            gv.gpuvm_run_scatter_increment_masked(b.vm, dev(idx2), dev(m.astype(np.uint8)), n_upd)
            gv.gpuvm_check(b.vm)
            check_invariants(b, read_only=False)
            gv.gpuvm_flush(b.vm)
            assert np.array_equal(b.arr, want), name
            assert int(b.arr.sum()) == int(m.sum())


def test_masked_launchers_report_bad_indices(gpu):
    data = inputs.u32_values(21, 0, 1 << 14)
    with Backing(data, 4096, 8 * 4096) as b:
        idx = np.array([5, 1 << 14, 7], np.uint32)                      # the middle one is out of range ...
        d_out = torch.zeros(3, dtype=torch.int32, device="cuda")
        gv.gpuvm_run_gather_masked(b.vm, dev(idx), dev(np.array([1, 0, 1], np.uint8)), 3, d_out)
        gv.gpuvm_check(b.vm)                                            # ... but masked out: fine
        gv.gpuvm_run_gather_masked(b.vm, dev(idx), dev(np.array([1, 1, 1], np.uint8)), 3, d_out)
        with pytest.raises(gv.GpuvmError) as e:
            gv.gpuvm_check(b.vm)
        assert e.value.code == gv.ERANGE

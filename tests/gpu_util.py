"""Helpers shared by the GPU parity tests: device buffers (torch = plumbing),
pinned backing stores, and the invariants read back from the device tables."""
import numpy as np
import torch

import paper_2411_05309_amd as gv


def dev(arr):
    """numpy -> device tensor with the same bits (uint32/uint64 as int32/int64)."""
    a = np.ascontiguousarray(arr)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    elif a.dtype == np.uint64:
        a = a.view(np.int64)
    return torch.from_numpy(a).cuda()


def host(t, dtype):
    return t.cpu().numpy().view(dtype)


class Backing:
    """Pinned host array + a gpuvm handle over it."""

    def __init__(self, data, page_bytes, frame_pool_bytes, policy=gv.POLICY_CLOCK):
        self.arr = gv.pinned_array(data.shape, data.dtype)
        self.arr[...] = data
        self.vm = gv.gpuvm_create(self.arr.ctypes.data, self.arr.nbytes, page_bytes, frame_pool_bytes, policy)
        self.page_bytes = page_bytes
        self.n_frames = frame_pool_bytes // page_bytes
        self.n_pages = -(-self.arr.nbytes // page_bytes)

    def close(self):
        if self.vm:
            gv.gpuvm_destroy(self.vm)
            self.vm = None
            gv.free_pinned(self.arr)

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def check_invariants(b, read_only=True, pristine=None, remote_first=False):
    """Quiesced-state invariants of the page table / frame table / counters."""
    gv.gpuvm_check(b.vm)
    pte, owner, hand = gv.gpuvm_dump_tables(b.vm)
    st = gv.gpuvm_stats(b.vm)
    f = gv.decode_pte(pte)
    assert np.all(f["pin"] == 0), "a reference count is left over"
    assert np.all((f["state"] == gv.ST_INVALID) | (f["state"] == gv.ST_RESIDENT)), "LOADING/EVICTING left over"
    res = np.nonzero(f["state"] == gv.ST_RESIDENT)[0]
    assert len(res) <= b.n_frames
    frames = f["frame"][res]
    assert np.all(frames < b.n_frames)
    assert len(np.unique(frames)) == len(res), "two pages share a frame"
    assert np.all(owner[frames] == res), "frame table and page table disagree"
    inv = f["state"] == gv.ST_INVALID
    # (in remote-first mode the frame bits of an INVALID entry count its reads in place)
    keep = np.uint64(gv.PTE_GEN_MASK) | (np.uint64((1 << 64) - (1 << gv.PTE_FRAME_SHIFT)) if remote_first else np.uint64(0))
    assert np.all((pte[inv] & ~keep) == 0), "stale bits on an INVALID entry"
    # a page's install generation counts its faults (mod 4096)
    if st["faults"] < 4096:                      # no single page can have wrapped
        assert int(f["gen"].sum()) == st["faults"]
    assert st["faults"] - st["evictions"] == len(res)
    assert st["writebacks_evict"] <= st["evictions"]
    last_len = b.arr.nbytes - (b.n_pages - 1) * b.page_bytes
    fetched = st["faults"] - st["faults_no_fetch"]          # pages installed for a full overwrite are not read
    assert fetched >= 0
    if last_len == b.page_bytes:
        assert st["bytes_in"] == fetched * b.page_bytes
    else:
        assert fetched * b.page_bytes - (b.page_bytes - last_len) * fetched <= st["bytes_in"] <= fetched * b.page_bytes
    if read_only:
        assert st["writebacks_evict"] == 0 and st["writebacks_flush"] == 0 and st["bytes_out"] == 0
        assert not np.any(f["dirty"])
        if pristine is not None:
            assert np.array_equal(b.arr, pristine), "a read-only run changed host memory"
    return st, f, owner, hand

"""gpuvm_create_in: pool and tables carved out of a device allocation the caller
owns (here a torch tensor) behave exactly like the ones gpuvm_create allocates -
the same deterministic replay, the same free-running results and invariants -
and nothing is written outside the stated number of bytes."""
import numpy as np
import pytest
import torch

import oracle
import paper_2411_05309_amd as gv
from paper_2411_05309_amd import inputs

from gpu_util import Backing, check_invariants, dev, host

pytestmark = pytest.mark.gpu


class CarvedBacking(Backing):
    """A Backing whose handle lives in a caller-owned torch tensor, with a canary behind it."""

    def __init__(self, data, page_bytes, frame_pool_bytes, policy=gv.POLICY_CLOCK, canary=4096):
        self.arr = gv.pinned_array(data.shape, data.dtype)
        self.arr[...] = data
        self.need = gv.gpuvm_workspace_bytes(self.arr.nbytes, page_bytes, frame_pool_bytes)
        assert self.need >= frame_pool_bytes // page_bytes * page_bytes + 8 * -(-self.arr.nbytes // page_bytes)
        self.ws = torch.full((self.need + canary,), 0x5A, dtype=torch.uint8, device="cuda")
        assert self.ws.data_ptr() % 256 == 0
        self.vm = gv.gpuvm_create_in(self.arr.ctypes.data, self.arr.nbytes, page_bytes, frame_pool_bytes, policy,
                                     self.ws, self.need)
        self.page_bytes = page_bytes
        self.n_frames = frame_pool_bytes // page_bytes
        self.n_pages = -(-self.arr.nbytes // page_bytes)

    def canary_intact(self):
        return bool(torch.all(self.ws[self.need:] == 0x5A).item())


def test_workspace_size_and_refusals(gpu):
    assert gv.gpuvm_workspace_bytes(1 << 20, 3000, 1 << 16) == 0              # page size not a power of two
    assert gv.gpuvm_workspace_bytes(1 << 20, 4096, 4096) == 0                  # fewer than two frames
    assert gv.gpuvm_workspace_bytes(0, 4096, 1 << 16) == 0
    need = gv.gpuvm_workspace_bytes(1 << 20, 4096, 16 * 4096)
    assert 16 * 4096 + 256 * 8 + 16 * 4 <= need <= 16 * 4096 + 256 * 8 + 16 * 4 + 16 * 8 * 64 + 8 * 256
    data = inputs.u32_values(1, 0, 1 << 18)
    arr = gv.pinned_array(data.shape, data.dtype)
    try:
        ws = torch.zeros(need + 512, dtype=torch.uint8, device="cuda")
        for bad_ws, bad_len in ((ws[1:], need), (ws, need - 1), (None, need)):
            with pytest.raises(gv.GpuvmError) as e:
                gv.gpuvm_create_in(arr.ctypes.data, arr.nbytes, 4096, 16 * 4096, gv.POLICY_CLOCK, bad_ws, bad_len)
            assert e.value.code == gv.EINVAL
        with pytest.raises(gv.GpuvmError) as e:                                # host memory is no workspace
            gv.gpuvm_create_in(arr.ctypes.data, arr.nbytes, 4096, 16 * 4096, gv.POLICY_CLOCK, arr.ctypes.data, need)
        assert e.value.code == gv.EINVAL
    finally:
        gv.free_pinned(arr)


@pytest.mark.parametrize("policy", [gv.POLICY_CLOCK, gv.POLICY_FIFO])
def test_carved_handle_replays_like_an_allocated_one(gpu, policy):
    n_elems, page, frames, n_idx, phase_len = (1 << 16) + 100, 4096, 16, 6007, 7
    data = inputs.u32_values(1, 0, n_elems)
    r = inputs.zipf_ranks(4, 0, n_idx, n_elems, 1.2) - 1
    idx = ((r * 2654435761) % n_elems).astype(np.uint32)
    want, want_sum = oracle.gather(data, idx)
    results = []
    for cls in (Backing, CarvedBacking):
        with cls(data, page, frames * page, policy) as b:
            d_out = torch.zeros(n_idx, dtype=torch.int32, device="cuda")
            d_sum = torch.zeros(1, dtype=torch.int64, device="cuda")
            gv.gpuvm_run_gather_phased(b.vm, dev(idx), n_idx, phase_len, d_out, d_sum)
            assert np.array_equal(host(d_out, np.uint32), want) and int(host(d_sum, np.uint64)[0]) == want_sum
            st, f, owner, hand = check_invariants(b, read_only=True, pristine=data)
            results.append((st, owner.copy(), hand))
            if cls is CarvedBacking:
                assert b.canary_intact()
    (st_a, owner_a, hand_a), (st_c, owner_c, hand_c) = results
    assert st_a == st_c and np.array_equal(owner_a, owner_c) and hand_a == hand_c
    spread = frames // 2 if policy == gv.POLICY_CLOCK else 0
    sim = oracle.PagingSim(page // 8, frames, oracle.CLOCK if policy == gv.POLICY_CLOCK else oracle.FIFO,
                           n_words=-(-data.nbytes // 8), spread=spread)
    sim.run((idx.astype(np.uint64) * 4) // 8, phase_len=phase_len)
    assert st_c["faults"] == sim.counters["faults"] and st_c["evictions"] == sim.counters["evictions"]


def test_carved_handle_free_running_and_lifetime(gpu):
    n64, page, frames, n_upd = 1 << 15, 4096, 16, 40000
    idx = ((inputs.zipf_ranks(6, 0, n_upd, n64, 0.9) - 1) * 40503 % n64).astype(np.uint32)
    want = np.zeros(n64, np.uint64)
    oracle.scatter_increment(want, idx)
    b = CarvedBacking(np.zeros(n64, np.uint64), page, frames * page)
    try:
        gv.gpuvm_run_scatter_increment(b.vm, dev(idx), n_upd)
        st, *_ = check_invariants(b, read_only=False)
        assert st["writebacks_evict"] > 0
        gv.gpuvm_flush(b.vm)
        assert np.array_equal(b.arr, want)
        ridx = inputs.u32_indices(9, 0, 5000, n64 * 2)
        d_out = torch.zeros(5000, dtype=torch.int32, device="cuda")
        gv.gpuvm_run_gather(b.vm, dev(ridx), 5000, d_out, None)             # the same handle read as uint32 words
        gv.gpuvm_check(b.vm)
        assert np.array_equal(host(d_out, np.uint32), oracle.gather(want.view(np.uint32), ridx)[0])
        gv.gpuvm_reset(b.vm)
        assert b.canary_intact()
    finally:
        ws = b.ws
        b.close()
    ws.fill_(7)                                                              # destroy left the caller's memory alone
    torch.cuda.synchronize()
    assert int(ws[0].item()) == 7

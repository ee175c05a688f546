"""Model-based test of the free-running path: a seeded random sequence of
gathers, increments, fault-ahead requests, flushes and resets on ONE paged
array with a small pool, under every policy and both write-back orders.  The
model is the definition on plain memory (the oracle's gather and histogram on a
numpy array); after every flush the pinned host array must equal it, every
gather must return the model's values, and the tables must satisfy the
quiesced-state invariants."""
import numpy as np
import pytest
import torch

import oracle
import paper_2411_05309_amd as gv
from paper_2411_05309_amd import inputs

from gpu_util import Backing, check_invariants, dev, host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("wb_mode,remote_bytes", [(gv.WB_SERIAL, 0), (gv.WB_OVERLAPPED, 0), (gv.WB_SERIAL, 4), (gv.WB_SERIAL, 1024)])
@pytest.mark.parametrize("policy", [gv.POLICY_CLOCK, gv.POLICY_FIFO, gv.POLICY_FIFO_WAIT, gv.POLICY_CLOCK_WRITE_AWARE, gv.POLICY_GCLOCK])
@pytest.mark.parametrize("n64,page,frames,seed", [
    ((1 << 16) + 37, 4096, 24, 1),       # 129 pages (the last one short) over 24 frames
    (1 << 17, 65536, 8, 2),              # 16 pages of 64 KiB over the smallest pool
    ((1 << 18) + 5, 4096, 256, 3),       # 513 pages over 256 frames: 128 waves, every wave with many pages per access
])
def test_random_operation_sequence_matches_the_model(gpu, policy, wb_mode, remote_bytes, n64, page, frames, seed):
    model = inputs.u32_values(seed, 0, 2 * n64).view(np.uint64).copy()      # arbitrary initial content
    n_pages = -(-model.nbytes // page)
    pick = inputs.u32_indices(100 + seed, 0, 64, 1 << 16)                   # the op sequence, seeded
    with Backing(model, page, frames * page, policy) as b:
        gv.gpuvm_set_writeback_mode(b.vm, wb_mode)
        gv.gpuvm_set_remote_first(b.vm, remote_bytes)           # reads that miss may be served in place
        dirty_since_flush = False
        for step, r in enumerate(pick):
            op = int(r) % 8
            n = 200 + int(r >> 3) % 3000
            if op <= 2:                                                     # gather uint32 words
                idx = inputs.u32_indices(1000 + step, seed, n, 1 << 30) % np.uint32(2 * n64)
                idx = idx.astype(np.uint32)
                want, want_sum = oracle.gather(model.view(np.uint32), idx)
                d_out = torch.zeros(n, dtype=torch.int32, device="cuda")
                d_sum = torch.zeros(1, dtype=torch.int64, device="cuda")
                gv.gpuvm_run_gather(b.vm, dev(idx), n, d_out, d_sum)
                gv.gpuvm_check(b.vm)
                assert np.array_equal(host(d_out, np.uint32), want), (step, "gather")
                assert int(host(d_sum, np.uint64)[0]) == want_sum
            elif op <= 5:                                                   # increments of uint64 elements
                idx = (inputs.zipf_ranks(2000 + step, seed, n, n64, 0.9) - 1).astype(np.uint64)
                idx = ((idx * 40503) % n64).astype(np.uint32)
                oracle.scatter_increment(model, idx)
                gv.gpuvm_run_scatter_increment(b.vm, dev(idx), n)
                dirty_since_flush = True
            elif op == 6:                                                   # fault-ahead of a page range
                first = int(r >> 8) % n_pages
                gv.gpuvm_run_prefetch(b.vm, first, min(frames // 2, n_pages - first))
            else:                                                           # flush or reset: host memory catches up
                (gv.gpuvm_reset if (r >> 8) & 1 else gv.gpuvm_flush)(b.vm)
                assert np.array_equal(b.arr, model), (step, "host array after flush")
                dirty_since_flush = False
            if step % 8 == 7:
                st, f, *_ = check_invariants(b, read_only=False, remote_first=remote_bytes > 0)
                if not dirty_since_flush:
                    assert not np.any(f["dirty"])
        gv.gpuvm_flush(b.vm)
        st, *_ = check_invariants(b, read_only=False, remote_first=remote_bytes > 0)
        assert (st["remote_reads"] > 0) == (remote_bytes > 0)
        assert np.array_equal(b.arr, model)

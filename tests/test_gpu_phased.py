"""Deterministic barrier-phased mode: fault / hit / eviction / write-back
counts, ring cursor and the final frame table must equal the oracle's
sequential FIFO / CLOCK replay, and the application output its definition."""
import numpy as np
import pytest
import torch

import oracle
import paper_2411_05309_amd as gv
from paper_2411_05309_amd import inputs

from gpu_util import Backing, check_invariants, dev, host

pytestmark = pytest.mark.gpu

_POL = {gv.POLICY_FIFO: oracle.FIFO, gv.POLICY_CLOCK: oracle.CLOCK, gv.POLICY_CLOCK_WRITE_AWARE: oracle.CLOCK_WA,
        gv.POLICY_GCLOCK: oracle.GCLOCK}


# (policy, hands): hands = e puts the CLOCK policies' front hand frames * e / 8 ahead of the cursor, 0 = one hand
_CASES = [(gv.POLICY_CLOCK, 4), (gv.POLICY_CLOCK, 0), (gv.POLICY_CLOCK, 7), (gv.POLICY_CLOCK, 1), (gv.POLICY_FIFO, 0),
          (gv.POLICY_GCLOCK, 0)]
_CASES_W = _CASES + [(gv.POLICY_CLOCK_WRITE_AWARE, 4), (gv.POLICY_CLOCK_WRITE_AWARE, 0)]


def _spread(policy, frames, hands):
    return frames * hands // 8 if policy in (gv.POLICY_CLOCK, gv.POLICY_CLOCK_WRITE_AWARE) else 0


def _set_hands(b, policy, frames, hands):
    if policy in (gv.POLICY_CLOCK, gv.POLICY_CLOCK_WRITE_AWARE):
        if hands != 4:
            gv.gpuvm_set_clock_hands(b.vm, hands)              # 4 is the default
    else:
        with pytest.raises(gv.GpuvmError):
            gv.gpuvm_set_clock_hands(b.vm, 4)                  # no reference bit, no front hand
    assert gv.clock_spread(b.vm) == _spread(policy, frames, hands)


def _compare_with_replay(b, sim, frames):
    st, f, owner, hand = check_invariants(b, read_only=False)
    c = sim.counters
    for gpu_name, sim_name in [("faults", "faults"), ("hits", "hits"), ("evictions", "evictions"),
                               ("writebacks_evict", "writebacks_evict"), ("alloc_skips", "skips"),
                               ("alloc_sweeps", "sweeps"), ("phases", "phases")]:
        assert st[gpu_name] == c[sim_name], (gpu_name, st, c)
    s = sim.state()
    want_owner = np.where(s["owner"] < 0, gv.NO_PAGE, s["owner"]).astype(np.uint32)
    assert np.array_equal(owner, want_owner)
    assert hand % frames == sim.hand
    res = np.nonzero(f["state"] == gv.ST_RESIDENT)[0]
    assert np.array_equal(f["frame"][res], s["where"][res])
    assert np.array_equal(f["dirty"][res], s["dirty"][s["where"][res]])
    assert np.array_equal(f["ref"][res], s["ref"][s["where"][res]])
    assert np.array_equal(f["defer"][res], s["defer"][s["where"][res]])
    return st


@pytest.mark.parametrize("policy,hands", _CASES)
@pytest.mark.parametrize("n_elems,page,frames,n_idx,phase_len", [
    (1 << 18, 4096, 64, 20000, 48),        # 256 pages over 64 frames, phases pin most of the pool
    ((1 << 16) + 100, 4096, 16, 5003, 7),  # short last page, ragged last phase
    (1 << 16, 4096, 128, 4000, 64),        # fits
    (1 << 20, 4096, 256, 30000, 200),
])
def test_gather_phased_equals_sequential_replay(gpu, policy, hands, n_elems, page, frames, n_idx, phase_len):
    data = inputs.u32_values(1, 0, n_elems)
    # skewed indices so that CLOCK and FIFO differ and pinned frames are passed over
    r = inputs.zipf_ranks(4, 0, n_idx, n_elems, 1.2) - 1
    idx = ((r * 2654435761) % n_elems).astype(np.uint32)
    want, want_sum = oracle.gather(data, idx)
    sim = oracle.PagingSim(page // 8, frames, _POL[policy], n_words=-(-data.nbytes // 8), spread=_spread(policy, frames, hands))
    sim.run((idx.astype(np.uint64) * 4) // 8, phase_len=phase_len)
    with Backing(data, page, frames * page, policy) as b:
        _set_hands(b, policy, frames, hands)
        d_idx = dev(idx)
        d_out = torch.zeros(n_idx, dtype=torch.int32, device="cuda")
        d_sum = torch.zeros(1, dtype=torch.int64, device="cuda")
        gv.gpuvm_run_gather_phased(b.vm, d_idx, n_idx, phase_len, d_out, d_sum)
        assert np.array_equal(host(d_out, np.uint32), want)
        assert int(host(d_sum, np.uint64)[0]) == want_sum
        st = _compare_with_replay(b, sim, frames)
        assert st["writebacks_evict"] == 0
        assert np.array_equal(b.arr, data)


@pytest.mark.parametrize("policy,hands", _CASES)
def test_embedding_shaped_page_sequence_equals_sequential_replay(gpu, policy, hands):
    """The embedding-bag configuration at reduced scale in deterministic mode: the
    page sequence of its row reads (scrambled Zipf(1.05) ids, 512-byte rows, 128
    rows per 64 KiB page, pool a quarter of the table, one bag of 32 rows per
    phase) goes through the phased gather as one word per row; fault, hit and
    eviction counts and the final frame table equal the sequential replay."""
    rows, dim, page, bags, bag_len = 50_001, 128, 65536, 600, 32
    table = inputs.f32_uniform(11, 0, rows * dim)
    frames = (table.nbytes // 4) // page
    ids = inputs.bag_row_ids(5, 0, bags * bag_len, rows, 1.05)
    idx = (ids.astype(np.uint64) * dim).astype(np.uint32)                   # first word of each row
    data = table.view(np.uint32)
    want, want_sum = oracle.gather(data, idx)
    sim = oracle.PagingSim(page // 8, frames, _POL[policy], n_words=-(-data.nbytes // 8), spread=_spread(policy, frames, hands))
    sim.run((idx.astype(np.uint64) * 4) // 8, phase_len=bag_len)
    with Backing(data, page, frames * page, policy) as b:
        _set_hands(b, policy, frames, hands)
        d_out = torch.zeros(idx.size, dtype=torch.int32, device="cuda")
        gv.gpuvm_run_gather_phased(b.vm, dev(idx), idx.size, bag_len, d_out, None)
        assert np.array_equal(host(d_out, np.uint32), want)
        st = _compare_with_replay(b, sim, frames)
        assert st["phases"] == bags and st["evictions"] > 0 and st["hits"] > 0


@pytest.mark.parametrize("wb_mode", [gv.WB_OVERLAPPED, gv.WB_SERIAL])
@pytest.mark.parametrize("policy,hands", _CASES_W)
@pytest.mark.parametrize("n_elems,page,frames,n_upd,phase_len", [
    (1 << 15, 4096, 16, 20000, 12),
    ((1 << 14) + 9, 4096, 8, 6001, 5),
])
def test_scatter_phased_equals_sequential_replay(gpu, policy, hands, n_elems, page, frames, n_upd, phase_len, wb_mode):
    r = inputs.zipf_ranks(6, 0, n_upd, n_elems, 0.9) - 1
    idx = ((r * 40503) % n_elems).astype(np.uint32)
    want = np.zeros(n_elems, np.uint64)
    sim = oracle.PagingSim(page // 8, frames, _POL[policy], host=want, spread=_spread(policy, frames, hands))
    sim.run(idx.astype(np.uint64), op=oracle.ADD, val=1, phase_len=phase_len)
    with Backing(np.zeros(n_elems, np.uint64), page, frames * page, policy) as b:
        _set_hands(b, policy, frames, hands)
        gv.gpuvm_set_writeback_mode(b.vm, wb_mode)
        gv.gpuvm_run_scatter_increment_phased(b.vm, dev(idx), n_upd, phase_len)
        st = _compare_with_replay(b, sim, frames)
        assert st["writebacks_evict"] > 0
        gv.gpuvm_flush(b.vm)
        sim.flush()
        assert gv.gpuvm_stats(b.vm)["writebacks_flush"] == sim.counters["writebacks_flush"]
        assert np.array_equal(b.arr, want)
        direct = np.zeros(n_elems, np.uint64)
        oracle.scatter_increment(direct, idx)
        assert np.array_equal(b.arr, direct)


def test_phased_mode_refuses_the_waiting_policy(gpu):
    data = inputs.u32_values(1, 0, 1 << 16)
    with Backing(data, 4096, 8 * 4096, gv.POLICY_FIFO_WAIT) as b:
        d_out = torch.zeros(8, dtype=torch.int32, device="cuda")
        with pytest.raises(gv.GpuvmError) as e:
            gv.gpuvm_run_gather_phased(b.vm, dev(np.arange(8, dtype=np.uint32)), 8, 4, d_out, None)
        assert e.value.code == gv.EINVAL


def test_phase_with_more_pages_than_frames_is_refused(gpu):
    data = inputs.u32_values(1, 0, 1 << 16)
    with Backing(data, 4096, 8 * 4096) as b:
        idx = (np.arange(32, dtype=np.uint32) * 1024)            # 32 distinct pages, 8 frames
        d_out = torch.zeros(32, dtype=torch.int32, device="cuda")
        with pytest.raises(gv.GpuvmError) as e:
            gv.gpuvm_run_gather_phased(b.vm, dev(idx), 32, 32, d_out, None)
        assert e.value.code == gv.EDEADLK


def test_refused_phase_leaves_the_data_alone(gpu):
    """A deterministic scatter whose second phase touches more pages than there are
    frames: the launch reports GPUVM_EDEADLK, the refused phase and every later one
    change nothing (no update lands in some other page's frame), and after a
    reset the host array holds exactly the first phase's increments."""
    n64, page, frames, phase_len = 1 << 15, 4096, 8, 32
    per_page = page // 8
    good = (np.arange(phase_len, dtype=np.uint32) % 4) * per_page + 5       # 4 pages
    wide = np.arange(phase_len, dtype=np.uint32) * per_page + 9             # 32 pages > 8 frames
    idx = np.concatenate([good, wide, good]).astype(np.uint32)
    want = np.zeros(n64, np.uint64)
    oracle.scatter_increment(want, good)
    with Backing(np.zeros(n64, np.uint64), page, frames * page) as b:
        with pytest.raises(gv.GpuvmError) as e:
            gv.gpuvm_run_scatter_increment_phased(b.vm, dev(idx), idx.size, phase_len)
        assert e.value.code == gv.EDEADLK
        gv.gpuvm_reset(b.vm)                                       # writes the dirty frames back, clears the error
        gv.gpuvm_check(b.vm)
        assert np.array_equal(b.arr, want)
        gv.gpuvm_run_scatter_increment_phased(b.vm, dev(good), good.size, phase_len)   # the handle works again
        gv.gpuvm_flush(b.vm)
        assert np.array_equal(b.arr, 2 * want)


def test_gather_phased_full_size_config(gpu):
    """The headline configuration (64 MiB, 4 KiB pages, 4096 frames, 2^20 uniform
    indices) in phases of 1024 accesses: counts, cursor and the final frame
    table equal the sequential CLOCK replay."""
    n_elems, n_idx, page, frames, phase_len = 1 << 24, 1 << 20, 4096, 4096, 1024
    data = inputs.u32_values(0x9E3779B9, 0, n_elems)
    idx = inputs.u32_indices(1, 0, n_idx, n_elems)
    want, want_sum = oracle.gather(data, idx)
    sim = oracle.PagingSim(page // 8, frames, oracle.CLOCK, n_words=data.nbytes // 8, spread=frames // 2)   # the default: two hands
    sim.run((idx.astype(np.uint64) * 4) // 8, phase_len=phase_len)
    # independent-reference sanity: ~3/4 of the distinct pages of a phase miss
    assert 0.7 * n_idx < sim.counters["faults"] < 0.8 * n_idx
    with Backing(data, page, frames * page, gv.POLICY_CLOCK) as b:
        assert gv.clock_spread(b.vm) == frames // 2
        d_out = torch.zeros(n_idx, dtype=torch.int32, device="cuda")
        d_sum = torch.zeros(1, dtype=torch.int64, device="cuda")
        gv.gpuvm_run_gather_phased(b.vm, dev(idx), n_idx, phase_len, d_out, d_sum)
        assert np.array_equal(host(d_out, np.uint32), want)
        assert int(host(d_sum, np.uint64)[0]) == want_sum
        _compare_with_replay(b, sim, frames)

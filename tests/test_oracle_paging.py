"""Pins for the oracle's paged-memory simulator (CPU only).

What fixes the expected values here is never the simulator itself:
  * textbook FIFO fault counts (Belady's anomaly string; the 20-reference
    string of the standard OS textbook),
  * closed forms (compulsory misses only; cyclic scan),
  * two independently written models from the textbook descriptions of the
    policies -- FIFO as a bounded queue, second chance as a queue whose head is
    re-appended with its bit cleared -- compared on exhaustive tiny traces,
  * traces worked by hand from the stated reading (derivations below),
  * invariants checked after every phase of random runs, and the data that
    must survive eviction + write-back + flush.
"""
import itertools
import os
from collections import deque

import numpy as np
import pytest

import oracle
from oracle import ADD, CLOCK, FIFO, READ, WRITE, PagingSim

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold(name):
    rows = []
    with open(os.path.join(GOLD, name)) as fh:
        for line in fh:
            line = line.split("#")[0].split()
            if line:
                rows.append(line)
    return rows


def _run_pages(pages, frames, policy, writes=None, phase_len=1, n_pages=None, spread=0):
    """Page-granular trace through the simulator (one word per page)."""
    n_pages = n_pages or (max(pages) + 1)
    sim = PagingSim(1, frames, policy, n_words=n_pages, spread=spread)
    op = None if writes is None else np.where(np.asarray(writes), WRITE, READ).astype(np.uint8)
    sim.run(np.asarray(pages, np.uint64), op=op, phase_len=phase_len)
    return sim


# ---------------------------------------------------------------- textbook

def test_belady_anomaly_fifo():
    rows = _gold("belady_fifo.txt")
    refs = [int(x) for x in rows[0][1:]]
    for row in rows[1:]:
        frames, faults, owner = int(row[1]), int(row[2]), [int(x) for x in row[3:]]
        sim = _run_pages(refs, frames, FIFO)
        assert sim.counters["faults"] == faults
        assert sim.counters["hits"] == len(refs) - faults
        assert sim.state()["owner"].tolist() == owner
        # every reference bit is set when the hand arrives, so CLOCK walks one
        # full turn and takes the same victim: same faults, same placement
        simc = _run_pages(refs, frames, CLOCK)
        assert simc.counters["faults"] == faults
        assert simc.state()["owner"].tolist() == owner


def test_os_textbook_string_fifo():
    rows = _gold("os_textbook_fifo.txt")
    refs = [int(x) for x in rows[0][1:]]
    frames, faults = int(rows[1][1]), int(rows[1][2])
    assert _run_pages(refs, frames, FIFO).counters["faults"] == faults


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("policy", [FIFO, CLOCK])
def test_compulsory_misses_only(policy):
    rng = np.random.default_rng(5)
    pages = rng.integers(0, 40, 2000)
    sim = _run_pages(pages.tolist(), 40, policy, n_pages=40)
    c = sim.counters
    assert c["faults"] == len(set(pages.tolist()))
    assert c["evictions"] == 0 and c["writebacks_evict"] == 0
    assert c["hits"] == len(pages) - c["faults"]
    # frames are handed out in ring order: the i-th new page sits in frame i
    first = list(dict.fromkeys(pages.tolist()))
    assert sim.state()["owner"][:len(first)].tolist() == first


@pytest.mark.parametrize("policy", [FIFO, CLOCK])
@pytest.mark.parametrize("n,f,t", [(10, 3, 4), (17, 16, 3), (64, 16, 3), (5, 1, 2)])
def test_cyclic_scan(policy, n, f, t):
    """N pages scanned T times with F < N frames: every access faults."""
    sim = _run_pages(list(range(n)) * t, f, policy)
    c = sim.counters
    assert c["faults"] == t * n and c["hits"] == 0
    assert c["evictions"] == t * n - f
    assert c["writebacks_evict"] == 0 and c["skips"] == 0


def test_streaming_config_closed_form():
    """The streaming workload: 8 GiB in 64 KiB pages, 2 GiB pool, 3 passes."""
    n, f, t = 131072, 32768, 3
    sim = PagingSim(1, f, CLOCK, n_words=n)
    sim.run(np.tile(np.arange(n, dtype=np.uint64), t))
    c = sim.counters
    assert c["faults"] == 393216 and c["evictions"] == 360448
    assert c["faults"] * 65536 == 24 << 30


# ---------------------------------------------------------------- independent models

def fifo_queue_model(refs, frames):
    """FIFO as every textbook states it: a queue of resident pages."""
    q, faults = deque(), 0
    for p in refs:
        if p in q:
            continue
        faults += 1
        if len(q) == frames:
            q.popleft()
        q.append(p)
    return faults, set(q)


def second_chance_queue_model(refs, frames):
    """Second chance as a FIFO queue: the oldest page is inspected; if its R
    bit is set it is cleared and the page goes to the back as if it had just
    arrived; otherwise it is evicted.  R is set on load and on every use."""
    q, rbit, faults = deque(), {}, 0
    for p in refs:
        if p in rbit:
            rbit[p] = 1
            continue
        faults += 1
        if len(q) == frames:
            while True:
                old = q.popleft()
                if rbit[old]:
                    rbit[old] = 0
                    q.append(old)
                else:
                    del rbit[old]
                    break
        q.append(p)
        rbit[p] = 1
    return faults, set(q)


def test_exhaustive_small_traces_against_queue_models():
    checked = 0
    for npages, frames, length in [(3, 2, 6), (4, 2, 6), (4, 3, 7), (5, 3, 6)]:
        for refs in itertools.product(range(npages), repeat=length):
            f_faults, f_set = fifo_queue_model(refs, frames)
            c_faults, c_set = second_chance_queue_model(refs, frames)
            sf = _run_pages(list(refs), frames, FIFO, n_pages=npages)
            sc = _run_pages(list(refs), frames, CLOCK, n_pages=npages)
            assert sf.counters["faults"] == f_faults, refs
            assert sc.counters["faults"] == c_faults, refs
            assert set(sf.state()["owner"][sf.state()["owner"] >= 0].tolist()) == f_set
            assert set(sc.state()["owner"][sc.state()["owner"] >= 0].tolist()) == c_set
            checked += 1
    assert checked > 20000


def test_random_long_traces_against_queue_models():
    rng = np.random.default_rng(11)
    for _ in range(40):
        npages = int(rng.integers(4, 60))
        frames = int(rng.integers(1, npages))
        # skewed references so that CLOCK and FIFO really differ
        refs = np.minimum(rng.geometric(0.15, 3000) - 1, npages - 1).tolist()
        ff, fs = fifo_queue_model(refs, frames)
        cf, cs = second_chance_queue_model(refs, frames)
        sf = _run_pages(refs, frames, FIFO, n_pages=npages)
        sc = _run_pages(refs, frames, CLOCK, n_pages=npages)
        assert sf.counters["faults"] == ff and sc.counters["faults"] == cf
        own = sc.state()["owner"]
        assert set(own[own >= 0].tolist()) == cs
        own = sf.state()["owner"]
        assert set(own[own >= 0].tolist()) == fs


def test_clock_keeps_a_reused_page_that_fifo_drops():
    # 3 frames.  1 2 3 fill; 4 turns the hand once (clearing all bits) and
    # replaces 1.  Then 2 is used again (bit set), 5 must replace 3 (bit clear
    # at the hand), not 2; FIFO replaces 2 (the oldest).  6th reference to 2:
    # hit under CLOCK, fault under FIFO.
    refs = [1, 2, 3, 4, 2, 5, 2]
    assert _run_pages(refs, 3, FIFO).counters["faults"] == 6
    assert _run_pages(refs, 3, CLOCK).counters["faults"] == 5


# ---------------------------------------------------------------- two-handed CLOCK

def two_hands_rotating_queue_model(refs, frames, spread, bit_on_load=1):
    """The two-handed clock told as a rotating queue: the ring of frames, seen
    from the cursor, is a queue whose head is the frame under the cursor (None =
    never used).  Each step of the cursor first lets the front hand clear the R
    bit of the element `spread` places behind the head of the queue, then looks
    at the head: an empty frame or a page with a clear bit gives way to the new
    page, which goes to the back; a page with its bit set loses the bit and goes
    to the back itself.  R is set on load (`bit_on_load`) and on every use."""
    q, rbit, faults, passes = deque([None] * frames), {}, 0, 0
    for p in refs:
        if p in rbit:
            rbit[p] = 1
            continue
        faults += 1
        while True:
            if spread % frames and q[spread % frames] is not None:
                rbit[q[spread % frames]] = 0
            head = q.popleft()
            if head is not None and rbit[head]:
                rbit[head] = 0
                q.append(head)
                passes += 1
                continue
            if head is not None:
                del rbit[head]
            q.append(p)
            rbit[p] = bit_on_load
            break
    return faults, {x for x in q if x is not None}, passes


def test_two_hands_exhaustive_small_traces_against_the_rotating_queue():
    checked = 0
    for npages, frames, length in [(3, 2, 6), (4, 3, 7), (5, 3, 6), (5, 4, 6)]:
        for spread in range(1, frames):
            for refs in itertools.product(range(npages), repeat=length):
                faults, resident, passes = two_hands_rotating_queue_model(refs, frames, spread)
                sim = _run_pages(list(refs), frames, CLOCK, n_pages=npages, spread=spread)
                assert sim.counters["faults"] == faults, (refs, spread)
                assert sim.counters["sweeps"] == passes, (refs, spread)
                own = sim.state()["owner"]
                assert set(own[own >= 0].tolist()) == resident, (refs, spread)
                checked += 1
    assert checked > 40000


def test_two_hands_long_skewed_traces_against_the_rotating_queue():
    rng = np.random.default_rng(21)
    differs = 0
    for _ in range(40):
        npages = int(rng.integers(6, 80))
        frames = int(rng.integers(2, npages))
        spread = int(rng.integers(1, frames))
        refs = np.minimum(rng.geometric(0.12, 4000) - 1, npages - 1).tolist()
        faults, resident, passes = two_hands_rotating_queue_model(refs, frames, spread)
        sim = _run_pages(refs, frames, CLOCK, n_pages=npages, spread=spread)
        assert sim.counters["faults"] == faults and sim.counters["sweeps"] == passes
        own = sim.state()["owner"]
        assert set(own[own >= 0].tolist()) == resident
        differs += faults != second_chance_queue_model(refs, frames)[0]
    assert differs > 20                      # the second hand really changes the outcome


def test_with_a_front_hand_the_bit_set_on_load_decides_nothing():
    """A page enters at the back of the queue, F - 1 places behind the head; the
    front hand, 1 <= S <= F - 1 places behind the head, clears its bit after
    F - 1 - S steps, before the page can reach the head.  So whether a load sets
    the bit or not changes no decision: same faults, same passes, same resident
    set.  With one hand the bit on load does matter."""
    checked = 0
    for npages, frames, length in [(3, 2, 6), (4, 3, 7), (5, 4, 6)]:
        for spread in range(1, frames):
            for refs in itertools.product(range(npages), repeat=length):
                assert (two_hands_rotating_queue_model(refs, frames, spread, bit_on_load=0)
                        == two_hands_rotating_queue_model(refs, frames, spread, bit_on_load=1)), (refs, spread)
                checked += 1
    assert checked > 20000
    rng = np.random.default_rng(23)
    for _ in range(30):
        npages = int(rng.integers(6, 80))
        frames = int(rng.integers(2, npages))
        spread = int(rng.integers(1, frames))
        refs = np.minimum(rng.geometric(0.12, 3000) - 1, npages - 1).tolist()
        faults, resident, passes = two_hands_rotating_queue_model(refs, frames, spread, bit_on_load=0)
        sim = _run_pages(refs, frames, CLOCK, n_pages=npages, spread=spread)
        assert sim.counters["faults"] == faults and sim.counters["sweeps"] == passes
        own = sim.state()["owner"]
        assert set(own[own >= 0].tolist()) == resident
    refs = [1, 2, 3, 4, 2, 5, 2]
    assert (two_hands_rotating_queue_model(refs, 3, 0, bit_on_load=0)
            != two_hands_rotating_queue_model(refs, 3, 0, bit_on_load=1))


def test_front_hand_on_the_cursor_is_the_one_handed_clock():
    """A spread of 0 or of a whole ring puts the front hand on the cursor's own
    frame: there is none, and the policy is the second chance of the textbook."""
    rng = np.random.default_rng(22)
    for _ in range(20):
        npages = int(rng.integers(4, 50))
        frames = int(rng.integers(1, npages))
        refs = np.minimum(rng.geometric(0.15, 2000) - 1, npages - 1).tolist()
        want = second_chance_queue_model(refs, frames)[0]
        for spread in (0, frames, 3 * frames):
            assert _run_pages(refs, frames, CLOCK, n_pages=npages, spread=spread).counters["faults"] == want
    with pytest.raises(ValueError):
        PagingSim(1, 4, FIFO, n_words=8, spread=2)           # no reference bit, no front hand


@pytest.mark.parametrize("n,f,t", [(10, 3, 4), (17, 16, 3), (64, 16, 3), (1000, 256, 2)])
def test_two_hands_pass_nothing_on_a_scan(n, f, t):
    """Cyclic scan: the front hand has cleared every bit before the cursor
    arrives, so the closed form of the scan holds with zero passes - where one
    hand goes once round clearing bits at the start of every lap."""
    for spread in sorted({1, f // 2, f - 1} - {0}):
        c = _run_pages(list(range(n)) * t, f, CLOCK, spread=spread).counters
        assert c["faults"] == t * n and c["evictions"] == t * n - f and c["hits"] == 0
        assert c["sweeps"] == 0 and c["skips"] == 0
    one = _run_pages(list(range(n)) * t, f, CLOCK).counters
    assert one["faults"] == t * n and one["sweeps"] >= f


def test_hand_trace_two_hands_f4():
    """4 frames, front hand 2 ahead, trace 1 2 3 4 2 5 1 3 5 6 (bits as r0..r3).

    Fill: 1 -> frame 0 (front hand on empty frame 2), 2 -> frame 1 (front on
    empty 3), 3 -> frame 2 (front on frame 0: r0 cleared), 4 -> frame 3 (front
    on 1: r1 cleared).  Bits 0 0 1 1, cursor 0.  2 hits: r1 set.
    5: cursor 0, front clears r2; frame 0 (page 1) has a clear bit: evicted, 5
    installed.  Frames 5 2 3 4, bits 1 1 0 1, cursor 1.
    1: cursor 1, front clears r3; frame 1 (page 2) has its bit set: cleared and
    passed (1st pass).  Cursor 2, front clears r0 (page 5); frame 2 (page 3) is
    clear: evicted, 1 installed.  Frames 5 2 1 4, bits 0 0 1 0, cursor 3.
    3: cursor 3, front on frame 1 (already clear); frame 3 (page 4) clear:
    evicted, 3 installed.  Frames 5 2 1 3, bits 0 0 1 1, cursor 0.  5 hits: r0.
    6: cursor 0, front clears r2; frame 0 (page 5) set: cleared, passed (2nd
    pass).  Cursor 1, front clears r3; frame 1 (page 2) clear: evicted, 6
    installed.  Frames 5 6 1 3.  8 faults, 2 hits, 4 evictions, 2 passes.

    One hand: the fill leaves all bits set; 2 hits.  5 clears four bits (4
    passes) and takes frame 0.  1 takes frame 1 (page 2, clear).  3 and 5 hit.
    6: frame 2 (page 3) set: 5th pass; frame 3 (page 4) clear: evicted.  Frames
    5 1 3 6; 7 faults, 3 hits, 3 evictions.
    """
    rows = _gold("trace_two_hands_f4.txt")
    acc = rows[0][1:]
    pages = [int(a[:-1]) for a in acc]
    for row in rows[1:]:
        assert row[1] == "spread"
        _check_expect(_run_pages(pages, 4, CLOCK, spread=int(row[2])), _parse_expect(row[2:]))


# ---------------------------------------------------------------- hand-worked traces

def _parse_expect(row):
    d, i = {}, 1
    while row[i] != "owner":
        d[row[i]] = int(row[i + 1])
        i += 2
    d["owner"] = [int(x) for x in row[i + 1:]]
    return d


def _check_expect(sim, exp):
    sim.flush()
    c = sim.counters
    for k, v in exp.items():
        if k == "owner":
            assert sim.state()["owner"].tolist() == v
        else:
            assert c[k] == v, (k, c)


def test_hand_trace_dirty_f3():
    """3 frames, phase length 1: 1R 2W 3R 1R 4R 1R 5R 2R 1W 3R.

    FIFO: 1,2,3 fill frames 0,1,2 (2 dirty).  1R hits.  4 takes frame 0
    (drops 1, clean).  1 faults again, takes frame 1 (page 2 is dirty: first
    write-back).  5 takes frame 2 (drops 3).  2 takes frame 0 (drops 4).  1W
    hits in frame 1 and dirties it.  3 takes frame 1 (page 1 dirty: second
    write-back).  8 faults, 2 hits, 5 evictions, 2 write-backs, frames hold
    2,3,5, nothing dirty is left for the flush.

    CLOCK: after the fill all bits are set; 1R changes nothing.  4 clears the
    bits of frames 0,1,2 (3 sweeps) and takes frame 0.  1 takes frame 1 (bit
    clear; page 2 dirty: write-back).  5 takes frame 2.  2: hand at 0, bits of
    0,1,2 are set (installed since): 3 more sweeps, takes frame 0.  1W hits in
    frame 1, sets its bit, dirties it.  3: hand at 1, bit set -> cleared (7th
    sweep), frame 2 has a clear bit: drops 5.  Frames hold 2,1,3; page 1 is
    still dirty: one flush write-back.
    """
    rows = _gold("trace_dirty_f3.txt")
    acc = rows[0][1:]
    pages = [int(a[:-1]) for a in acc]
    writes = [a[-1] == "W" for a in acc]
    for row, pol in ((rows[1], FIFO), (rows[2], CLOCK)):
        _check_expect(_run_pages(pages, 3, pol, writes), _parse_expect(row))


def test_hand_trace_phased_f4():
    """4 frames, three phases of four accesses (derivation: the distinct pages
    of a phase are pinned while it lasts; hits are pinned first, faults are
    served in ascending page order; a pinned frame is passed over).

    Phase 1 {0,1,2}: frames 0,1,2; hand 3; page 1 dirty.
    Phase 2 {1,3,4,5}: 1 hits (pinned).  3 takes the empty frame 3.  4: FIFO
    takes frame 0 (drops 0); CLOCK first clears frame 0, passes pinned 1,
    clears 2, passes pinned 3, then takes frame 0.  5: frame 1 is pinned,
    frame 2 (page 2) is taken.  4 is dirty.  Frames 4,1,5,3, hand 3.
    Phase 3 {0,1,4,6}: 1 and 4 hit.  0: FIFO takes frame 3 (drops 3); CLOCK
    clears 3, passes pinned 0 and 1, clears 2, takes frame 3.  6: passes
    pinned 0 and 1, takes frame 2 (drops 5).  0 is dirty.
    Totals: 8 faults, 3 hits, 4 evictions, no eviction write-back (victims
    0,2,3,5 were clean), flush writes 1, 4 and 0.  Passed-over pinned frames:
    FIFO 1+2 = 3, CLOCK 3+4 = 7; CLOCK bit clearings 2+2 = 4.
    """
    rows = _gold("trace_phased_f4.txt")
    phases = [r[1:] for r in rows if r[0] == "phase"]
    for row in rows:
        if row[0] not in ("fifo", "clock"):
            continue
        sim = PagingSim(1, 4, FIFO if row[0] == "fifo" else CLOCK, n_words=7)
        for ph in phases:
            pages = np.array([int(a[:-1]) for a in ph], np.uint64)
            op = np.array([WRITE if a[-1] == "W" else READ for a in ph], np.uint8)
            sim.phase(pages, op)
        _check_expect(sim, _parse_expect(row))


# ---------------------------------------------------------------- invariants + data

def _check_invariants(sim, n_frames):
    st, c = sim.state(), sim.counters
    owner, where = st["owner"], st["where"]
    res = np.nonzero(where >= 0)[0]
    assert len(res) <= n_frames
    assert len(set(where[res].tolist())) == len(res)          # one frame per page
    assert np.all(owner[where[res]] == res)                   # and back
    assert np.count_nonzero(owner >= 0) == len(res)
    assert np.all(st["pin"] == 0)
    assert c["faults"] - c["evictions"] == len(res)
    assert np.all(st["dirty"][owner < 0] == 0)


@pytest.mark.parametrize("policy,two_hands", [(FIFO, False), (CLOCK, False), (CLOCK, True)])
def test_random_phases_invariants_and_data(policy, two_hands):
    rng = np.random.default_rng(3 + policy + 10 * two_hands)
    for trial in range(25):
        page_words = int(rng.choice([1, 4, 16]))
        n_words = int(rng.integers(20, 400))
        n_pages = -(-n_words // page_words)
        frames = int(rng.integers(2, max(3, n_pages)))
        phase_len = int(rng.integers(1, frames + 1))
        host = rng.integers(0, 1 << 40, n_words).astype(np.uint64)
        model = host.copy()                 # the same ops on plain memory
        sim = PagingSim(page_words, frames, policy, host=host, spread=frames // 2 if two_hands else 0)
        for _ in range(30):
            k = phase_len
            idx = rng.integers(0, n_words, k).astype(np.uint64)
            op = rng.integers(0, 3, k).astype(np.uint8)
            val = rng.integers(0, 1000, k).astype(np.uint64)
            got = sim.phase(idx, op, val)
            for i in range(k):              # plain sequential semantics
                before = model[idx[i]]
                if op[i] == READ:
                    assert got[i] == before
                elif op[i] == WRITE:
                    model[idx[i]] = val[i]
                else:
                    assert got[i] == before
                    model[idx[i]] = before + val[i]
            _check_invariants(sim, frames)
        sim.flush()
        assert np.all(sim.state()["dirty"] == 0)
        assert np.array_equal(host, model)


def test_scatter_through_paging_equals_bincount():
    rng = np.random.default_rng(9)
    n_words, k = 4096, 50000
    idx = np.minimum(rng.zipf(1.3, k) - 1, n_words - 1).astype(np.uint64)
    for policy in (FIFO, CLOCK):
        host = np.zeros(n_words, np.uint64)
        sim = PagingSim(64, 8, policy, host=host)
        sim.run(idx, op=ADD, val=1, phase_len=8)
        c = sim.counters
        assert c["writebacks_evict"] > 0
        assert c["writebacks_evict"] <= c["evictions"]
        sim.flush()
        assert np.array_equal(host, np.bincount(idx.astype(np.int64), minlength=n_words).astype(np.uint64))
        assert int(host.sum()) == k


def test_readonly_trace_never_writes_back():
    rng = np.random.default_rng(2)
    host = rng.integers(0, 1 << 60, 1000).astype(np.uint64)
    keep = host.copy()
    sim = PagingSim(8, 5, CLOCK, host=host)
    idx = rng.integers(0, 1000, 5000).astype(np.uint64)
    got = sim.run(idx, phase_len=4)
    assert np.array_equal(got, keep[idx.astype(np.int64)])
    sim.flush()
    c = sim.counters
    assert c["writebacks_evict"] == 0 and c["writebacks_flush"] == 0
    assert np.array_equal(host, keep)


def test_short_last_page_and_errors():
    host = np.arange(10, dtype=np.uint64)           # pages of 4: 4 + 4 + 2 words
    sim = PagingSim(4, 2, FIFO, host=host)
    sim.run(np.array([9, 0, 5, 9], np.uint64), op=np.array([ADD, READ, READ, READ], np.uint8), val=7)
    sim.flush()
    assert host[9] == 16 and host[:9].tolist() == list(range(9))
    with pytest.raises(IndexError):
        sim.phase(np.array([10], np.uint64))
    with pytest.raises(ValueError):                 # 3 distinct pages, 2 frames
        sim.phase(np.array([0, 4, 8], np.uint64))


def test_pinned_frames_are_never_victims():
    # 2 frames; phase {0,1} then phase {1,2}: page 1 is pinned by the second
    # phase, so page 2 must replace page 0 whatever the policy.
    for policy in (FIFO, CLOCK):
        sim = PagingSim(1, 2, policy, n_words=3)
        sim.phase(np.array([0, 1], np.uint64))
        sim.phase(np.array([1, 2], np.uint64))
        assert sorted(sim.state()["owner"].tolist()) == [1, 2]
        assert sim.counters["hits"] == 1 and sim.counters["faults"] == 3


# ---------------------------------------------------------------- write-aware CLOCK

def write_aware_queue_model(refs, writes, frames):
    """Second chance as a queue, with one more chance for a page that was written:
    the oldest page goes to the back with its R bit cleared if R is set; else, if
    it is dirty and has not been spared yet, it is spared once; else it is evicted."""
    q, st, faults, wbs = deque(), {}, 0, 0           # st[page] = [R, dirty, spared]
    for p, w in zip(refs, writes):
        if p in st:
            st[p][0] = 1
            st[p][1] |= int(w)
            continue
        faults += 1
        if len(q) == frames:
            while True:
                old = q.popleft()
                r, d, sp = st[old]
                if r:
                    st[old][0] = 0
                    q.append(old)
                elif d and not sp:
                    st[old][2] = 1
                    q.append(old)
                else:
                    wbs += d
                    del st[old]
                    break
        q.append(p)
        st[p] = [1, int(w), 0]
    return faults, wbs, set(q)


def test_write_aware_clock_equals_clock_without_writes():
    for npages, frames, length in [(4, 2, 6), (4, 3, 7), (5, 3, 6)]:
        for refs in itertools.product(range(npages), repeat=length):
            a = _run_pages(list(refs), frames, CLOCK, n_pages=npages)
            b = _run_pages(list(refs), frames, oracle.CLOCK_WA, n_pages=npages)
            assert a.counters == b.counters and a.state()["owner"].tolist() == b.state()["owner"].tolist()


def test_write_aware_clock_against_queue_model():
    rng = np.random.default_rng(21)
    for _ in range(60):
        npages = int(rng.integers(4, 40))
        frames = int(rng.integers(1, npages))
        n = 2000
        refs = np.minimum(rng.geometric(0.12, n) - 1, npages - 1).tolist()
        writes = (rng.random(n) < 0.3).tolist()
        f, w, resident = write_aware_queue_model(refs, writes, frames)
        sim = _run_pages(refs, frames, oracle.CLOCK_WA, writes, n_pages=npages)
        assert sim.counters["faults"] == f and sim.counters["writebacks_evict"] == w
        own = sim.state()["owner"]
        assert set(own[own >= 0].tolist()) == resident


def test_write_aware_clock_spares_the_written_page():
    # 2 frames: 1W 2R 3R.  The hand clears both bits, comes back to page 1 (dirty,
    # not yet spared: spared), takes clean page 2.  Plain CLOCK evicts page 1 and
    # pays a write-back.
    wa = _run_pages([1, 2, 3], 2, oracle.CLOCK_WA, [True, False, False], n_pages=5)
    ck = _run_pages([1, 2, 3], 2, CLOCK, [True, False, False], n_pages=5)
    assert sorted(wa.state()["owner"].tolist()) == [1, 3] and wa.counters["writebacks_evict"] == 0
    assert sorted(ck.state()["owner"].tolist()) == [2, 3] and ck.counters["writebacks_evict"] == 1
    # spared once only: 4R finds page 1 with its chance used up
    wa.run(np.array([4], np.uint64))
    assert wa.counters["writebacks_evict"] == 1 and sorted(wa.state()["owner"].tolist()) == [3, 4]


# ---------------------------------------------------------------- generalized CLOCK (use count 0..2)

def gclock_queue_model(refs, frames, cap=2):
    """Written independently of the simulator: resident pages in a queue, each
    with a use count that starts at 0 and grows by one per later use up to `cap`;
    to make room the front page is re-appended with its count lowered while the
    count is positive, and leaves at 0.  Returns faults, passes, resident set."""
    q, cnt = deque(), {}
    faults = passes = 0
    for p in refs:
        if p in cnt:
            cnt[p] = min(cnt[p] + 1, cap)
            continue
        faults += 1
        if len(q) == frames:
            while True:
                old = q.popleft()
                if cnt[old] > 0:
                    cnt[old] -= 1
                    passes += 1
                    q.append(old)
                else:
                    del cnt[old]
                    break
        q.append(p)
        cnt[p] = 0
    return faults, passes, set(q)


def test_gclock_against_queue_model_exhaustive_and_random():
    for npages, frames, length in [(4, 2, 7), (4, 3, 7), (5, 3, 6)]:
        for refs in itertools.product(range(npages), repeat=length):
            f, passes, resident = gclock_queue_model(refs, frames)
            sim = _run_pages(list(refs), frames, oracle.GCLOCK, n_pages=npages)
            own = sim.state()["owner"]
            assert (sim.counters["faults"], sim.counters["sweeps"], set(own[own >= 0].tolist())) == (f, passes, resident), refs
    rng = np.random.default_rng(31)
    for _ in range(60):
        npages = int(rng.integers(4, 40))
        frames = int(rng.integers(1, npages))
        refs = np.minimum(rng.geometric(0.12, 2000) - 1, npages - 1).tolist()
        f, passes, resident = gclock_queue_model(refs, frames)
        sim = _run_pages(refs, frames, oracle.GCLOCK, n_pages=npages)
        own = sim.state()["owner"]
        assert (sim.counters["faults"], sim.counters["sweeps"], set(own[own >= 0].tolist())) == (f, passes, resident)


def test_gclock_is_fifo_without_reuse_and_never_sweeps_on_a_scan():
    # pages are installed with count 0: a cyclic scan (no page used again while
    # resident) takes every frame at the hand's first visit - FIFO's faults,
    # evictions and placement, and not one pass
    for n, frames, turns in [(10, 3, 4), (64, 16, 3), (7, 6, 5)]:
        refs = list(range(n)) * turns
        g = _run_pages(refs, frames, oracle.GCLOCK)
        f = _run_pages(refs, frames, FIFO)
        assert g.counters["faults"] == f.counters["faults"] == turns * n
        assert g.counters["evictions"] == turns * n - frames and g.counters["sweeps"] == 0
        assert g.state()["owner"].tolist() == f.state()["owner"].tolist()
    # CLOCK pays one pass per eviction on the same scan (every bit is set at install)
    c = _run_pages(list(range(10)) * 4, 3, CLOCK)
    assert c.counters["sweeps"] > 0


def test_gclock_hand_worked_trace():
    # 2 frames, trace 1 1 1 2 3 4 5.  Page 1 is used twice more after its install:
    # count 2 (the cap).  3 faults: frame 0 (page 1) 2 -> 1, passed; frame 1 (page 2,
    # count 0) taken.  4 faults: page 1 1 -> 0, passed; page 3 taken.  5 faults: page 1
    # at 0, taken.  Two earned chances, two passes, then it goes.
    sim = _run_pages([1, 1, 1, 2, 3], 2, oracle.GCLOCK, n_pages=6)
    assert sim.state()["owner"].tolist() == [1, 3] and sim.counters["sweeps"] == 1
    st = sim.state()
    assert (int(st["ref"][0]), int(st["defer"][0])) == (1, 0)                 # count 1
    sim.run(np.array([4], np.uint64))
    assert sim.state()["owner"].tolist() == [1, 4] and sim.counters["sweeps"] == 2
    sim.run(np.array([5], np.uint64))
    assert sim.state()["owner"].tolist() == [5, 4] and sim.counters["sweeps"] == 2
    assert sim.counters["faults"] == 5 and sim.counters["hits"] == 2 and sim.counters["evictions"] == 3
    # CLOCK on the first five references: both bits are set at install, the hand
    # clears them in turn and takes page 1, the one that was used three times
    ck = _run_pages([1, 1, 1, 2, 3], 2, CLOCK, n_pages=6)
    assert ck.state()["owner"].tolist() == [3, 2] and ck.counters["sweeps"] == 2
    # the count is capped: ten uses earn no more than two passes
    many = _run_pages([1] * 10 + [2, 3, 4, 5], 2, oracle.GCLOCK, n_pages=6)
    assert 1 not in many.state()["owner"].tolist() and many.counters["sweeps"] == 2


def test_waiting_policy_has_no_sequential_replay():
    with pytest.raises(ValueError):
        PagingSim(1, 4, 2, n_words=8)

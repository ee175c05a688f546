// Protocol stress of the fault path on the CPU: N threads, each a one-lane
// wavefront, run seeded random loads, atomic adds, stores, optimistic page
// reads, page-level pinned writes and fault-ahead touches through the accessors of gpuvm_device.h (the
// header itself, compiled for the host through shim.h) over a pool far smaller
// than the data set.  Checked while running: a counter never reads below the
// increments that had completed before the read began nor above those that had
// been announced before it ended; a thread reads back what it stored, through
// any number of evictions and write-backs.  Checked at the end: no error was
// recorded, every reference count is zero, page table and frame table agree,
// and after writing the dirty frames back the host array holds exactly
// initial value + number of increments, and the last stored values.
//
// usage: driver policy threads frames page_bytes pages ops_per_thread seed writeback_mode yield_every remote_touches clock_hands
#include "shim.h"
#include GPUVM_DEVICE_HEADER

#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>

typedef unsigned long long u64;

static gpuvm_dev_t vm;
static std::vector<u64> init_val;
static std::atomic<u64> *announced, *completed;      // increments per shared element
static std::atomic<int> failures{0};

static void fail(const char *what, u64 a, u64 b, u64 c) {
    if (failures.fetch_add(1) < 10) fprintf(stderr, "FAIL %s: %llu %llu %llu\n", what, a, b, c);
}

struct rng_t {
    u64 s;
    u64 next() { s ^= s >> 12; s ^= s << 25; s ^= s >> 27; return s * 2685821657736338717ull; }
};

int main(int argc, char **argv) {
    if (argc != 12) { fprintf(stderr, "usage: see the head of driver.cpp\n"); return 2; }
    const unsigned policy = atoi(argv[1]), threads = atoi(argv[2]), frames = atoi(argv[3]);
    const unsigned page_bytes = atoi(argv[4]), pages = atoi(argv[5]), ops = atoi(argv[6]);
    const u64 seed = strtoull(argv[7], nullptr, 10);
    const unsigned wb_mode = atoi(argv[8]);
    shim_yield_every = atoi(argv[9]);
    const unsigned remote_touches = atoi(argv[10]);         // 0: every miss migrates; else reads in place before migration
    const unsigned clock_hands = atoi(argv[11]) & GPUVM_F_HANDS_MASK;   // CLOCK policies: front hand this many eighths of the ring ahead, 0 = one hand
    if (frames < 2 * threads || frames < 8) { fprintf(stderr, "need frames >= max(8, 2 * threads)\n"); return 2; }

    const u64 per_page = page_bytes / 8;
    const u64 n_shared = (u64)pages * per_page - 5;            // short last page: 40 bytes missing
    const u64 priv = 64;                                       // private elements per thread, spread over pages
    std::vector<u64> host(n_shared), pte(pages, 0), stats(GPUVM_STAT_SLOTS * GPUVM_S_COUNT, 0), hand(2, 0);
    std::vector<unsigned> owner(frames, GPUVM_NO_PAGE);
    std::vector<char> pool((size_t)frames * page_bytes, (char)0xAB);
    init_val.resize(n_shared);
    for (u64 i = 0; i < n_shared; ++i) host[i] = init_val[i] = i * 7 + 1;
    announced = new std::atomic<u64>[n_shared]();
    completed = new std::atomic<u64>[n_shared]();
    unsigned shift = 0;
    while ((1u << shift) < page_bytes) ++shift;
    vm.pte = pte.data(); vm.frame_owner = owner.data(); vm.hand = hand.data(); vm.stats = stats.data();
    vm.frames = pool.data(); vm.host = (char *)host.data();
    vm.bytes = n_shared * 8; vm.n_pages = pages; vm.n_frames = frames; vm.page_shift = shift;
    vm.policy = policy; vm.spin_limit = 1u << 30; vm.flags = (wb_mode ? GPUVM_F_OVERLAPPED_WRITEBACK : 0) | (remote_touches << GPUVM_F_REMOTE_SHIFT) | (clock_hands << GPUVM_F_HANDS_SHIFT);

    // element i is private to thread t if i % stride == t (t < threads) and i / stride < priv
    const u64 stride = n_shared / priv;
    auto owner_of = [&](u64 i) -> int { return (i % stride < threads && i / stride < priv) ? (int)(i % stride) : -1; };
    std::vector<std::vector<u64>> last(threads, std::vector<u64>(priv, 0));

    auto body = [&](unsigned t) {
        blockIdx.x = t >> 1;                                      // two waves per workgroup share a counter shard
        rng_t r{seed * 1000003ull + t * 7919ull + 1};
        for (unsigned k = 0; k < priv; ++k) last[t][k] = init_val[k * stride + t];
        for (unsigned n = 0; n < ops && failures.load() == 0; ++n) {
            const u64 x = r.next();
            // skewed choice of element: half of the accesses go to one sixteenth of the pages
            u64 i = (x >> 8) % n_shared;
            if (x & 0x80) i = (x >> 8) % (n_shared / 16);
            const unsigned op = x & 7;
            if (op == 7) {                                        // store to / read back a private element
                const unsigned k = (x >> 40) % priv;
                const u64 e = k * stride + t;
                if (x & 0x100) {                                  // through a cursor: the page stays pinned between the two
                    gpuvm_cursor_t c = gpuvm_cursor_begin();
                    const u64 got = gpuvm_cursor_load<u64>(vm, c, e, true);
                    if (got != last[t][k]) fail("private element read back (cursor)", e, got, last[t][k]);
                    last[t][k] = x | 1;
                    gpuvm_cursor_store<u64>(vm, c, e, last[t][k], true);
                    gpuvm_cursor_end(vm, c);
                    continue;
                }
                const u64 got = gpuvm_load<u64>(vm, e);
                if (got != last[t][k]) fail("private element read back", e, got, last[t][k]);
                last[t][k] = x | 1;
                gpuvm_store<u64>(vm, e, last[t][k]);
                continue;
            }
            if (owner_of(i) >= 0) continue;                       // shared operations leave private elements alone
            if (op <= 1) {                                        // increment through the element accessor
                announced[i].fetch_add(1);
                gpuvm_atomic_add<u64>(vm, i, 1ull);
                completed[i].fetch_add(1);
            } else if (op == 2) {                                 // increment by a page-level writer (pinned)
                const unsigned page = (unsigned)((i * 8) >> shift);
                announced[i].fetch_add(1);
                char *p = gpuvm_acquire(vm, page, true);
                __hip_atomic_fetch_add(reinterpret_cast<u64 *>(p + ((i * 8) & (page_bytes - 1))), 1ull, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                gpuvm_release(vm, page);
                completed[i].fetch_add(1);
            } else if (op == 3 && (x & 0x100)) {                  // two reads in one optimistic transaction
                const u64 j = (x >> 20) % n_shared;
                if (owner_of(j) >= 0) continue;
                const u64 lo_i = completed[i].load(), lo_j = completed[j].load();
                const unsigned long long elems[2] = {i, j};
                const bool wants[2] = {true, true};
                u64 got[2];
                gpuvm_load_n<u64, 2>(vm, elems, wants, got);
                const u64 hi_i = announced[i].load(), hi_j = announced[j].load();
                if (got[0] < init_val[i] + lo_i || got[0] > init_val[i] + hi_i) fail("batched read out of bounds", i, got[0], init_val[i]);
                if (got[1] < init_val[j] + lo_j || got[1] > init_val[j] + hi_j) fail("batched read out of bounds", j, got[1], init_val[j]);
            } else if (op == 4 && (x & 0x100)) {                  // a short walk with a cursor (may cross into the next page)
                gpuvm_cursor_t c = gpuvm_cursor_begin();
                for (u64 e = i; e < i + 6 && e < n_shared; ++e) {
                    if (owner_of(e) >= 0) continue;
                    const u64 lo = completed[e].load();
                    const u64 got = gpuvm_cursor_load<u64>(vm, c, e, true);
                    const u64 hi = announced[e].load();
                    if (got < init_val[e] + lo || got > init_val[e] + hi) fail("cursor read out of bounds", e, got, init_val[e]);
                }
                gpuvm_cursor_end(vm, c);
            } else if (op <= 4) {                                 // read through the element accessor
                const u64 lo = completed[i].load();
                const u64 got = gpuvm_load<u64>(vm, i);
                const u64 hi = announced[i].load();
                if (got < init_val[i] + lo || got > init_val[i] + hi) fail("counter out of bounds", i, got, init_val[i]);
            } else if (op == 5) {                                 // optimistic page-level read
                const unsigned page = (unsigned)((i * 8) >> shift);
                const unsigned off = (unsigned)((i * 8) & (page_bytes - 1));
                const u64 lo = completed[i].load();
                unsigned long long token;
                const char *p = gpuvm_peek(vm, page, &token);
                if (p) {
                    const gpuvm_detail::u32x2 v = gpuvm_frame_load_b64(vm, p, off);
                    if (gpuvm_peek_valid(vm, page, token)) {
                        const u64 got = ((u64)v.y << 32) | v.x;
                        const u64 hi = announced[i].load();
                        if (got < init_val[i] + lo || got > init_val[i] + hi) fail("validated peek out of bounds", i, got, init_val[i]);
                    }
                }
            } else if (x & 0x200) {                               // a one-visit page-level read: pinned, no reference mark
                const unsigned page = (unsigned)((i * 8) >> shift);
                const unsigned off = (unsigned)((i * 8) & (page_bytes - 1));
                const u64 lo = completed[i].load();
                const char *p = gpuvm_acquire_cold(vm, page, false, true);
                const gpuvm_detail::u32x2 v = gpuvm_frame_load_b64(vm, p, off);
                gpuvm_release(vm, page);
                const u64 got = ((u64)v.y << 32) | v.x;
                const u64 hi = announced[i].load();
                if (hand[1] == 0 && (got < init_val[i] + lo || got > init_val[i] + hi)) fail("pinned page read out of bounds", i, got, init_val[i]);
            } else {                                              // fault-ahead
                gpuvm_touch(vm, (unsigned)((i * 8) >> shift));
            }
        }
    };
    std::vector<std::thread> pool_threads;
    for (unsigned t = 0; t < threads; ++t) pool_threads.emplace_back(body, t);
    for (auto &th : pool_threads) th.join();

    // quiesced state
    if (hand[1] != 0) fail("kernel-side error recorded", hand[1], 0, 0);
    std::vector<int> seen(frames, 0);
    u64 resident = 0, dirty = 0;
    for (unsigned p = 0; p < pages; ++p) {
        const u64 w = pte[p];
        const unsigned st = (unsigned)((w & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT);
        if (w & GPUVM_PTE_PIN_MASK) fail("reference count left", p, w, 0);
        if (st == GPUVM_ST_INVALID) {
            const u64 touch_bits = remote_touches ? ~0ull << GPUVM_PTE_FRAME_SHIFT : 0ull;   // count of reads in place
            if (w & ~((u64)GPUVM_PTE_GEN_MASK | touch_bits)) fail("stale bits on an INVALID entry", p, w, 0);
            if (remote_touches && (w >> GPUVM_PTE_FRAME_SHIFT) >= remote_touches) fail("more reads in place than a migration costs", p, w, remote_touches);
        } else if (st == GPUVM_ST_RESIDENT) {
            const unsigned f = (unsigned)(w >> GPUVM_PTE_FRAME_SHIFT);
            if (f >= frames || owner[f] != p || seen[f]++) fail("page table and frame table disagree", p, f, f < frames ? owner[f] : 0);
            ++resident;
            if (w & GPUVM_PTE_DIRTY) {                            // what gpuvm_flush does
                ++dirty;
                const u64 len = gpuvm_detail::page_len(vm, p);
                memcpy((char *)host.data() + ((size_t)p << shift), pool.data() + ((size_t)f << shift), len);
            }
        } else {
            fail("page left LOADING or EVICTING", p, w, 0);
        }
    }
    u64 tot[GPUVM_S_COUNT] = {0};
    for (int s = 0; s < GPUVM_STAT_SLOTS; ++s)
        for (int c = 0; c < GPUVM_S_COUNT; ++c) tot[c] += stats[(size_t)s * GPUVM_S_COUNT + c];
    if (tot[GPUVM_S_FAULTS] - (tot[GPUVM_S_FAULTS] - tot[GPUVM_S_FRESH]) != resident) fail("faults - evictions != resident", tot[GPUVM_S_FAULTS], (tot[GPUVM_S_FAULTS] - tot[GPUVM_S_FRESH]), resident);
    u64 incs = 0;
    for (u64 i = 0; i < n_shared; ++i) {
        const int o = owner_of(i);
        const u64 want = o >= 0 ? last[o][i / stride] : init_val[i] + completed[i].load();
        if (host[i] != want) fail("final host value", i, host[i], want);
        incs += completed[i].load();
    }
    printf("{\"failures\": %d, \"faults\": %llu, \"evictions\": %llu, \"writebacks_evict\": %llu, \"loading_waits\": %llu, "
           "\"alloc_skips\": %llu, \"alloc_sweeps\": %llu, \"resident\": %llu, \"dirty_at_end\": %llu, \"increments\": %llu, "
           "\"remote_reads\": %llu}\n",
           failures.load(), tot[GPUVM_S_FAULTS], (tot[GPUVM_S_FAULTS] - tot[GPUVM_S_FRESH]), tot[GPUVM_S_WB_EVICT], tot[GPUVM_S_WAITS],
           tot[GPUVM_S_SKIPS], tot[GPUVM_S_SWEEPS], resident, dirty, incs, tot[GPUVM_S_REMOTE]);
    return failures.load() ? 1 : 0;
}

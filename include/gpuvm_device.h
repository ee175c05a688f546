/*
 * gpuvm_device.h - device-side accessors of GPUVM for gfx950 (HIP only).
 *
 * Include from a .hip file, take a gpuvm_dev_t by value as a kernel argument
 * and index the paged data set like an array (paper: the gpuvm<T> class of the
 * vector-addition listing; System Overview steps 1-7):
 *
 *     float a = gpuvm_load<float>(vm, i);         // any lane, any divergence
 *     gpuvm_store<float>(vm, i, a + 1.0f);
 *     gpuvm_atomic_add<unsigned long long>(vm, i, 1ull);
 *     float b = gpuvm_load_if<float>(vm, i, in_range);   // whole wave calls, predicate per lane
 *
 * or, for code in which a whole wavefront works on one page at a time,
 *
 *     char *p = gpuvm_acquire(vm, page, write);   // same page in every lane
 *     ... gpuvm_frame_load_b32/b64/b128(vm, p, byte_offset) ...
 *     gpuvm_release(vm, page);
 *
 * Execution model.  A CDNA wavefront has no independent thread scheduling, so
 * the fault path is wave-uniform: reads of resident pages are served lane by
 * lane without any reference count (optimistic, validated by the page's
 * word); for writes and for whatever missed, the accessor loops over the
 * distinct pages its active lanes touch (wavefront dedup, paper: Page access
 * synchronization); for each page the first lane of the group is the leader
 * and performs every atomic, and all active lanes move the page together (the
 * substitute for the paper's NIC work request).  While it waits or allocates
 * a wave holds at most ONE frame (a pinned page, or the frame it is filling),
 * so frames in use never exceed the number of waves in flight; the launchers
 * keep that below half the frame pool, which is what makes "pass over a
 * pinned frame" always find a victim.  A kernel of your own has to do the
 * same: launch no more wavefronts than gpuvm_max_waves() returns for every
 * handle the kernel touches (grid-stride over the work), and let a wave hold
 * at most one gpuvm_acquire per handle at a time.
 *
 * Page-table word (one 64-bit atomic per page, all updates are atomics that
 * leave the pin count of concurrent users intact):
 *     bits  0..19  pin    reference counter: waves that use or wait for the page
 *     bits 20..31  gen    install generation, +1 every time the page becomes RESIDENT
 *     bit   32     REF    CLOCK reference bit (generalized CLOCK: first bit of the use count)
 *     bit   33     DIRTY  frame differs from host memory
 *     bits 34..35  state  0 INVALID, 1 LOADING, 2 RESIDENT, 3 EVICTING
 *     bit   36     DEFER  write-aware CLOCK: the hand has spared this dirty page once
 *                         (generalized CLOCK: second bit of the use count)
 *     bits 37..63  frame  valid while RESIDENT / EVICTING; while INVALID: the number
 *                         of reads served in place since the page was last evicted
 *                         (remote-first mode, otherwise 0)
 * Frame table: frame_owner[f] = page whose data the frame holds (0xFFFFFFFF
 * before first use).  hand[0] is the global head cursor of the frame ring;
 * ticket t names frame t mod n_frames (paper: Eviction scheme - the leader
 * atomically takes the next mapping and may not choose a frame).
 * hand[1] holds the first error a kernel recorded; hand[2] is a work counter
 * of the library's own launchers (zero at launch) and of no concern to
 * kernels written against this header.
 *
 * Coherence and ordering.  Each XCD of the MI355X has its own L2, and the
 * L1/L2 are not kept coherent with each other by hardware for ordinary loads
 * and stores; agent-scope fences would do it, but they write back / invalidate
 * a whole L2 each time and serialise the fault path.  Instead every access to
 * frame memory carries the agent-scope cache bits (sc1): the mover stores the
 * page write-through, element loads/stores/atomics are relaxed agent-scope
 * atomics, and wave-level users read frames with gpuvm_frame_load*().  Host
 * memory is read and written at system scope (sc0 sc1).  Page-table atomics
 * are relaxed at agent scope.  Ordering then needs no cache maintenance, only
 * completion: s_waitcnt vmcnt(0) after the page was copied and before it is
 * published RESIDENT; after a write-back and before the victim becomes INVALID
 * (the re-fault's reads follow the posted writes on the same link); after a
 * user's last access and before its pin is dropped.  A reader's frame address
 * depends on the value its page-table atomic returned.
 */
#ifndef GPUVM_DEVICE_H
#define GPUVM_DEVICE_H

#include <hip/hip_runtime.h>
#include "gpuvm.h"

#define GPUVM_PTE_PIN_MASK    0x00000000000FFFFFull
#define GPUVM_PTE_GEN_SHIFT   20
#define GPUVM_PTE_GEN_MASK    0x00000000FFF00000ull
#define GPUVM_PTE_KEEP_MASK   (GPUVM_PTE_PIN_MASK | GPUVM_PTE_GEN_MASK)   /* survives INVALID */
#define GPUVM_PTE_IDENT_MASK  (GPUVM_PTE_GEN_MASK | GPUVM_PTE_STATE_MASK | ~((1ull << GPUVM_PTE_FRAME_SHIFT) - 1))
#define GPUVM_PTE_REF         (1ull << 32)
#define GPUVM_PTE_DIRTY       (1ull << 33)
#define GPUVM_PTE_STATE_SHIFT 34
#define GPUVM_PTE_STATE_MASK  (3ull << GPUVM_PTE_STATE_SHIFT)
#define GPUVM_PTE_DEFER       (1ull << 36)   /* write-aware CLOCK: dirty page already spared once;
                                                 generalized CLOCK: second bit of the use count    */
#define GPUVM_PTE_FRAME_SHIFT 37
#define GPUVM_ST_INVALID  0ull
#define GPUVM_ST_LOADING  1ull
#define GPUVM_ST_RESIDENT 2ull
#define GPUVM_ST_EVICTING 3ull
#define GPUVM_NO_PAGE 0xFFFFFFFFu

/* slots of one shard of gpuvm_dev_t::stats.  The eight counters a fault
 * touches come first and share 64 bytes, so that one fault updates them with
 * ONE atomic instruction (lane r adds to slot r); gpuvm_stats() sorts the
 * slots into the order of gpuvm_stats_t.  Bytes are not counted per fault:
 * every page moved is page_bytes long except the last page of the data set if
 * it is short, whose fetches and write-backs are counted in SHORT_IN / SHORT_OUT.
 * Evictions are not counted either: a fault takes a frame that was never used
 * (FRESH, at most n_frames times after a reset) or evicts a victim, so
 * evictions = faults - fresh, and a fault in the steady state adds to FAULTS only. */
enum {
    GPUVM_S_FAULTS = 0, GPUVM_S_FRESH, GPUVM_S_WB_EVICT, GPUVM_S_SHORT_IN,
    GPUVM_S_SHORT_OUT, GPUVM_S_SKIPS, GPUVM_S_SWEEPS, GPUVM_S_NOFETCH,
    GPUVM_S_WB_FLUSH, GPUVM_S_HITS, GPUVM_S_GROUPS, GPUVM_S_COALESCED,
    GPUVM_S_WAITS, GPUVM_S_PHASES, GPUVM_S_REMOTE, GPUVM_S_COUNT = 16
};
#define GPUVM_S_FAULT_SLOTS 8

__device__ __forceinline__ bool gpuvm_uses_ref(unsigned int policy) {
    return policy == GPUVM_POLICY_CLOCK || policy == GPUVM_POLICY_CLOCK_WRITE_AWARE;
}
/* Two-handed CLOCK: the frame the front hand stands on while the cursor is on
 * frame f - n_frames * e / 8 positions ahead, e = 1..7 from the handle's flags;
 * e = 0 puts it on f itself, which means there is no front hand (one-handed
 * CLOCK). */
__device__ __forceinline__ unsigned int gpuvm_clock_spread(const gpuvm_dev_t &vm) {
    const unsigned int eighths = (vm.flags >> GPUVM_F_HANDS_SHIFT) & GPUVM_F_HANDS_MASK;
    return gpuvm_uses_ref(vm.policy) ? (unsigned int)(((unsigned long long)vm.n_frames * eighths) >> 3) : 0u;
}
__device__ __forceinline__ unsigned int gpuvm_front_hand(const gpuvm_dev_t &vm, unsigned int f) {
    const unsigned int g = f + gpuvm_clock_spread(vm);
    return g >= vm.n_frames ? g - vm.n_frames : g;
}
/* What a use of a resident page adds to its word: the reference bit under the
 * CLOCK policies; under the generalized CLOCK one step of the use count, which
 * is the number of set bits among REF and DEFER (0..2), so that uses and the
 * hand can race without ever producing a meaningless combination. */
__device__ __forceinline__ unsigned long long gpuvm_use_mark(unsigned int policy, unsigned long long word) {
    if (policy == GPUVM_POLICY_GCLOCK)
        return !(word & GPUVM_PTE_REF) ? GPUVM_PTE_REF : !(word & GPUVM_PTE_DEFER) ? GPUVM_PTE_DEFER : 0ull;
    return gpuvm_uses_ref(policy) && !(word & GPUVM_PTE_REF) ? GPUVM_PTE_REF : 0ull;
}

namespace gpuvm_detail {

#define GPUVM_DEV __device__ __forceinline__

GPUVM_DEV unsigned long long a_load(const unsigned long long *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
GPUVM_DEV unsigned int a_load(const unsigned int *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
GPUVM_DEV void a_store(unsigned int *p, unsigned int v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
GPUVM_DEV unsigned long long a_add(unsigned long long *p, unsigned long long v) {
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
GPUVM_DEV unsigned long long a_or(unsigned long long *p, unsigned long long v) {
    return __hip_atomic_fetch_or(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
GPUVM_DEV unsigned long long a_and(unsigned long long *p, unsigned long long v) {
    return __hip_atomic_fetch_and(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
GPUVM_DEV unsigned long long a_xor(unsigned long long *p, unsigned long long v) {
    return __hip_atomic_fetch_xor(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
GPUVM_DEV bool a_cas(unsigned long long *p, unsigned long long *expected, unsigned long long desired) {
    return __hip_atomic_compare_exchange_strong(p, expected, desired, __ATOMIC_RELAXED,
                                                __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

/* completion of everything this wave has issued to memory (loads returned,
 * stores and atomics acknowledged at their scope); also a compiler barrier */
GPUVM_DEV void wait_vm() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

GPUVM_DEV unsigned int bcast(unsigned int v) { return __builtin_amdgcn_readfirstlane(v); }
GPUVM_DEV unsigned long long bcast(unsigned long long v) {
    unsigned int lo = __builtin_amdgcn_readfirstlane((unsigned int)v);
    unsigned int hi = __builtin_amdgcn_readfirstlane((unsigned int)(v >> 32));
    return ((unsigned long long)hi << 32) | lo;
}

/* the lanes that are executing right now, and this lane's place among them */
struct wave_t {
    unsigned long long active;
    unsigned int rank, count;
    bool leader;
};
GPUVM_DEV wave_t wave_now() {
    wave_t w;
    w.active = __builtin_amdgcn_ballot_w64(true);
    unsigned int below = __builtin_amdgcn_mbcnt_hi((unsigned int)(w.active >> 32),
                          __builtin_amdgcn_mbcnt_lo((unsigned int)w.active, 0u));
    w.rank = below;
    w.count = (unsigned int)__popcll(w.active);
    w.leader = below == 0;
    return w;
}

GPUVM_DEV unsigned long long *stat_shard(const gpuvm_dev_t &vm) {
    return vm.stats + (size_t)(blockIdx.x & (GPUVM_STAT_SLOTS - 1)) * GPUVM_S_COUNT;
}
GPUVM_DEV void stat_add(const gpuvm_dev_t &vm, int which, unsigned long long v) {
    __hip_atomic_fetch_add(stat_shard(vm) + which, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

/* the counters of one fault, all at once: the values are wave-uniform, active
 * lane r adds the r-th of them to slot r of the shard (one instruction for a
 * full wave; a wave with fewer than eight active lanes takes several turns) */
GPUVM_DEV void stat_add_fault(const gpuvm_dev_t &vm, unsigned int rank, unsigned int count,
                              unsigned long long fresh, unsigned long long wb, unsigned long long short_in,
                              unsigned long long short_out, unsigned long long skips, unsigned long long sweeps,
                              unsigned long long nofetch) {
    unsigned long long *shard = stat_shard(vm);
    for (unsigned int r = rank; r < GPUVM_S_FAULT_SLOTS; r += count) {
        const unsigned long long v = r == GPUVM_S_FAULTS ? 1ull : r == GPUVM_S_FRESH ? fresh
                                   : r == GPUVM_S_WB_EVICT ? wb : r == GPUVM_S_SHORT_IN ? short_in
                                   : r == GPUVM_S_SHORT_OUT ? short_out : r == GPUVM_S_SKIPS ? skips
                                   : r == GPUVM_S_SWEEPS ? sweeps : nofetch;
        if (v) __hip_atomic_fetch_add(shard + r, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

/* first error wins; every bounded wait polls this word so that one wave that
 * gives up releases all the others */
GPUVM_DEV void raise_error(const gpuvm_dev_t &vm, int code) {
    unsigned long long expected = 0;
    a_cas(vm.hand + 1, &expected, (unsigned long long)(unsigned int)(-code));
}
GPUVM_DEV bool aborted(const gpuvm_dev_t &vm) { return a_load(vm.hand + 1) != 0; }

GPUVM_DEV unsigned int page_len(const gpuvm_dev_t &vm, unsigned int page) {
    unsigned long long lo = (unsigned long long)page << vm.page_shift;
    unsigned long long left = vm.bytes - lo;
    unsigned long long full = 1ull << vm.page_shift;
    return (unsigned int)(left < full ? left : full);
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

/* cache-scope bits of a buffer instruction's aux operand on gfx942/gfx950 */
#define GPUVM_AUX_AGENT  16   /* sc1: coherent across the XCDs of this GPU */
#define GPUVM_AUX_SYSTEM 17   /* sc0 sc1: coherent with the host           */

/* Buffer descriptor over [base, base + bytes): raw (stride 0) addressing,
 * out-of-range lanes read 0 / write nothing. */
GPUVM_DEV __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned int bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

/* Whole-wave copy: the active lanes move `bytes` from src to dst, 16 bytes per
 * lane per instruction, lanes on consecutive addresses (one instruction of a
 * full wave covers 1 KiB), up to 8 loads in flight per lane before the first
 * store.  This is the page mover (both directions) and the write-back.
 * LD / ST are the cache scopes of the two sides. */
template <int UNROLL, int LD, int ST>
GPUVM_DEV void copy_tier(__amdgpu_buffer_rsrc_t rd, __amdgpu_buffer_rsrc_t rs, unsigned int &o,
                         unsigned int stride, unsigned int vec_bytes) {
    for (; o + (UNROLL - 1) * stride < vec_bytes; o += UNROLL * stride) {
        u32x4 r[UNROLL];
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) r[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, o + j * stride, 0, LD);
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) __builtin_amdgcn_raw_buffer_store_b128(r[j], rd, o + j * stride, 0, ST);
    }
}
template <int LD, int ST>
GPUVM_DEV void wave_copy(char *dst, const char *src, unsigned int bytes, const wave_t &w) {
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(src, bytes), rd = make_rsrc(dst, bytes);
    const unsigned int stride = w.count * 16u;
    const unsigned int vec_bytes = bytes & ~15u;
    unsigned int o = w.rank * 16u;
    copy_tier<8, LD, ST>(rd, rs, o, stride, vec_bytes);   /* 64 KiB page, full wave: 8 rounds of 8 KiB */
    copy_tier<4, LD, ST>(rd, rs, o, stride, vec_bytes);   /* 4 KiB page, full wave: one round          */
    copy_tier<2, LD, ST>(rd, rs, o, stride, vec_bytes);
    copy_tier<1, LD, ST>(rd, rs, o, stride, vec_bytes);
    /* < 16 bytes left over (a short last page); the wave may have fewer active lanes than that */
    for (unsigned int t = vec_bytes + w.rank; t < bytes; t += w.count)
        __builtin_amdgcn_raw_buffer_store_b8(__builtin_amdgcn_raw_buffer_load_b8(rs, t, 0, LD), rd, t, 0, ST);
}
/* Whole-wave exchange for a fault whose victim is dirty: the old content of the
 * frame goes to `host_old` while the new page comes from `host_new`, with the
 * loads of both directions in flight together, so the fault pays one trip over
 * the link instead of two in a row.  Every lane reads a piece of the frame
 * before it overwrites that same piece (the store of the new piece is issued
 * after the store of the old one, which needs the loaded data).  Both pages
 * are `bytes` long, a multiple of 16. */
template <int UNROLL>
GPUVM_DEV void swap_tier(__amdgpu_buffer_rsrc_t rf, __amdgpu_buffer_rsrc_t ro, __amdgpu_buffer_rsrc_t rn,
                         unsigned int &o, unsigned int stride, unsigned int bytes) {
    for (; o + (UNROLL - 1) * stride < bytes; o += UNROLL * stride) {
        u32x4 vo[UNROLL], vn[UNROLL];
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) vn[j] = __builtin_amdgcn_raw_buffer_load_b128(rn, o + j * stride, 0, GPUVM_AUX_SYSTEM);
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) vo[j] = __builtin_amdgcn_raw_buffer_load_b128(rf, o + j * stride, 0, GPUVM_AUX_AGENT);
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) __builtin_amdgcn_raw_buffer_store_b128(vo[j], ro, o + j * stride, 0, GPUVM_AUX_SYSTEM);
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) __builtin_amdgcn_raw_buffer_store_b128(vn[j], rf, o + j * stride, 0, GPUVM_AUX_AGENT);
    }
}
GPUVM_DEV void swap_frame_with_host(char *frame, char *host_old, const char *host_new, unsigned int bytes,
                                    const wave_t &w) {
    const __amdgpu_buffer_rsrc_t rf = make_rsrc(frame, bytes), ro = make_rsrc(host_old, bytes),
                                 rn = make_rsrc(host_new, bytes);
    const unsigned int stride = w.count * 16u;
    unsigned int o = w.rank * 16u;
    swap_tier<4>(rf, ro, rn, o, stride, bytes);       /* 8 loads in flight per lane, like wave_copy */
    swap_tier<1>(rf, ro, rn, o, stride, bytes);
}
GPUVM_DEV void copy_host_to_frame(char *frame, const char *host, unsigned int bytes, const wave_t &w) {
    wave_copy<GPUVM_AUX_SYSTEM, GPUVM_AUX_AGENT>(frame, host, bytes, w);
}
GPUVM_DEV void copy_frame_to_host(char *host, const char *frame, unsigned int bytes, const wave_t &w) {
    wave_copy<GPUVM_AUX_AGENT, GPUVM_AUX_SYSTEM>(host, frame, bytes, w);
}

/* Remote-first mode: should this read of a page that is not resident be served
 * in place?  Yes while the page is INVALID and its reads in place have not yet
 * cost what a migration costs; then the touch is counted (a CAS: the word may
 * change state under us, and the count shares its bits with the frame index of
 * a resident page).  No: the caller migrates the page.  One lane calls this. */
GPUVM_DEV bool touch_in_place(const gpuvm_dev_t &vm, unsigned int page) {
    const unsigned long long limit = vm.flags >> GPUVM_F_REMOTE_SHIFT;
    unsigned long long cur = a_load(vm.pte + page);
    /* (a failed CAS returns the word as it is now; waves that walk an index array in
     * step can meet on one word, so a few failures are not yet a reason to migrate) */
    for (int tries = 0; tries < 32; ++tries) {
        if (((cur & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) != GPUVM_ST_INVALID) return false;
        if ((cur >> GPUVM_PTE_FRAME_SHIFT) + 1 >= limit) return false;
        if (a_cas(vm.pte + page, &cur, cur + (1ull << GPUVM_PTE_FRAME_SHIFT))) {
            stat_add(vm, GPUVM_S_REMOTE, 1);
            return true;
        }
    }
    return false;
}

/* The cursor stands on frame f, whose owner entry read q and whose page word
 * read pq: take the frame if the policy allows (true: victim / wb are set, the
 * victim's word is claimed), else pass it (false).  A clean victim becomes
 * INVALID with the claiming CAS itself - its frame holds nothing that host
 * memory does not, and the frame table keeps naming it until the new owner is
 * recorded, which makes the frame look busy to anybody else; a dirty victim
 * becomes EVICTING and turns INVALID once its write-back has completed. */
GPUVM_DEV bool claim_or_pass(const gpuvm_dev_t &vm, unsigned int f, unsigned int q, unsigned long long pq,
                             unsigned int &victim, unsigned int &wb, unsigned int &skips, unsigned int &sweeps,
                             bool &redraw, bool &waiting) {
    if (q == GPUVM_NO_PAGE ||                                  /* first install still under way */
        ((pq & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) != GPUVM_ST_RESIDENT ||
        (unsigned int)(pq >> GPUVM_PTE_FRAME_SHIFT) != f ||
        (pq & GPUVM_PTE_PIN_MASK) != 0) {                      /* busy or in use */
        if (vm.policy == GPUVM_POLICY_FIFO_WAIT) {             /* the paper's rule: wait for this frame */
            if (!waiting) { waiting = true; stat_add(vm, GPUVM_S_WAITS, 1); }
            redraw = false;
            __builtin_amdgcn_s_sleep(4);
        } else {
            ++skips;                                           /* this build's default: pass it over */
        }
        return false;
    }
    if (gpuvm_uses_ref(vm.policy) && (pq & GPUVM_PTE_REF)) {
        a_and(vm.pte + q, ~GPUVM_PTE_REF);                    /* second chance */
        ++sweeps;
        return false;
    }
    if (vm.policy == GPUVM_POLICY_GCLOCK && (pq & (GPUVM_PTE_REF | GPUVM_PTE_DEFER))) {
        a_and(vm.pte + q, ~((pq & GPUVM_PTE_DEFER) ? GPUVM_PTE_DEFER : GPUVM_PTE_REF));   /* count - 1 */
        ++sweeps;
        return false;
    }
    if (vm.policy == GPUVM_POLICY_CLOCK_WRITE_AWARE && (pq & GPUVM_PTE_DIRTY) && !(pq & GPUVM_PTE_DEFER)) {
        /* a written page costs a write-back: spare it once and look for a
         * clean victim first (a CAS: without a pin the page may leave) */
        unsigned long long expect = pq;
        a_cas(vm.pte + q, &expect, pq | GPUVM_PTE_DEFER);
        ++sweeps;
        return false;
    }
    /* claim the victim; fails if anybody pinned it in the meantime */
    const bool dirty = (pq & GPUVM_PTE_DIRTY) != 0;
    if (!a_cas(vm.pte + q, &pq, dirty ? pq | GPUVM_PTE_STATE_MASK : pq & GPUVM_PTE_KEEP_MASK)) {
        if (vm.policy == GPUVM_POLICY_FIFO_WAIT) redraw = false; else ++skips;
        return false;
    }
    victim = q;
    wb = dirty ? 1u : 0u;
    return true;
}

/* Frame allocation + eviction + migration for `page`, whose state word this
 * wave has just moved INVALID -> LOADING.  Returns the frame, or GPUVM_NO_PAGE
 * if a bounded wait ran out (error recorded).
 * Atomics of one fault on the leader's dependent chain: the ticket, the claim
 * of the victim; off the chain (nobody waits for their result): the front
 * hand's bit clearing, the victim's INVALID (dirty victims only - a clean one
 * becomes INVALID with the claim itself), the publishing xor, the counters. */
GPUVM_DEV unsigned int fault(const gpuvm_dev_t &vm, unsigned int page, bool write, unsigned int gen,
                             const wave_t &w, bool fetch = true, unsigned long long *deferred = nullptr) {
    unsigned int f = 0, victim = GPUVM_NO_PAGE, wb = 0, ok = 1, n_skips = 0, n_sweeps = 0;
    if (w.leader) {
        unsigned int skips = 0, sweeps = 0;
        bool redraw = true, waiting = false;
        const unsigned long long budget = 8ull * vm.n_frames + vm.spin_limit;
        /* what the frame after the cursor's looked like when the cursor's own was read:
         * if this frame is passed and the next ticket is the next frame (nobody else
         * drew in between), the pass costs the ticket's round trip only */
        unsigned long long ahead_ticket = ~0ull, ahead_pq = 0;
        unsigned int ahead_q = GPUVM_NO_PAGE;
        for (unsigned long long tries = 0;; ++tries) {
            if (tries > budget || ((tries & 1023) == 1023 && aborted(vm))) {
                raise_error(vm, GPUVM_EDEADLK);
                ok = 0;
                break;
            }
            unsigned int q, qg = GPUVM_NO_PAGE, g = f;
            if (redraw) {
                const unsigned long long t = a_add(vm.hand, 1ull);
                f = (unsigned int)(t % vm.n_frames);
                /* the two hands move together: the frame-table entries are read at once
                 * (cursor, the frame after it, front hand), then their pages' words */
                g = gpuvm_front_hand(vm, f);
                const bool first_turn = t < vm.n_frames;
                const bool known = t == ahead_ticket;
                const unsigned int f1 = f + 1 == vm.n_frames ? 0u : f + 1;
                q = first_turn ? GPUVM_NO_PAGE : known ? ahead_q : a_load(vm.frame_owner + f);
                const unsigned int q1 = t + 1 < vm.n_frames ? GPUVM_NO_PAGE : a_load(vm.frame_owner + f1);
                if (g != f) qg = a_load(vm.frame_owner + g);
                unsigned long long pg = qg == GPUVM_NO_PAGE ? 0ull : a_load(vm.pte + qg);
                if (first_turn) {                             /* first turn: frame never used */
                    if ((pg & GPUVM_PTE_REF) && (unsigned int)(pg >> GPUVM_PTE_FRAME_SHIFT) == g &&
                        ((pg & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) == GPUVM_ST_RESIDENT)
                        a_and(vm.pte + qg, ~GPUVM_PTE_REF);
                    break;
                }
                unsigned long long pq0 = q == GPUVM_NO_PAGE ? 0ull : known ? ahead_pq : a_load(vm.pte + q);
                ahead_pq = q1 == GPUVM_NO_PAGE ? 0ull : a_load(vm.pte + q1);
                ahead_q = q1;
                ahead_ticket = t + 1;
                if ((pg & GPUVM_PTE_REF) && (unsigned int)(pg >> GPUVM_PTE_FRAME_SHIFT) == g &&
                    ((pg & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) == GPUVM_ST_RESIDENT)
                    a_and(vm.pte + qg, ~GPUVM_PTE_REF);       /* front hand: the bit starts its last lap */
                if (claim_or_pass(vm, f, q, pq0, victim, wb, skips, sweeps, redraw, waiting)) break;
                continue;
            }
            redraw = true;                                    /* the waiting policy looks at its frame again */
            q = a_load(vm.frame_owner + f);
            const unsigned long long pq = q == GPUVM_NO_PAGE ? 0ull : a_load(vm.pte + q);
            if (claim_or_pass(vm, f, q, pq, victim, wb, skips, sweeps, redraw, waiting)) break;
        }
        n_skips = skips; n_sweeps = sweeps;
    }
    ok = bcast(ok);
    if (!ok) {
        if (w.leader) a_and(vm.pte + page, GPUVM_PTE_KEEP_MASK);         /* back to INVALID */
        return GPUVM_NO_PAGE;
    }
    f = bcast(f); victim = bcast(victim); wb = bcast(wb);
    char *frame = vm.frames + ((size_t)f << vm.page_shift);
    const unsigned int len = page_len(vm, page);
    const unsigned int full = 1u << vm.page_shift;
    unsigned int vlen = 0;
    bool fetched = false;
    if (wb) {                                                 /* only a dirty victim is still EVICTING here */
        vlen = page_len(vm, victim);
        if ((vm.flags & GPUVM_F_OVERLAPPED_WRITEBACK) && fetch && vlen == len && (len & 15u) == 0) {
            /* write-back and fetch share one pass over the frame */
            swap_frame_with_host(frame, vm.host + ((size_t)victim << vm.page_shift),
                                 vm.host + ((size_t)page << vm.page_shift), len, w);
            fetched = true;
        } else {
            copy_frame_to_host(vm.host + ((size_t)victim << vm.page_shift), frame, vlen, w);
        }
        wait_vm();                                            /* posted before the victim can be re-read */
        if (w.leader) a_and(vm.pte + victim, GPUVM_PTE_KEEP_MASK);      /* INVALID; waiters keep their pins */
    }
    if (fetch && !fetched) copy_host_to_frame(frame, vm.host + ((size_t)page << vm.page_shift), len, w);
    if (w.leader) a_store(vm.frame_owner + f, page);
    wait_vm();                                                /* the page is in the frame */
    /* only this wave changes anything but the pin field while the page is
     * LOADING, so one xor moves state, frame, flags and generation at once */
    const unsigned long long flip =
        ((GPUVM_ST_LOADING ^ GPUVM_ST_RESIDENT) << GPUVM_PTE_STATE_SHIFT) |
        ((unsigned long long)f << GPUVM_PTE_FRAME_SHIFT) |
        /* the reference bit of a new page: clear under the generalized CLOCK (use
         * count 0), set otherwise.  With a front hand the bit could be left clear
         * without changing any decision (that hand goes by before the cursor
         * returns) and the hand would save an atomic - but then every wave that
         * reads a fresh page finds the bit clear and tries to set it, and when
         * hundreds of waves read the same new page at the same moment (the
         * column-order product) those attempts queue on the page's word: 33.8 ms
         * against 22.6 on a 16384 x 16384 matrix. */
        (vm.policy == GPUVM_POLICY_GCLOCK ? 0ull : GPUVM_PTE_REF) |
        (write ? GPUVM_PTE_DIRTY : 0ull) |
        ((unsigned long long)(gen ^ ((gen + 1u) & 0xFFFu)) << GPUVM_PTE_GEN_SHIFT);
    if (deferred) {
        /* the caller accesses the frame first and then publishes and drops its
         * reference with ONE add: the bits above the pin field are known exactly
         * (LOADING, this generation, nothing else), so new - old - 1 is exact */
        const unsigned long long before = (GPUVM_ST_LOADING << GPUVM_PTE_STATE_SHIFT) |
                                          ((unsigned long long)gen << GPUVM_PTE_GEN_SHIFT);
        *deferred = (before ^ flip) - before - 1ull;
    } else if (w.leader) {
        a_xor(vm.pte + page, flip);                           /* publish: RESIDENT */
    }
    stat_add_fault(vm, w.rank, w.count, victim == GPUVM_NO_PAGE, wb, fetch && len != full, wb && vlen != full,
                   bcast(n_skips), bcast(n_sweeps), fetch ? 0u : 1u);
    return f;
}

/* lookup + pin of one page for the whole wave; see gpuvm_acquire.  `hint` is
 * what the caller last read from the page's word, if it has (GPUVM_NO_HINT
 * otherwise): when that says INVALID, reference count and INVALID -> LOADING
 * are tried as one CAS on it instead of an add followed by a CAS. */
#define GPUVM_NO_HINT (~0ull)
GPUVM_DEV char *acquire_page(const gpuvm_dev_t &vm, unsigned int page_any, bool write, bool fetch,
                             unsigned long long hint = GPUVM_NO_HINT, unsigned long long *deferred = nullptr,
                             bool mark = true) {
    const wave_t w = wave_now();
    const unsigned int page = bcast(page_any);
    unsigned long long *pte = vm.pte + page;
    unsigned long long cur = 0;
    unsigned int how = 0;                     /* 0 hit, 1 this wave faults, 2 gave up */
    if (w.leader) {
        if (hint != GPUVM_NO_HINT && ((hint & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) == GPUVM_ST_INVALID) {
            cur = hint;
            const unsigned long long mine = ((hint & GPUVM_PTE_KEEP_MASK) + 1ull) | (GPUVM_ST_LOADING << GPUVM_PTE_STATE_SHIFT);
            if (a_cas(pte, &cur, mine)) { cur = mine; how = 1; }
        }
        if (how == 0) cur = a_add(pte, 1ull) + 1ull;        /* lookup and reference count in one atomic */
        unsigned int spins = 0;
        while (how == 0) {
            const unsigned long long st = (cur & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT;
            if (st == GPUVM_ST_RESIDENT) break;
            if (st == GPUVM_ST_INVALID) {     /* inter-wave arbitration: one wave locks the entry */
                /* (the bits above the state may hold a count of reads in place: it ends here) */
                if (a_cas(pte, &cur, (cur & GPUVM_PTE_KEEP_MASK) | (GPUVM_ST_LOADING << GPUVM_PTE_STATE_SHIFT))) { how = 1; break; }
                continue;
            }
            if (spins == 0) stat_add(vm, GPUVM_S_WAITS, 1);
            if (++spins > vm.spin_limit || ((spins & 63) == 63 && aborted(vm))) {
                raise_error(vm, GPUVM_EDEADLK);
                how = 2;
                break;
            }
            __builtin_amdgcn_s_sleep(4);
            cur = a_load(pte);
        }
    }
    how = bcast(how);
    if (how == 2) return vm.frames;
    cur = bcast(cur);
    unsigned int f;
    if (how == 1) {
        f = fault(vm, page, write, (unsigned int)(cur >> GPUVM_PTE_GEN_SHIFT) & 0xFFFu, w, fetch, deferred);
        if (f == GPUVM_NO_PAGE) { if (deferred) *deferred = 0; return vm.frames; }
    } else {
        f = (unsigned int)(cur >> GPUVM_PTE_FRAME_SHIFT);
        if (w.leader) {
            unsigned long long need = 0;
            if (write && !(cur & GPUVM_PTE_DIRTY)) need |= GPUVM_PTE_DIRTY;
            if (mark) need |= gpuvm_use_mark(vm.policy, cur);
            if (need) a_or(pte, need);
            if (vm.flags & GPUVM_F_ACCESS_STATS) stat_add(vm, GPUVM_S_HITS, 1);
        }
    }
    return vm.frames + ((size_t)f << vm.page_shift);
}

}  // namespace gpuvm_detail

/* Pin `page` (the same value in every active lane) and return the address of
 * its frame, migrating it first if it is not in GPU memory.  `write` = the
 * caller will modify the page.  Must be followed by gpuvm_release before the
 * wave acquires another page of the same handle.  After a recorded error the
 * returned pointer is a valid dummy (frame 0) so that callers never
 * dereference garbage. */
__device__ __forceinline__ char *gpuvm_acquire(const gpuvm_dev_t &vm, unsigned int page_any, bool write) {
    return gpuvm_detail::acquire_page(vm, page_any, write, true);
}

/* gpuvm_acquire for callers that expect the page NOT to be resident (a scan, a
 * fault-ahead, the first touch of a page per round): the page's word is read
 * first, and if it says INVALID the reference and the INVALID -> LOADING lock are
 * taken with one CAS on that value instead of an add followed by a CAS - one
 * atomic less per fault; a resident page costs one more load than gpuvm_acquire.
 * gpuvm_acquire_hinted takes the word from a caller that has read it already
 * (the token of a gpuvm_peek that did not validate).
 * `last_use`: the caller will not come back to the page for a long time (one
 * visit per page and round); a hit then leaves the replacement policy's mark
 * as it is, so that the page is not kept in preference to pages that are still
 * waiting for their visit. */
__device__ __forceinline__ char *gpuvm_acquire_hinted(const gpuvm_dev_t &vm, unsigned int page_any, bool write,
                                                      unsigned long long word) {
    return gpuvm_detail::acquire_page(vm, page_any, write, true, gpuvm_detail::bcast(word));
}
__device__ __forceinline__ char *gpuvm_acquire_cold(const gpuvm_dev_t &vm, unsigned int page_any, bool write,
                                                    bool last_use = false) {
    const unsigned int page = gpuvm_detail::bcast(page_any);
    unsigned long long word = 0;
    if (gpuvm_detail::wave_now().leader) word = gpuvm_detail::a_load(vm.pte + page);
    return gpuvm_detail::acquire_page(vm, page, write, true, gpuvm_detail::bcast(word), nullptr, !last_use);
}

/* The same for a caller that will store every byte of the page before it
 * releases it: on a miss the frame is installed without reading the page from
 * the host (its old content would be overwritten anyway), which saves one page
 * of link traffic per fault.  The frame's bytes are undefined until written;
 * the page is DIRTY from the start.  Not in the paper, whose write faults
 * always fetch. */
__device__ __forceinline__ char *gpuvm_acquire_overwrite(const gpuvm_dev_t &vm, unsigned int page_any) {
    return gpuvm_detail::acquire_page(vm, page_any, true, false);
}

/* Drop the pin taken by gpuvm_acquire, once everything the wave issued to the
 * page has completed. */
__device__ __forceinline__ void gpuvm_release(const gpuvm_dev_t &vm, unsigned int page_any) {
    using namespace gpuvm_detail;
    const wave_t w = wave_now();
    const unsigned int page = bcast(page_any);
    wait_vm();
    if (w.leader) a_add(vm.pte + page, ~0ull);                /* pin - 1 */
}

/* Fault-ahead: make `page` resident (if it is not) and let go of it at once;
 * the data is not touched.  For waves that run ahead of the ones that will
 * use the page, the device-side counterpart of a prefetch hint. */
__device__ __forceinline__ void gpuvm_touch(const gpuvm_dev_t &vm, unsigned int page_any) {
    (void)gpuvm_acquire_cold(vm, page_any, false);
    gpuvm_release(vm, page_any);
}

/* Optimistic page-level read for wave-level users (same page in every lane):
 * gpuvm_peek returns the frame of `page` if it is RESIDENT right now, without
 * taking a reference, and the page's word in *token; read the frame with
 * gpuvm_frame_load_*(), then ask gpuvm_peek_valid: true means the frame held
 * the page during all of those reads (state, frame and install generation are
 * unchanged), false means the values must be thrown away and the page taken
 * with gpuvm_acquire.  Nothing is pinned, so readers of a hot page do not
 * serialise on its word and never hold up an eviction.
 *
 * The same in four steps, for callers that keep several such reads in flight
 * (all the words, then all the frame reads, one wait, all the re-checks):
 *   token = gpuvm_peek_begin(vm, page);  frame = gpuvm_token_frame(vm, token);
 *   ... gpuvm_frame_load_*(vm, frame, ..) if frame != nullptr ...
 *   gpuvm_wait_reads();  again = gpuvm_peek_begin(vm, page);
 *   ok = gpuvm_peek_same(vm, page, token, again);
 * Every lane loads the word itself (one address, one request), so there is no
 * leader and no broadcast between the steps. */
__device__ __forceinline__ unsigned long long gpuvm_peek_begin(const gpuvm_dev_t &vm, unsigned int page) {
    return gpuvm_detail::a_load(vm.pte + page);
}
__device__ __forceinline__ const char *gpuvm_token_frame(const gpuvm_dev_t &vm, unsigned long long token) {
    if (((token & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) != GPUVM_ST_RESIDENT) return nullptr;
    return vm.frames + ((size_t)(token >> GPUVM_PTE_FRAME_SHIFT) << vm.page_shift);
}
__device__ __forceinline__ void gpuvm_wait_reads() { gpuvm_detail::wait_vm(); }
__device__ __forceinline__ bool gpuvm_peek_same(const gpuvm_dev_t &vm, unsigned int page, unsigned long long token,
                                                unsigned long long again) {
    using namespace gpuvm_detail;
    const bool same = ((again ^ token) & GPUVM_PTE_IDENT_MASK) == 0 &&
                      ((token & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) == GPUVM_ST_RESIDENT;
    const unsigned long long mark = same ? gpuvm_use_mark(vm.policy, again) : 0ull;
    if (mark && wave_now().leader) {
        unsigned long long expect = again;                    /* second-chance bit / use count, best effort */
        a_cas(vm.pte + page, &expect, again | mark);
    }
    if (same && (vm.flags & GPUVM_F_ACCESS_STATS) && wave_now().leader) stat_add(vm, GPUVM_S_HITS, 1);
    return same;
}
__device__ __forceinline__ const char *gpuvm_peek(const gpuvm_dev_t &vm, unsigned int page_any,
                                                  unsigned long long *token) {
    const unsigned int page = gpuvm_detail::bcast(page_any);
    *token = gpuvm_peek_begin(vm, page);
    return gpuvm_token_frame(vm, *token);
}
__device__ __forceinline__ bool gpuvm_peek_valid(const gpuvm_dev_t &vm, unsigned int page_any,
                                                 unsigned long long token) {
    const unsigned int page = gpuvm_detail::bcast(page_any);
    gpuvm_wait_reads();                                       /* the reads have returned */
    return gpuvm_peek_same(vm, page, token, gpuvm_peek_begin(vm, page));
}

/* Coherent reads of frame memory for wave-level users of gpuvm_acquire:
 * `frame` is the pointer gpuvm_acquire returned (the same in every lane),
 * `byte_off` the lane's offset into the page.  Offsets beyond the page read 0. */
__device__ __forceinline__ unsigned int gpuvm_frame_load_b32(const gpuvm_dev_t &vm, const char *frame, unsigned int byte_off) {
    return __builtin_amdgcn_raw_buffer_load_b32(gpuvm_detail::make_rsrc(frame, 1u << vm.page_shift), byte_off, 0, GPUVM_AUX_AGENT);
}
__device__ __forceinline__ gpuvm_detail::u32x2 gpuvm_frame_load_b64(const gpuvm_dev_t &vm, const char *frame, unsigned int byte_off) {
    return __builtin_amdgcn_raw_buffer_load_b64(gpuvm_detail::make_rsrc(frame, 1u << vm.page_shift), byte_off, 0, GPUVM_AUX_AGENT);
}
__device__ __forceinline__ gpuvm_detail::u32x4 gpuvm_frame_load_b128(const gpuvm_dev_t &vm, const char *frame, unsigned int byte_off) {
    return __builtin_amdgcn_raw_buffer_load_b128(gpuvm_detail::make_rsrc(frame, 1u << vm.page_shift), byte_off, 0, GPUVM_AUX_AGENT);
}
/* Coherent stores to a frame held through gpuvm_acquire(.., true) or
 * gpuvm_acquire_overwrite.  Offsets beyond the page write nothing. */
__device__ __forceinline__ void gpuvm_frame_store_b32(const gpuvm_dev_t &vm, char *frame, unsigned int byte_off, unsigned int v) {
    __builtin_amdgcn_raw_buffer_store_b32(v, gpuvm_detail::make_rsrc(frame, 1u << vm.page_shift), byte_off, 0, GPUVM_AUX_AGENT);
}
__device__ __forceinline__ void gpuvm_frame_store_b128(const gpuvm_dev_t &vm, char *frame, unsigned int byte_off, gpuvm_detail::u32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, gpuvm_detail::make_rsrc(frame, 1u << vm.page_shift), byte_off, 0, GPUVM_AUX_AGENT);
}

namespace gpuvm_detail {

/* for the counters only: number of distinct pages among the wanting lanes */
GPUVM_DEV unsigned int count_page_groups(unsigned int page, bool want) {
    unsigned int n_groups = 0;
    bool ungrouped = want;
    for (;;) {
        const unsigned long long todo = __builtin_amdgcn_ballot_w64(ungrouped);
        if (todo == 0) break;
        const unsigned int first = (unsigned int)__ffsll((long long)todo) - 1u;
        if (page == (unsigned int)__builtin_amdgcn_readlane(page, first)) ungrouped = false;
        ++n_groups;
    }
    return n_groups;
}

/* second half of an optimistic read: `word` is what the lane read from the
 * page's entry before it read the frame, the frame reads have returned; true
 * if the entry still names the same installation of the page.  Sets the
 * second-chance bit if the hand has cleared it (best effort: a CAS, because
 * without a pin the page may leave at any moment and a plain OR could then
 * mark an entry that is no longer RESIDENT); `may_mark` names the one lane
 * that does so when the whole wave reads one page. */
GPUVM_DEV bool optimistic_read_stands(const gpuvm_dev_t &vm, unsigned int page, unsigned long long word,
                                      unsigned long long again, bool may_mark) {
    const bool still = ((again ^ word) & GPUVM_PTE_IDENT_MASK) == 0;
    const unsigned long long mark = still && may_mark ? gpuvm_use_mark(vm.policy, again) : 0ull;
    if (mark) {
        unsigned long long expect = again;
        a_cas(vm.pte + page, &expect, again | mark);
    }
    return still;
}

/* miss pass: the lanes in `pending` go through gpuvm_acquire one page at a
 * time (all active lanes help to move each page), so that the wave never holds
 * more than one frame while it waits or allocates */
struct no_remote {};      /* tag: this access has no in-place form (writes, atomics) */
template <typename T, typename Op, typename Remote>
GPUVM_DEV void access_missing(const gpuvm_dev_t &vm, unsigned int page, unsigned int off, bool write, bool pending,
                              unsigned long long word, Op op, Remote remote) {
    /* The word of the page that comes after this one, read while this one's fault
     * is under way: what the hit pass saw is a fault or more old by the time a
     * later group's turn comes, and a stale word costs the lookup two atomics
     * more (the CAS on it fails, an add and a second CAS follow). */
    unsigned long long fresh = 0;
    unsigned int fresh_page = GPUVM_NO_PAGE;
    for (;;) {
        const unsigned long long todo = __builtin_amdgcn_ballot_w64(pending);
        if (todo == 0) break;
        const unsigned int first = (unsigned int)__ffsll((long long)todo) - 1u;
        const unsigned int group_page = __builtin_amdgcn_readlane(page, first);
        /* what the group's first lane last saw in the page's word (the hit pass read it) */
        const unsigned long long hint = fresh_page == group_page ? bcast(fresh) :
            ((unsigned long long)(unsigned int)__builtin_amdgcn_readlane((unsigned int)(word >> 32), first) << 32) |
            (unsigned int)__builtin_amdgcn_readlane((unsigned int)word, first);
        {
            const unsigned long long later = __builtin_amdgcn_ballot_w64(pending && page != group_page);
            fresh_page = later ? (unsigned int)__builtin_amdgcn_readlane(page, (unsigned int)__ffsll((long long)later) - 1u)
                               : GPUVM_NO_PAGE;
            if (later) fresh = a_load(vm.pte + fresh_page);           /* one address for the whole wave */
        }
        if constexpr (!__is_same(Remote, no_remote)) {
            /* remote-first: the group's first lane asks whether the page has earned
             * its migration yet; if not, the lanes read host memory in place */
            if (vm.flags >> GPUVM_F_REMOTE_SHIFT) {
                unsigned int in_place = 0;
                if (__lane_id() == first) in_place = touch_in_place(vm, group_page) ? 1u : 0u;
                in_place = __builtin_amdgcn_readlane(in_place, first);
                if (in_place) {
                    if (pending && page == group_page) {
                        remote(reinterpret_cast<T *>(vm.host + ((size_t)group_page << vm.page_shift) + off));
                        pending = false;
                    }
                    continue;
                }
            }
        }
        /* a page this wave faults in is published only after the group's lanes have
         * had their access: publishing and dropping the reference are one atomic */
        unsigned long long publish = 0;
        char *frame = acquire_page(vm, group_page, write, true, hint, &publish);
        if (pending && page == group_page) {
            op(reinterpret_cast<T *>(frame + off));
            pending = false;
        }
        wait_vm();
        if (wave_now().leader) a_add(vm.pte + group_page, publish ? publish : ~0ull);
    }
}

}  // namespace gpuvm_detail

/* Element access with wavefront dedup: calls op(T*) once in every active lane
 * whose `want` is true, on the lane's element.  Lanes with want == false take
 * no element but help to move pages; calling this with all lanes of the wave
 * active (and `want` as the predicate) is what keeps a fault one link round
 * trip wide - under divergence only the active lanes can copy.
 *
 * Hit pass (all lanes at once):
 *   - reads are optimistic and need no grouping: every lane loads its page's
 *     word (lanes on one page load one address, which the memory pipeline
 *     merges), reads its element from the frame the word names and loads the
 *     word again; if state, frame and install generation are unchanged the
 *     frame held the page all the while (eviction changes the word before the
 *     frame is reused, re-installation bumps the generation) and the value
 *     stands.  No atomic, no reference count: readers of a hot page do not
 *     serialise on its word and never block its eviction;
 *   - writes pin: the lanes are grouped by page with ALU work only (lowest lane
 *     of a page = its leader), every leader takes a reference with one
 *     fetch_add, all in the same instruction; resident groups update their
 *     elements, wait, mark the page DIRTY and unpin.  No wave waits while it
 *     holds these pins.
 * Miss pass: lanes whose page was not resident (or whose optimistic read did
 * not validate) are grouped by page - one leader, one fault per page and wave -
 * and go through gpuvm_acquire one page at a time, so that a wave never holds
 * more than one frame while it waits or allocates.  A read may come with a
 * second functor, `remote`: in remote-first mode (gpuvm_set_remote_first) it
 * is called on the element's address in host memory instead, for as long as
 * the page has not earned its migration. */
template <typename T, typename Op, typename Remote = gpuvm_detail::no_remote>
__device__ __forceinline__ void gpuvm_access(const gpuvm_dev_t &vm, unsigned long long elem, bool write, bool want,
                                             Op op, Remote remote = Remote{}) {
    using namespace gpuvm_detail;
    const unsigned long long byte = elem * sizeof(T);
    const unsigned int page = (unsigned int)(byte >> vm.page_shift);              /* address split */
    const unsigned int off = (unsigned int)(byte & ((1ull << vm.page_shift) - 1));
    const unsigned int lane = __lane_id();
    bool resident;
    unsigned int n_groups = 0;
    unsigned long long seen = 0;              /* the page's word as this lane last saw it, without a pin of ours */

    if (!write) {
        /* hit pass, reads.  One page for the whole wave (unit stride, a row
         * segment): its first wanting lane loads the word for everybody.  Several
         * pages: every lane on its own - the loads of lanes that share a page
         * fall on one address, so no grouping is needed. */
        const unsigned long long wanting = __builtin_amdgcn_ballot_w64(want);
        const unsigned int first = wanting ? (unsigned int)__ffsll((long long)wanting) - 1u : 0u;
        const bool one_page =
            __builtin_amdgcn_ballot_w64(want && page != (unsigned int)__builtin_amdgcn_readlane(page, first)) == 0;
        auto load_word = [&]() {
            unsigned long long w = 0;
            if (one_page) {
                if (want && lane == first) w = a_load(vm.pte + page);
                const unsigned int lo = __builtin_amdgcn_readlane((unsigned int)w, first);
                const unsigned int hi = __builtin_amdgcn_readlane((unsigned int)(w >> 32), first);
                w = ((unsigned long long)hi << 32) | lo;
            } else if (want) {
                w = a_load(vm.pte + page);
            }
            return w;
        };
        const unsigned long long word = load_word();
        resident = want && ((word & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) == GPUVM_ST_RESIDENT;
        if (resident)
            op(reinterpret_cast<T *>(vm.frames + ((size_t)(word >> GPUVM_PTE_FRAME_SHIFT) << vm.page_shift) + off));
        wait_vm();
        seen = word;
        if (__builtin_amdgcn_ballot_w64(resident)) {
            const unsigned long long again = load_word();
            if (resident) { resident = optimistic_read_stands(vm, page, word, again, !one_page || lane == first); seen = again; }
        }
    } else {
        /* hit pass, writes: group the wanting lanes by page (leader_lane = lowest
         * lane with my page) so that a page takes one reference per wave */
        unsigned int leader_lane = lane;
        {
            bool ungrouped = want;
            for (;;) {
                const unsigned long long todo = __builtin_amdgcn_ballot_w64(ungrouped);
                if (todo == 0) break;
                const unsigned int first = (unsigned int)__ffsll((long long)todo) - 1u;
                const unsigned int group_page = __builtin_amdgcn_readlane(page, first);
                if (ungrouped && page == group_page) { leader_lane = first; ungrouped = false; }
                ++n_groups;
            }
        }
        const bool is_leader = want && leader_lane == lane;
        unsigned long long word = 0;
        if (is_leader) word = a_add(vm.pte + page, 1ull);
        {
            const unsigned int lo = __shfl((unsigned int)word, (int)leader_lane, 64);
            const unsigned int hi = __shfl((unsigned int)(word >> 32), (int)leader_lane, 64);
            word = ((unsigned long long)hi << 32) | lo;
        }
        resident = want && ((word & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) == GPUVM_ST_RESIDENT;
        if (resident)
            op(reinterpret_cast<T *>(vm.frames + ((size_t)(word >> GPUVM_PTE_FRAME_SHIFT) << vm.page_shift) + off));
        wait_vm();
        if (is_leader) {
            if (resident) {
                unsigned long long need = 0;
                if (!(word & GPUVM_PTE_DIRTY)) need |= GPUVM_PTE_DIRTY;
                need |= gpuvm_use_mark(vm.policy, word);
                if (need) a_or(vm.pte + page, need);
            }
            a_add(vm.pte + page, ~0ull);                      /* unpin, or give the pin back */
        }
        seen = word;                          /* before our pin = after we gave it back, unless somebody else came by */
    }
    if (vm.flags & GPUVM_F_ACCESS_STATS) {
        /* pages, not lanes: a page with any lane still missing counts as a miss */
        if (!write) n_groups = count_page_groups(page, want);
        const unsigned int n_missing = count_page_groups(page, want && !resident);
        const unsigned long long wanting = __builtin_amdgcn_ballot_w64(want);
        if (wave_now().leader) {
            stat_add(vm, GPUVM_S_GROUPS, n_groups);
            stat_add(vm, GPUVM_S_COALESCED, (unsigned long long)__popcll(wanting) - n_groups);
            stat_add(vm, GPUVM_S_HITS, n_groups - n_missing);
        }
    }
    access_missing<T>(vm, page, off, write, want && !resident, seen, op, remote);
}

/* Elements are 4 or 8 bytes wide and are read, written and updated with
 * relaxed agent-scope atomics, which is what keeps frame data coherent
 * between the XCDs without cache maintenance.  The *_if forms take the lane's
 * predicate and are meant to be called by all lanes of the wave together. */
template <typename T>
__device__ __forceinline__ T gpuvm_load_if(const gpuvm_dev_t &vm, unsigned long long elem, bool want) {
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "gpuvm_load: 4- or 8-byte elements");
    T v{};
    gpuvm_access<T>(vm, elem, false, want,
                    [&](T *p) { v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); },
                    [&](T *p) { v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM); });   /* in place */
    return v;
}
template <typename T>
__device__ __forceinline__ T gpuvm_load(const gpuvm_dev_t &vm, unsigned long long elem) {
    return gpuvm_load_if<T>(vm, elem, true);
}

template <typename T>
__device__ __forceinline__ void gpuvm_store_if(const gpuvm_dev_t &vm, unsigned long long elem, T v, bool want) {
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "gpuvm_store: 4- or 8-byte elements");
    gpuvm_access<T>(vm, elem, true, want, [&](T *p) {
        __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    });
}
template <typename T>
__device__ __forceinline__ void gpuvm_store(const gpuvm_dev_t &vm, unsigned long long elem, T v) {
    gpuvm_store_if<T>(vm, elem, v, true);
}

/* data[elem] += v with a device-scope atomic on the frame; returns nothing. */
template <typename T>
__device__ __forceinline__ void gpuvm_atomic_add_if(const gpuvm_dev_t &vm, unsigned long long elem, T v, bool want) {
    gpuvm_access<T>(vm, elem, true, want, [&](T *p) {
        __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    });
}
template <typename T>
__device__ __forceinline__ void gpuvm_atomic_add(const gpuvm_dev_t &vm, unsigned long long elem, T v) {
    gpuvm_atomic_add_if<T>(vm, elem, v, true);
}

/* Several independent reads per lane in one optimistic transaction: the N page
 * words, then the N elements, one wait, the N re-checks - N loads in flight per
 * lane where gpuvm_load has one.  For code whose wave count is bounded by a
 * small pool, so that more waves cannot hide the latency of the three dependent
 * loads of a read.  Lanes whose read did not validate, or whose page is not
 * resident, go through the miss pass one element index at a time.  Called by
 * all lanes of the wave together; want[k] is the lane's predicate for elem[k]. */
template <typename T, int N>
__device__ __forceinline__ void gpuvm_load_n(const gpuvm_dev_t &vm, const unsigned long long (&elem)[N],
                                             const bool (&want)[N], T (&out)[N]) {
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "gpuvm_load_n: 4- or 8-byte elements");
    using namespace gpuvm_detail;
    unsigned int page[N], off[N];
    unsigned long long word[N], seen[N];
    bool resident[N];
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const unsigned long long byte = elem[k] * sizeof(T);
        page[k] = (unsigned int)(byte >> vm.page_shift);
        off[k] = (unsigned int)(byte & ((1ull << vm.page_shift) - 1));
        word[k] = want[k] ? a_load(vm.pte + page[k]) : 0ull;
        out[k] = T{};
    }
#pragma unroll
    for (int k = 0; k < N; ++k) {
        resident[k] = want[k] && ((word[k] & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) == GPUVM_ST_RESIDENT;
        if (resident[k])
            out[k] = __hip_atomic_load(reinterpret_cast<T *>(vm.frames + ((size_t)(word[k] >> GPUVM_PTE_FRAME_SHIFT) << vm.page_shift) + off[k]),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    wait_vm();
#pragma unroll
    for (int k = 0; k < N; ++k) seen[k] = resident[k] ? a_load(vm.pte + page[k]) : word[k];
#pragma unroll
    for (int k = 0; k < N; ++k)
        if (resident[k]) resident[k] = optimistic_read_stands(vm, page[k], word[k], seen[k], true);
#pragma unroll
    for (int k = 0; k < N; ++k) {
        if (vm.flags & GPUVM_F_ACCESS_STATS) {
            const unsigned int n_groups = count_page_groups(page[k], want[k]);
            const unsigned int n_missing = count_page_groups(page[k], want[k] && !resident[k]);
            const unsigned long long wanting = __builtin_amdgcn_ballot_w64(want[k]);
            if (wave_now().leader) {
                stat_add(vm, GPUVM_S_GROUPS, n_groups);
                stat_add(vm, GPUVM_S_COALESCED, (unsigned long long)__popcll(wanting) - n_groups);
                stat_add(vm, GPUVM_S_HITS, n_groups - n_missing);
            }
        }
        T &slot = out[k];
        access_missing<T>(vm, page[k], off[k], false, want[k] && !resident[k], seen[k],
                          [&](T *p) { slot = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); },
                          [&](T *p) { slot = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM); });
    }
}

/* A wave's cursor over a paged array, for code that walks it with unit stride
 * (or stays inside one page for many calls): the wave keeps ONE page pinned
 * between calls - the paper's reference counter, held for as long as the wave
 * stands on the page - so that a call that stays on the page is a compare and a
 * load, with no look at the page table at all.  Moving to another page drops
 * the pin and takes the next one (faulting the page in if need be); a call whose
 * lanes stand on several pages drops the pin and goes through gpuvm_load /
 * gpuvm_store lane by lane.  All lanes of the wave call together with the
 * lane's predicate in `want`; the cursor itself is the same in every lane.
 * The pin counts against the wave's one-frame-per-handle budget like a
 * gpuvm_acquire, and like it must be given back: gpuvm_cursor_end() before the
 * wave leaves, and no gpuvm_acquire on the same handle while a cursor is open. */
struct gpuvm_cursor_t {
    unsigned int page;        /* GPUVM_NO_PAGE: nothing pinned */
    bool dirty;               /* the pinned page is already marked DIRTY */
    char *frame;
};
__device__ __forceinline__ gpuvm_cursor_t gpuvm_cursor_begin() { return gpuvm_cursor_t{GPUVM_NO_PAGE, false, nullptr}; }
__device__ __forceinline__ void gpuvm_cursor_end(const gpuvm_dev_t &vm, gpuvm_cursor_t &c) {
    if (c.page != GPUVM_NO_PAGE) gpuvm_release(vm, c.page);
    c.page = GPUVM_NO_PAGE;
}
namespace gpuvm_detail {
/* true: the cursor now stands on the one page all wanting lanes are on (frame
 * pinned, DIRTY set if write); false: the lanes are on several pages, or nobody
 * wants anything - the cursor holds nothing and the caller takes the general path */
GPUVM_DEV bool cursor_seek(const gpuvm_dev_t &vm, gpuvm_cursor_t &c, unsigned int page, bool want, bool write) {
    const unsigned long long wanting = __builtin_amdgcn_ballot_w64(want);
    if (wanting == 0) return false;
    const bool count = (vm.flags & GPUVM_F_ACCESS_STATS) != 0;
    if (__builtin_amdgcn_ballot_w64(want && page != c.page) == 0) {          /* still on the pinned page */
        if (count && wave_now().leader) {
            stat_add(vm, GPUVM_S_GROUPS, 1);
            stat_add(vm, GPUVM_S_COALESCED, (unsigned long long)__popcll(wanting) - 1);
            stat_add(vm, GPUVM_S_HITS, 1);
        }
        if (write && !c.dirty) {
            if (wave_now().leader) a_or(vm.pte + c.page, GPUVM_PTE_DIRTY);  /* pinned: the word cannot leave RESIDENT */
            c.dirty = true;
        }
        return true;
    }
    const unsigned int first = (unsigned int)__ffsll((long long)wanting) - 1u;
    const unsigned int p = __builtin_amdgcn_readlane(page, first);
    if (c.page != GPUVM_NO_PAGE) { gpuvm_release(vm, c.page); c.page = GPUVM_NO_PAGE; }
    if (__builtin_amdgcn_ballot_w64(want && page != p) != 0) return false;   /* several pages */
    if (count && wave_now().leader) {                                         /* (acquire_page counts the hit, or the fault) */
        stat_add(vm, GPUVM_S_GROUPS, 1);
        stat_add(vm, GPUVM_S_COALESCED, (unsigned long long)__popcll(wanting) - 1);
    }
    c.frame = acquire_page(vm, p, write, true);
    c.page = p;
    c.dirty = write;
    return true;
}
}  // namespace gpuvm_detail
template <typename T>
__device__ __forceinline__ T gpuvm_cursor_load(const gpuvm_dev_t &vm, gpuvm_cursor_t &c, unsigned long long elem, bool want) {
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "gpuvm_cursor_load: 4- or 8-byte elements");
    const unsigned long long byte = elem * sizeof(T);
    const unsigned int page = (unsigned int)(byte >> vm.page_shift);
    const unsigned int off = (unsigned int)(byte & ((1ull << vm.page_shift) - 1));
    if (gpuvm_detail::cursor_seek(vm, c, page, want, false))
        return want ? __hip_atomic_load(reinterpret_cast<T *>(c.frame + off), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : T{};
    return gpuvm_load_if<T>(vm, elem, want);
}
template <typename T>
__device__ __forceinline__ void gpuvm_cursor_store(const gpuvm_dev_t &vm, gpuvm_cursor_t &c, unsigned long long elem, T v, bool want) {
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "gpuvm_cursor_store: 4- or 8-byte elements");
    const unsigned long long byte = elem * sizeof(T);
    const unsigned int page = (unsigned int)(byte >> vm.page_shift);
    const unsigned int off = (unsigned int)(byte & ((1ull << vm.page_shift) - 1));
    if (gpuvm_detail::cursor_seek(vm, c, page, want, true)) {
        if (want) __hip_atomic_store(reinterpret_cast<T *>(c.frame + off), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    gpuvm_store_if<T>(vm, elem, v, want);
}

/* Array-like view for kernels written in the style of the paper's listing
 * (System Overview: an array-like structure, so that c[i] = a[i] + b[i] needs
 * no other change): v[i] reads, v[i] = x stores, v[i] += x adds atomically.
 * at(i, want) is the same with the lane's predicate, for code that keeps the
 * whole wave on the access so that all lanes help to move pages. */
template <typename T>
struct gpuvm_array {
    gpuvm_dev_t vm;
    struct ref {
        const gpuvm_dev_t &vm;
        unsigned long long i;
        bool want;
        __device__ __forceinline__ operator T() const { return gpuvm_load_if<T>(vm, i, want); }
        __device__ __forceinline__ const ref &operator=(T v) const { gpuvm_store_if<T>(vm, i, v, want); return *this; }
        __device__ __forceinline__ const ref &operator=(const ref &o) const { return *this = (T)o; }
        __device__ __forceinline__ const ref &operator+=(T v) const { gpuvm_atomic_add_if<T>(vm, i, v, want); return *this; }
    };
    __device__ __forceinline__ ref operator[](unsigned long long i) const { return ref{vm, i, true}; }
    __device__ __forceinline__ ref at(unsigned long long i, bool want) const { return ref{vm, want ? i : 0ull, want}; }
    __device__ __forceinline__ unsigned long long size() const { return vm.bytes / sizeof(T); }
};

#endif /* GPUVM_DEVICE_H */

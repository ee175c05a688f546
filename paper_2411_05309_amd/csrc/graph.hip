// libgpuvm - graph workloads over a paged CSR col_idx array: BFS (vertex chunks and edge-balanced), connected components, SSSP with paged weights.
// The fault path itself (page-table lookup, wavefront dedup, frame allocation,
// eviction, write-back, migration) is in include/gpuvm_device.h and is inlined
// into every kernel, the way the paper inlines its runtime into the application
// kernels (System Overview; Register usage).
#include "gpuvm_internal.h"

using namespace gpuvm_detail;

// One BFS level, topology driven: a wave scans 64 consecutive vertices; the
// edges of each vertex on the current level are read from the paged col_idx
// array by the whole wave, page by page, keeping one page pinned at a time.
__global__ __launch_bounds__(kBlock) void k_bfs_level(gpuvm_dev_t vm, const int64_t *__restrict__ row_ptr,
                                                       int64_t nv, int32_t *level, int32_t cur, int *changed) {
    const unsigned int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * kBlock) >> 6;
    const unsigned int elems_shift = vm.page_shift - 2;                // int32 per page
    int found = 0;
    for (int64_t base = wave * 64; base < nv; base += nwaves * 64) {
        const int64_t v = base + lane;
        int64_t beg = 0, end = 0;
        if (v < nv && level[v] == cur) { beg = row_ptr[v]; end = row_ptr[v + 1]; }
        unsigned long long todo = __builtin_amdgcn_ballot_w64(end > beg);
        unsigned int held = GPUVM_NO_PAGE;
        const char *ptr = nullptr;
        while (todo) {
            const unsigned int l = (unsigned int)__ffsll((long long)todo) - 1u;
            todo &= todo - 1;
            const int64_t b = ((int64_t)__builtin_amdgcn_readlane((int)(beg >> 32), l) << 32) |
                              (unsigned int)__builtin_amdgcn_readlane((int)beg, l);
            const int64_t e = ((int64_t)__builtin_amdgcn_readlane((int)(end >> 32), l) << 32) |
                              (unsigned int)__builtin_amdgcn_readlane((int)end, l);
            for (int64_t pos = b; pos < e;) {
                const unsigned int page = (unsigned int)(pos >> elems_shift);
                const int64_t page_first = (int64_t)page << elems_shift;
                const int64_t page_stop = page_first + ((int64_t)1 << elems_shift);
                const int64_t stop = e < page_stop ? e : page_stop;
                if (page != held) {
                    if (held != GPUVM_NO_PAGE) gpuvm_release(vm, held);
                    ptr = gpuvm_acquire(vm, page, false);
                    held = page;
                }
                for (int64_t i = pos + lane; i < stop; i += 64) {
                    const int32_t u = (int32_t)gpuvm_frame_load_b32(vm, ptr, (unsigned int)(i - page_first) << 2);
                    if ((uint64_t)(uint32_t)u >= (uint64_t)nv) { raise_error(vm, GPUVM_ERANGE); continue; }   // malformed neighbour id
                    if (level[u] < 0) { level[u] = cur + 1; found = 1; }
                }
                pos = stop;
            }
        }
        if (held != GPUVM_NO_PAGE) gpuvm_release(vm, held);
    }
    if (__builtin_amdgcn_ballot_w64(found != 0) && lane == 0) *changed = 1;
}

// ---- edge-balanced BFS (the paper's Balanced CSR idea, Graph Workloads: equal
// chunks of edges per worker so that faults do not serialise behind the huge
// neighbour lists).  The chunk is one page of col_idx: a wave owns page p for
// the level, so every page is faulted by at most one wave per level and no
// vertex, however large, is walked by a single wave.
// page_owner[p] = vertex that owns the first edge of page p (owner[n_pages] = nv-1).
__global__ void k_bfs_page_owner(const int64_t *__restrict__ row_ptr, int64_t nv, unsigned int n_pages,
                                 unsigned int elems_shift, unsigned int *page_owner) {
    const unsigned int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p > n_pages) return;
    if (p == n_pages) { page_owner[p] = (unsigned int)(nv - 1); return; }
    const int64_t e = (int64_t)p << elems_shift;
    int64_t lo = 0, hi = nv;                      // last v with row_ptr[v] <= e
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (row_ptr[mid] <= e) lo = mid; else hi = mid;
    }
    page_owner[p] = (unsigned int)lo;
}

// Page-owned edge walk shared by the edge-balanced graph kernels: wave w owns
// pages w, w + nwaves, ... of the paged col_idx array for this round; inside a
// page it visits the edge segments of the vertices for which active(v) holds.
// Short segments are walked one lane per vertex, long ones by the whole wave.
// visit(v, u, byte_off, ptr2, in_place): edge v -> u stored at byte_off of the
// page; ptr2 is the same page of a second paged array (edge weights) or null - a
// frame, or host memory if in_place.
// DIRECT = true is the zero-copy baseline: the same walk reading col_idx in
// place in pinned host memory (system-scope loads), no page table, no frames.
// In remote-first mode (gpuvm_set_remote_first on the handle of col_idx) the
// choice is made page by page, for both arrays together: a page that is not resident and whose
// active segments would cost less over the link read in place (64 bytes per
// short list at least, 4 bytes per edge, times two for the low rate of
// scattered reads) than the page itself is read in place; everything else is
// paged in as usual.  The sparse levels of a BFS,
// where a 64 KiB page is wanted for a handful of edges, are the case.
// The pages of col_idx in which some active vertex owns edges: a mark per page and
// the marked pages as a list (in no particular order), so that a round costs what
// its frontier's pages cost - not a scan over the owner ranges of every vertex -
// and the waves share the pages of a sparse round evenly.
struct page_list_t {
    unsigned int *mark;                            // [n_pages] 0 / 1
    unsigned int *list;                            // [n_pages] the marked pages
    unsigned int *order;                           // [n_pages] the round's pages that are not resident when it begins
    unsigned int *ring;                            // [n_frames] those that are, by their frame's distance from the cursor
    unsigned int *count;                           // [0] how many marked; [1] resident, [2] not; next to take: [3] of ring, [4] of order
};
__device__ __forceinline__ void mark_page(const page_list_t &next, unsigned int p) {
    if (next.mark[p] == 0 && atomicExch(next.mark + p, 1u) == 0) next.list[atomicAdd(next.count, 1u)] = p;
}

// A round's pages sorted for the waves: those that are not resident, in about
// the order given (label propagation gains from ascending pages), and those that
// the previous round left in the pool, each in the slot of its frame's distance
// from the cursor - the order in which the allocator will come to evict them.
// `every_page`: the round's pages are all pages (no list).  `in_place`: the round
// reads host memory in place, whatever the pool holds.  count[1..4] are zero and
// ring[] is all GPUVM_NO_PAGE.
__global__ __launch_bounds__(256) void k_sort_round(gpuvm_dev_t vm, page_list_t work, bool every_page, bool in_place) {
    const unsigned int n = every_page ? vm.n_pages : *work.count;
    const unsigned int cursor = (unsigned int)(a_load(vm.hand) % vm.n_frames);
    for (unsigned int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) {
        const unsigned int page = every_page ? i : work.list[i];
        const unsigned long long w = a_load(vm.pte + page);
        if (!in_place && ((w & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) == GPUVM_ST_RESIDENT) {
            const unsigned int f = (unsigned int)(w >> GPUVM_PTE_FRAME_SHIFT);
            if (f < vm.n_frames) {
                work.ring[f >= cursor ? f - cursor : f + vm.n_frames - cursor] = page;
                atomicAdd(work.count + 1, 1u);
                continue;
            }
        }
        work.order[atomicAdd(work.count + 2, 1u)] = page;
    }
}

// `work`: this round's pages as k_sort_round left them.  The waves take them one
// at a time from two shared counters: two resident pages for every page that has
// to be faulted in, for as long as there are both.  The resident pages go in the
// order in which the cursor will reach their frames and are let go without a
// mark (gpuvm_acquire_cold, last_use), so the faults evict what has been used
// already and stay behind the waves that use the rest: up to a pool's worth of
// pages per round that do not cross the link again, used while the link is busy
// with the others.
template <bool DIRECT = false, class Active, class Visit>
__device__ __forceinline__ void walk_owned_pages(const gpuvm_dev_t &vm, const gpuvm_dev_t *vm2,
                                                 const int64_t *__restrict__ row_ptr,
                                                 const unsigned int *__restrict__ page_owner,
                                                 const page_list_t &work, bool every_page,
                                                 Active active, Visit visit) {
    const unsigned int lane = threadIdx.x & 63;
    const unsigned int elems_shift = vm.page_shift - 2;
    const int64_t n_edges = (int64_t)(vm.bytes >> 2);
    constexpr int kSmall = 32;                    // lists up to this length: one lane each
    // scattered short reads in place run well below the link's bulk rate; on the
    // scale-26 BFS a factor of 2 was the fastest of 1, 1.5, 2, 3, 4, 8
    // (206, 146, 139, 142, 146, 157 ms; 197 ms with every page migrated)
    constexpr unsigned long long kInPlacePenalty = 2;
    const unsigned int n_miss = work.count[2];
    auto do_page = [&](const unsigned int page) {
        const int64_t e_lo = (int64_t)page << elems_shift;
        const int64_t e_hi = min((long long)n_edges, (long long)(e_lo + ((int64_t)1 << elems_shift)));
        const int64_t v_first = page_owner[page], v_last = page_owner[page + 1];
        const char *ptr = nullptr, *ptr2 = nullptr;
        bool in_place = DIRECT;
        if (!DIRECT && (vm.flags >> GPUVM_F_REMOTE_SHIFT) &&
            ((a_load(vm.pte + page) & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) != GPUVM_ST_RESIDENT) {
            // what would the active segments of this page cost if read in place?
            unsigned long long cost = 0;
            for (int64_t vb = v_first; vb <= v_last && cost * kInPlacePenalty < (1ull << vm.page_shift); vb += 64) {
                const int64_t v = vb + lane;
                long long len = 0;
                if (v <= v_last && active(v))
                    len = min((long long)row_ptr[v + 1], (long long)e_hi) - max((long long)row_ptr[v], (long long)e_lo);
                unsigned long long c = len > 0 ? max(64ull, (unsigned long long)len * 4ull) : 0ull;   // per array: the page count cancels
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, 64);
                cost += c;
            }
            in_place = cost * kInPlacePenalty < (1ull << vm.page_shift);
            if (in_place && cost && lane == 0) stat_add(vm, GPUVM_S_REMOTE, 1);
        }
        for (int64_t vb = v_first; vb <= v_last; vb += 64) {
            const int64_t v = vb + lane;
            int64_t beg = 0, end = 0;
            if (v <= v_last && active(v)) {
                beg = max((long long)row_ptr[v], (long long)e_lo);
                end = min((long long)row_ptr[v + 1], (long long)e_hi);
            }
            const int len = end > beg ? (int)(end - beg) : 0;
            if (__builtin_amdgcn_ballot_w64(len > 0) == 0) continue;
            if (!ptr) {
                ptr = in_place ? vm.host + ((size_t)page << vm.page_shift) : gpuvm_acquire_cold(vm, page, false, true);
                if (vm2) ptr2 = in_place ? vm2->host + ((size_t)page << vm2->page_shift) : gpuvm_acquire_cold(*vm2, page, false, true);
            }
            auto edge_at = [&](unsigned int o) {
                return in_place ? (int32_t)__builtin_amdgcn_raw_buffer_load_b32(make_rsrc(ptr, 1u << vm.page_shift), o, 0, GPUVM_AUX_SYSTEM)
                                : (int32_t)gpuvm_frame_load_b32(vm, ptr, o);
            };
            const bool small = len > 0 && len <= kSmall;
            int longest = small ? len : 0;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) longest = max(longest, __shfl_xor(longest, off, 64));
            const unsigned int my_off = (unsigned int)(beg - e_lo) << 2;
            for (int j = 0; j < longest; ++j) {
                if (small && j < len) {
                    const unsigned int o = my_off + ((unsigned int)j << 2);
                    visit(v, edge_at(o), o, ptr2, in_place);
                }
            }
            unsigned long long todo = __builtin_amdgcn_ballot_w64(len > kSmall);
            while (todo) {
                const unsigned int l = (unsigned int)__ffsll((long long)todo) - 1u;
                todo &= todo - 1;
                const unsigned int off0 = (unsigned int)__builtin_amdgcn_readlane((int)my_off, l);
                const unsigned int n = (unsigned int)__builtin_amdgcn_readlane(len, l);
                const int64_t vl = vb + l;
                for (unsigned int i = lane; i < n; i += 64) {
                    const unsigned int o = off0 + (i << 2);
                    visit(vl, edge_at(o), o, ptr2, in_place);
                }
            }
        }
        if (ptr && !in_place) {
            gpuvm_release(vm, page);
            if (vm2) gpuvm_release(*vm2, page);
        }
    };
    bool ring_left = !DIRECT && work.count[1] != 0, order_left = true;
    // (every wave starts with two resident pages: the allocator takes frames the
    // moment a fault draws its ticket, a wave needs a while per page - starting a
    // third of the waves on faults loses a third of the hits; one resident page per
    // fault instead of two loses about as many on the scale-26 BFS - 146 K faults
    // against 134 K - and three per fault change nothing)
    for (unsigned int turn = 0; ring_left || order_left;) {
        const bool from_ring = ring_left && (turn % 3 != 2 || !order_left);
        unsigned int k = 0;
        if (lane == 0) k = atomicAdd(work.count + (from_ring ? 3 : 4), 1u);
        k = bcast(k);
        if (k >= (from_ring ? vm.n_frames : n_miss)) {
            if (from_ring) ring_left = false; else order_left = false;
            continue;
        }
        const unsigned int page = from_ring ? work.ring[k] : work.order[k];
        if (page == GPUVM_NO_PAGE) continue;          // a frame that holds none of this round's pages
        do_page(page);
        ++turn;
    }
}

// A vertex has just become active for the next round: mark the pages of col_idx
// that hold its edges.
__device__ __forceinline__ void mark_pages_of(const int64_t *__restrict__ row_ptr, int64_t u, unsigned int elems_shift,
                                              const page_list_t &next) {
    const int64_t b = row_ptr[u], e = row_ptr[u + 1];
    if (e <= b) return;
    for (int64_t p = b >> elems_shift; p <= (e - 1) >> elems_shift; ++p) mark_page(next, (unsigned int)p);
}

__global__ void k_mark_pages_of(const int64_t *__restrict__ row_ptr, int64_t u, unsigned int elems_shift,
                                page_list_t next) {
    if (blockIdx.x == 0 && threadIdx.x == 0) mark_pages_of(row_ptr, u, elems_shift, next);
}

template <bool DIRECT>
__global__ __launch_bounds__(kBlock) void k_bfs_level_balanced(gpuvm_dev_t vm, const int64_t *__restrict__ row_ptr,
                                                                const unsigned int *__restrict__ page_owner, int64_t nv,
                                                                page_list_t work, page_list_t next,
                                                                int32_t *level, int32_t cur, int *changed) {
    int found = 0;
    const unsigned int elems_shift = vm.page_shift - 2;
    walk_owned_pages<DIRECT>(vm, nullptr, row_ptr, page_owner, work, false,
                     [&](int64_t v) { return level[v] == cur; },
                     [&](int64_t, int32_t u, unsigned int, const char *, bool) {
                         if ((uint64_t)(uint32_t)u >= (uint64_t)nv) { raise_error(vm, GPUVM_ERANGE); return; }   // malformed neighbour id
                         if (level[u] < 0) {
                             level[u] = cur + 1;
                             found = 1;
                             mark_pages_of(row_ptr, u, elems_shift, next);         // several lanes may find u: same marks
                         }
                     });
    if (__builtin_amdgcn_ballot_w64(found != 0) && (threadIdx.x & 63) == 0) *changed = 1;
}

// Connected components (weak) by label propagation: every round walks every
// edge (v, u) and pulls both labels down to the smaller one; the fixed point
// labels each vertex with the smallest vertex id of its component.
__global__ __launch_bounds__(kBlock) void k_cc_round_balanced(gpuvm_dev_t vm, const int64_t *__restrict__ row_ptr,
                                                               const unsigned int *__restrict__ page_owner, int64_t nv,
                                                               page_list_t work, int32_t *label, int *changed) {
    int found = 0;
    walk_owned_pages(vm, nullptr, row_ptr, page_owner, work, true,
                     [&](int64_t) { return true; },
                     [&](int64_t v, int32_t u, unsigned int, const char *, bool) {
                         if ((uint64_t)(uint32_t)u >= (uint64_t)nv) { raise_error(vm, GPUVM_ERANGE); return; }
                         const int32_t lv = __hip_atomic_load(label + v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                         const int32_t lu = __hip_atomic_load(label + u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                         if (lv < lu) {
                             __hip_atomic_fetch_min(label + u, lv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                             found = 1;
                         } else if (lu < lv) {
                             __hip_atomic_fetch_min(label + v, lu, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                             found = 1;
                         }
                     });
    if (__builtin_amdgcn_ballot_w64(found != 0) && (threadIdx.x & 63) == 0) *changed = 1;
}

// Single-source shortest paths, frontier-based Bellman-Ford: a round relaxes
// the out-edges of the vertices whose distance fell in the previous round.
// Edge weights are a second paged array with the layout of col_idx.
__global__ __launch_bounds__(kBlock) void k_sssp_round_balanced(gpuvm_dev_t vm, gpuvm_dev_t vmw,
                                                                 const int64_t *__restrict__ row_ptr,
                                                                 const unsigned int *__restrict__ page_owner, int64_t nv,
                                                                 page_list_t work, page_list_t next,
                                                                 uint32_t *dist, const unsigned char *act_cur,
                                                                 unsigned char *act_next, int *changed) {
    int found = 0;
    const unsigned int elems_shift = vm.page_shift - 2;
    walk_owned_pages(vm, &vmw, row_ptr, page_owner, work, false,
                     [&](int64_t v) { return act_cur[v] != 0; },
                     [&](int64_t v, int32_t u, unsigned int off, const char *pw, bool in_place) {
                         if ((uint64_t)(uint32_t)u >= (uint64_t)nv) { raise_error(vm, GPUVM_ERANGE); return; }
                         const uint32_t w = in_place ? __builtin_amdgcn_raw_buffer_load_b32(make_rsrc(pw, 1u << vmw.page_shift), off, 0, GPUVM_AUX_SYSTEM)
                                                     : gpuvm_frame_load_b32(vmw, pw, off);
                         const uint32_t dv = __hip_atomic_load(dist + v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                         if (dv != 0xFFFFFFFFu) {
                             const uint32_t nd = dv + w;
                             const uint32_t old = __hip_atomic_fetch_min(dist + u, nd, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                             if (nd < old) {
                                 if (!act_next[u]) mark_pages_of(row_ptr, u, elems_shift, next);   // first to lower it this round (or racing with the first)
                                 act_next[u] = 1;
                                 found = 1;
                             }
                         }
                     });
    if (__builtin_amdgcn_ballot_w64(found != 0) && (threadIdx.x & 63) == 0) *changed = 1;
}

__global__ void k_iota32(int32_t *p, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = (int32_t)i;
}

// the two page lists of a handle (allocated by ensure_page_owner)
static page_list_t page_list_of(const gpuvm_t *vm, int which) {
    const size_t np = vm->dev.n_pages;
    unsigned int *base = vm->page_marks + (size_t)which * (3 * np + vm->dev.n_frames + 64);
    return page_list_t{base, base + np, base + 2 * np, base + 3 * np, base + 3 * np + vm->dev.n_frames};
}
// before a round's kernel: its pages in the order the waves take them
static void order_pages(const gpuvm_t *vm, int which, bool every_page, hipStream_t s, bool in_place = false) {
    const page_list_t l = page_list_of(vm, which);
    k_fill32<<<1, 64, 0, s>>>(l.count + 1, 4, 0u);
    k_fill32<<<64, 256, 0, s>>>(l.ring, vm->dev.n_frames, GPUVM_NO_PAGE);
    k_sort_round<<<std::max(1u, std::min(256u, (vm->dev.n_pages + 255) / 256)), 256, 0, s>>>(vm->dev, l, every_page, in_place);
}
static void clear_page_list(const gpuvm_t *vm, int which, hipStream_t s) {
    const page_list_t l = page_list_of(vm, which);
    k_fill32<<<64, 256, 0, s>>>(l.mark, vm->dev.n_pages, 0u);
    k_fill32<<<1, 64, 0, s>>>(l.count, 1, 0u);
}

extern "C" {

static int ensure_page_owner(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv, hipStream_t s);

static int run_bfs(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv, int64_t src, int32_t *d_level,
                   int *n_levels_out, void *stream, bool balanced, bool direct = false) {
    if (!vm || !d_row_ptr || !d_level || nv <= 0 || src < 0 || src >= nv || nv > 0x7FFFFFFF) return GPUVM_EINVAL;
    if (vm->dev.bytes % 4) return GPUVM_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    // the zero-copy baseline holds no frames: its waves are bounded by the device only
    const int waves = direct ? vm->cus * vm->waves_per_cu
                             : launch_waves(vm, balanced ? (size_t)vm->dev.n_pages : (size_t)((nv + 63) / 64));
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    if (balanced) {
        int rc0 = ensure_page_owner(vm, d_row_ptr, nv, s);
        if (rc0) return rc0;
    }
    k_fill32<<<1024, 256, 0, s>>>((unsigned int *)d_level, (size_t)nv, 0xFFFFFFFFu);
    k_fill32<<<1, 64, 0, s>>>((unsigned int *)d_level + src, 1, 0u);
    if (balanced) {                                            // the source's pages are the first round's work
        clear_page_list(vm, 0, s);
        k_mark_pages_of<<<1, 64, 0, s>>>(d_row_ptr, src, vm->dev.page_shift - 2, page_list_of(vm, 0));
    }
    int levels = 0;
    for (int32_t cur = 0;; ++cur) {
        int changed = 0;
        const page_list_t work = balanced ? page_list_of(vm, cur & 1) : page_list_t{};
        const page_list_t next = balanced ? page_list_of(vm, (cur + 1) & 1) : page_list_t{};
        k_fill32<<<1, 64, 0, s>>>((unsigned int *)vm->bfs_changed, 1, 0u);
        if (balanced) {
            clear_page_list(vm, (cur + 1) & 1, s);
            order_pages(vm, cur & 1, false, s, direct);
        }
        if (direct)
            k_bfs_level_balanced<true><<<grid_for_waves(waves), kBlock, 0, s>>>(vm->dev, d_row_ptr, vm->page_owner, nv,
                                                                                 work, next, d_level, cur, vm->bfs_changed);
        else if (balanced)
            k_bfs_level_balanced<false><<<grid_for_waves(waves), kBlock, 0, s>>>(vm->dev, d_row_ptr, vm->page_owner, nv,
                                                                                  work, next, d_level, cur, vm->bfs_changed);
        else
            k_bfs_level<<<grid_for_waves(waves), kBlock, 0, s>>>(vm->dev, d_row_ptr, nv, d_level, cur, vm->bfs_changed);
        HIP_TRY(hipMemcpyAsync(&changed, vm->bfs_changed, sizeof(int), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        ++levels;
        if (!changed || cur == 0x7FFFFFFE) break;
        int rc = check_kernel_error(vm);
        if (rc) return rc;
    }
    if (n_levels_out) *n_levels_out = levels;
    return check_kernel_error(vm);
}

int gpuvm_run_bfs(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv, int64_t src, int32_t *d_level,
                  int *n_levels_out, void *stream) {
    return run_bfs(vm, d_row_ptr, nv, src, d_level, n_levels_out, stream, false);
}

int gpuvm_run_bfs_balanced(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv, int64_t src, int32_t *d_level,
                           int *n_levels_out, void *stream) {
    return run_bfs(vm, d_row_ptr, nv, src, d_level, n_levels_out, stream, true);
}

int gpuvm_bench_bfs_zero_copy(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv, int64_t src, int32_t *d_level,
                              int *n_levels_out, void *stream) {
    return run_bfs(vm, d_row_ptr, nv, src, d_level, n_levels_out, stream, true, true);
}

static int ensure_page_owner(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv, hipStream_t s) {
    if (!vm->page_owner) HIP_TRY(hipMalloc(&vm->page_owner, ((size_t)vm->dev.n_pages + 1) * sizeof(unsigned int)));
    // two page lists, this round's and the next one's: marks, list, order, ring, counters (padded)
    if (!vm->page_marks) HIP_TRY(hipMalloc(&vm->page_marks, 2 * (3 * (size_t)vm->dev.n_pages + vm->dev.n_frames + 64) * sizeof(unsigned int)));
    const unsigned int n = vm->dev.n_pages + 1;
    k_bfs_page_owner<<<(n + 255) / 256, 256, 0, s>>>(d_row_ptr, nv, vm->dev.n_pages, vm->dev.page_shift - 2, vm->page_owner);
    return GPUVM_OK;
}

int gpuvm_run_cc_balanced(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv, int32_t *d_label, int *n_rounds_out,
                          void *stream) {
    if (!vm || !d_row_ptr || !d_label || nv <= 0 || nv > 0x7FFFFFFF || vm->dev.bytes % 4) return GPUVM_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int waves = launch_waves(vm, vm->dev.n_pages);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    int rc = ensure_page_owner(vm, d_row_ptr, nv, s);
    if (rc) return rc;
    k_iota32<<<1024, 256, 0, s>>>(d_label, (size_t)nv);
    int rounds = 0;
    for (;;) {
        int changed = 0;
        k_fill32<<<1, 64, 0, s>>>((unsigned int *)vm->bfs_changed, 1, 0u);
        order_pages(vm, 0, true, s);
        k_cc_round_balanced<<<grid_for_waves(waves), kBlock, 0, s>>>(vm->dev, d_row_ptr, vm->page_owner, nv,
                                                                      page_list_of(vm, 0), d_label, vm->bfs_changed);
        HIP_TRY(hipMemcpyAsync(&changed, vm->bfs_changed, sizeof(int), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        ++rounds;
        rc = check_kernel_error(vm);
        if (rc) return rc;
        if (!changed || rounds > 1000000) break;
    }
    if (n_rounds_out) *n_rounds_out = rounds;
    return GPUVM_OK;
}

int gpuvm_run_sssp_balanced(gpuvm_t *vm, gpuvm_t *vm_weights, const int64_t *d_row_ptr, int64_t nv, int64_t src,
                            uint32_t *d_dist, int *n_rounds_out, void *stream) {
    if (!vm || !vm_weights || vm == vm_weights || !d_row_ptr || !d_dist || nv <= 0 || nv > 0x7FFFFFFF || src < 0 ||
        src >= nv)
        return GPUVM_EINVAL;
    if (vm->dev.bytes % 4 || vm_weights->dev.bytes != vm->dev.bytes || vm_weights->dev.page_shift != vm->dev.page_shift)
        return GPUVM_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int waves = std::min(launch_waves(vm, vm->dev.n_pages), launch_waves(vm_weights, vm->dev.n_pages));
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    int rc = ensure_page_owner(vm, d_row_ptr, nv, s);
    if (rc) return rc;
    unsigned char *act = nullptr;                           // two activity maps, swapped every round
    HIP_TRY(hipMalloc(&act, 2 * (size_t)nv));
    k_fill8<<<1024, 256, 0, s>>>(act, 2 * (size_t)nv, 0);
    k_fill8<<<1, 64, 0, s>>>(act + src, 1, 1);
    clear_page_list(vm, 0, s);
    k_mark_pages_of<<<1, 64, 0, s>>>(d_row_ptr, src, vm->dev.page_shift - 2, page_list_of(vm, 0));
    k_fill32<<<1024, 256, 0, s>>>(d_dist, (size_t)nv, 0xFFFFFFFFu);
    k_fill32<<<1, 64, 0, s>>>(d_dist + src, 1, 0u);
    int rounds = 0;
    rc = GPUVM_OK;
    for (;;) {
        int changed = 0;
        unsigned char *cur = act + (size_t)(rounds & 1) * nv, *next = act + (size_t)((rounds + 1) & 1) * nv;
        const page_list_t work = page_list_of(vm, rounds & 1), work_next = page_list_of(vm, (rounds + 1) & 1);
        k_fill32<<<1, 64, 0, s>>>((unsigned int *)vm->bfs_changed, 1, 0u);
        k_fill8<<<1024, 256, 0, s>>>(next, (size_t)nv, 0);
        clear_page_list(vm, (rounds + 1) & 1, s);
        order_pages(vm, rounds & 1, false, s);
        k_sssp_round_balanced<<<grid_for_waves(waves), kBlock, 0, s>>>(vm->dev, vm_weights->dev, d_row_ptr,
                                                                        vm->page_owner, nv, work, work_next, d_dist, cur, next,
                                                                        vm->bfs_changed);
        hipError_t e = hipMemcpyAsync(&changed, vm->bfs_changed, sizeof(int), hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) { rc = GPUVM_EHIP; break; }
        ++rounds;
        rc = check_kernel_error(vm);
        if (!rc) rc = check_kernel_error(vm_weights);
        if (rc || !changed || rounds > 1000000) break;
    }
    (void)hipFree(act);
    if (n_rounds_out) *n_rounds_out = rounds;
    return rc;
}

}  // extern "C"

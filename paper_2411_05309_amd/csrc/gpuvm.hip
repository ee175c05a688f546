// libgpuvm: host side of the GPUVM hot path for MI355X (gfx950) - life cycle,
// flush/reset/stats, and the kernels + launchers of the five workloads, the
// deterministic barrier-phased mode and the roofline microbenchmarks.
// The fault path itself (page-table lookup, wavefront dedup, frame allocation,
// eviction, write-back, migration) is in include/gpuvm_device.h and is inlined
// into every kernel here, the way the paper inlines its runtime into the
// application kernels (System Overview; Register usage).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "gpuvm.h"
#include "gpuvm_device.h"

using namespace gpuvm_detail;

namespace {

constexpr int kBlock = 256;               // 4 wavefronts per workgroup
constexpr int kWavesPerBlock = kBlock / 64;
constexpr uint32_t kDefaultSpinLimit = 1u << 22;

struct phase_job {                        // one fault of a deterministic phase
    unsigned int page, frame, victim, writeback;
};

}  // namespace

struct gpuvm {
    gpuvm_dev_t dev;
    int device;
    int cus;
    int waves_per_cu;
    size_t page_bytes;
    // deterministic mode scratch (allocated on first use)
    unsigned int *stamp = nullptr;        // [n_pages] phase tag of the last toucher
    unsigned char *first = nullptr;       // [phase_cap] access i was first on its page
    unsigned int *miss = nullptr;         // [phase_cap] missing pages, then sorted
    unsigned int *miss_sorted = nullptr;
    phase_job *jobs = nullptr;            // [phase_cap]
    unsigned int *phase_ctr = nullptr;    // [0] misses, [1] hits, [2] jobs
    size_t phase_cap = 0;
    unsigned int phase_tag = 0;
    int *bfs_changed = nullptr;
    unsigned int *page_owner = nullptr;   // [n_pages + 1], edge-balanced BFS
};

#define HIP_TRY(expr)                                                            \
    do {                                                                         \
        hipError_t e_ = (expr);                                                  \
        if (e_ != hipSuccess) {                                                  \
            fprintf(stderr, "libgpuvm: %s failed: %s (%s:%d)\n", #expr,          \
                    hipGetErrorString(e_), __FILE__, __LINE__);                  \
            return e_ == hipErrorOutOfMemory ? GPUVM_ENOMEM : GPUVM_EHIP;        \
        }                                                                        \
    } while (0)

// ------------------------------------------------------------------ utility kernels

__global__ void k_fill64(unsigned long long *p, size_t n, unsigned long long v) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
__global__ void k_fill32(unsigned int *p, size_t n, unsigned int v) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// One wavefront per frame: write a DIRTY page back and clear the bit.  Runs
// alone (no other kernel on the handle), so plain table reads are enough.
__global__ __launch_bounds__(kBlock) void k_flush(gpuvm_dev_t vm) {
    const wave_t w = wave_now();
    const unsigned int wave = (blockIdx.x * kBlock + threadIdx.x) >> 6;
    const unsigned int nwaves = (gridDim.x * kBlock) >> 6;
    for (unsigned int f = wave; f < vm.n_frames; f += nwaves) {
        const unsigned int q = vm.frame_owner[f];
        if (q == GPUVM_NO_PAGE) continue;
        const unsigned long long pq = vm.pte[q];
        if (((pq & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) != GPUVM_ST_RESIDENT ||
            (unsigned int)(pq >> GPUVM_PTE_FRAME_SHIFT) != f || !(pq & GPUVM_PTE_DIRTY))
            continue;
        const unsigned int len = page_len(vm, q);
        copy_frame_to_host(vm.host + ((size_t)q << vm.page_shift), vm.frames + ((size_t)f << vm.page_shift), len, w);
        if (w.leader) {
            a_and(vm.pte + q, ~GPUVM_PTE_DIRTY);
            stat_add(vm, GPUVM_S_WB_FLUSH, 1);
            stat_add(vm, GPUVM_S_BYTES_OUT, len);
        }
    }
    wait_vm();
}

// ------------------------------------------------------------------ workload kernels

__device__ __forceinline__ unsigned long long wave_sum(unsigned long long v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// Random gather: one access per lane per iteration, grid-stride.
__global__ __launch_bounds__(kBlock) void k_gather(gpuvm_dev_t vm, const uint32_t *__restrict__ idx, size_t n,
                                                    uint32_t *__restrict__ out, unsigned long long *sum,
                                                    unsigned long long n_elems) {
    const size_t nthreads = (size_t)gridDim.x * kBlock;
    unsigned long long acc = 0;
    const size_t n_up = (n + 63) & ~(size_t)63;                  // whole waves iterate together
    for (size_t k = (size_t)blockIdx.x * kBlock + threadIdx.x; k < n_up; k += nthreads) {
        unsigned long long i = k < n ? idx[k] : 0;
        bool want = k < n;
        if (want && i >= n_elems) { raise_error(vm, GPUVM_ERANGE); want = false; }
        const uint32_t v = gpuvm_load_if<uint32_t>(vm, i, want);
        if (want) { out[k] = v; acc += v; }
    }
    if (sum) {
        // every lane of the wave reaches this point (the loop has ended for all)
        acc = wave_sum(acc);
        if ((threadIdx.x & 63) == 0 && acc)
            __hip_atomic_fetch_add(sum, acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Scatter-increment: data[idx[k]] += 1 through the paged view.
__global__ __launch_bounds__(kBlock) void k_scatter_inc(gpuvm_dev_t vm, const uint32_t *__restrict__ idx, size_t n,
                                                         unsigned long long n_elems) {
    const size_t nthreads = (size_t)gridDim.x * kBlock;
    const size_t n_up = (n + 63) & ~(size_t)63;
    for (size_t k = (size_t)blockIdx.x * kBlock + threadIdx.x; k < n_up; k += nthreads) {
        unsigned long long i = k < n ? idx[k] : 0;
        bool want = k < n;
        if (want && i >= n_elems) { raise_error(vm, GPUVM_ERANGE); want = false; }
        gpuvm_atomic_add_if<unsigned long long>(vm, i, 1ull, want);
    }
}

// The paper's own example (vector-addition listing): C[i] = A[i] + B[i] with all
// three vectors paged; C is written through gpuvm_store, so its pages become
// DIRTY and are written back at eviction or flush.
// Work distribution: a wave takes one page-sized stripe of the index range at a
// time (consecutive stripes to consecutive waves), so that the waves in flight
// fault on different pages; with a plain grid-stride loop all of them would
// stand on the same handful of pages and wait for one fetch at a time.
__global__ __launch_bounds__(kBlock) void k_vector_add(gpuvm_dev_t a, gpuvm_dev_t b, gpuvm_dev_t c, size_t n) {
    const unsigned int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const size_t nwaves = ((size_t)gridDim.x * kBlock) >> 6;
    const size_t stripe = (size_t)1 << (c.page_shift - 2);               // floats per page of C
    for (size_t lo = wave * stripe; lo < n; lo += nwaves * stripe) {
        const size_t hi = lo + stripe < n ? lo + stripe : n;
        for (size_t i0 = lo; i0 < hi; i0 += 64) {
            const size_t i = i0 + lane;
            const bool want = i < hi;
            const float x = gpuvm_load_if<float>(a, want ? i : 0, want);
            const float y = gpuvm_load_if<float>(b, want ? i : 0, want);
            gpuvm_store_if<float>(c, want ? i : 0, x + y, want);
        }
    }
}

// Streaming read-reduce: wave w takes pages w, w + nwaves, ...; the page's
// floats are summed in fp64 and added to the sum of the block it belongs to.
__global__ __launch_bounds__(kBlock) void k_stream_reduce(gpuvm_dev_t vm, unsigned int pages_per_block,
                                                           double *sums) {
    const unsigned int lane = threadIdx.x & 63;
    const unsigned int wave = (blockIdx.x * kBlock + threadIdx.x) >> 6;
    const unsigned int nwaves = (gridDim.x * kBlock) >> 6;
    for (unsigned int page = wave; page < vm.n_pages; page += nwaves) {
        const unsigned int len = page_len(vm, page);
        const unsigned int nvec = len >> 4;                           // float4 items
        const char *p = gpuvm_acquire(vm, page, false);
        double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
        for (unsigned int i = lane; i < nvec; i += 64) {
            const u32x4 v = gpuvm_frame_load_b128(vm, p, i << 4);
            a0 += (double)__uint_as_float(v.x); a1 += (double)__uint_as_float(v.y);
            a2 += (double)__uint_as_float(v.z); a3 += (double)__uint_as_float(v.w);
        }
        // floats beyond the last full float4 of a short last page
        if ((nvec << 4) + (lane << 2) < len)
            a0 += (double)__uint_as_float(gpuvm_frame_load_b32(vm, p, (nvec << 4) + (lane << 2)));
        gpuvm_release(vm, page);
        double s = (a0 + a1) + (a2 + a3);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
        if (lane == 0)
            __hip_atomic_fetch_add(sums + page / pages_per_block, s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

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
// visit(v, u, byte_off, ptr2): edge v -> u stored at byte_off of the page; ptr2
// is the frame of the same page of a second paged array (edge weights) or null.
template <class Active, class Visit>
__device__ __forceinline__ void walk_owned_pages(const gpuvm_dev_t &vm, const gpuvm_dev_t *vm2,
                                                 const int64_t *__restrict__ row_ptr,
                                                 const unsigned int *__restrict__ page_owner,
                                                 Active active, Visit visit) {
    const unsigned int lane = threadIdx.x & 63;
    const unsigned int wave = (blockIdx.x * kBlock + threadIdx.x) >> 6;
    const unsigned int nwaves = (gridDim.x * kBlock) >> 6;
    const unsigned int elems_shift = vm.page_shift - 2;
    const int64_t n_edges = (int64_t)(vm.bytes >> 2);
    constexpr int kSmall = 32;                    // lists up to this length: one lane each
    for (unsigned int page = wave; page < vm.n_pages; page += nwaves) {
        const int64_t e_lo = (int64_t)page << elems_shift;
        const int64_t e_hi = min((long long)n_edges, (long long)(e_lo + ((int64_t)1 << elems_shift)));
        const int64_t v_first = page_owner[page], v_last = page_owner[page + 1];
        const char *ptr = nullptr, *ptr2 = nullptr;
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
                ptr = gpuvm_acquire(vm, page, false);
                if (vm2) ptr2 = gpuvm_acquire(*vm2, page, false);
            }
            const bool small = len > 0 && len <= kSmall;
            int longest = small ? len : 0;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) longest = max(longest, __shfl_xor(longest, off, 64));
            const unsigned int my_off = (unsigned int)(beg - e_lo) << 2;
            for (int j = 0; j < longest; ++j) {
                if (small && j < len) {
                    const unsigned int o = my_off + ((unsigned int)j << 2);
                    visit(v, (int32_t)gpuvm_frame_load_b32(vm, ptr, o), o, ptr2);
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
                    visit(vl, (int32_t)gpuvm_frame_load_b32(vm, ptr, o), o, ptr2);
                }
            }
        }
        if (ptr) {
            gpuvm_release(vm, page);
            if (vm2) gpuvm_release(*vm2, page);
        }
    }
}

__global__ __launch_bounds__(kBlock) void k_bfs_level_balanced(gpuvm_dev_t vm, const int64_t *__restrict__ row_ptr,
                                                                const unsigned int *__restrict__ page_owner,
                                                                int32_t *level, int32_t cur, int *changed) {
    int found = 0;
    walk_owned_pages(vm, nullptr, row_ptr, page_owner,
                     [&](int64_t v) { return level[v] == cur; },
                     [&](int64_t, int32_t u, unsigned int, const char *) {
                         if (level[u] < 0) { level[u] = cur + 1; found = 1; }
                     });
    if (__builtin_amdgcn_ballot_w64(found != 0) && (threadIdx.x & 63) == 0) *changed = 1;
}

// Connected components (weak) by label propagation: every round walks every
// edge (v, u) and pulls both labels down to the smaller one; the fixed point
// labels each vertex with the smallest vertex id of its component.
__global__ __launch_bounds__(kBlock) void k_cc_round_balanced(gpuvm_dev_t vm, const int64_t *__restrict__ row_ptr,
                                                               const unsigned int *__restrict__ page_owner,
                                                               int32_t *label, int *changed) {
    int found = 0;
    walk_owned_pages(vm, nullptr, row_ptr, page_owner,
                     [&](int64_t) { return true; },
                     [&](int64_t v, int32_t u, unsigned int, const char *) {
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
                                                                 const unsigned int *__restrict__ page_owner,
                                                                 uint32_t *dist, const unsigned char *act_cur,
                                                                 unsigned char *act_next, int *changed) {
    int found = 0;
    walk_owned_pages(vm, &vmw, row_ptr, page_owner,
                     [&](int64_t v) { return act_cur[v] != 0; },
                     [&](int64_t v, int32_t u, unsigned int off, const char *pw) {
                         const uint32_t w = gpuvm_frame_load_b32(vmw, pw, off);
                         const uint32_t dv = __hip_atomic_load(dist + v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                         if (dv != 0xFFFFFFFFu) {
                             const uint32_t nd = dv + w;
                             const uint32_t old = __hip_atomic_fetch_min(dist + u, nd, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                             if (nd < old) { act_next[u] = 1; found = 1; }
                         }
                     });
    if (__builtin_amdgcn_ballot_w64(found != 0) && (threadIdx.x & 63) == 0) *changed = 1;
}

__global__ void k_iota32(int32_t *p, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = (int32_t)i;
}
__global__ void k_fill8(unsigned char *p, size_t n, unsigned char v) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// Embedding bag, sum pooling: one wave per bag; a row of 64*VPL floats is read
// as VPL consecutive floats per lane; rows are added in listed order in fp32.
template <int VPL>
__global__ __launch_bounds__(kBlock) void k_embedding_bag(gpuvm_dev_t vm, const int32_t *__restrict__ ids,
                                                           size_t bags, unsigned int bag_len, float *__restrict__ out,
                                                           unsigned long long n_rows) {
    typedef float vec_t __attribute__((ext_vector_type(VPL)));
    const unsigned int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const size_t nwaves = ((size_t)gridDim.x * kBlock) >> 6;
    const unsigned int row_bytes = 64u * VPL * 4u;
    for (size_t bag = wave; bag < bags; bag += nwaves) {
        vec_t acc = 0.0f;
        for (unsigned int j0 = 0; j0 < bag_len; j0 += 64) {
            const unsigned int nj = min(64u, bag_len - j0);
            int my_id = 0;
            if (lane < nj) my_id = ids[bag * bag_len + j0 + lane];
            for (unsigned int j = 0; j < nj; ++j) {
                const unsigned long long id = (unsigned int)__builtin_amdgcn_readlane(my_id, j);
                if (id >= n_rows) { if (lane == 0) raise_error(vm, GPUVM_ERANGE); continue; }
                const unsigned long long byte = id * row_bytes;
                const unsigned int page = (unsigned int)(byte >> vm.page_shift);
                const unsigned int off = (unsigned int)(byte & ((1ull << vm.page_shift) - 1));
                const char *p = gpuvm_acquire(vm, page, false);
                vec_t v;
                const unsigned int o = off + lane * (VPL * 4u);
                if constexpr (VPL == 1) {
                    v = __uint_as_float(gpuvm_frame_load_b32(vm, p, o));
                } else if constexpr (VPL == 2) {
                    const u32x2 r = gpuvm_frame_load_b64(vm, p, o);
                    v.x = __uint_as_float(r.x); v.y = __uint_as_float(r.y);
                } else {
                    const u32x4 r = gpuvm_frame_load_b128(vm, p, o);
                    v.x = __uint_as_float(r.x); v.y = __uint_as_float(r.y);
                    v.z = __uint_as_float(r.z); v.w = __uint_as_float(r.w);
                }
                gpuvm_release(vm, page);
                acc += v;
            }
        }
        *reinterpret_cast<vec_t *>(out + bag * (64u * VPL) + lane * VPL) = acc;
    }
}

// Transposed matrix-vector product y = A^T x over a paged row-major fp32 matrix:
// a thread owns a column and walks down the rows, so consecutive accesses of a
// thread are a whole row apart (the column-order pattern of the paper's
// transfer-bound applications, which has no spatial locality per thread); the
// 64 lanes of a wave read 256 consecutive bytes of one row.  fp64 accumulation.
__global__ __launch_bounds__(kBlock) void k_matvec_t(gpuvm_dev_t vm, unsigned long long rows, unsigned long long cols,
                                                      unsigned int skew, const float *__restrict__ x,
                                                      double *__restrict__ y) {
    const size_t nthreads = (size_t)gridDim.x * kBlock;
    const unsigned long long cols_up = (cols + 63) & ~63ull;           // whole waves stay together
    for (unsigned long long j = (size_t)blockIdx.x * kBlock + threadIdx.x; j < cols_up; j += nthreads) {
        double acc = 0.0;
        const bool want = j < cols;
        // Waves that walk down the same rows in lock step would all wait for
        // the same one or two pages at a time; starting each block of columns
        // a few rows apart keeps `skew` rows of pages in flight instead.
        const unsigned long long r0 = (j >> 6) % skew;
        for (unsigned long long k = 0; k < rows; ++k) {
            const unsigned long long i = k + r0 < rows ? k + r0 : k + r0 - rows;
            acc += (double)gpuvm_load_if<float>(vm, want ? i * cols + j : 0, want) * (double)x[i];
        }
        if (want) y[j] = acc;
    }
}

// Filter-then-gather over two paged uint32 columns (the paper's query pattern:
// scan one column, fetch another only for the few rows that pass): for rows
// with key > threshold add val[row] to a 64-bit sum and count the row.  The key
// column is streamed page by page by whole waves; the value column is reached
// through the element accessor by the (sparse, divergent) matching lanes.
__global__ __launch_bounds__(kBlock) void k_filter_sum(gpuvm_dev_t vmk, gpuvm_dev_t vmv, unsigned int threshold,
                                                        unsigned long long *count, unsigned long long *sum) {
    const unsigned int lane = threadIdx.x & 63;
    const unsigned int wave = (blockIdx.x * kBlock + threadIdx.x) >> 6;
    const unsigned int nwaves = (gridDim.x * kBlock) >> 6;
    const unsigned int elems_shift = vmk.page_shift - 2;
    unsigned long long my_count = 0, my_sum = 0;
    for (unsigned int page = wave; page < vmk.n_pages; page += nwaves) {
        const unsigned int n = page_len(vmk, page) >> 2;
        const unsigned long long first = (unsigned long long)page << elems_shift;
        const char *p = gpuvm_acquire(vmk, page, false);
        for (unsigned int i0 = 0; i0 < n; i0 += 64) {
            const unsigned int i = i0 + lane;
            const bool hit = i < n && gpuvm_frame_load_b32(vmk, p, i << 2) > threshold;
            if (__builtin_amdgcn_ballot_w64(hit) == 0) continue;
            const uint32_t v = gpuvm_load_if<uint32_t>(vmv, hit ? first + i : 0, hit);   // all lanes help to fault
            if (hit) {
                my_sum += v;
                my_count += 1;
            }
        }
        gpuvm_release(vmk, page);
    }
    my_sum = wave_sum(my_sum);
    my_count = wave_sum(my_count);
    if (lane == 0 && my_count) {
        __hip_atomic_fetch_add(sum, my_sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(count, my_count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ------------------------------------------------------------------ roofline kernels

__global__ __launch_bounds__(kBlock) void k_bench_copy(char *dst, const char *src, size_t bytes, size_t chunk) {
    const wave_t w = wave_now();
    const size_t wave = ((size_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const size_t nwaves = ((size_t)gridDim.x * kBlock) >> 6;
    const size_t nchunks = (bytes + chunk - 1) / chunk;
    for (size_t c = wave; c < nchunks; c += nwaves) {
        const size_t lo = c * chunk;
        const unsigned int len = (unsigned int)(chunk < bytes - lo ? chunk : bytes - lo);
        wave_copy<GPUVM_AUX_SYSTEM, GPUVM_AUX_SYSTEM>(dst + lo, src + lo, len, w);
    }
}

__global__ __launch_bounds__(kBlock) void k_bench_read(const char *src, size_t bytes, size_t chunk,
                                                        unsigned long long *sink) {
    const unsigned int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const size_t nwaves = ((size_t)gridDim.x * kBlock) >> 6;
    const size_t nchunks = (bytes + chunk - 1) / chunk;
    u32x4 acc = {0, 0, 0, 0};
    for (size_t c = wave; c < nchunks; c += nwaves) {
        const size_t lo = c * chunk;
        const unsigned int nvec = (unsigned int)((chunk < bytes - lo ? chunk : bytes - lo) >> 4);
        const u32x4 *p = reinterpret_cast<const u32x4 *>(src + lo);
        unsigned int i = lane;
        for (; i + 7 * 64 < nvec; i += 8 * 64) {
            u32x4 r[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) r[j] = p[i + j * 64];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc ^= r[j];
        }
        for (; i < nvec; i += 64) acc ^= p[i];
    }
    unsigned long long v = ((unsigned long long)(acc.x ^ acc.z) << 32) | (acc.y ^ acc.w);
    if (v == 0x9E3779B97F4A7C15ull) sink[0] = v;   // practically never: keeps the loads alive
}

// One wave, a chain of dependent 16-byte-per-lane loads (1 KiB per hop, the
// mover's instruction): the unloaded round-trip time of the memory behind src.
__global__ __launch_bounds__(64) void k_bench_latency(const char *src, unsigned int bytes, unsigned int hops,
                                                       unsigned int zero, unsigned long long *out) {
    const unsigned int lane = threadIdx.x & 63;
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(src, bytes);
    unsigned int off = lane * 16u, acc = 0;
    const unsigned int span = bytes - 1024u;
    const unsigned long long t0 = wall_clock64();
    for (unsigned int h = 0; h < hops; ++h) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, GPUVM_AUX_SYSTEM);
        acc ^= v.x;
        off = (off + 69632u + (v.x & zero)) % span / 1024u * 1024u + lane * 16u;   // next hop needs this one's data
    }
    const unsigned long long t1 = wall_clock64();
    if (lane == 0) { out[0] = t1 - t0; out[1] = acc; }
}

__global__ __launch_bounds__(kBlock) void k_bench_gather_plain(const uint32_t *__restrict__ data,
                                                                const uint32_t *__restrict__ idx, size_t n,
                                                                uint32_t *__restrict__ out) {
    const size_t nthreads = (size_t)gridDim.x * kBlock;
    for (size_t k = (size_t)blockIdx.x * kBlock + threadIdx.x; k < n; k += nthreads) out[k] = data[idx[k]];
}

// ------------------------------------------------------------------ deterministic phases

// (A) first toucher of each page in this phase pins it if resident, else lists it.
__global__ __launch_bounds__(kBlock) void k_phase_lookup(gpuvm_dev_t vm, const uint32_t *__restrict__ idx, size_t k,
                                                          unsigned int elem_shift, unsigned long long n_elems,
                                                          unsigned int tag, unsigned int *stamp, unsigned char *first,
                                                          unsigned int *miss, unsigned int *ctr) {
    const size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= k) return;
    first[i] = 0;
    const unsigned long long e = idx[i];
    if (e >= n_elems) { raise_error(vm, GPUVM_ERANGE); return; }
    const unsigned int page = (unsigned int)((e << elem_shift) >> vm.page_shift);
    if (atomicExch(stamp + page, tag) == tag) return;                 // somebody else was first
    first[i] = 1;
    const unsigned long long pq = a_load(vm.pte + page);
    if (((pq & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) == GPUVM_ST_RESIDENT) {
        a_add(vm.pte + page, 1ull);                                   // one more user
        if (!(pq & GPUVM_PTE_REF)) a_or(vm.pte + page, GPUVM_PTE_REF);
        atomicAdd(ctr + 1, 1u);
    } else {
        miss[atomicAdd(ctr + 0, 1u)] = page;
    }
}

// (B) one workgroup: rank-sort the missing pages, then ONE thread serves them
// in ascending order, walking the frame ring like a sequential replay.
__global__ __launch_bounds__(1024) void k_phase_assign(gpuvm_dev_t vm, const unsigned int *miss, unsigned int *sorted,
                                                        phase_job *jobs, unsigned int *ctr) {
    const unsigned int n = ctr[0];
    for (unsigned int i = threadIdx.x; i < n; i += blockDim.x) {
        const unsigned int x = miss[i];
        unsigned int r = 0;
        for (unsigned int j = 0; j < n; ++j) r += miss[j] < x;        // pages are distinct
        sorted[r] = x;
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    unsigned long long *st = vm.stats;                                // shard 0
    st[GPUVM_S_PHASES] += 1;
    st[GPUVM_S_HITS] += ctr[1];
    if ((unsigned long long)n + ctr[1] > vm.n_frames) { raise_error(vm, GPUVM_EDEADLK); ctr[2] = 0; ctr[0] = 0; ctr[1] = 0; return; }
    unsigned long long hand = vm.hand[0];
    unsigned int done = 0;
    for (unsigned int i = 0; i < n; ++i) {
        const unsigned int p = sorted[i];
        unsigned int f, victim = GPUVM_NO_PAGE, wb = 0;
        unsigned long long guard = 0;
        for (;;) {
            if (++guard > 3ull * vm.n_frames + 3) { raise_error(vm, GPUVM_EDEADLK); goto out; }
            f = (unsigned int)(hand % vm.n_frames);
            ++hand;
            const unsigned int q = vm.frame_owner[f];
            if (q == GPUVM_NO_PAGE) break;
            const unsigned long long pq = vm.pte[q];
            if (pq & GPUVM_PTE_PIN_MASK) { st[GPUVM_S_SKIPS] += 1; continue; }
            if (vm.policy == GPUVM_POLICY_CLOCK && (pq & GPUVM_PTE_REF)) {
                vm.pte[q] = pq & ~GPUVM_PTE_REF;
                st[GPUVM_S_SWEEPS] += 1;
                continue;
            }
            victim = q;
            wb = (pq & GPUVM_PTE_DIRTY) ? 1u : 0u;
            st[GPUVM_S_EVICTIONS] += 1;
            if (wb) { st[GPUVM_S_WB_EVICT] += 1; st[GPUVM_S_BYTES_OUT] += page_len(vm, q); }
            vm.pte[q] = pq & GPUVM_PTE_GEN_MASK;                      // INVALID
            break;
        }
        vm.frame_owner[f] = p;
        vm.pte[p] = (GPUVM_ST_RESIDENT << GPUVM_PTE_STATE_SHIFT) | ((unsigned long long)f << GPUVM_PTE_FRAME_SHIFT) |
                    GPUVM_PTE_REF | ((vm.pte[p] + (1ull << GPUVM_PTE_GEN_SHIFT)) & GPUVM_PTE_GEN_MASK) |
                    1ull;                                             // next generation, pinned once
        st[GPUVM_S_FAULTS] += 1;
        st[GPUVM_S_BYTES_IN] += page_len(vm, p);
        jobs[done].page = p; jobs[done].frame = f; jobs[done].victim = victim; jobs[done].writeback = wb;
        ++done;
    }
out:
    vm.hand[0] = hand;
    ctr[2] = done;
    ctr[0] = 0;
    ctr[1] = 0;
}

// (C) one wave per fault: write the dirty victim back, then migrate the page.
__global__ __launch_bounds__(kBlock) void k_phase_migrate(gpuvm_dev_t vm, const phase_job *jobs, const unsigned int *ctr) {
    const wave_t w = wave_now();
    const unsigned int wave = (blockIdx.x * kBlock + threadIdx.x) >> 6;
    const unsigned int nwaves = (gridDim.x * kBlock) >> 6;
    const unsigned int n = ctr[2];
    for (unsigned int j = wave; j < n; j += nwaves) {
        const phase_job job = jobs[j];
        char *frame = vm.frames + ((size_t)job.frame << vm.page_shift);
        if (job.writeback)
            copy_frame_to_host(vm.host + ((size_t)job.victim << vm.page_shift), frame, page_len(vm, job.victim), w);
        if (job.writeback) wait_vm();
        copy_host_to_frame(frame, vm.host + ((size_t)job.page << vm.page_shift), page_len(vm, job.page), w);
    }
    wait_vm();
}

// (D) the accesses themselves (every page of the phase is resident and pinned),
// then the first toucher of each page drops the phase's pin.
template <int OP>   // 0: gather uint32, 1: increment uint64
__global__ __launch_bounds__(kBlock) void k_phase_access(gpuvm_dev_t vm, const uint32_t *__restrict__ idx, size_t k,
                                                          unsigned long long n_elems, const unsigned char *first,
                                                          uint32_t *out, unsigned long long *sum) {
    const size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    unsigned long long acc = 0;
    if (i < k && idx[i] < n_elems) {
        const unsigned long long byte = (unsigned long long)idx[i] << (OP == 0 ? 2 : 3);
        const unsigned int page = (unsigned int)(byte >> vm.page_shift);
        const unsigned int off = (unsigned int)(byte & ((1ull << vm.page_shift) - 1));
        const unsigned long long pq = a_load(vm.pte + page);
        char *p = vm.frames + ((size_t)(pq >> GPUVM_PTE_FRAME_SHIFT) << vm.page_shift) + off;
        if (OP == 0) {
            const uint32_t v = __hip_atomic_load(reinterpret_cast<const uint32_t *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            out[i] = v;
            acc = v;
        } else {
            __hip_atomic_fetch_add(reinterpret_cast<unsigned long long *>(p), 1ull, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            if (!(pq & GPUVM_PTE_DIRTY)) a_or(vm.pte + page, GPUVM_PTE_DIRTY);
        }
        if (first[i]) {
            // the pin only guards the page during this phase's frame assignment,
            // which is over; nothing is evicted before the next phase's kernels
            a_add(vm.pte + page, ~0ull);
        }
    }
    if (OP == 0 && sum) {
        acc = wave_sum(acc);
        if ((threadIdx.x & 63) == 0 && acc)
            __hip_atomic_fetch_add(sum, acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ------------------------------------------------------------------ host helpers

namespace {

int check_kernel_error(gpuvm_t *vm) {
    unsigned long long word = 0;
    HIP_TRY(hipMemcpy(&word, vm->dev.hand + 1, sizeof(word), hipMemcpyDeviceToHost));
    return word ? -(int)word : GPUVM_OK;
}

int grid_for_waves(int waves) { return std::max(1, waves / kWavesPerBlock); }

int launch_waves(const gpuvm_t *vm, size_t work_waves) {
    // waves in flight: enough to fill the device, never more than half the
    // frames, whole workgroups; 0 if not even one workgroup may run
    long long cap = std::min<long long>((long long)vm->cus * vm->waves_per_cu, vm->dev.n_frames / 2);
    cap = (cap / kWavesPerBlock) * kWavesPerBlock;
    const long long need = (long long)((std::max<size_t>(work_waves, 1) + kWavesPerBlock - 1) / kWavesPerBlock) * kWavesPerBlock;
    return (int)std::min(cap, need);
}

int ensure_phase_scratch(gpuvm_t *vm, size_t phase_len) {
    if (!vm->stamp) {
        HIP_TRY(hipMalloc(&vm->stamp, (size_t)vm->dev.n_pages * sizeof(unsigned int)));
        HIP_TRY(hipMalloc(&vm->phase_ctr, 4 * sizeof(unsigned int)));
        k_fill32<<<256, 256>>>(vm->stamp, vm->dev.n_pages, 0u);
        k_fill32<<<1, 64>>>(vm->phase_ctr, 4, 0u);
        HIP_TRY(hipDeviceSynchronize());
    }
    if (phase_len > vm->phase_cap) {
        if (vm->first) { (void)hipFree(vm->first); (void)hipFree(vm->miss); (void)hipFree(vm->miss_sorted); (void)hipFree(vm->jobs); }
        vm->first = nullptr; vm->phase_cap = 0;
        HIP_TRY(hipMalloc(&vm->first, phase_len));
        HIP_TRY(hipMalloc(&vm->miss, phase_len * sizeof(unsigned int)));
        HIP_TRY(hipMalloc(&vm->miss_sorted, phase_len * sizeof(unsigned int)));
        HIP_TRY(hipMalloc(&vm->jobs, phase_len * sizeof(phase_job)));
        vm->phase_cap = phase_len;
    }
    return GPUVM_OK;
}

template <int OP>
int run_phased(gpuvm_t *vm, const uint32_t *d_idx, size_t n, size_t phase_len, uint32_t *d_out,
               uint64_t *d_sum, void *stream) {
    if (!vm || (!d_idx && n) || phase_len == 0 || phase_len > (1u << 16)) return GPUVM_EINVAL;
    if (vm->dev.policy == GPUVM_POLICY_FIFO_WAIT) return GPUVM_EINVAL;   // a sequential agent cannot wait
    if (OP == 0 && !d_out && n) return GPUVM_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    int rc = ensure_phase_scratch(vm, phase_len);
    if (rc) return rc;
    const unsigned int elem_shift = OP == 0 ? 2 : 3;
    const unsigned long long n_elems = vm->dev.bytes >> elem_shift;
    const int mig_waves = std::max(kWavesPerBlock, launch_waves(vm, phase_len));
    for (size_t lo = 0; lo < n; lo += phase_len) {
        const size_t k = std::min(phase_len, n - lo);
        const int grid = (int)((k + kBlock - 1) / kBlock);
        if (++vm->phase_tag == 0) {                       // tag wrapped: forget old stamps
            k_fill32<<<256, 256, 0, s>>>(vm->stamp, vm->dev.n_pages, 0u);
            vm->phase_tag = 1;
        }
        k_phase_lookup<<<grid, kBlock, 0, s>>>(vm->dev, d_idx + lo, k, elem_shift, n_elems, vm->phase_tag,
                                               vm->stamp, vm->first, vm->miss, vm->phase_ctr);
        k_phase_assign<<<1, 1024, 0, s>>>(vm->dev, vm->miss, vm->miss_sorted, vm->jobs, vm->phase_ctr);
        k_phase_migrate<<<grid_for_waves(mig_waves), kBlock, 0, s>>>(vm->dev, vm->jobs, vm->phase_ctr);
        k_phase_access<OP><<<grid, kBlock, 0, s>>>(vm->dev, d_idx + lo, k, n_elems, vm->first,
                                                   d_out ? d_out + lo : nullptr, (unsigned long long *)d_sum);
    }
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(s));
    return check_kernel_error(vm);
}

}  // namespace

// ------------------------------------------------------------------ C ABI

extern "C" {

const char *gpuvm_strerror(int code) {
    switch (code) {
        case GPUVM_OK: return "ok";
        case GPUVM_EINVAL: return "invalid argument";
        case GPUVM_ENOMEM: return "out of memory";
        case GPUVM_EPIN: return "host buffer is not pinned GPU-mapped memory";
        case GPUVM_EDEADLK: return "frame pool too small for the waves in flight, or a bounded in-kernel wait ran out";
        case GPUVM_EHIP: return "HIP runtime error";
        case GPUVM_ERANGE: return "index outside the data set";
        default: return "unknown gpuvm error";
    }
}

int gpuvm_host_alloc(size_t bytes, void **out) {
    if (!out || bytes == 0) return GPUVM_EINVAL;
    *out = nullptr;
    hipError_t e = hipHostMalloc(out, bytes, hipHostMallocDefault);
    if (e != hipSuccess) { (void)hipGetLastError(); *out = nullptr; return GPUVM_ENOMEM; }
    return GPUVM_OK;
}

int gpuvm_host_free(void *p) {
    if (!p) return GPUVM_OK;
    HIP_TRY(hipHostFree(p));
    return GPUVM_OK;
}

int gpuvm_create(void *host_buf, size_t bytes, size_t page_bytes, size_t frame_pool_bytes, int policy,
                 gpuvm_t **out) {
    if (!out) return GPUVM_EINVAL;
    *out = nullptr;
    if (!host_buf || bytes == 0) return GPUVM_EINVAL;
    if (page_bytes < 4096 || page_bytes > (1u << 20) || (page_bytes & (page_bytes - 1))) return GPUVM_EINVAL;
    if (policy != GPUVM_POLICY_FIFO && policy != GPUVM_POLICY_CLOCK && policy != GPUVM_POLICY_FIFO_WAIT) return GPUVM_EINVAL;
    const size_t n_frames = frame_pool_bytes / page_bytes;
    const size_t n_pages = (bytes + page_bytes - 1) / page_bytes;
    if (n_frames < 2 || n_frames >= (1u << 28) || n_pages >= 0xFFFFFFFFull) return GPUVM_EINVAL;

    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, host_buf) != hipSuccess) { (void)hipGetLastError(); return GPUVM_EPIN; }
    if (attr.type != hipMemoryTypeHost || !attr.devicePointer) return GPUVM_EPIN;
    // the whole range must lie inside the pinned allocation
    hipPointerAttribute_t last;
    if (hipPointerGetAttributes(&last, (char *)host_buf + bytes - 1) != hipSuccess ||
        last.type != hipMemoryTypeHost) { (void)hipGetLastError(); return GPUVM_EPIN; }

    gpuvm_t *vm = new (std::nothrow) gpuvm();
    if (!vm) return GPUVM_ENOMEM;
    memset(&vm->dev, 0, sizeof(vm->dev));
    HIP_TRY(hipGetDevice(&vm->device));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, vm->device));
    vm->cus = prop.multiProcessorCount;
    vm->waves_per_cu = 8;
    if (const char *e = getenv("GPUVM_WAVES_PER_CU")) vm->waves_per_cu = std::max(1, std::min(32, atoi(e)));
    vm->page_bytes = page_bytes;
    gpuvm_dev_t &d = vm->dev;
    d.host = (char *)attr.devicePointer;
    d.bytes = bytes;
    d.n_pages = (uint32_t)n_pages;
    d.n_frames = (uint32_t)n_frames;
    d.page_shift = (uint32_t)__builtin_ctzll(page_bytes);
    d.policy = (uint32_t)policy;
    d.spin_limit = kDefaultSpinLimit;
    d.flags = 0;
    int rc = GPUVM_OK;
    auto alloc = [&](void **p, size_t sz) {
        if (rc) return;
        if (hipMalloc(p, sz) != hipSuccess) { (void)hipGetLastError(); rc = GPUVM_ENOMEM; }
    };
    alloc((void **)&d.frames, n_frames * page_bytes);
    alloc((void **)&d.pte, n_pages * sizeof(unsigned long long));
    alloc((void **)&d.frame_owner, n_frames * sizeof(unsigned int));
    alloc((void **)&d.hand, 2 * sizeof(unsigned long long));
    alloc((void **)&d.stats, (size_t)GPUVM_STAT_SLOTS * GPUVM_S_COUNT * sizeof(unsigned long long));
    alloc((void **)&vm->bfs_changed, sizeof(int));
    if (rc) { gpuvm_destroy(vm); return rc; }
    k_fill64<<<256, 256>>>(d.pte, n_pages, 0ull);
    k_fill32<<<256, 256>>>(d.frame_owner, n_frames, GPUVM_NO_PAGE);
    k_fill64<<<1, 64>>>(d.hand, 2, 0ull);
    k_fill64<<<4, 256>>>(d.stats, (size_t)GPUVM_STAT_SLOTS * GPUVM_S_COUNT, 0ull);
    if (hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); gpuvm_destroy(vm); return GPUVM_EHIP; }
    *out = vm;
    return GPUVM_OK;
}

int gpuvm_destroy(gpuvm_t *vm) {
    if (!vm) return GPUVM_OK;
    (void)hipDeviceSynchronize();
    gpuvm_dev_t &d = vm->dev;
    (void)hipFree(d.frames); (void)hipFree(d.pte); (void)hipFree(d.frame_owner); (void)hipFree(d.hand); (void)hipFree(d.stats);
    (void)hipFree(vm->stamp); (void)hipFree(vm->first); (void)hipFree(vm->miss); (void)hipFree(vm->miss_sorted); (void)hipFree(vm->jobs);
    (void)hipFree(vm->phase_ctr); (void)hipFree(vm->bfs_changed); (void)hipFree(vm->page_owner);
    delete vm;
    return GPUVM_OK;
}

int gpuvm_device_handle(const gpuvm_t *vm, gpuvm_dev_t *out) {
    if (!vm || !out) return GPUVM_EINVAL;
    *out = vm->dev;
    return GPUVM_OK;
}

int gpuvm_configure(gpuvm_t *vm, uint32_t spin_limit, int access_stats) {
    if (!vm) return GPUVM_EINVAL;
    vm->dev.spin_limit = spin_limit ? spin_limit : kDefaultSpinLimit;
    vm->dev.flags = access_stats ? (vm->dev.flags | GPUVM_F_ACCESS_STATS) : (vm->dev.flags & ~GPUVM_F_ACCESS_STATS);
    return GPUVM_OK;
}

int gpuvm_set_waves_per_cu(gpuvm_t *vm, int waves_per_cu) {
    if (!vm || waves_per_cu < 1 || waves_per_cu > 32) return GPUVM_EINVAL;
    vm->waves_per_cu = waves_per_cu;
    return GPUVM_OK;
}

int gpuvm_max_waves(const gpuvm_t *vm) {
    if (!vm) return GPUVM_EINVAL;
    return launch_waves(vm, (size_t)1 << 40);
}

int gpuvm_flush(gpuvm_t *vm, void *stream) {
    if (!vm) return GPUVM_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int waves = std::max(kWavesPerBlock, std::min<int>(vm->cus * 8, (int)std::min<size_t>(vm->dev.n_frames, 1 << 20)));
    k_flush<<<grid_for_waves(waves), kBlock, 0, s>>>(vm->dev);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(s));
    return check_kernel_error(vm);
}

int gpuvm_reset(gpuvm_t *vm, void *stream) {
    if (!vm) return GPUVM_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int waves = std::max(kWavesPerBlock, std::min<int>(vm->cus * 8, (int)std::min<size_t>(vm->dev.n_frames, 1 << 20)));
    k_flush<<<grid_for_waves(waves), kBlock, 0, s>>>(vm->dev);
    gpuvm_dev_t &d = vm->dev;
    k_fill64<<<256, 256, 0, s>>>(d.pte, d.n_pages, 0ull);
    k_fill32<<<256, 256, 0, s>>>(d.frame_owner, d.n_frames, GPUVM_NO_PAGE);
    k_fill64<<<1, 64, 0, s>>>(d.hand, 2, 0ull);
    k_fill64<<<4, 256, 0, s>>>(d.stats, (size_t)GPUVM_STAT_SLOTS * GPUVM_S_COUNT, 0ull);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(s));
    return GPUVM_OK;
}

int gpuvm_stats(gpuvm_t *vm, gpuvm_stats_t *out) {
    if (!vm || !out) return GPUVM_EINVAL;
    HIP_TRY(hipDeviceSynchronize());
    std::vector<unsigned long long> raw((size_t)GPUVM_STAT_SLOTS * GPUVM_S_COUNT);
    HIP_TRY(hipMemcpy(raw.data(), vm->dev.stats, raw.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
    uint64_t tot[GPUVM_S_COUNT] = {0};
    for (int s = 0; s < GPUVM_STAT_SLOTS; ++s)
        for (int c = 0; c < GPUVM_S_COUNT; ++c) tot[c] += raw[(size_t)s * GPUVM_S_COUNT + c];
    static_assert(sizeof(gpuvm_stats_t) == GPUVM_S_COUNT * sizeof(uint64_t), "stats layout");
    memcpy(out, tot, sizeof(tot));
    return check_kernel_error(vm);
}

int gpuvm_stats_clear(gpuvm_t *vm) {
    if (!vm) return GPUVM_EINVAL;
    HIP_TRY(hipDeviceSynchronize());
    k_fill64<<<4, 256>>>(vm->dev.stats, (size_t)GPUVM_STAT_SLOTS * GPUVM_S_COUNT, 0ull);
    HIP_TRY(hipDeviceSynchronize());
    return GPUVM_OK;
}

int gpuvm_dump_tables(gpuvm_t *vm, uint64_t *pte_out, uint32_t *owner_out, uint64_t *hand_out) {
    if (!vm) return GPUVM_EINVAL;
    HIP_TRY(hipDeviceSynchronize());
    if (pte_out) HIP_TRY(hipMemcpy(pte_out, vm->dev.pte, (size_t)vm->dev.n_pages * 8, hipMemcpyDeviceToHost));
    if (owner_out) HIP_TRY(hipMemcpy(owner_out, vm->dev.frame_owner, (size_t)vm->dev.n_frames * 4, hipMemcpyDeviceToHost));
    if (hand_out) HIP_TRY(hipMemcpy(hand_out, vm->dev.hand, 8, hipMemcpyDeviceToHost));
    return check_kernel_error(vm);
}

int gpuvm_check(gpuvm_t *vm, void *stream) {
    if (!vm) return GPUVM_EINVAL;
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    return check_kernel_error(vm);
}

// ---- free-running launchers

int gpuvm_run_gather(gpuvm_t *vm, const uint32_t *d_idx, size_t n, uint32_t *d_out, uint64_t *d_sum,
                     void *stream) {
    if (!vm || (n && (!d_idx || !d_out))) return GPUVM_EINVAL;
    if (n == 0) return GPUVM_OK;
    const int waves = launch_waves(vm, (n + 63) / 64);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    k_gather<<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm->dev, d_idx, n, d_out,
                                                                         (unsigned long long *)d_sum,
                                                                         vm->dev.bytes / 4);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_run_scatter_increment(gpuvm_t *vm, const uint32_t *d_idx, size_t n, void *stream) {
    if (!vm || (n && !d_idx)) return GPUVM_EINVAL;
    if (n == 0) return GPUVM_OK;
    const int waves = launch_waves(vm, (n + 63) / 64);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    k_scatter_inc<<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm->dev, d_idx, n, vm->dev.bytes / 8);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_run_vector_add(gpuvm_t *vm_a, gpuvm_t *vm_b, gpuvm_t *vm_c, size_t n, void *stream) {
    if (!vm_a || !vm_b || !vm_c || vm_a == vm_c || vm_b == vm_c) return GPUVM_EINVAL;
    if (n * 4 > vm_a->dev.bytes || n * 4 > vm_b->dev.bytes || n * 4 > vm_c->dev.bytes) return GPUVM_ERANGE;
    if (n == 0) return GPUVM_OK;
    const size_t work = (n * 4 + vm_c->page_bytes - 1) / vm_c->page_bytes;       // page-sized stripes
    const int waves = std::min({launch_waves(vm_a, work), launch_waves(vm_b, work), launch_waves(vm_c, work)});
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    k_vector_add<<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm_a->dev, vm_b->dev, vm_c->dev, n);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_run_stream_reduce(gpuvm_t *vm, size_t block_elems, double *d_sums, void *stream) {
    if (!vm || !d_sums || block_elems == 0) return GPUVM_EINVAL;
    const size_t block_bytes = block_elems * 4;
    if (block_bytes % vm->page_bytes || vm->dev.bytes % 4) return GPUVM_EINVAL;
    const unsigned int ppb = (unsigned int)(block_bytes / vm->page_bytes);
    const size_t nblocks = (vm->dev.n_pages + ppb - 1) / ppb;
    const int waves = launch_waves(vm, vm->dev.n_pages);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    hipStream_t s = (hipStream_t)stream;
    k_fill64<<<64, 256, 0, s>>>((unsigned long long *)d_sums, nblocks, 0ull);   // +0.0
    k_stream_reduce<<<grid_for_waves(waves), kBlock, 0, s>>>(vm->dev, ppb, d_sums);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

static int ensure_page_owner(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv, hipStream_t s);

static int run_bfs(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv, int64_t src, int32_t *d_level,
                   int *n_levels_out, void *stream, bool balanced) {
    if (!vm || !d_row_ptr || !d_level || nv <= 0 || src < 0 || src >= nv || nv > 0x7FFFFFFF) return GPUVM_EINVAL;
    if (vm->dev.bytes % 4) return GPUVM_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int waves = launch_waves(vm, balanced ? (size_t)vm->dev.n_pages : (size_t)((nv + 63) / 64));
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    if (balanced) {
        int rc0 = ensure_page_owner(vm, d_row_ptr, nv, s);
        if (rc0) return rc0;
    }
    k_fill32<<<1024, 256, 0, s>>>((unsigned int *)d_level, (size_t)nv, 0xFFFFFFFFu);
    k_fill32<<<1, 64, 0, s>>>((unsigned int *)d_level + src, 1, 0u);
    int levels = 0;
    for (int32_t cur = 0;; ++cur) {
        int changed = 0;
        k_fill32<<<1, 64, 0, s>>>((unsigned int *)vm->bfs_changed, 1, 0u);
        if (balanced)
            k_bfs_level_balanced<<<grid_for_waves(waves), kBlock, 0, s>>>(vm->dev, d_row_ptr, vm->page_owner, d_level,
                                                                           cur, vm->bfs_changed);
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

static int ensure_page_owner(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv, hipStream_t s) {
    if (!vm->page_owner) HIP_TRY(hipMalloc(&vm->page_owner, ((size_t)vm->dev.n_pages + 1) * sizeof(unsigned int)));
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
        k_cc_round_balanced<<<grid_for_waves(waves), kBlock, 0, s>>>(vm->dev, d_row_ptr, vm->page_owner, d_label,
                                                                      vm->bfs_changed);
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
    k_fill32<<<1024, 256, 0, s>>>(d_dist, (size_t)nv, 0xFFFFFFFFu);
    k_fill32<<<1, 64, 0, s>>>(d_dist + src, 1, 0u);
    int rounds = 0;
    rc = GPUVM_OK;
    for (;;) {
        int changed = 0;
        unsigned char *cur = act + (size_t)(rounds & 1) * nv, *next = act + (size_t)((rounds + 1) & 1) * nv;
        k_fill32<<<1, 64, 0, s>>>((unsigned int *)vm->bfs_changed, 1, 0u);
        k_fill8<<<1024, 256, 0, s>>>(next, (size_t)nv, 0);
        k_sssp_round_balanced<<<grid_for_waves(waves), kBlock, 0, s>>>(vm->dev, vm_weights->dev, d_row_ptr,
                                                                        vm->page_owner, d_dist, cur, next,
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

int gpuvm_run_embedding_bag(gpuvm_t *vm, size_t dim, const int32_t *d_ids, size_t bags, size_t bag_len,
                            float *d_out, void *stream) {
    if (!vm || !d_ids || !d_out || bag_len == 0 || bag_len > 0xFFFFFFFFu) return GPUVM_EINVAL;
    if (dim != 64 && dim != 128 && dim != 256) return GPUVM_EINVAL;
    const size_t row_bytes = dim * 4;
    if (vm->page_bytes % row_bytes || vm->dev.bytes % row_bytes) return GPUVM_EINVAL;
    if (bags == 0) return GPUVM_OK;
    const int waves = launch_waves(vm, bags);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    const int grid = grid_for_waves(waves);
    hipStream_t s = (hipStream_t)stream;
    const unsigned long long n_rows = vm->dev.bytes / row_bytes;
    if (dim == 64) k_embedding_bag<1><<<grid, kBlock, 0, s>>>(vm->dev, d_ids, bags, (unsigned int)bag_len, d_out, n_rows);
    else if (dim == 128) k_embedding_bag<2><<<grid, kBlock, 0, s>>>(vm->dev, d_ids, bags, (unsigned int)bag_len, d_out, n_rows);
    else k_embedding_bag<4><<<grid, kBlock, 0, s>>>(vm->dev, d_ids, bags, (unsigned int)bag_len, d_out, n_rows);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_run_matvec_t(gpuvm_t *vm, size_t rows, size_t cols, const float *d_x, double *d_y, void *stream) {
    if (!vm || !d_x || !d_y || rows == 0 || cols == 0) return GPUVM_EINVAL;
    if (rows * cols * 4 != vm->dev.bytes) return GPUVM_EINVAL;
    const int waves = launch_waves(vm, (cols + 63) / 64);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    // rows of A the pool can hold; the start rows are spread over a window well inside it
    const size_t rows_in_pool = (size_t)vm->dev.n_frames * vm->page_bytes / (cols * 4);
    const unsigned int skew = (unsigned int)std::max<size_t>(1, std::min<size_t>({(size_t)64, rows_in_pool / 4, rows}));
    k_matvec_t<<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm->dev, rows, cols, skew, d_x, d_y);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_run_filter_sum(gpuvm_t *vm_key, gpuvm_t *vm_val, uint32_t threshold, uint64_t *d_count, uint64_t *d_sum,
                         void *stream) {
    if (!vm_key || !vm_val || vm_key == vm_val || !d_count || !d_sum) return GPUVM_EINVAL;
    if (vm_key->dev.bytes % 4 || vm_val->dev.bytes != vm_key->dev.bytes) return GPUVM_EINVAL;
    const int waves = std::min(launch_waves(vm_key, vm_key->dev.n_pages), launch_waves(vm_val, vm_key->dev.n_pages));
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    hipStream_t s = (hipStream_t)stream;
    k_fill64<<<1, 64, 0, s>>>((unsigned long long *)d_count, 1, 0ull);
    k_fill64<<<1, 64, 0, s>>>((unsigned long long *)d_sum, 1, 0ull);
    k_filter_sum<<<grid_for_waves(waves), kBlock, 0, s>>>(vm_key->dev, vm_val->dev, threshold,
                                                          (unsigned long long *)d_count, (unsigned long long *)d_sum);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

// ---- deterministic launchers

int gpuvm_run_gather_phased(gpuvm_t *vm, const uint32_t *d_idx, size_t n, size_t phase_len, uint32_t *d_out,
                            uint64_t *d_sum, void *stream) {
    return run_phased<0>(vm, d_idx, n, phase_len, d_out, d_sum, stream);
}

int gpuvm_run_scatter_increment_phased(gpuvm_t *vm, const uint32_t *d_idx, size_t n, size_t phase_len,
                                       void *stream) {
    return run_phased<1>(vm, d_idx, n, phase_len, nullptr, nullptr, stream);
}

// ---- roofline microbenchmarks

static int bench_waves(int waves) {
    if (waves <= 0) {
        int dev = 0, cus = 256;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            cus = prop.multiProcessorCount;
        waves = cus * 8;
    }
    return std::max(kWavesPerBlock, (waves / kWavesPerBlock) * kWavesPerBlock);
}

int gpuvm_bench_copy(void *dst, const void *src, size_t bytes, size_t chunk_bytes, int waves, void *stream) {
    if (!dst || !src || bytes == 0 || chunk_bytes < 16 || chunk_bytes % 16 || chunk_bytes > (1u << 30)) return GPUVM_EINVAL;
    k_bench_copy<<<grid_for_waves(bench_waves(waves)), kBlock, 0, (hipStream_t)stream>>>((char *)dst, (const char *)src,
                                                                                          bytes, chunk_bytes);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_bench_read(const void *src, size_t bytes, size_t chunk_bytes, int waves, uint64_t *d_sink, void *stream) {
    if (!src || !d_sink || bytes == 0 || chunk_bytes < 16 || chunk_bytes % 16 || chunk_bytes > (1u << 30)) return GPUVM_EINVAL;
    k_bench_read<<<grid_for_waves(bench_waves(waves)), kBlock, 0, (hipStream_t)stream>>>((const char *)src, bytes,
                                                                                          chunk_bytes,
                                                                                          (unsigned long long *)d_sink);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_bench_latency(const void *src, size_t bytes, int hops, double *ns_per_hop_out, void *stream) {
    if (!src || !ns_per_hop_out || bytes < (1u << 20) || bytes > (1u << 31) || hops < 1) return GPUVM_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    unsigned long long *d_out = nullptr, h_out[2] = {0, 0};
    HIP_TRY(hipMalloc(&d_out, 2 * sizeof(unsigned long long)));
    int dev = 0, khz = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    k_bench_latency<<<1, 64, 0, s>>>((const char *)src, (unsigned int)bytes, (unsigned int)hops, 0u, d_out);
    hipError_t e = hipMemcpyAsync(h_out, d_out, sizeof(h_out), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipFree(d_out);
    if (e != hipSuccess || khz <= 0) return GPUVM_EHIP;
    *ns_per_hop_out = (double)h_out[0] * 1e6 / (double)khz / (double)hops;
    return GPUVM_OK;
}

int gpuvm_bench_gather_plain(const uint32_t *d_data, const uint32_t *d_idx, size_t n, uint32_t *d_out, void *stream) {
    if (!d_data || !d_idx || !d_out) return GPUVM_EINVAL;
    if (n == 0) return GPUVM_OK;
    const int grid = (int)std::min<size_t>((n + kBlock - 1) / kBlock, 256 * 32);
    k_bench_gather_plain<<<grid, kBlock, 0, (hipStream_t)stream>>>(d_data, d_idx, n, d_out);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

}  // extern "C"

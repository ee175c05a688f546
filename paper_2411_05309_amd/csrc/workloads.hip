// libgpuvm - kernels and launchers of the array workloads: random gather, scatter-increment, vector addition, streaming reduce, embedding bag, column-order product, filter-then-gather.
// The fault path itself (page-table lookup, wavefront dedup, frame allocation,
// eviction, write-back, migration) is in include/gpuvm_device.h and is inlined
// into every kernel, the way the paper inlines its runtime into the application
// kernels (System Overview; Register usage).
#include "gpuvm_internal.h"

#include <atomic>

using namespace gpuvm_detail;

// Random gather.  A wave takes a contiguous run of the index array, 64 indices
// per step, and reads through a cursor: when all of a step's indices fall on the
// page the wave already stands on (a sorted or unit-stride index array) the read
// needs no look at the page table; otherwise - the random case - every lane
// goes through gpuvm_load on its own.
// PER_LANE = 1: one access per lane per step - the form for a pool smaller than
// the data set: a wave that collects four times as many misses per step finds
// fewer of them resident by the time it reaches them (10 % more faults on the
// 4x oversubscribed gather).  PER_LANE = 4 is for a pool that holds every page,
// where nothing is ever evicted and the run is hits after the first touch: four
// reads in flight per lane (four cursor reads when every 64-lane group of the
// step stays on one page, one batched optimistic read otherwise).
template <int PER_LANE>
__global__ __launch_bounds__(kBlock) void k_gather(gpuvm_dev_t vm, const uint32_t *__restrict__ idx, size_t n,
                                                    uint32_t *__restrict__ out, unsigned long long *sum,
                                                    unsigned long long n_elems) {
    const unsigned int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const size_t nwaves = ((size_t)gridDim.x * kBlock) >> 6;
    const size_t step = 64 * PER_LANE;
    const size_t per_wave = ((n + nwaves - 1) / nwaves + step - 1) / step * step;   // whole steps
    const size_t lo = wave * per_wave, hi = lo + per_wave < n ? lo + per_wave : n;
    unsigned long long acc = 0;
    if constexpr (PER_LANE == 1) {
        // the waves take runs of 256 indices from a shared counter (hand[2], zero at
        // launch): how many of a wave's indices miss is a matter of chance, and with
        // fixed shares the waves that drew the most misses finish alone, the link idle
        gpuvm_cursor_t cur = gpuvm_cursor_begin();
        constexpr size_t kRun = 256;
        for (;;) {
            unsigned int r = 0;
            if (lane == 0) r = (unsigned int)__hip_atomic_fetch_add(vm.hand + 2, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const size_t run_lo = (size_t)bcast(r) * kRun;
            if (run_lo >= n) break;
            const size_t run_hi = run_lo + kRun < n ? run_lo + kRun : n;
            for (size_t k0 = run_lo; k0 < run_hi; k0 += 64) {
                const size_t k = k0 + lane;
                unsigned long long i = k < run_hi ? idx[k] : 0;
                bool want = k < run_hi;
                if (want && i >= n_elems) { raise_error(vm, GPUVM_ERANGE); want = false; }
                const uint32_t v = gpuvm_cursor_load<uint32_t>(vm, cur, i, want);
                if (want) { out[k] = v; acc += v; }
            }
        }
        gpuvm_cursor_end(vm, cur);
    } else {
        gpuvm_cursor_t cur = gpuvm_cursor_begin();
        uint32_t ahead[PER_LANE];                                // the next step's indices, loaded a step early
#pragma unroll
        for (int j = 0; j < PER_LANE; ++j) ahead[j] = lo + j * 64 + lane < hi ? idx[lo + j * 64 + lane] : 0u;
        for (size_t k0 = lo; k0 < hi; k0 += step) {
            unsigned long long i[PER_LANE];
            bool want[PER_LANE], stay = cur.page != GPUVM_NO_PAGE;
#pragma unroll
            for (int j = 0; j < PER_LANE; ++j) {
                const size_t k = k0 + j * 64 + lane;
                want[j] = k < hi;
                i[j] = ahead[j];
                ahead[j] = k + step < hi ? idx[k + step] : 0u;
                if (want[j] && i[j] >= n_elems) { raise_error(vm, GPUVM_ERANGE); want[j] = false; }
                stay = stay && !(want[j] && (unsigned int)((i[j] * 4) >> vm.page_shift) != cur.page);
            }
            if (__builtin_amdgcn_ballot_w64(!stay) == 0) {
                // the whole step stays on the page the wave stands on: PER_LANE loads in flight, nothing else
                uint32_t v[PER_LANE];
#pragma unroll
                for (int j = 0; j < PER_LANE; ++j)
                    v[j] = want[j] ? __hip_atomic_load(reinterpret_cast<const uint32_t *>(cur.frame + ((i[j] * 4) & ((1ull << vm.page_shift) - 1))),
                                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
#pragma unroll
                for (int j = 0; j < PER_LANE; ++j)
                    if (want[j]) { out[k0 + j * 64 + lane] = v[j]; acc += v[j]; }
            } else {
                // one group of 64 after the other through the cursor (one copy of the general path)
#pragma nounroll
                for (int j = 0; j < PER_LANE; ++j) {
                    const unsigned long long ij = j == 0 ? i[0] : j == 1 ? i[1] : j == 2 ? i[2] : i[PER_LANE - 1];
                    const bool wj = j == 0 ? want[0] : j == 1 ? want[1] : j == 2 ? want[2] : want[PER_LANE - 1];
                    const uint32_t v = gpuvm_cursor_load<uint32_t>(vm, cur, ij, wj);
                    if (wj) { out[k0 + j * 64 + lane] = v; acc += v; }
                }
            }
        }
        gpuvm_cursor_end(vm, cur);
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

// The accessors under divergence, as in thread-per-element code with a
// condition around the access (the style of the paper's listing): only the
// lanes whose mask byte is set enter gpuvm_load / gpuvm_atomic_add, so lookups,
// faults and page copies run with whatever lanes happen to be active - down to
// one - and the last wave of the grid is a partial one.
__global__ __launch_bounds__(kBlock) void k_gather_masked(gpuvm_dev_t vm, const uint32_t *__restrict__ idx,
                                                           const unsigned char *__restrict__ mask, size_t n,
                                                           uint32_t *__restrict__ out, unsigned long long n_elems) {
    const size_t nthreads = (size_t)gridDim.x * kBlock;
    for (size_t k = (size_t)blockIdx.x * kBlock + threadIdx.x; k < n; k += nthreads) {
        if (!mask[k]) continue;
        const unsigned long long i = idx[k];
        if (i >= n_elems) { raise_error(vm, GPUVM_ERANGE); continue; }
        out[k] = gpuvm_load<uint32_t>(vm, i);
    }
}
__global__ __launch_bounds__(kBlock) void k_scatter_inc_masked(gpuvm_dev_t vm, const uint32_t *__restrict__ idx,
                                                                const unsigned char *__restrict__ mask, size_t n,
                                                                unsigned long long n_elems) {
    const size_t nthreads = (size_t)gridDim.x * kBlock;
    for (size_t k = (size_t)blockIdx.x * kBlock + threadIdx.x; k < n; k += nthreads) {
        if (!mask[k]) continue;
        const unsigned long long i = idx[k];
        if (i >= n_elems) { raise_error(vm, GPUVM_ERANGE); continue; }
        gpuvm_atomic_add<unsigned long long>(vm, i, 1ull);
    }
}

// The paper's own example (vector-addition listing): C[i] = A[i] + B[i] with all
// three vectors paged; C is written through gpuvm_store, so its pages become
// DIRTY and are written back at eviction or flush.
// Work distribution: a wave takes one page-sized stripe of the index range at a
// time (consecutive stripes to consecutive waves), so that the waves in flight
// fault on different pages; with a plain grid-stride loop all of them would
// stand on the same handful of pages and wait for one fetch at a time.
template <bool OVERWRITE>
__global__ __launch_bounds__(kBlock) void k_vector_add(gpuvm_dev_t a, gpuvm_dev_t b, gpuvm_dev_t c, size_t n) {
    const unsigned int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const size_t nwaves = ((size_t)gridDim.x * kBlock) >> 6;
    const size_t stripe = (size_t)1 << (c.page_shift - 2);               // floats per page of C
    // the wave walks its stripe with a cursor per vector: the page it stands on stays
    // pinned from one step to the next, so a step is three compares, two loads and a store
    gpuvm_cursor_t ca = gpuvm_cursor_begin(), cb = gpuvm_cursor_begin(), cc = gpuvm_cursor_begin();
    for (size_t lo = wave * stripe; lo < n; lo += nwaves * stripe) {
        const size_t hi = lo + stripe < n ? lo + stripe : n;
        // OVERWRITE: the stripe is exactly one page of C and the wave stores all
        // of it (the launcher admits only an n that ends on a page boundary or
        // where C ends), so the page needs no fetch.  The pin on C's page is
        // held across faults on A and B, which draw on pools of their own.
        const unsigned int page_c = (unsigned int)(lo >> (c.page_shift - 2));
        char *fc = OVERWRITE ? gpuvm_acquire_overwrite(c, page_c) : nullptr;
        for (size_t i0 = lo; i0 < hi; i0 += 64) {
            const size_t i = i0 + lane;
            const bool want = i < hi;
            const float x = gpuvm_cursor_load<float>(a, ca, want ? i : 0, want);
            const float y = gpuvm_cursor_load<float>(b, cb, want ? i : 0, want);
            if (OVERWRITE) {
                if (want) gpuvm_frame_store_b32(c, fc, (unsigned int)(i - lo) * 4u, __float_as_uint(x + y));
            } else {
                gpuvm_cursor_store<float>(c, cc, want ? i : 0, x + y, want);         // the listing's c[i] = a[i] + b[i]
            }
        }
        if (OVERWRITE) gpuvm_release(c, page_c);
    }
    gpuvm_cursor_end(a, ca);
    gpuvm_cursor_end(b, cb);
    if (!OVERWRITE) gpuvm_cursor_end(c, cc);
}

// Fault-ahead of a page range: wave w touches pages first + w, first + w + nwaves, ...
__global__ __launch_bounds__(kBlock) void k_prefetch(gpuvm_dev_t vm, unsigned int first, unsigned int count) {
    const unsigned int wave = (blockIdx.x * kBlock + threadIdx.x) >> 6;
    const unsigned int nwaves = (gridDim.x * kBlock) >> 6;
    for (unsigned int j = wave; j < count; j += nwaves) gpuvm_touch(vm, first + j);
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
        const char *p = gpuvm_acquire_cold(vm, page, false);     // a scan: the page is rarely there already
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

// Embedding bag, sum pooling: one wave per bag; a row of 64*VPL floats is read
// as VPL consecutive floats per lane; rows are added in listed order in fp32.
// DIRECT = true is the zero-copy baseline: the rows are read in place in pinned
// host memory (system-scope loads), no page table, no frames.
template <int VPL, bool DIRECT = false>
__global__ __launch_bounds__(kBlock) void k_embedding_bag(gpuvm_dev_t vm, const int32_t *__restrict__ ids,
                                                           size_t bags, unsigned int bag_len, float *__restrict__ out,
                                                           unsigned long long n_rows) {
    typedef float vec_t __attribute__((ext_vector_type(VPL)));
    const unsigned int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const size_t nwaves = ((size_t)gridDim.x * kBlock) >> 6;
    const unsigned int row_bytes = 64u * VPL * 4u;
    constexpr int kRowBatch = 4;
    typedef std::integral_constant<bool, DIRECT> from_frame_t;       // frames, unless the whole kernel reads in place
    typedef std::integral_constant<bool, true> from_host_t;
    auto load_row = [&](const char *p, unsigned int o, auto in_host) {
        vec_t r4;
        constexpr int aux = decltype(in_host)::value ? GPUVM_AUX_SYSTEM : GPUVM_AUX_AGENT;
        const __amdgpu_buffer_rsrc_t rsrc = make_rsrc(p, 1u << vm.page_shift);
        if constexpr (VPL == 1) {
            r4 = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, o, 0, aux));
        } else if constexpr (VPL == 2) {
            const u32x2 r = __builtin_amdgcn_raw_buffer_load_b64(rsrc, o, 0, aux);
            r4.x = __uint_as_float(r.x); r4.y = __uint_as_float(r.y);
        } else {
            const u32x4 r = __builtin_amdgcn_raw_buffer_load_b128(rsrc, o, 0, aux);
            r4.x = __uint_as_float(r.x); r4.y = __uint_as_float(r.y);
            r4.z = __uint_as_float(r.z); r4.w = __uint_as_float(r.w);
        }
        return r4;
    };
    for (size_t bag = wave; bag < bags; bag += nwaves) {
        vec_t acc = 0.0f;
        for (unsigned int j0 = 0; j0 < bag_len; j0 += 64) {
            const unsigned int nj = min(64u, bag_len - j0);
            int my_id = 0;
            if (lane < nj) my_id = ids[bag * bag_len + j0 + lane];
            // kRowBatch rows at a time: their table words, their row reads and
            // their re-checks are in flight together; hot rows are read without
            // a reference, a miss (or a page that left meanwhile) goes through
            // the pinned path; the rows are added in listed order either way
            for (unsigned int j0b = 0; j0b < nj; j0b += kRowBatch) {
                unsigned int page[kRowBatch], o[kRowBatch];
                unsigned long long token[kRowBatch], again[kRowBatch];
                const char *p[kRowBatch];
                vec_t v[kRowBatch];
                bool live[kRowBatch];
#pragma unroll
                for (int b = 0; b < kRowBatch; ++b) {
                    const unsigned int j = j0b + b;
                    const unsigned long long id = (unsigned int)__builtin_amdgcn_readlane(my_id, j < nj ? j : 0);
                    live[b] = j < nj && id < n_rows;
                    if (j < nj && id >= n_rows && lane == 0) raise_error(vm, GPUVM_ERANGE);
                    const unsigned long long byte = (live[b] ? id : 0ull) * row_bytes;
                    page[b] = (unsigned int)(byte >> vm.page_shift);
                    o[b] = (unsigned int)(byte & ((1ull << vm.page_shift) - 1)) + lane * (VPL * 4u);
                    token[b] = DIRECT ? 0ull : gpuvm_peek_begin(vm, page[b]);
                }
                if constexpr (DIRECT) {
#pragma unroll
                    for (int b = 0; b < kRowBatch; ++b) {
                        v[b] = 0.0f;
                        if (live[b]) v[b] = load_row(vm.host + ((size_t)page[b] << vm.page_shift), o[b], from_host_t{});
                    }
#pragma unroll
                    for (int b = 0; b < kRowBatch; ++b)
                        if (live[b]) acc += v[b];
                    continue;
                }
#pragma unroll
                for (int b = 0; b < kRowBatch; ++b) {
                    p[b] = live[b] ? gpuvm_token_frame(vm, token[b]) : nullptr;
                    v[b] = 0.0f;
                    if (p[b]) v[b] = load_row(p[b], o[b], from_frame_t{});
                }
                gpuvm_wait_reads();
#pragma unroll
                for (int b = 0; b < kRowBatch; ++b) again[b] = gpuvm_peek_begin(vm, page[b]);
#pragma unroll
                for (int b = 0; b < kRowBatch; ++b) {
                    if (!live[b]) continue;
                    if (!(p[b] && gpuvm_peek_same(vm, page[b], token[b], again[b]))) {
                        // remote-first: a page that has not earned its migration yet
                        // gives up its row in place, 512 bytes over the link
                        unsigned int in_place = 0;
                        if ((vm.flags >> GPUVM_F_REMOTE_SHIFT) && lane == 0) in_place = touch_in_place(vm, page[b]) ? 1u : 0u;
                        if (__builtin_amdgcn_readfirstlane(in_place)) {
                            v[b] = load_row(vm.host + ((size_t)page[b] << vm.page_shift), o[b], from_host_t{});
                            gpuvm_wait_reads();
                        } else {
                            const char *q = gpuvm_acquire_hinted(vm, page[b], false, again[b]);
                            v[b] = load_row(q, o[b], from_frame_t{});
                            gpuvm_release(vm, page[b]);
                        }
                    }
                    acc += v[b];
                }
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
//
// Every page is wanted by all the waves whose columns lie in it, each at the
// moment it reaches that row.  Two things keep this from degenerating:
//  - fault-ahead helpers (the first `helper_blocks` workgroups) touch the pages
//    of the rows to come (acquire, release) in parallel, so that the compute
//    waves find them resident instead of fetching them one after the other;
//  - a sliding window: every compute wave publishes the row it has reached in
//    progress[wave]; nobody - helper or compute wave - goes further than
//    `window` rows beyond the slowest compute wave.  Without it a wave that
//    falls behind by more than the pool holds finds its pages evicted, has to
//    fetch every one itself and falls further behind (measured: 2-3x the
//    traffic, 8x the time).  The slowest wave is never held back, so the
//    window always moves; waiting is bounded by spin_limit all the same.
constexpr unsigned int kRowProgressLen = 8192;        // progress words of a handle's own array

// Scratch of gpuvm_run_matvec_t_noalloc: the row each compute wave has reached,
// one word per wave, in place of the array the allocating entry point keeps per
// handle.  One copy per GPU, held until the process ends; every call on a GPU
// shares it, so calls that overlap on one GPU race.
constexpr unsigned int kNoAllocWaves = GPUVM_NOALLOC_MAX_COLS / 64;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned int scratch[kNoAllocWaves];
static std::atomic<unsigned int *> scratch_of_device[kMaxDevices];

__device__ __forceinline__ unsigned int slowest_row(const unsigned int *progress, unsigned int n_compute_waves) {
    unsigned int lo = 0xFFFFFFFFu;
    for (unsigned int i = threadIdx.x & 63; i < n_compute_waves; i += 64) lo = min(lo, a_load(progress + i));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) lo = min(lo, (unsigned int)__shfl_xor((int)lo, off, 64));
    return lo;
}

__global__ __launch_bounds__(kBlock) void k_matvec_t(gpuvm_dev_t vm, unsigned long long rows, unsigned long long cols,
                                                      unsigned int skew, unsigned int helper_blocks,
                                                      unsigned int window, unsigned int *progress,
                                                      const float *__restrict__ x, double *__restrict__ y) {
    const unsigned int lane = threadIdx.x & 63;
    // compute waves that own a block of 64 columns; the grid is rounded up to whole
    // workgroups, and a wave without columns never publishes a row: it must not
    // count as the slowest one
    const unsigned int n_compute_waves =
        (unsigned int)min((unsigned long long)(((gridDim.x - helper_blocks) * kBlock) >> 6), (cols + 63) >> 6);
    if (blockIdx.x < helper_blocks) {
        const unsigned int hw = (blockIdx.x * kBlock + threadIdx.x) >> 6;
        const unsigned int nh = (helper_blocks * kBlock) >> 6;
        const unsigned long long row_bytes = cols * 4;
        unsigned int at = 0;
        for (unsigned int page = hw; page < vm.n_pages; page += nh) {
            const unsigned long long row = ((unsigned long long)page << vm.page_shift) / row_bytes;
            for (unsigned int polls = 0; row > (unsigned long long)at + window && polls < vm.spin_limit; ++polls) {
                at = slowest_row(progress, n_compute_waves);
                if (row <= (unsigned long long)at + window || ((polls & 255) == 255 && aborted(vm))) break;
                __builtin_amdgcn_s_sleep(32);
            }
            if (row + skew < at) continue;                    // every compute wave is already past it
            gpuvm_touch(vm, page);
        }
        return;
    }
    const unsigned int cwave = ((blockIdx.x - helper_blocks) * kBlock + threadIdx.x) >> 6;
    const size_t nthreads = (size_t)(gridDim.x - helper_blocks) * kBlock;
    const unsigned long long cols_up = (cols + 63) & ~63ull;           // whole waves stay together
    for (unsigned long long j = (size_t)(blockIdx.x - helper_blocks) * kBlock + threadIdx.x; j < cols_up; j += nthreads) {
        double acc = 0.0;
        const bool want = j < cols;
        // a small spread of the start rows keeps the compute waves from hitting
        // one page word all at the same instant
        const unsigned long long r0 = (j >> 6) % skew;
        unsigned int slowest = 0;
        for (unsigned long long k = 0; k < rows; ++k) {
            const unsigned long long i = k + r0 < rows ? k + r0 : k + r0 - rows;
            if (window && (k & 15) == 0) {
                if (lane == 0) a_store(progress + cwave, (unsigned int)k);
                for (unsigned int polls = 0; k > (unsigned long long)slowest + window / 2 && polls < vm.spin_limit; ++polls) {
                    slowest = slowest_row(progress, n_compute_waves);
                    if (k <= (unsigned long long)slowest + window / 2 || ((polls & 255) == 255 && aborted(vm))) break;
                    __builtin_amdgcn_s_sleep(32);
                }
            }
            acc += (double)gpuvm_load_if<float>(vm, want ? i * cols + j : 0, want) * (double)x[i];
        }
        if (want) y[j] = acc;
        if (window && lane == 0) a_store(progress + cwave, 0xFFFFFFF0u);   // done: never the slowest again
    }
}

// Matrix-vector product y = A x over a paged row-major fp32 matrix, a thread
// per ROW (the first product of the paper's MVT / the first step of its ATAX):
// the 64 lanes of a wave stand on 64 different rows, i.e. on 64 different
// pages, and each walks along its own row, 64 (or 16) bytes per access.
// A page is used by one lane only, for page_bytes / 16 consecutive steps, and
// all lanes reach their next page at the same step.  Reads go through the
// element accessor: 64 optimistic hits per step, and at a page boundary 64
// faults per wave, one after the other.  The launcher keeps the rows in flight
// (one page each) below the pool size; beyond that every step would fault.
// fp64 accumulation, columns ascending.
template <int FLOATS> struct f32_chunk_t { float v[FLOATS]; };
template <int FLOATS>     // floats per access: 64 or 16 (256 or 64 bytes in flight per lane and step), or 4
__global__ __launch_bounds__(kBlock) void k_matvec_rows(gpuvm_dev_t vm, unsigned long long rows, unsigned long long cols,
                                                         const float *__restrict__ x, double *__restrict__ y) {
    typedef f32_chunk_t<FLOATS> chunk_t;
    const size_t nthreads = (size_t)gridDim.x * kBlock;
    const unsigned long long rows_up = (rows + 63) & ~63ull;      // whole waves iterate together
    for (unsigned long long r = (size_t)blockIdx.x * kBlock + threadIdx.x; r < rows_up; r += nthreads) {
        const bool want = r < rows;
        double acc = 0.0;
        for (unsigned long long j = 0; j < cols; j += FLOATS) {
            unsigned long long w[FLOATS / 2] = {};
            gpuvm_access<chunk_t>(vm, want ? (r * cols + j) / FLOATS : 0, false, want, [&](chunk_t *p) {
                unsigned long long *q = reinterpret_cast<unsigned long long *>(p);
#pragma unroll
                for (int k = 0; k < FLOATS / 2; ++k)
                    w[k] = __hip_atomic_load(q + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            });
#pragma unroll
            for (int k = 0; k < FLOATS / 2; ++k) {
                acc += (double)__uint_as_float((unsigned int)w[k]) * (double)x[j + 2 * k];
                acc += (double)__uint_as_float((unsigned int)(w[k] >> 32)) * (double)x[j + 2 * k + 1];
            }
        }
        if (want) y[r] = acc;
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
        const char *p = gpuvm_acquire_cold(vmk, page, false);
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

extern "C" {

int gpuvm_run_gather(gpuvm_t *vm, const uint32_t *d_idx, size_t n, uint32_t *d_out, uint64_t *d_sum,
                     void *stream) {
    if (!vm || (n && (!d_idx || !d_out))) return GPUVM_EINVAL;
    if (n == 0) return GPUVM_OK;
    // every page fits, so nothing is ever evicted and the run is hits after the first
    // touch: four reads in flight per lane, and as many waves as the device holds
    // (hits are bound by latency, not by the link) unless the caller chose a count
    const bool all_fit = vm->dev.n_frames >= vm->dev.n_pages;
    int waves = launch_waves(vm, (n + 63) / 64);
    if (all_fit && !vm->waves_chosen) {
        long long cap = (long long)vm->cus * 32;                  // (no bound by the frames: nothing is ever evicted)
        const long long need = (long long)((n + 255) / 256 + kWavesPerBlock - 1) / kWavesPerBlock * kWavesPerBlock;
        waves = (int)std::max<long long>(std::min(cap, need), std::min<long long>(waves, kWavesPerBlock));
    }
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    if (all_fit && n >= (size_t)waves * 256)
        k_gather<4><<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm->dev, d_idx, n, d_out,
                                                                                (unsigned long long *)d_sum, vm->dev.bytes / 4);
    else {
        k_fill64<<<1, 64, 0, (hipStream_t)stream>>>(vm->dev.hand + 2, 1, 0ull);     // the runs' counter (a fill kernel: capturable)
        k_gather<1><<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm->dev, d_idx, n, d_out,
                                                                                (unsigned long long *)d_sum, vm->dev.bytes / 4);
    }
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_run_gather_masked(gpuvm_t *vm, const uint32_t *d_idx, const uint8_t *d_mask, size_t n, uint32_t *d_out,
                            void *stream) {
    if (!vm || (n && (!d_idx || !d_mask || !d_out))) return GPUVM_EINVAL;
    if (n == 0) return GPUVM_OK;
    const int waves = launch_waves(vm, (n + 63) / 64);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    k_gather_masked<<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm->dev, d_idx, d_mask, n, d_out,
                                                                                vm->dev.bytes / 4);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_run_scatter_increment_masked(gpuvm_t *vm, const uint32_t *d_idx, const uint8_t *d_mask, size_t n,
                                       void *stream) {
    if (!vm || (n && (!d_idx || !d_mask))) return GPUVM_EINVAL;
    if (n == 0) return GPUVM_OK;
    const int waves = launch_waves_duplex(vm, (n + 63) / 64);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    k_scatter_inc_masked<<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(dev_for_writers(vm, waves), d_idx, d_mask, n,
                                                                                     vm->dev.bytes / 8);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_run_scatter_increment(gpuvm_t *vm, const uint32_t *d_idx, size_t n, void *stream) {
    if (!vm || (n && !d_idx)) return GPUVM_EINVAL;
    if (n == 0) return GPUVM_OK;
    const int waves = launch_waves_duplex(vm, (n + 63) / 64);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    k_scatter_inc<<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(dev_for_writers(vm, waves), d_idx, n, vm->dev.bytes / 8);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

static int run_vector_add(gpuvm_t *vm_a, gpuvm_t *vm_b, gpuvm_t *vm_c, size_t n, bool overwrite, void *stream) {
    if (!vm_a || !vm_b || !vm_c || vm_a == vm_c || vm_b == vm_c) return GPUVM_EINVAL;
    if (n * 4 > vm_a->dev.bytes || n * 4 > vm_b->dev.bytes || n * 4 > vm_c->dev.bytes) return GPUVM_ERANGE;
    // without a fetch the last page touched must be stored completely: n ends
    // on a page boundary of C or where C itself ends
    if (overwrite && (n * 4) % vm_c->page_bytes != 0 && n * 4 != vm_c->dev.bytes) return GPUVM_EINVAL;
    if (n == 0) return GPUVM_OK;
    const size_t work = (n * 4 + vm_c->page_bytes - 1) / vm_c->page_bytes;       // page-sized stripes
    const int waves = std::min({launch_waves(vm_a, work), launch_waves(vm_b, work), launch_waves(vm_c, work)});
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    if (overwrite)
        k_vector_add<true><<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm_a->dev, vm_b->dev, dev_for_writers(vm_c, waves), n);
    else
        k_vector_add<false><<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm_a->dev, vm_b->dev, dev_for_writers(vm_c, waves), n);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_run_vector_add(gpuvm_t *vm_a, gpuvm_t *vm_b, gpuvm_t *vm_c, size_t n, void *stream) {
    return run_vector_add(vm_a, vm_b, vm_c, n, false, stream);
}

int gpuvm_run_vector_add_overwrite(gpuvm_t *vm_a, gpuvm_t *vm_b, gpuvm_t *vm_c, size_t n, void *stream) {
    return run_vector_add(vm_a, vm_b, vm_c, n, true, stream);
}

int gpuvm_run_prefetch(gpuvm_t *vm, size_t first_page, size_t n_pages, void *stream) {
    if (!vm) return GPUVM_EINVAL;
    if (first_page > vm->dev.n_pages || n_pages > vm->dev.n_pages - first_page) return GPUVM_ERANGE;
    if (n_pages == 0) return GPUVM_OK;
    const int waves = launch_waves_streaming(vm, n_pages);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    k_prefetch<<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm->dev, (unsigned int)first_page,
                                                                           (unsigned int)n_pages);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_run_stream_reduce(gpuvm_t *vm, size_t block_elems, double *d_sums, void *stream) {
    if (!vm || !d_sums || block_elems == 0) return GPUVM_EINVAL;
    const size_t block_bytes = block_elems * 4;
    if (block_bytes % vm->page_bytes || vm->dev.bytes % 4) return GPUVM_EINVAL;
    const unsigned int ppb = (unsigned int)(block_bytes / vm->page_bytes);
    const size_t nblocks = (vm->dev.n_pages + ppb - 1) / ppb;
    const int waves = launch_waves_streaming(vm, vm->dev.n_pages);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    hipStream_t s = (hipStream_t)stream;
    k_fill64<<<64, 256, 0, s>>>((unsigned long long *)d_sums, nblocks, 0ull);   // +0.0
    k_stream_reduce<<<grid_for_waves(waves), kBlock, 0, s>>>(vm->dev, ppb, d_sums);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

static int run_embedding_bag(gpuvm_t *vm, size_t dim, const int32_t *d_ids, size_t bags, size_t bag_len,
                             float *d_out, void *stream, bool direct) {
    if (!vm || !d_ids || !d_out || bag_len == 0 || bag_len > 0xFFFFFFFFu) return GPUVM_EINVAL;
    if (dim != 64 && dim != 128 && dim != 256) return GPUVM_EINVAL;
    const size_t row_bytes = dim * 4;
    if (vm->page_bytes % row_bytes || vm->dev.bytes % row_bytes) return GPUVM_EINVAL;
    if (bags == 0) return GPUVM_OK;
    // the zero-copy baseline holds no frames: its waves are bounded by the device only
    const int waves = direct ? vm->cus * vm->waves_per_cu : launch_waves_streaming(vm, bags);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    const int grid = grid_for_waves(waves);
    hipStream_t s = (hipStream_t)stream;
    const unsigned long long n_rows = vm->dev.bytes / row_bytes;
    const unsigned int len = (unsigned int)bag_len;
    if (direct) {
        if (dim == 64) k_embedding_bag<1, true><<<grid, kBlock, 0, s>>>(vm->dev, d_ids, bags, len, d_out, n_rows);
        else if (dim == 128) k_embedding_bag<2, true><<<grid, kBlock, 0, s>>>(vm->dev, d_ids, bags, len, d_out, n_rows);
        else k_embedding_bag<4, true><<<grid, kBlock, 0, s>>>(vm->dev, d_ids, bags, len, d_out, n_rows);
    } else {
        if (dim == 64) k_embedding_bag<1><<<grid, kBlock, 0, s>>>(vm->dev, d_ids, bags, len, d_out, n_rows);
        else if (dim == 128) k_embedding_bag<2><<<grid, kBlock, 0, s>>>(vm->dev, d_ids, bags, len, d_out, n_rows);
        else k_embedding_bag<4><<<grid, kBlock, 0, s>>>(vm->dev, d_ids, bags, len, d_out, n_rows);
    }
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_run_embedding_bag(gpuvm_t *vm, size_t dim, const int32_t *d_ids, size_t bags, size_t bag_len,
                            float *d_out, void *stream) {
    return run_embedding_bag(vm, dim, d_ids, bags, bag_len, d_out, stream, false);
}

int gpuvm_bench_embedding_bag_zero_copy(gpuvm_t *vm, size_t dim, const int32_t *d_ids, size_t bags, size_t bag_len,
                                        float *d_out, void *stream) {
    return run_embedding_bag(vm, dim, d_ids, bags, bag_len, d_out, stream, true);
}

// progress == nullptr: the array of the handle, allocated on first use
static int run_matvec_t(gpuvm_t *vm, size_t rows, size_t cols, const float *d_x, double *d_y, void *stream,
                        unsigned int *progress, unsigned int progress_len) {
    if (!vm || !d_x || !d_y || rows == 0 || cols == 0) return GPUVM_EINVAL;
    if (rows * cols * 4 != vm->dev.bytes) return GPUVM_EINVAL;
    if (rows >= 0xFFFFFFF0ull) return GPUVM_EINVAL;
    const int cap = launch_waves(vm, (size_t)1 << 40);
    const int waves = launch_waves(vm, (cols + 63) / 64);
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    // rows of A the pool can hold; start rows, the helpers' lead and the spread of
    // the compute waves all stay well inside it
    const size_t rows_in_pool = (size_t)vm->dev.n_frames * vm->page_bytes / (cols * 4);
    const unsigned int skew = (unsigned int)std::max<size_t>(1, std::min<size_t>({(size_t)64, rows_in_pool / 4, rows}));
    // one pass over the rows per wave is what the window reasons about
    const bool single_pass = (size_t)waves * 64 >= cols;
    // Under the two-handed CLOCK a page keeps the reference bit it is installed with for the part of
    // the ring the front hand has not covered yet, (8 - e) / 8 of it; a page that is
    // still being used after that is marked again and outlives its turn by a whole
    // lap, dead weight that the rows in flight then lack.  So every use of a page -
    // from the helper that brings it in to the slowest wave, window + window / 2 rows
    // later - has to fall inside that part: window = 2/3 of it, rounded down to a
    // quarter of the pool for the default half-ring spread.  One hand, FIFO and the
    // generalized CLOCK keep half the pool.
    const unsigned int eighths = (vm->dev.flags >> GPUVM_F_HANDS_SHIFT) & GPUVM_F_HANDS_MASK;
    const bool two_hands = eighths && (vm->dev.policy == GPUVM_POLICY_CLOCK || vm->dev.policy == GPUVM_POLICY_CLOCK_WRITE_AWARE);
    // ... and no further ahead than 64 MiB of rows: the link is full with a few MiB in
    // flight, and a longer lead only spreads the compute waves over more pages at a
    // time (a pool that holds everything: 28.1 -> 22.6 ms on 16384 x 16384, 86.6 ->
    // 75.6 ms on 32768 x 32768; a quarter of that: 77.8 -> 76.7 ms; 16 MiB is too
    // short for two-page rows, 81.7 ms)
    const size_t lead = std::min<size_t>(two_hands ? rows_in_pool * (8 - eighths) / 16 : rows_in_pool / 2,
                                         std::max<size_t>(16, ((size_t)64 << 20) / (cols * 4)));
    const unsigned int window = single_pass && rows_in_pool >= 16 ? (unsigned int)std::min<size_t>(std::max<size_t>(lead, 4), 0x7FFFFFFF) : 0;
    // fault-ahead helpers: what is left of the wave budget, at most two per compute unit
    const int helpers = window ? std::min(cap - waves, vm->cus * 2) / kWavesPerBlock * kWavesPerBlock : 0;
    hipStream_t s = (hipStream_t)stream;
    if (!progress) {
        if (!vm->row_progress) HIP_TRY(hipMalloc(&vm->row_progress, kRowProgressLen * sizeof(unsigned int)));
        progress = vm->row_progress;
        progress_len = kRowProgressLen;
    }
    if ((unsigned int)waves > progress_len) return GPUVM_EINVAL;      // one word per compute wave
    k_fill32<<<8, 256, 0, s>>>(progress, progress_len, 0u);            // a fill kernel, not a memset: capturable
    k_matvec_t<<<grid_for_waves(waves) + helpers / kWavesPerBlock, kBlock, 0, s>>>(
        vm->dev, rows, cols, skew, (unsigned int)(helpers / kWavesPerBlock), window, progress, d_x, d_y);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

int gpuvm_run_matvec_t(gpuvm_t *vm, size_t rows, size_t cols, const float *d_x, double *d_y, void *stream) {
    return run_matvec_t(vm, rows, cols, d_x, d_y, stream, nullptr, 0);
}

int gpuvm_run_matvec_t_noalloc(gpuvm_t *vm, size_t rows, size_t cols, const float *d_x, double *d_y, void *stream) {
    if (!vm) return GPUVM_EINVAL;
    if (cols > (size_t)GPUVM_NOALLOC_MAX_COLS) {
        fprintf(stderr, "libgpuvm: gpuvm_run_matvec_t_noalloc: %zu columns exceed the %d that the static scratch "
                        "array holds progress words for; use gpuvm_run_matvec_t\n", cols, GPUVM_NOALLOC_MAX_COLS);
        return GPUVM_ERANGE;
    }
    // the address of this device's copy of the array, looked up once per device
    // with that device current (the array's name is no device address in host code)
    int device = -1;
    HIP_TRY(hipGetDevice(&device));
    if (device != vm->device || device < 0 || device >= kMaxDevices) return GPUVM_EINVAL;
    unsigned int *p = scratch_of_device[device].load(std::memory_order_acquire);
    if (!p) {
        HIP_TRY(hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)));
        if (!p) return GPUVM_EHIP;
        scratch_of_device[device].store(p, std::memory_order_release);
    }
    return run_matvec_t(vm, rows, cols, d_x, d_y, stream, p, kNoAllocWaves);
}

int gpuvm_run_matvec(gpuvm_t *vm, size_t rows, size_t cols, const float *d_x, double *d_y, void *stream) {
    if (!vm || !d_x || !d_y || rows == 0 || cols == 0 || cols % 4) return GPUVM_EINVAL;
    if (rows * cols * 4 != vm->dev.bytes) return GPUVM_EINVAL;
    // every lane in flight holds on to one page of its row: keep them within 3/4 of the pool
    const int fit = (int)std::min<size_t>(vm->dev.n_frames * 3 / 4 / 64, 1 << 20) / kWavesPerBlock * kWavesPerBlock;
    const int waves = std::min(launch_waves(vm, (rows + 63) / 64), std::max(fit, kWavesPerBlock));
    if (waves < kWavesPerBlock) return GPUVM_EDEADLK;
    // the fewer waves the pool allows, the more each optimistic read has to carry: its three
    // dependent loads are all that is in flight per lane (256 bytes per read: 46 ms instead of 78
    // on a 1 GiB matrix with a pool of a twelfth, 16 waves; no difference when the link is the bound)
    if (cols % 64 == 0 && waves < vm->cus * 2)
        k_matvec_rows<64><<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm->dev, rows, cols, d_x, d_y);
    else if (cols % 16 == 0)
        k_matvec_rows<16><<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm->dev, rows, cols, d_x, d_y);
    else
        k_matvec_rows<4><<<grid_for_waves(waves), kBlock, 0, (hipStream_t)stream>>>(vm->dev, rows, cols, d_x, d_y);
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

}  // extern "C"

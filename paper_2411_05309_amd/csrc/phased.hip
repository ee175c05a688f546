// libgpuvm - deterministic barrier-phased mode: the same accesses cut into phases whose faults one sequential agent serves in ascending page order, so that counts and the frame table equal a sequential replay.
// The fault path itself (page-table lookup, wavefront dedup, frame allocation,
// eviction, write-back, migration) is in include/gpuvm_device.h and is inlined
// into every kernel, the way the paper inlines its runtime into the application
// kernels (System Overview; Register usage).
#include "gpuvm_internal.h"

using namespace gpuvm_detail;

// (A) first toucher of each page in this phase pins it if resident, else lists it.
__global__ __launch_bounds__(kBlock) void k_phase_lookup(gpuvm_dev_t vm, const uint32_t *__restrict__ idx, size_t k,
                                                          unsigned int elem_shift, unsigned long long n_elems,
                                                          unsigned int tag, unsigned int *stamp, unsigned char *first,
                                                          unsigned int *miss, unsigned int *ctr) {
    const size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= k) return;
    first[i] = 0;
    if (aborted(vm)) return;                                          // an earlier phase failed: touch nothing more
    const unsigned long long e = idx[i];
    if (e >= n_elems) { raise_error(vm, GPUVM_ERANGE); return; }
    const unsigned int page = (unsigned int)((e << elem_shift) >> vm.page_shift);
    if (atomicExch(stamp + page, tag) == tag) return;                 // somebody else was first
    first[i] = 1;
    const unsigned long long pq = a_load(vm.pte + page);
    if (((pq & GPUVM_PTE_STATE_MASK) >> GPUVM_PTE_STATE_SHIFT) == GPUVM_ST_RESIDENT) {
        a_add(vm.pte + page, 1ull);                                   // one more user
        const unsigned long long mark = vm.policy == GPUVM_POLICY_GCLOCK ? gpuvm_use_mark(vm.policy, pq)
                                                                           : (pq & GPUVM_PTE_REF) ? 0ull : GPUVM_PTE_REF;
        if (mark) a_or(vm.pte + page, mark);                          // used: reference bit / use count
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
    if (aborted(vm)) {                                                // uniform: the error word is only ever set once
        if (threadIdx.x == 0) { ctr[0] = 0; ctr[1] = 0; ctr[2] = 0; }
        return;
    }
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
            const unsigned int g = gpuvm_front_hand(vm, f);           // two-handed CLOCK: the front hand moves with the cursor
            if (g != f && vm.frame_owner[g] != GPUVM_NO_PAGE) vm.pte[vm.frame_owner[g]] &= ~GPUVM_PTE_REF;
            const unsigned int q = vm.frame_owner[f];
            if (q == GPUVM_NO_PAGE) { st[GPUVM_S_FRESH] += 1; break; }
            const unsigned long long pq = vm.pte[q];
            if (pq & GPUVM_PTE_PIN_MASK) { st[GPUVM_S_SKIPS] += 1; continue; }
            if (gpuvm_uses_ref(vm.policy) && (pq & GPUVM_PTE_REF)) {
                vm.pte[q] = pq & ~GPUVM_PTE_REF;
                st[GPUVM_S_SWEEPS] += 1;
                continue;
            }
            if (vm.policy == GPUVM_POLICY_GCLOCK && (pq & (GPUVM_PTE_REF | GPUVM_PTE_DEFER))) {
                vm.pte[q] = pq & ~((pq & GPUVM_PTE_DEFER) ? GPUVM_PTE_DEFER : GPUVM_PTE_REF);   // use count - 1
                st[GPUVM_S_SWEEPS] += 1;
                continue;
            }
            if (vm.policy == GPUVM_POLICY_CLOCK_WRITE_AWARE && (pq & GPUVM_PTE_DIRTY) && !(pq & GPUVM_PTE_DEFER)) {
                vm.pte[q] = pq | GPUVM_PTE_DEFER;
                st[GPUVM_S_SWEEPS] += 1;
                continue;
            }
            victim = q;
            wb = (pq & GPUVM_PTE_DIRTY) ? 1u : 0u;
            if (wb) { st[GPUVM_S_WB_EVICT] += 1; st[GPUVM_S_SHORT_OUT] += page_len(vm, q) != (1u << vm.page_shift); }
            vm.pte[q] = pq & GPUVM_PTE_GEN_MASK;                      // INVALID
            break;
        }
        vm.frame_owner[f] = p;
        vm.pte[p] = (GPUVM_ST_RESIDENT << GPUVM_PTE_STATE_SHIFT) | ((unsigned long long)f << GPUVM_PTE_FRAME_SHIFT) |
                    (vm.policy == GPUVM_POLICY_GCLOCK ? 0ull : GPUVM_PTE_REF) |
                    ((vm.pte[p] + (1ull << GPUVM_PTE_GEN_SHIFT)) & GPUVM_PTE_GEN_MASK) |
                    1ull;                                             // next generation, pinned once
        st[GPUVM_S_FAULTS] += 1;
        st[GPUVM_S_SHORT_IN] += page_len(vm, p) != (1u << vm.page_shift);
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
        const unsigned int len = page_len(vm, job.page);
        if (job.writeback) {
            const unsigned int vlen = page_len(vm, job.victim);
            if ((vm.flags & GPUVM_F_OVERLAPPED_WRITEBACK) && vlen == len && (len & 15u) == 0) {
                swap_frame_with_host(frame, vm.host + ((size_t)job.victim << vm.page_shift),
                                     vm.host + ((size_t)job.page << vm.page_shift), len, w);
                continue;
            }
            copy_frame_to_host(vm.host + ((size_t)job.victim << vm.page_shift), frame, vlen, w);
            wait_vm();
        }
        copy_host_to_frame(frame, vm.host + ((size_t)job.page << vm.page_shift), len, w);
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
    // a phase that was refused (more pages than frames, or no victim found) has
    // installed nothing, or only some of its pages: its accesses are dropped
    // and no pin is given back that was never taken; the launch reports the
    // error and the handle is good again after gpuvm_reset
    const bool failed = aborted(vm);
    if (!failed && i < k && idx[i] < n_elems) {
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

namespace {

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

extern "C" {

int gpuvm_run_gather_phased(gpuvm_t *vm, const uint32_t *d_idx, size_t n, size_t phase_len, uint32_t *d_out,
                            uint64_t *d_sum, void *stream) {
    return run_phased<0>(vm, d_idx, n, phase_len, d_out, d_sum, stream);
}

int gpuvm_run_scatter_increment_phased(gpuvm_t *vm, const uint32_t *d_idx, size_t n, size_t phase_len,
                                       void *stream) {
    return run_phased<1>(vm, d_idx, n, phase_len, nullptr, nullptr, stream);
}

}  // extern "C"

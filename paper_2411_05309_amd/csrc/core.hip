// libgpuvm - life cycle of a paged view, flush / reset / counters, launch-shape helpers.
// The fault path itself (page-table lookup, wavefront dedup, frame allocation,
// eviction, write-back, migration) is in include/gpuvm_device.h and is inlined
// into every kernel, the way the paper inlines its runtime into the application
// kernels (System Overview; Register usage).
#include "gpuvm_internal.h"

using namespace gpuvm_detail;

#include <new>
#include <vector>

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
            // the write-aware policy's 'spared once' mark goes with the dirty bit; under the
            // generalized CLOCK the same bit is half of the use count and stays
            a_and(vm.pte + q, ~(GPUVM_PTE_DIRTY | (vm.policy == GPUVM_POLICY_GCLOCK ? 0ull : GPUVM_PTE_DEFER)));
            stat_add(vm, GPUVM_S_WB_FLUSH, 1);
            if (len != (1u << vm.page_shift)) stat_add(vm, GPUVM_S_SHORT_OUT, 1);
        }
    }
    wait_vm();
}

int check_kernel_error(gpuvm_t *vm) {
    unsigned long long word = 0;
    HIP_TRY(hipMemcpy(&word, vm->dev.hand + 1, sizeof(word), hipMemcpyDeviceToHost));
    return word ? -(int)word : GPUVM_OK;
}

int grid_for_waves(int waves) { return std::max(1, waves / kWavesPerBlock); }

int launch_waves(const gpuvm_t *vm, size_t work_waves) {
    // waves in flight: enough to fill the device, never more than half the
    // frames, whole workgroups; 0 if not even one workgroup may run.  A pool that
    // holds every page needs no such bound: a page faults once, into a frame that
    // was never used, and nobody ever has to find a victim.
    const bool all_fit = vm->dev.n_frames >= vm->dev.n_pages;
    long long cap = std::min<long long>((long long)vm->cus * vm->waves_per_cu, all_fit ? (1ll << 30) : vm->dev.n_frames / 2);
    cap = (cap / kWavesPerBlock) * kWavesPerBlock;
    const long long need = (long long)((std::max<size_t>(work_waves, 1) + kWavesPerBlock - 1) / kWavesPerBlock) * kWavesPerBlock;
    return (int)std::min(cap, need);
}

// For launches that are streams of page faults with little work per page (the
// streaming reduce, the embedding bag, fault-ahead) on a pool smaller than the data
// set.  The link is full with some 75 KB in flight; what is in flight beyond a few
// MiB only queues in the memory system, in front of the frame stores and the table
// atomics: the streaming configuration reaches 57.2 GB/s with 512 waves on 64 KiB
// pages (a wave has 8 KiB outstanding) against 55.5 with 2048, the embedding
// configuration 12.3 s against 12.75.  Kernels that also compute between their
// faults (the graph walks) or serve hits lane by lane (the gather) keep the full
// count.  A wave count chosen by the caller stands.
int launch_waves_streaming(const gpuvm_t *vm, size_t work_waves) {
    const int all = launch_waves(vm, work_waves);
    if (vm->waves_chosen) return all;
    if (vm->dev.n_frames >= vm->dev.n_pages) {
        // every page fits: hits after the first touch, bound by the latency of HBM and
        // of the one pin per page - 16 waves per CU read resident 64 KiB pages at 5.3 TB/s
        // (a plain read of the same bytes: 5.7), 8 at 3.5, 32 at 4.9
        const long long cap = (long long)vm->cus * 16;
        const long long need = (long long)((std::max<size_t>(work_waves, 1) + kWavesPerBlock - 1) / kWavesPerBlock) * kWavesPerBlock;
        return (int)std::min(cap, need);
    }
    const size_t per_wave = std::min<size_t>(vm->page_bytes, 8192);
    const int sweet = (int)((4u << 20) / per_wave) / kWavesPerBlock * kWavesPerBlock;
    return std::max(std::min(all, sweet), std::min(all, kWavesPerBlock));
}

// For launches whose faults write back as much as they fetch.  With both
// directions of the link busy, throughput peaks at about 4 MiB of page traffic
// in flight (512 waves on 64 KiB pages, of which a wave has 8 KiB outstanding;
// 1024 waves on 4 KiB pages) and is some 8 % lower with the 8-16 MiB that suit
// one-way traffic.  A wave count chosen by the caller stands.
int launch_waves_duplex(const gpuvm_t *vm, size_t work_waves) {
    const int all = launch_waves(vm, work_waves);
    if (vm->waves_chosen) return all;
    const size_t per_wave = std::min<size_t>(vm->page_bytes, 8192);
    const int sweet = (int)((4u << 20) / per_wave) / kWavesPerBlock * kWavesPerBlock;
    return std::max(std::min(all, sweet), std::min(all, kWavesPerBlock));
}

// Unless the caller chose an order, a launch that dirties pages with few waves in
// flight overlaps the write-back of a dirty victim with the fetch (one pass over
// the frame, both directions in flight): measured, a run is about 10 % shorter
// up to 64 waves on 4 KiB pages and 3-13 % from 32 to 256 waves on 64 KiB pages,
// and no shorter (a few per cent longer on 4 KiB pages) once the link is full,
// where the paper's order - write back, then fetch - stays.  The limit is the
// wave count at which the link fills: 64 waves, 256 from 64 KiB pages on.
gpuvm_dev_t dev_for_writers(const gpuvm_t *vm, int waves) {
    gpuvm_dev_t d = vm->dev;
    const int limit = vm->page_bytes >= 65536 ? 256 : 64;
    if (!vm->wb_chosen && waves <= limit) d.flags |= GPUVM_F_OVERLAPPED_WRITEBACK;
    return d;
}

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

// Layout of pool and tables inside one device allocation (every part on a 256-byte boundary).
namespace {
struct table_layout { size_t frames, pte, owner, hand, stats, flag, total; };
bool geometry_ok(size_t bytes, size_t page_bytes, size_t frame_pool_bytes) {
    if (bytes == 0) return false;
    if (page_bytes < 4096 || page_bytes > (1u << 20) || (page_bytes & (page_bytes - 1))) return false;
    const size_t n_frames = frame_pool_bytes / page_bytes;
    const size_t n_pages = (bytes + page_bytes - 1) / page_bytes;
    return n_frames >= 2 && n_frames < (1u << 27) && n_pages < 0xFFFFFFFFull;
}
table_layout layout_for(size_t bytes, size_t page_bytes, size_t frame_pool_bytes) {
    const size_t n_frames = frame_pool_bytes / page_bytes, n_pages = (bytes + page_bytes - 1) / page_bytes;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    table_layout l;
    l.frames = 0;
    l.pte = up(n_frames * page_bytes);
    l.owner = l.pte + up(n_pages * sizeof(unsigned long long));
    l.hand = l.owner + up(n_frames * sizeof(unsigned int));
    l.stats = l.hand + up(4 * sizeof(unsigned long long));
    l.flag = l.stats + up((size_t)GPUVM_STAT_SLOTS * GPUVM_S_COUNT * sizeof(unsigned long long));
    l.total = l.flag + up(sizeof(int));
    return l;
}
}  // namespace

static int create_view(void *host_buf, size_t bytes, size_t page_bytes, size_t frame_pool_bytes, int policy,
                       void *d_workspace, size_t workspace_bytes, gpuvm_t **out);

size_t gpuvm_workspace_bytes(size_t bytes, size_t page_bytes, size_t frame_pool_bytes) {
    return geometry_ok(bytes, page_bytes, frame_pool_bytes) ? layout_for(bytes, page_bytes, frame_pool_bytes).total : 0;
}

int gpuvm_create(void *host_buf, size_t bytes, size_t page_bytes, size_t frame_pool_bytes, int policy,
                 gpuvm_t **out) {
    return create_view(host_buf, bytes, page_bytes, frame_pool_bytes, policy, nullptr, 0, out);
}

int gpuvm_create_in(void *host_buf, size_t bytes, size_t page_bytes, size_t frame_pool_bytes, int policy,
                    void *d_workspace, size_t workspace_bytes, gpuvm_t **out) {
    if (out) *out = nullptr;
    if (!d_workspace || ((uintptr_t)d_workspace & 255)) return GPUVM_EINVAL;
    return create_view(host_buf, bytes, page_bytes, frame_pool_bytes, policy, d_workspace, workspace_bytes, out);
}

static int create_view(void *host_buf, size_t bytes, size_t page_bytes, size_t frame_pool_bytes, int policy,
                       void *d_workspace, size_t workspace_bytes, gpuvm_t **out) {
    if (!out) return GPUVM_EINVAL;
    *out = nullptr;
    if (!host_buf || !geometry_ok(bytes, page_bytes, frame_pool_bytes)) return GPUVM_EINVAL;
    if (policy < GPUVM_POLICY_FIFO || policy > GPUVM_POLICY_GCLOCK) return GPUVM_EINVAL;
    const size_t n_frames = frame_pool_bytes / page_bytes;
    const size_t n_pages = (bytes + page_bytes - 1) / page_bytes;
    const table_layout lay = layout_for(bytes, page_bytes, frame_pool_bytes);
    if (d_workspace) {
        if (workspace_bytes < lay.total) return GPUVM_EINVAL;
        hipPointerAttribute_t wa;                                 // the workspace must be device memory, all of it
        if (hipPointerGetAttributes(&wa, d_workspace) != hipSuccess || wa.type != hipMemoryTypeDevice ||
            hipPointerGetAttributes(&wa, (char *)d_workspace + lay.total - 1) != hipSuccess || wa.type != hipMemoryTypeDevice) {
            (void)hipGetLastError();
            return GPUVM_EINVAL;
        }
    }

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
    hipDeviceProp_t prop;
    if (hipGetDevice(&vm->device) != hipSuccess || hipGetDeviceProperties(&prop, vm->device) != hipSuccess) {
        (void)hipGetLastError();
        delete vm;
        return GPUVM_EHIP;
    }
    vm->cus = prop.multiProcessorCount;
    vm->waves_per_cu = 8;
    vm->waves_chosen = false;
    if (const char *e = getenv("GPUVM_WAVES_PER_CU")) {
        vm->waves_per_cu = std::max(1, std::min(32, atoi(e)));
        vm->waves_chosen = true;
    }
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
    // the CLOCK policies run two-handed by default: front hand half a ring ahead
    if (policy == GPUVM_POLICY_CLOCK || policy == GPUVM_POLICY_CLOCK_WRITE_AWARE)
        d.flags |= (uint32_t)GPUVM_CLOCK_HANDS_DEFAULT << GPUVM_F_HANDS_SHIFT;
    int rc = GPUVM_OK;
    if (d_workspace) {
        char *w = (char *)d_workspace;
        vm->owns_tables = false;
        d.frames = w + lay.frames;
        d.pte = (unsigned long long *)(w + lay.pte);
        d.frame_owner = (unsigned int *)(w + lay.owner);
        d.hand = (unsigned long long *)(w + lay.hand);
        d.stats = (unsigned long long *)(w + lay.stats);
        vm->bfs_changed = (int *)(w + lay.flag);
    } else {
        auto alloc = [&](void **p, size_t sz) {
            if (rc) return;
            if (hipMalloc(p, sz) != hipSuccess) { (void)hipGetLastError(); rc = GPUVM_ENOMEM; }
        };
        alloc((void **)&d.frames, n_frames * page_bytes);
        alloc((void **)&d.pte, n_pages * sizeof(unsigned long long));
        alloc((void **)&d.frame_owner, n_frames * sizeof(unsigned int));
        alloc((void **)&d.hand, 4 * sizeof(unsigned long long));
        alloc((void **)&d.stats, (size_t)GPUVM_STAT_SLOTS * GPUVM_S_COUNT * sizeof(unsigned long long));
        alloc((void **)&vm->bfs_changed, sizeof(int));
    }
    if (rc) { gpuvm_destroy(vm); return rc; }
    k_fill64<<<256, 256>>>(d.pte, n_pages, 0ull);
    k_fill32<<<256, 256>>>(d.frame_owner, n_frames, GPUVM_NO_PAGE);
    k_fill64<<<1, 64>>>(d.hand, 4, 0ull);
    k_fill64<<<4, 256>>>(d.stats, (size_t)GPUVM_STAT_SLOTS * GPUVM_S_COUNT, 0ull);
    if (hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); gpuvm_destroy(vm); return GPUVM_EHIP; }
    *out = vm;
    return GPUVM_OK;
}

int gpuvm_destroy(gpuvm_t *vm) {
    if (!vm) return GPUVM_OK;
    (void)hipDeviceSynchronize();
    gpuvm_dev_t &d = vm->dev;
    if (vm->owns_tables) {
        (void)hipFree(d.frames); (void)hipFree(d.pte); (void)hipFree(d.frame_owner); (void)hipFree(d.hand); (void)hipFree(d.stats);
        (void)hipFree(vm->bfs_changed);
    }
    (void)hipFree(vm->stamp); (void)hipFree(vm->first); (void)hipFree(vm->miss); (void)hipFree(vm->miss_sorted); (void)hipFree(vm->jobs);
    (void)hipFree(vm->phase_ctr); (void)hipFree(vm->page_owner); (void)hipFree(vm->page_marks); (void)hipFree(vm->row_progress);
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

int gpuvm_set_writeback_mode(gpuvm_t *vm, int mode) {
    if (!vm || (mode != GPUVM_WB_OVERLAPPED && mode != GPUVM_WB_SERIAL)) return GPUVM_EINVAL;
    vm->dev.flags = mode == GPUVM_WB_OVERLAPPED ? (vm->dev.flags | GPUVM_F_OVERLAPPED_WRITEBACK)
                                                : (vm->dev.flags & ~GPUVM_F_OVERLAPPED_WRITEBACK);
    vm->wb_chosen = true;
    return GPUVM_OK;
}

int gpuvm_set_clock_hands(gpuvm_t *vm, int spread_eighths) {
    if (!vm || spread_eighths < 0 || spread_eighths > (int)GPUVM_F_HANDS_MASK) return GPUVM_EINVAL;
    const bool has_bit = vm->dev.policy == GPUVM_POLICY_CLOCK || vm->dev.policy == GPUVM_POLICY_CLOCK_WRITE_AWARE;
    if (spread_eighths && !has_bit) return GPUVM_EINVAL;
    vm->dev.flags = (vm->dev.flags & ~(GPUVM_F_HANDS_MASK << GPUVM_F_HANDS_SHIFT)) | ((uint32_t)spread_eighths << GPUVM_F_HANDS_SHIFT);
    return GPUVM_OK;
}

int gpuvm_set_remote_first(gpuvm_t *vm, size_t bytes_per_touch) {
    if (!vm) return GPUVM_EINVAL;
    uint32_t touches = 0;
    if (bytes_per_touch) {
        // rent or buy: migrate once the reads in place have cost one page
        const size_t per_touch = std::max<size_t>(bytes_per_touch, 128);
        touches = (uint32_t)std::min<size_t>(std::max<size_t>(vm->page_bytes / per_touch, 2), (1u << 24) - 1);
    }
    vm->dev.flags = (vm->dev.flags & ((1u << GPUVM_F_REMOTE_SHIFT) - 1)) | (touches << GPUVM_F_REMOTE_SHIFT);
    return GPUVM_OK;
}

int gpuvm_set_waves_per_cu(gpuvm_t *vm, int waves_per_cu) {
    if (!vm || waves_per_cu < 1 || waves_per_cu > 32) return GPUVM_EINVAL;
    vm->waves_per_cu = waves_per_cu;
    vm->waves_chosen = true;
    return GPUVM_OK;
}

int gpuvm_max_waves(const gpuvm_t *vm) {
    if (!vm) return GPUVM_EINVAL;
    return launch_waves(vm, (size_t)1 << 40);
}

int gpuvm_max_waves_streaming(const gpuvm_t *vm) {
    if (!vm) return GPUVM_EINVAL;
    return launch_waves_streaming(vm, (size_t)1 << 40);
}

int gpuvm_max_waves_duplex(const gpuvm_t *vm) {
    if (!vm) return GPUVM_EINVAL;
    return launch_waves_duplex(vm, (size_t)1 << 40);
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
    memset(out, 0, sizeof(*out));
    out->faults = tot[GPUVM_S_FAULTS];           out->evictions = tot[GPUVM_S_FAULTS] - tot[GPUVM_S_FRESH];
    out->writebacks_evict = tot[GPUVM_S_WB_EVICT]; out->writebacks_flush = tot[GPUVM_S_WB_FLUSH];
    // every page moved is page_bytes long, except the last page of the data set if it is short
    const uint64_t page = vm->page_bytes, missing = (uint64_t)vm->dev.n_pages * page - vm->dev.bytes;
    out->bytes_in = (tot[GPUVM_S_FAULTS] - tot[GPUVM_S_NOFETCH]) * page - tot[GPUVM_S_SHORT_IN] * missing;
    out->bytes_out = (tot[GPUVM_S_WB_EVICT] + tot[GPUVM_S_WB_FLUSH]) * page - tot[GPUVM_S_SHORT_OUT] * missing;
    out->hits = tot[GPUVM_S_HITS];               out->wave_page_groups = tot[GPUVM_S_GROUPS];
    out->lanes_coalesced = tot[GPUVM_S_COALESCED]; out->loading_waits = tot[GPUVM_S_WAITS];
    out->alloc_skips = tot[GPUVM_S_SKIPS];       out->alloc_sweeps = tot[GPUVM_S_SWEEPS];
    out->phases = tot[GPUVM_S_PHASES];           out->faults_no_fetch = tot[GPUVM_S_NOFETCH];
    out->remote_reads = tot[GPUVM_S_REMOTE];
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

}  // extern "C"

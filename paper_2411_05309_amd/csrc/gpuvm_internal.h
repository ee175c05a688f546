// Internal declarations shared by the translation units of libgpuvm (not part
// of the boundary): the handle behind gpuvm_t, launch-shape helpers, error
// plumbing and the small fill kernels every unit needs.
#ifndef GPUVM_INTERNAL_H
#define GPUVM_INTERNAL_H

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "gpuvm.h"
#include "gpuvm_device.h"

constexpr int kBlock = 256;               // 4 wavefronts per workgroup
constexpr int kWavesPerBlock = kBlock / 64;
constexpr uint32_t kDefaultSpinLimit = 1u << 22;

struct phase_job {                        // one fault of a deterministic phase
    unsigned int page, frame, victim, writeback;
};

struct gpuvm {
    gpuvm_dev_t dev;
    int device;
    int cus;
    int waves_per_cu;
    bool waves_chosen;            // set by the caller (or the environment): launchers do not second-guess it
    bool wb_chosen = false;       // write-back order set by the caller: launchers do not second-guess it
    bool owns_tables = true;      // false: pool and tables were carved from the caller's workspace (gpuvm_create_in)
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
    unsigned int *page_marks = nullptr;   // two page lists (mark per page, list, taking order, counters), edge-balanced BFS / CC / SSSP: this round's and the next one's
    unsigned int *row_progress = nullptr; // [8192] row reached by each compute wave (column-order product)
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

// Launch shape and kernel-side errors (core.hip).
int check_kernel_error(gpuvm_t *vm);      // reads the error word a kernel may have recorded (synchronous copy)
int grid_for_waves(int waves);            // workgroups for that many wavefronts
int launch_waves(const gpuvm_t *vm, size_t work_waves);          // waves to keep in flight; 0 = pool too small
int launch_waves_streaming(const gpuvm_t *vm, size_t work_waves);   // for launches that are plain streams of page faults
int launch_waves_duplex(const gpuvm_t *vm, size_t work_waves);   // the same for launches that write back as much as they fetch
gpuvm_dev_t dev_for_writers(const gpuvm_t *vm, int waves);       // device view for a launch that dirties pages, with `waves` in flight

// Fill kernels (a copy per translation unit; used instead of hipMemsetAsync so
// that a caller may capture the launchers in a graph).
static __global__ void k_fill64(unsigned long long *p, size_t n, unsigned long long v) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
static __global__ void k_fill32(unsigned int *p, size_t n, unsigned int v) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
static __global__ void k_fill8(unsigned char *p, size_t n, unsigned char v) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

__device__ __forceinline__ unsigned long long wave_sum(unsigned long long v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

#endif  // GPUVM_INTERNAL_H

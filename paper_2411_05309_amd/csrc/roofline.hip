// libgpuvm - roofline microbenchmarks: wavefront copy / read of host or device memory, load latency, plain gather.
// The fault path itself (page-table lookup, wavefront dedup, frame allocation,
// eviction, write-back, migration) is in include/gpuvm_device.h and is inlined
// into every kernel, the way the paper inlines its runtime into the application
// kernels (System Overview; Register usage).
#include "gpuvm_internal.h"

using namespace gpuvm_detail;

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

// The same copy staged through LDS instead of registers: every wave owns 8 KiB
// of LDS, fills it with eight direct-to-LDS loads (global_load_lds_dwordx4: lane
// i's 16 bytes land at the slot's base + 16 i, no VGPR holds them), waits, and
// writes the 8 KiB out with LDS reads and stores.  The alternative design of the
// page mover, kept as a microbenchmark so that the choice between the two can
// be measured.  `bytes` and `chunk` are multiples of 16.
__global__ __launch_bounds__(kBlock) void k_bench_copy_lds(char *dst, const char *src, size_t bytes, size_t chunk) {
    __shared__ __attribute__((aligned(16))) unsigned int stage[kWavesPerBlock][8][256];
    const unsigned int lane = threadIdx.x & 63, wv = bcast(threadIdx.x >> 6);
    const size_t wave = bcast((unsigned int)(((size_t)blockIdx.x * kBlock + threadIdx.x) >> 6));   // wave-uniform, in SGPRs
    const size_t nwaves = ((size_t)gridDim.x * kBlock) >> 6;
    const size_t nchunks = (bytes + chunk - 1) / chunk;
    for (size_t c = wave; c < nchunks; c += nwaves) {
        const size_t lo = c * chunk;
        const size_t len = chunk < bytes - lo ? chunk : bytes - lo;
        const __amdgpu_buffer_rsrc_t rd = make_rsrc(dst + lo, (unsigned int)len);
        for (size_t o = 0; o < len; o += 8192) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const size_t at = o + (size_t)j * 1024 + lane * 16u;
                if (at < len)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + lo + at),
                                                     (__attribute__((address_space(3))) void *)&stage[wv][j][0], 16, 0,
                                                     GPUVM_AUX_SYSTEM);
            }
            wait_vm();                                        // the loads have landed in LDS
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const size_t at = o + (size_t)j * 1024 + lane * 16u;
                if (at < len) {
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(&stage[wv][j][lane * 4u]);
                    __builtin_amdgcn_raw_buffer_store_b128(v, rd, (unsigned int)at, 0, GPUVM_AUX_SYSTEM);
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // LDS read out before the next round overwrites it
        }
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

// data[idx[k]] += 1 on a plain uint64 array with no page table: in HBM the
// ceiling for scatter hits, in pinned host memory (system-scope atomics
// executed over the link) the zero-copy form of the scatter-increment.
__global__ __launch_bounds__(kBlock) void k_bench_scatter_plain(unsigned long long *data, const uint32_t *__restrict__ idx,
                                                                 size_t n) {
    const size_t nthreads = (size_t)gridDim.x * kBlock;
    for (size_t k = (size_t)blockIdx.x * kBlock + threadIdx.x; k < n; k += nthreads)
        __hip_atomic_fetch_add(data + idx[k], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

extern "C" {

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

int gpuvm_bench_copy_lds(void *dst, const void *src, size_t bytes, size_t chunk_bytes, int waves, void *stream) {
    if (!dst || !src || bytes == 0 || bytes % 16 || chunk_bytes < 16 || chunk_bytes % 16 || chunk_bytes > (1u << 30)) return GPUVM_EINVAL;
    k_bench_copy_lds<<<grid_for_waves(bench_waves(waves)), kBlock, 0, (hipStream_t)stream>>>((char *)dst, (const char *)src,
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

int gpuvm_bench_scatter_plain(uint64_t *data, const uint32_t *d_idx, size_t n, void *stream) {
    if (!data || !d_idx) return GPUVM_EINVAL;
    if (n == 0) return GPUVM_OK;
    const int grid = (int)std::min<size_t>((n + kBlock - 1) / kBlock, 256 * 32);
    k_bench_scatter_plain<<<grid, kBlock, 0, (hipStream_t)stream>>>((unsigned long long *)data, d_idx, n);
    HIP_TRY(hipGetLastError());
    return GPUVM_OK;
}

}  // extern "C"

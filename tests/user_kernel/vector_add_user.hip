// A kernel as a user of the library would write it: the paper's vector-addition
// listing against the two public headers only (include/gpuvm.h for the host
// calls, include/gpuvm_device.h for the array-like view), built into a library
// of its own.  Test infrastructure: it shows that the boundary is usable from
// outside the library's sources, and it runs the accessors in plain
// thread-per-element code (divergent tail, operator[] loads and stores).
#include "gpuvm_device.h"

// c[i] = a[i] + b[i], one element per thread and grid-stride.  The only change
// against the same kernel on plain pointers is the type of a, b and c.
__global__ void k_user_vector_add(gpuvm_array<float> a, gpuvm_array<float> b, gpuvm_array<float> c, size_t n) {
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += nthreads)
        c[i] = a[i] + b[i];
}

// x[i] *= s in place: a load and a store of the same element of one array.
__global__ void k_user_scale(gpuvm_array<float> x, float s, size_t n) {
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += nthreads)
        x[i] = x[i] * s;
}

// y[i] += x[i] with a cursor per array: a wave takes a contiguous run of the
// index range and keeps the page it stands on pinned from one step to the next
// (gpuvm_cursor_load / gpuvm_cursor_store), the way sequential code would.
__global__ void k_user_accumulate(gpuvm_dev_t x, gpuvm_dev_t y, size_t n) {
    const unsigned int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const size_t nwaves = ((size_t)gridDim.x * blockDim.x) >> 6;
    const size_t per_wave = ((n + nwaves - 1) / nwaves + 63) / 64 * 64;
    const size_t lo = wave * per_wave, hi = lo + per_wave < n ? lo + per_wave : n;
    gpuvm_cursor_t cx = gpuvm_cursor_begin(), cy = gpuvm_cursor_begin();
    for (size_t i0 = lo; i0 < hi; i0 += 64) {
        const size_t i = i0 + lane;
        const bool want = i < hi;
        const float a = gpuvm_cursor_load<float>(x, cx, want ? i : 0, want);
        const float b = gpuvm_cursor_load<float>(y, cy, want ? i : 0, want);
        gpuvm_cursor_store<float>(y, cy, want ? i : 0, a + b, want);
    }
    gpuvm_cursor_end(x, cx);
    gpuvm_cursor_end(y, cy);
}

// out[k] = data[i0[k]] + data[i1[k]] (uint32, wrapping): two independent reads per
// lane in one optimistic transaction (gpuvm_load_n).
__global__ void k_user_gather_pairs(gpuvm_dev_t data, const unsigned int *i0, const unsigned int *i1, size_t n,
                                    unsigned int *out) {
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    const size_t n_up = (n + 63) & ~(size_t)63;                   // whole waves call the accessor together
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < n_up; k += nthreads) {
        const bool w = k < n;
        const unsigned long long elem[2] = {w ? i0[k] : 0ull, w ? i1[k] : 0ull};
        const bool want[2] = {w, w};
        unsigned int v[2];
        gpuvm_load_n<unsigned int, 2>(data, elem, want, v);
        if (w) out[k] = v[0] + v[1];
    }
}

// The one rule a user's launch has to follow: no more wavefronts in flight than
// gpuvm_max_waves() allows on every handle the kernel touches (each wave may
// hold a frame while it waits for another one to come free).
static int grid_blocks(std::initializer_list<gpuvm_t *> vms, int block) {
    int waves = 1 << 30;
    for (gpuvm_t *vm : vms) waves = std::min(waves, gpuvm_max_waves(vm));
    return waves * 64 / block;
}

extern "C" __attribute__((visibility("default")))
int user_vector_add(gpuvm_t *a, gpuvm_t *b, gpuvm_t *c, size_t n, void *stream) {
    gpuvm_dev_t da, db, dc;
    if (gpuvm_device_handle(a, &da) || gpuvm_device_handle(b, &db) || gpuvm_device_handle(c, &dc)) return GPUVM_EINVAL;
    const int blocks = grid_blocks({a, b, c}, 256);
    if (blocks < 1) return GPUVM_EDEADLK;
    k_user_vector_add<<<blocks, 256, 0, (hipStream_t)stream>>>(gpuvm_array<float>{da}, gpuvm_array<float>{db},
                                                                gpuvm_array<float>{dc}, n);
    return hipGetLastError() == hipSuccess ? GPUVM_OK : GPUVM_EHIP;
}

extern "C" __attribute__((visibility("default")))
int user_scale(gpuvm_t *x, float s, size_t n, void *stream) {
    gpuvm_dev_t dx;
    if (gpuvm_device_handle(x, &dx)) return GPUVM_EINVAL;
    const int blocks = grid_blocks({x}, 256);
    if (blocks < 1) return GPUVM_EDEADLK;
    k_user_scale<<<blocks, 256, 0, (hipStream_t)stream>>>(gpuvm_array<float>{dx}, s, n);
    return hipGetLastError() == hipSuccess ? GPUVM_OK : GPUVM_EHIP;
}

extern "C" __attribute__((visibility("default")))
int user_accumulate(gpuvm_t *x, gpuvm_t *y, size_t n, void *stream) {
    gpuvm_dev_t dx, dy;
    if (x == y || gpuvm_device_handle(x, &dx) || gpuvm_device_handle(y, &dy)) return GPUVM_EINVAL;
    const int blocks = grid_blocks({x, y}, 256);
    if (blocks < 1) return GPUVM_EDEADLK;
    k_user_accumulate<<<blocks, 256, 0, (hipStream_t)stream>>>(dx, dy, n);
    return hipGetLastError() == hipSuccess ? GPUVM_OK : GPUVM_EHIP;
}

extern "C" __attribute__((visibility("default")))
int user_gather_pairs(gpuvm_t *data, const unsigned int *d_i0, const unsigned int *d_i1, size_t n, unsigned int *d_out,
                      void *stream) {
    gpuvm_dev_t dd;
    if (gpuvm_device_handle(data, &dd)) return GPUVM_EINVAL;
    const int blocks = grid_blocks({data}, 256);
    if (blocks < 1) return GPUVM_EDEADLK;
    k_user_gather_pairs<<<blocks, 256, 0, (hipStream_t)stream>>>(dd, d_i0, d_i1, n, d_out);
    return hipGetLastError() == hipSuccess ? GPUVM_OK : GPUVM_EHIP;
}

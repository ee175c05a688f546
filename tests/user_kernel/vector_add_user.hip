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

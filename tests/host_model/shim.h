// Host build of include/gpuvm_device.h for the protocol stress test: every
// "wavefront" is ONE lane run by one CPU thread, so the wave-level intrinsics
// collapse to their one-lane meaning and the inter-wave protocol (page-table
// word, ring cursor, eviction claim, optimistic reads, write-back) runs as
// written, under the preemptive interleavings of host threads.  Test
// infrastructure only: nothing in the library includes this file.
#pragma once
#include <sched.h>
#include <stdint.h>
#include <string.h>

#define __device__
#define __forceinline__ inline __attribute__((always_inline))
#define __HIP_MEMORY_SCOPE_SINGLETHREAD 1
#define __HIP_MEMORY_SCOPE_WAVEFRONT 2
#define __HIP_MEMORY_SCOPE_WORKGROUP 3
#define __HIP_MEMORY_SCOPE_AGENT 4
#define __HIP_MEMORY_SCOPE_SYSTEM 5

struct shim_dim3 { unsigned int x, y, z; };
static thread_local shim_dim3 threadIdx = {0, 0, 0};
static thread_local shim_dim3 blockIdx = {0, 0, 0};      // set per thread: selects the counter shard
static thread_local unsigned int shim_tick = 0;
static unsigned int shim_yield_every = 0;                // 0 = never

static inline void shim_maybe_yield() {
    if (shim_yield_every && ++shim_tick % shim_yield_every == 0) sched_yield();
}

// one-lane wave
#define __builtin_amdgcn_ballot_w64(p) ((unsigned long long)((p) ? 1ull : 0ull))
#define __builtin_amdgcn_mbcnt_lo(mask, base) (base)
#define __builtin_amdgcn_mbcnt_hi(mask, base) (base)
#define __builtin_amdgcn_readfirstlane(v) (v)
#define __builtin_amdgcn_readlane(v, lane) (v)
#define __builtin_amdgcn_s_sleep(n) sched_yield()
#define __lane_id() 0u
#define __shfl(v, lane, width) (v)
#define __popcll(x) __builtin_popcountll(x)
#define __ffsll(x) __builtin_ffsll(x)

// raw buffer addressing: base + byte offset, out-of-range lanes read 0 / write nothing
struct shim_rsrc { char *base; unsigned int bytes; };
#define __amdgpu_buffer_rsrc_t shim_rsrc
#define __builtin_amdgcn_make_buffer_rsrc(p, stride, n, flags) (shim_rsrc{(char *)(p), (unsigned int)(n)})

typedef unsigned int shim_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int shim_u32x2 __attribute__((ext_vector_type(2)));
template <typename T>
static inline T shim_buf_load(shim_rsrc r, unsigned int off) {
    shim_maybe_yield();
    T v;
    memset(&v, 0, sizeof v);
    if ((unsigned long long)off + sizeof(T) <= r.bytes) memcpy(&v, r.base + off, sizeof v);
    return v;
}
template <typename T>
static inline void shim_buf_store(T v, shim_rsrc r, unsigned int off) {
    shim_maybe_yield();
    if ((unsigned long long)off + sizeof(T) <= r.bytes) memcpy(r.base + off, &v, sizeof v);
}
#define __builtin_amdgcn_raw_buffer_load_b128(r, off, soff, aux) shim_buf_load<shim_u32x4>(r, off)
#define __builtin_amdgcn_raw_buffer_load_b64(r, off, soff, aux) shim_buf_load<shim_u32x2>(r, off)
#define __builtin_amdgcn_raw_buffer_load_b32(r, off, soff, aux) shim_buf_load<unsigned int>(r, off)
#define __builtin_amdgcn_raw_buffer_load_b8(r, off, soff, aux) shim_buf_load<unsigned char>(r, off)
#define __builtin_amdgcn_raw_buffer_store_b128(v, r, off, soff, aux) shim_buf_store<shim_u32x4>(v, r, off)
#define __builtin_amdgcn_raw_buffer_store_b32(v, r, off, soff, aux) shim_buf_store<unsigned int>(v, r, off)
#define __builtin_amdgcn_raw_buffer_store_b8(v, r, off, soff, aux) shim_buf_store<unsigned char>(v, r, off)

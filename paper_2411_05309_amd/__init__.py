"""GPUVM hot path for MI355X: thin ctypes binding over ``libgpuvm.so``.

Argument marshalling only -- every step of the path (page-table lookup,
wavefront dedup, frame allocation, eviction, write-back, page migration, the
workload itself) runs in the HIP kernels behind the C ABI declared in
``include/gpuvm.h``; function names here are the C names.  There is no CPU
fallback: ``load()`` raises if the library has not been built
(``python -m paper_2411_05309_amd.build`` or ``__graft_entry__.build()``).

torch is used by callers for device memory and streams only; pointers cross
this boundary as plain integers (``tensor.data_ptr()``).
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgpuvm.so")

OK, EINVAL, ENOMEM, EPIN, EDEADLK, EHIP, ERANGE = 0, -1, -2, -3, -4, -5, -6
POLICY_FIFO, POLICY_CLOCK, POLICY_FIFO_WAIT, POLICY_CLOCK_WRITE_AWARE, POLICY_GCLOCK = 0, 1, 2, 3, 4
WB_SERIAL, WB_OVERLAPPED = 0, 1
STAT_NAMES = ("faults", "evictions", "writebacks_evict", "writebacks_flush",
              "bytes_in", "bytes_out", "hits", "wave_page_groups",
              "lanes_coalesced", "loading_waits", "alloc_skips", "alloc_sweeps",
              "phases", "faults_no_fetch", "remote_reads")

# page-table word layout (include/gpuvm_device.h)
PTE_PIN_MASK = 0xFFFFF
PTE_GEN_SHIFT = 20
PTE_GEN_MASK = 0xFFF00000
PTE_REF = 1 << 32
PTE_DIRTY = 1 << 33
PTE_STATE_SHIFT = 34
PTE_DEFER = 1 << 36
PTE_FRAME_SHIFT = 37
ST_INVALID, ST_LOADING, ST_RESIDENT, ST_EVICTING = 0, 1, 2, 3
NO_PAGE = 0xFFFFFFFF


class GpuvmError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        msg = _lib.gpuvm_strerror(code).decode() if _lib else str(code)
        super().__init__(f"{what}: {msg} ({code})")


class Stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in STAT_NAMES] + [("reserved", C.c_uint64 * 1)]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n in STAT_NAMES}


class Dev(C.Structure):
    _fields_ = [("pte", C.c_void_p), ("frame_owner", C.c_void_p), ("hand", C.c_void_p),
                ("stats", C.c_void_p), ("frames", C.c_void_p), ("host", C.c_void_p),
                ("bytes", C.c_uint64), ("n_pages", C.c_uint32), ("n_frames", C.c_uint32),
                ("page_shift", C.c_uint32), ("policy", C.c_uint32),
                ("spin_limit", C.c_uint32), ("flags", C.c_uint32)]


_lib = None

_SIGNATURES = {
    # name: (argtypes, restype)
    "gpuvm_host_alloc": ([C.c_size_t, C.POINTER(C.c_void_p)], C.c_int),
    "gpuvm_host_free": ([C.c_void_p], C.c_int),
    "gpuvm_create": ([C.c_void_p, C.c_size_t, C.c_size_t, C.c_size_t, C.c_int, C.POINTER(C.c_void_p)], C.c_int),
    "gpuvm_destroy": ([C.c_void_p], C.c_int),
    "gpuvm_workspace_bytes": ([C.c_size_t, C.c_size_t, C.c_size_t], C.c_size_t),
    "gpuvm_create_in": ([C.c_void_p, C.c_size_t, C.c_size_t, C.c_size_t, C.c_int, C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)], C.c_int),
    "gpuvm_device_handle": ([C.c_void_p, C.POINTER(Dev)], C.c_int),
    "gpuvm_configure": ([C.c_void_p, C.c_uint32, C.c_int], C.c_int),
    "gpuvm_set_writeback_mode": ([C.c_void_p, C.c_int], C.c_int),
    "gpuvm_set_clock_hands": ([C.c_void_p, C.c_int], C.c_int),
    "gpuvm_set_remote_first": ([C.c_void_p, C.c_size_t], C.c_int),
    "gpuvm_set_waves_per_cu": ([C.c_void_p, C.c_int], C.c_int),
    "gpuvm_check": ([C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_max_waves": ([C.c_void_p], C.c_int),
    "gpuvm_max_waves_duplex": ([C.c_void_p], C.c_int),
    "gpuvm_max_waves_streaming": ([C.c_void_p], C.c_int),
    "gpuvm_flush": ([C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_reset": ([C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_stats": ([C.c_void_p, C.POINTER(Stats)], C.c_int),
    "gpuvm_stats_clear": ([C.c_void_p], C.c_int),
    "gpuvm_dump_tables": ([C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_strerror": ([C.c_int], C.c_char_p),
    "gpuvm_run_gather": ([C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_run_gather_masked": ([C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_run_scatter_increment_masked": ([C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p], C.c_int),
    "gpuvm_run_prefetch": ([C.c_void_p, C.c_size_t, C.c_size_t, C.c_void_p], C.c_int),
    "gpuvm_run_vector_add": ([C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p], C.c_int),
    "gpuvm_run_vector_add_overwrite": ([C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p], C.c_int),
    "gpuvm_run_stream_reduce": ([C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_run_bfs": ([C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.POINTER(C.c_int), C.c_void_p], C.c_int),
    "gpuvm_run_bfs_balanced": ([C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.POINTER(C.c_int), C.c_void_p], C.c_int),
    "gpuvm_bench_bfs_zero_copy": ([C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.POINTER(C.c_int), C.c_void_p], C.c_int),
    "gpuvm_run_cc_balanced": ([C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.POINTER(C.c_int), C.c_void_p], C.c_int),
    "gpuvm_run_sssp_balanced": ([C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.POINTER(C.c_int), C.c_void_p], C.c_int),
    "gpuvm_run_embedding_bag": ([C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_size_t, C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_bench_embedding_bag_zero_copy": ([C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_size_t, C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_run_matvec_t": ([C.c_void_p, C.c_size_t, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_run_matvec_t_noalloc": ([C.c_void_p, C.c_size_t, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_run_matvec": ([C.c_void_p, C.c_size_t, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_run_filter_sum": ([C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_run_scatter_increment": ([C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p], C.c_int),
    "gpuvm_run_gather_phased": ([C.c_void_p, C.c_void_p, C.c_size_t, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_run_scatter_increment_phased": ([C.c_void_p, C.c_void_p, C.c_size_t, C.c_size_t, C.c_void_p], C.c_int),
    "gpuvm_bench_copy": ([C.c_void_p, C.c_void_p, C.c_size_t, C.c_size_t, C.c_int, C.c_void_p], C.c_int),
    "gpuvm_bench_copy_lds": ([C.c_void_p, C.c_void_p, C.c_size_t, C.c_size_t, C.c_int, C.c_void_p], C.c_int),
    "gpuvm_bench_read": ([C.c_void_p, C.c_size_t, C.c_size_t, C.c_int, C.c_void_p, C.c_void_p], C.c_int),
    "gpuvm_bench_latency": ([C.c_void_p, C.c_size_t, C.c_int, C.POINTER(C.c_double), C.c_void_p], C.c_int),
    "gpuvm_bench_scatter_plain": ([C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p], C.c_int),
    "gpuvm_bench_gather_plain": ([C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p], C.c_int),
}


def load():
    """dlopen libgpuvm.so and declare the C signatures; raises if it is not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -m paper_2411_05309_amd.build` (there is no CPU fallback)")
        lib = C.CDLL(LIB_PATH)
        for name, (argtypes, restype) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.argtypes, fn.restype = argtypes, restype
        _lib = lib
    return _lib


def _call(name, *args):
    rc = getattr(load(), name)(*args)
    if rc != OK:
        raise GpuvmError(rc, name)


def _ptr(x):
    """torch tensor / numpy array / int / None -> address."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return x.ctypes.data


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


# ---------------------------------------------------------------- C names

def gpuvm_strerror(code):
    return load().gpuvm_strerror(code).decode()


def gpuvm_host_alloc(nbytes):
    out = C.c_void_p()
    _call("gpuvm_host_alloc", nbytes, C.byref(out))
    return out.value


def gpuvm_host_free(ptr):
    _call("gpuvm_host_free", ptr)


def gpuvm_create(host_buf, nbytes, page_bytes, frame_pool_bytes, policy=POLICY_CLOCK):
    out = C.c_void_p()
    _call("gpuvm_create", _ptr(host_buf), nbytes, page_bytes, frame_pool_bytes, policy, C.byref(out))
    return out.value


def gpuvm_workspace_bytes(nbytes, page_bytes, frame_pool_bytes):
    return int(load().gpuvm_workspace_bytes(nbytes, page_bytes, frame_pool_bytes))


def gpuvm_create_in(host_buf, nbytes, page_bytes, frame_pool_bytes, policy, d_workspace, workspace_bytes):
    out = C.c_void_p()
    _call("gpuvm_create_in", _ptr(host_buf), nbytes, page_bytes, frame_pool_bytes, policy, _ptr(d_workspace), workspace_bytes,
          C.byref(out))
    return out.value


def gpuvm_destroy(vm):
    _call("gpuvm_destroy", vm)


def gpuvm_device_handle(vm):
    d = Dev()
    _call("gpuvm_device_handle", vm, C.byref(d))
    return d


def gpuvm_configure(vm, spin_limit=0, access_stats=False):
    _call("gpuvm_configure", vm, spin_limit, int(access_stats))


def gpuvm_set_writeback_mode(vm, mode):
    _call("gpuvm_set_writeback_mode", vm, mode)


def gpuvm_set_clock_hands(vm, spread_eighths):
    _call("gpuvm_set_clock_hands", vm, spread_eighths)


def clock_spread(vm):
    """Frames between the front hand and the cursor on this handle (0 = one hand)."""
    d = gpuvm_device_handle(vm)
    eighths = (d.flags >> 2) & 7
    uses_bit = d.policy in (POLICY_CLOCK, POLICY_CLOCK_WRITE_AWARE)
    return (d.n_frames * eighths) >> 3 if uses_bit else 0


def gpuvm_set_remote_first(vm, bytes_per_touch):
    _call("gpuvm_set_remote_first", vm, bytes_per_touch)


def gpuvm_set_waves_per_cu(vm, waves_per_cu):
    _call("gpuvm_set_waves_per_cu", vm, waves_per_cu)


def gpuvm_check(vm, stream=None):
    _call("gpuvm_check", vm, _stream(stream))


def gpuvm_max_waves(vm):
    return load().gpuvm_max_waves(vm)


def gpuvm_max_waves_duplex(vm):
    return load().gpuvm_max_waves_duplex(vm)


def gpuvm_max_waves_streaming(vm):
    return load().gpuvm_max_waves_streaming(vm)


def gpuvm_flush(vm, stream=None):
    _call("gpuvm_flush", vm, _stream(stream))


def gpuvm_reset(vm, stream=None):
    _call("gpuvm_reset", vm, _stream(stream))


def gpuvm_stats(vm):
    s = Stats()
    _call("gpuvm_stats", vm, C.byref(s))
    return s.as_dict()


def gpuvm_stats_clear(vm):
    _call("gpuvm_stats_clear", vm)


def gpuvm_dump_tables(vm):
    """(pte uint64[n_pages], owner uint32[n_frames], hand) as numpy arrays."""
    import numpy as np
    d = gpuvm_device_handle(vm)
    pte = np.empty(d.n_pages, np.uint64)
    owner = np.empty(d.n_frames, np.uint32)
    hand = np.zeros(1, np.uint64)
    _call("gpuvm_dump_tables", vm, pte.ctypes.data, owner.ctypes.data, hand.ctypes.data)
    return pte, owner, int(hand[0])


def gpuvm_run_gather(vm, d_idx, n, d_out, d_sum=None, stream=None):
    _call("gpuvm_run_gather", vm, _ptr(d_idx), n, _ptr(d_out), _ptr(d_sum), _stream(stream))


def gpuvm_run_gather_masked(vm, d_idx, d_mask, n, d_out, stream=None):
    _call("gpuvm_run_gather_masked", vm, _ptr(d_idx), _ptr(d_mask), n, _ptr(d_out), _stream(stream))


def gpuvm_run_scatter_increment_masked(vm, d_idx, d_mask, n, stream=None):
    _call("gpuvm_run_scatter_increment_masked", vm, _ptr(d_idx), _ptr(d_mask), n, _stream(stream))


def gpuvm_run_prefetch(vm, first_page, n_pages, stream=None):
    _call("gpuvm_run_prefetch", vm, first_page, n_pages, _stream(stream))


def gpuvm_run_vector_add_overwrite(vm_a, vm_b, vm_c, n, stream=None):
    _call("gpuvm_run_vector_add_overwrite", vm_a, vm_b, vm_c, n, _stream(stream))


def gpuvm_run_vector_add(vm_a, vm_b, vm_c, n, stream=None):
    _call("gpuvm_run_vector_add", vm_a, vm_b, vm_c, n, _stream(stream))


def gpuvm_run_stream_reduce(vm, block_elems, d_sums, stream=None):
    _call("gpuvm_run_stream_reduce", vm, block_elems, _ptr(d_sums), _stream(stream))


def gpuvm_run_bfs(vm, d_row_ptr, nv, src, d_level, stream=None):
    levels = C.c_int(0)
    _call("gpuvm_run_bfs", vm, _ptr(d_row_ptr), nv, src, _ptr(d_level), C.byref(levels), _stream(stream))
    return levels.value


def gpuvm_bench_bfs_zero_copy(vm, d_row_ptr, nv, src, d_level, stream=None):
    levels = C.c_int(0)
    _call("gpuvm_bench_bfs_zero_copy", vm, _ptr(d_row_ptr), nv, src, _ptr(d_level), C.byref(levels), _stream(stream))
    return levels.value


def gpuvm_run_bfs_balanced(vm, d_row_ptr, nv, src, d_level, stream=None):
    levels = C.c_int(0)
    _call("gpuvm_run_bfs_balanced", vm, _ptr(d_row_ptr), nv, src, _ptr(d_level), C.byref(levels), _stream(stream))
    return levels.value


def gpuvm_run_cc_balanced(vm, d_row_ptr, nv, d_label, stream=None):
    rounds = C.c_int(0)
    _call("gpuvm_run_cc_balanced", vm, _ptr(d_row_ptr), nv, _ptr(d_label), C.byref(rounds), _stream(stream))
    return rounds.value


def gpuvm_run_sssp_balanced(vm, vm_weights, d_row_ptr, nv, src, d_dist, stream=None):
    rounds = C.c_int(0)
    _call("gpuvm_run_sssp_balanced", vm, vm_weights, _ptr(d_row_ptr), nv, src, _ptr(d_dist), C.byref(rounds),
          _stream(stream))
    return rounds.value


def gpuvm_bench_embedding_bag_zero_copy(vm, dim, d_ids, bags, bag_len, d_out, stream=None):
    _call("gpuvm_bench_embedding_bag_zero_copy", vm, dim, _ptr(d_ids), bags, bag_len, _ptr(d_out), _stream(stream))


def gpuvm_run_embedding_bag(vm, dim, d_ids, bags, bag_len, d_out, stream=None):
    _call("gpuvm_run_embedding_bag", vm, dim, _ptr(d_ids), bags, bag_len, _ptr(d_out), _stream(stream))


def gpuvm_run_matvec(vm, rows, cols, d_x, d_y, stream=None):
    _call("gpuvm_run_matvec", vm, rows, cols, _ptr(d_x), _ptr(d_y), _stream(stream))


def gpuvm_run_matvec_t(vm, rows, cols, d_x, d_y, stream=None):
    _call("gpuvm_run_matvec_t", vm, rows, cols, _ptr(d_x), _ptr(d_y), _stream(stream))


def gpuvm_run_matvec_t_noalloc(vm, rows, cols, d_x, d_y, stream=None):
    _call("gpuvm_run_matvec_t_noalloc", vm, rows, cols, _ptr(d_x), _ptr(d_y), _stream(stream))


def gpuvm_run_filter_sum(vm_key, vm_val, threshold, d_count, d_sum, stream=None):
    _call("gpuvm_run_filter_sum", vm_key, vm_val, threshold, _ptr(d_count), _ptr(d_sum), _stream(stream))


def gpuvm_run_scatter_increment(vm, d_idx, n, stream=None):
    _call("gpuvm_run_scatter_increment", vm, _ptr(d_idx), n, _stream(stream))


def gpuvm_run_gather_phased(vm, d_idx, n, phase_len, d_out, d_sum=None, stream=None):
    _call("gpuvm_run_gather_phased", vm, _ptr(d_idx), n, phase_len, _ptr(d_out), _ptr(d_sum), _stream(stream))


def gpuvm_run_scatter_increment_phased(vm, d_idx, n, phase_len, stream=None):
    _call("gpuvm_run_scatter_increment_phased", vm, _ptr(d_idx), n, phase_len, _stream(stream))


def gpuvm_bench_copy(dst, src, nbytes, chunk_bytes, waves=0, stream=None):
    _call("gpuvm_bench_copy", _ptr(dst), _ptr(src), nbytes, chunk_bytes, waves, _stream(stream))


def gpuvm_bench_copy_lds(dst, src, nbytes, chunk_bytes, waves=0, stream=None):
    _call("gpuvm_bench_copy_lds", _ptr(dst), _ptr(src), nbytes, chunk_bytes, waves, _stream(stream))


def gpuvm_bench_read(src, nbytes, chunk_bytes, d_sink, waves=0, stream=None):
    _call("gpuvm_bench_read", _ptr(src), nbytes, chunk_bytes, waves, _ptr(d_sink), _stream(stream))


def gpuvm_bench_latency(src, nbytes, hops=2000, stream=None):
    ns = C.c_double(0.0)
    _call("gpuvm_bench_latency", _ptr(src), nbytes, hops, C.byref(ns), _stream(stream))
    return ns.value


def gpuvm_bench_scatter_plain(data, d_idx, n, stream=None):
    _call("gpuvm_bench_scatter_plain", _ptr(data), _ptr(d_idx), n, _stream(stream))


def gpuvm_bench_gather_plain(d_data, d_idx, n, d_out, stream=None):
    _call("gpuvm_bench_gather_plain", _ptr(d_data), _ptr(d_idx), n, _ptr(d_out), _stream(stream))


# ---------------------------------------------------------------- helpers (plumbing)

def pinned_array(shape, dtype):
    """numpy array over gpuvm_host_alloc memory; free with ``free_pinned``."""
    import numpy as np
    dtype = np.dtype(dtype)
    n = int(np.prod(shape))
    ptr = gpuvm_host_alloc(max(n * dtype.itemsize, 16))
    buf = (C.c_char * (n * dtype.itemsize)).from_address(ptr)
    arr = np.frombuffer(buf, dtype=dtype, count=n).reshape(shape)
    _PINNED[arr.ctypes.data] = ptr
    return arr


_PINNED = {}


def free_pinned(arr):
    ptr = _PINNED.pop(arr.ctypes.data, None)
    if ptr is not None:
        gpuvm_host_free(ptr)


def decode_pte(pte):
    """numpy view of the fields of page-table words."""
    import numpy as np
    pte = np.asarray(pte, np.uint64)
    return dict(pin=(pte & np.uint64(PTE_PIN_MASK)).astype(np.int64),
                gen=((pte & np.uint64(PTE_GEN_MASK)) >> np.uint64(PTE_GEN_SHIFT)).astype(np.int64),
                ref=((pte >> np.uint64(32)) & np.uint64(1)).astype(np.uint8),
                dirty=((pte >> np.uint64(33)) & np.uint64(1)).astype(np.uint8),
                state=((pte >> np.uint64(PTE_STATE_SHIFT)) & np.uint64(3)).astype(np.uint8),
                defer=((pte >> np.uint64(36)) & np.uint64(1)).astype(np.uint8),
                frame=(pte >> np.uint64(PTE_FRAME_SHIFT)).astype(np.int64))

#!/usr/bin/env python3
"""Benchmark of the GPUVM hot path on one MI355X.

A step is one cold-start pass of the whole path (address split, page-table
lookup + reference count, wavefront dedup, inter-wave arbitration, frame
allocation with eviction, dirty write-back, page migration, access, unpin)
over one batch of synthetic input.  Default workload: the random gather at 4x
oversubscription (64 MiB uint32 array in pinned host memory, 4 KiB pages,
16 MiB frame pool, 2^20 uniform indices).

Prints ONE JSON line: the metric (host-link GB/s serviced by GPU-thread page
faults, with faults/s and the fraction of the host-link roofline measured in
the same process), a `roofline` object for the dominant kernel (durations from
HIP events on the launch stream) and a `cpu_baseline` object (the CPU oracle
timed on the host cores).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PCIE5_X16_RAW_GBPS = 64.0      # nominal, per direction; the measured ceiling is what is used


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="gather", choices=["gather", "stream", "bfs", "cc", "sssp", "matvec_t", "matvec", "filter", "vector_add", "vector_add_overwrite", "embedding", "scatter"])
    ap.add_argument("--policy", default="clock", choices=["clock", "fifo", "fifo_wait", "clock_write_aware", "gclock"])
    ap.add_argument("--waves-per-cu", type=int, default=0)
    ap.add_argument("--clock-hands", type=int, default=None, metavar="EIGHTHS",
                    help="CLOCK policies: front hand this many eighths of the ring ahead of the cursor (0 = one hand; default 4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-baselines", action="store_true",
                    help="skip the same-GPU baselines, the hit-path measurements and the dedup step (profiling runs)")
    ap.add_argument("--bfs-naive", action="store_true", help="BFS with vertex-chunk instead of edge-balanced work")
    ap.add_argument("--remote-first", type=int, default=0, metavar="BYTES",
                    help="serve read misses in place until a page has cost its migration; BYTES = what a wavefront reads "
                         "from a page per access (4 for the gather, 512 for the embedding rows); 0 = the paper's behaviour")
    ap.add_argument("--sweep", default=None, choices=["oversubscription", "page_size", "policy", "writeback", "remote_first"],
                    help="instead of the benchmark line: one JSON line per point of a sweep")
    return ap.parse_args()


def ev_pair(torch):
    return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)


def measure_link(gv, torch, np):
    """Host-link read ceiling on this GPU: all-CU wavefront reads of a pinned
    buffer (the mover's own access pattern) and hipMemcpyAsync H2D; GB/s."""
    nbytes = 1 << 30
    h = gv.pinned_array((nbytes,), np.uint8)
    h[:] = 1
    d = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int64, device="cuda")
    ht = torch.from_numpy(h)
    res = {}
    for name, fn in (("wave_read_4k", lambda: gv.gpuvm_bench_read(h, nbytes, 4096, sink, 512)),
                     ("wave_read_64k", lambda: gv.gpuvm_bench_read(h, nbytes, 65536, sink, 512)),
                     ("wave_copy_4k", lambda: gv.gpuvm_bench_copy(d, h, nbytes, 4096, 512)),
                     ("wave_copy_lds_staged_4k", lambda: gv.gpuvm_bench_copy_lds(d, h, nbytes, 4096, 512)),
                     ("wave_copy_64k", lambda: gv.gpuvm_bench_copy(d, h, nbytes, 65536, 512)),
                     ("wave_copy_lds_staged_64k", lambda: gv.gpuvm_bench_copy_lds(d, h, nbytes, 65536, 512)),
                     ("hipMemcpy_h2d", lambda: d.copy_(ht, non_blocking=True)),
                     ("wave_copy_d2h_64k", lambda: gv.gpuvm_bench_copy(h, d, nbytes, 65536, 512)),
                     ("hipMemcpy_d2h", lambda: ht.copy_(d, non_blocking=True))):
        best = 0.0
        fn()
        torch.cuda.synchronize()
        for _ in range(3):
            e0, e1 = ev_pair(torch)
            e0.record(); fn(); e1.record()
            torch.cuda.synchronize()
            best = max(best, nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        res[name] = round(best, 2)
    e0, e1 = ev_pair(torch)
    d2 = torch.empty_like(d)
    gv.gpuvm_bench_copy(d2, d, nbytes, 65536, 4096)
    torch.cuda.synchronize()
    e0.record(); gv.gpuvm_bench_copy(d2, d, nbytes, 65536, 4096); e1.record()
    torch.cuda.synchronize()
    res["hbm_copy_rw"] = round(2 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    e0, e1 = ev_pair(torch)
    gv.gpuvm_bench_copy_lds(d2, d, nbytes, 65536, 4096)
    torch.cuda.synchronize()
    e0.record(); gv.gpuvm_bench_copy_lds(d2, d, nbytes, 65536, 4096); e1.record()
    torch.cuda.synchronize()
    res["hbm_copy_lds_staged_rw"] = round(2 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    # both directions at once (two streams of default priority): the ceiling for
    # a fault that writes a dirty victim back while other waves fetch.  256 waves
    # per direction is where two plain copies peak (48.5 GB/s each way; 45.5 with
    # 1024 per direction, 39.7 with 2048)
    h2 = gv.pinned_array((nbytes,), np.uint8)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    best = 0.0
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        gv.gpuvm_bench_copy(d, h, nbytes, 4096, 256, stream=s1)
        gv.gpuvm_bench_copy(h2, d2, nbytes, 4096, 256, stream=s2)
        torch.cuda.synchronize()
        best = max(best, nbytes / (time.perf_counter() - t0) / 1e9)
    res["duplex_each_direction"] = round(best, 2)
    # unloaded round trip of one 1 KiB wavefront load; with the bandwidth it gives
    # the bytes that must be in flight to fill the link (Little's law)
    lat_host = gv.gpuvm_bench_latency(h, nbytes, 4000)
    lat_hbm = gv.gpuvm_bench_latency(d, nbytes, 4000)
    res["host_load_latency_us"] = round(lat_host / 1e3, 3)
    res["hbm_load_latency_us"] = round(lat_hbm / 1e3, 3)
    res["bytes_in_flight_to_fill_link"] = int(res["wave_read_4k"] * 1e9 * lat_host * 1e-9)
    gv.free_pinned(h2)
    del d, d2, ht
    gv.free_pinned(h)
    return res


def measure_hit_path(gv, torch, np, inputs, oracle, hbm_copy_GBps):
    """Hits only: a 64 MiB uint32 array with a pool that holds all of it, warm, read
    through the paged view - uniform random indices on 4 KiB and on 64 KiB pages,
    and unit stride - against the same gather on a plain array in HBM.  Per
    element the gather moves 4 B of index, 4 B of data and 4 B of output; the
    roofline object prices those 12 B against the HBM copy rate measured in this
    process (random 4-byte reads cost a 64-byte sector each, which is why the
    plain array is far from it too)."""
    n_elems = 1 << 24
    data = inputs.u32_values(0x9E3779B9, 0, n_elems)
    arr = gv.pinned_array(data.shape, data.dtype)
    arr[...] = data
    d_plain = torch.from_numpy(data.view(np.int32)).cuda()
    res = {}

    def best_ms(fn, reps=7):
        ts = []
        for _ in range(reps):
            torch.cuda.synchronize()
            e0, e1 = ev_pair(torch)
            e0.record(); fn(); e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return min(ts)

    for name, page, idx in (("random_4KiB_pages", 4096, inputs.u32_indices(1, 0, 1 << 22, n_elems)),
                            ("random_64KiB_pages", 65536, inputs.u32_indices(1, 0, 1 << 22, n_elems)),
                            ("unit_stride_4KiB_pages", 4096, np.arange(n_elems, dtype=np.uint32)),
                            ("unit_stride_64KiB_pages", 65536, np.arange(n_elems, dtype=np.uint32))):
        n = idx.size
        d_idx = torch.from_numpy(idx.view(np.int32)).cuda()
        d_out = torch.zeros(n, dtype=torch.int32, device="cuda")
        want, _ = oracle.gather(data, idx)
        vm = gv.gpuvm_create(arr.ctypes.data, arr.nbytes, page, arr.nbytes, gv.POLICY_CLOCK)
        try:
            for _ in range(2):
                gv.gpuvm_run_gather(vm, d_idx, n, d_out, None)
            gv.gpuvm_check(vm)
            f0 = gv.gpuvm_stats(vm)["faults"]
            ms = best_ms(lambda: gv.gpuvm_run_gather(vm, d_idx, n, d_out, None))
            ok = bool(np.array_equal(d_out.cpu().numpy().view(np.uint32), want))
            new_faults = gv.gpuvm_stats(vm)["faults"] - f0
        finally:
            gv.gpuvm_destroy(vm)
        ms_plain = best_ms(lambda: gv.gpuvm_bench_gather_plain(d_plain, d_idx, n, d_out))
        ok_plain = bool(np.array_equal(d_out.cpu().numpy().view(np.uint32), want))
        gbps = 12 * n / ms / 1e6
        res[name] = {"G_elem_per_s": round(n / ms / 1e6, 2), "plain_array_G_elem_per_s": round(n / ms_plain / 1e6, 2),
                     "frac_of_plain_array": round(ms_plain / ms, 3), "best_ms": round(ms, 4), "elements": n,
                     "new_faults": new_faults, "parity": ok and ok_plain,
                     "roofline": {"bound": "hbm", "achieved": round(gbps, 1), "peak": hbm_copy_GBps, "unit": "GB/s",
                                  "frac": round(gbps / hbm_copy_GBps, 4), "algorithmic_bytes_per_element": 12}}
        del d_idx, d_out
    gv.free_pinned(arr)
    # the page-level hit path: a wave pins a resident page once and reads all of
    # it (the streaming reduce over an array that fits its pool, warm), against a
    # plain read of the same bytes from HBM
    n_f = 1 << 28
    x = inputs.f32_uniform(7, 0, n_f)
    arr = gv.pinned_array(x.shape, x.dtype)
    arr[...] = x
    block = 1 << 18
    d_s = torch.zeros(n_f // block, dtype=torch.float64, device="cuda")
    d_x = torch.from_numpy(x).cuda()
    sink = torch.zeros(1, dtype=torch.int64, device="cuda")
    vm = gv.gpuvm_create(arr.ctypes.data, arr.nbytes, 65536, arr.nbytes, gv.POLICY_CLOCK)
    try:
        for _ in range(2):
            gv.gpuvm_run_stream_reduce(vm, block, d_s)
        gv.gpuvm_check(vm)
        f0 = gv.gpuvm_stats(vm)["faults"]
        ms = best_ms(lambda: gv.gpuvm_run_stream_reduce(vm, block, d_s))
        new_faults = gv.gpuvm_stats(vm)["faults"] - f0
        want = oracle.stream_reduce(x, block, 1)[0]
        scale = oracle.stream_abs(x, block)
        ok = bool(np.all(np.abs(d_s.cpu().numpy() - want) <= 1e-11 * scale))
    finally:
        gv.gpuvm_destroy(vm)
    ms_plain = best_ms(lambda: gv.gpuvm_bench_read(d_x, arr.nbytes, 65536, sink, 4096))
    gbps = arr.nbytes / ms / 1e6
    res["whole_pages_64KiB"] = {"GBps": round(gbps, 1), "plain_read_GBps": round(arr.nbytes / ms_plain / 1e6, 1),
                                "frac_of_plain_read": round(ms_plain / ms, 3), "best_ms": round(ms, 4), "bytes": int(arr.nbytes),
                                "new_faults": new_faults, "parity": ok,
                                "roofline": {"bound": "hbm", "achieved": round(gbps, 1), "peak": 8000.0, "unit": "GB/s",
                                             "frac": round(gbps / 8000.0, 4), "algorithmic_bytes_per_element": 4,
                                             "peak_source": "published HBM3E peak of the MI355X"}}
    gv.free_pinned(arr)
    del d_x, d_s
    return res


class GatherWorkload:
    """Random gather: 64 MiB uint32 host array, 4 KiB pages, 16 MiB pool, 2^20 indices."""
    name = "random_gather_64MiB_u32_4KiB_pages_16MiB_pool_2^20_idx"
    n_elems, n_idx, page, pool = 1 << 24, 1 << 20, 4096, 16 << 20
    par_baseline = True                              # has an all-cores leg (oracle loops under a parallel-for)
    dtype = "u32"
    kernel = "k_gather"

    def __init__(self, gv, torch, np, inputs, policy):
        self.gv, self.torch, self.np = gv, torch, np
        self.data = inputs.u32_values(0x9E3779B9, 0, self.n_elems)
        self.idx = inputs.u32_indices(1, 0, self.n_idx, self.n_elems)
        self.arr = gv.pinned_array(self.data.shape, self.data.dtype)
        self.arr[...] = self.data
        self.vm = gv.gpuvm_create(self.arr.ctypes.data, self.arr.nbytes, self.page, self.pool, policy)
        self.d_idx = torch.from_numpy(self.idx.view(np.int32)).cuda()
        self.d_out = torch.zeros(self.n_idx, dtype=torch.int32, device="cuda")
        self.d_sum = torch.zeros(1, dtype=torch.int64, device="cuda")
        self.useful_bytes = 4 * self.n_idx

    def launch(self):
        self.gv.gpuvm_run_gather(self.vm, self.d_idx, self.n_idx, self.d_out, self.d_sum)

    def verify(self, oracle):
        want, _ = oracle.gather(self.data, self.idx)
        got = self.d_out.cpu().numpy().view(self.np.uint32)
        return bool(self.np.array_equal(got, want))

    def cpu_baseline(self, oracle, par=False):
        fn = oracle.par_gather if par else oracle.gather
        reps, t = 0, 0.0
        while t < (3.0 if par else 10.0) and reps < 5000:   # about ten seconds of CPU work on the oracle itself
            t0 = time.perf_counter()
            fn(self.data, self.idx)
            t += time.perf_counter() - t0
            reps += 1
        return t / reps, f"whole workload (2^20 gathers on the 64 MiB array), mean of {reps} runs"

    def config(self):
        return {"elements": self.n_elems, "indices": self.n_idx}

    def baselines(self, oracle):
        """The same gather with no paging layer: (a) zero-copy, the kernel
        dereferences the mapped pinned host array directly; (b) hipMallocManaged
        memory.  XNACK demand paging is not available on this machine, so (b) is
        what the runtime does without it (no page migration on fault)."""
        gv, torch, np = self.gv, self.torch, self.np
        want, _ = oracle.gather(self.data, self.idx)
        res = {}

        def timed(ptr):
            ts = []
            for _ in range(4):
                self.d_out.zero_()
                torch.cuda.synchronize()
                e0, e1 = ev_pair(torch)
                e0.record()
                gv.gpuvm_bench_gather_plain(ptr, self.d_idx, self.n_idx, self.d_out)
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            ok = bool(np.array_equal(self.d_out.cpu().numpy().view(np.uint32), want))
            return {"first_ms": round(ts[0], 4), "best_ms": round(min(ts), 4), "parity": ok}

        # hit path: the same gather when every page is resident (pool = data set, warm)
        vm2 = gv.gpuvm_create(self.arr.ctypes.data, self.arr.nbytes, self.page, self.arr.nbytes, 1)
        try:
            for _ in range(2):
                gv.gpuvm_run_gather(vm2, self.d_idx, self.n_idx, self.d_out, None)
            gv.gpuvm_check(vm2)
            f0 = gv.gpuvm_stats(vm2)["faults"]
            ts = []
            for _ in range(5):
                torch.cuda.synchronize()
                e0, e1 = ev_pair(torch)
                e0.record()
                gv.gpuvm_run_gather(vm2, self.d_idx, self.n_idx, self.d_out, None)
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            res["gpuvm_all_resident_hits_only"] = {
                "best_ms": round(min(ts), 4), "new_faults": gv.gpuvm_stats(vm2)["faults"] - f0,
                "G_elem_per_s": round(self.n_idx / (min(ts) * 1e-3) / 1e9, 3),
                "parity": bool(np.array_equal(self.d_out.cpu().numpy().view(np.uint32), want))}
        finally:
            gv.gpuvm_destroy(vm2)
        res["zero_copy_pinned_host"] = timed(self.arr.ctypes.data)
        dd = torch.from_numpy(self.data.view(np.int32)).cuda()
        res["resident_in_hbm_no_paging"] = timed(dd.data_ptr())
        try:
            import ctypes
            hip = ctypes.CDLL("libamdhip64.so")
            p = ctypes.c_void_p()
            rc = hip.hipMallocManaged(ctypes.byref(p), ctypes.c_size_t(self.arr.nbytes), ctypes.c_uint(1))
            if rc != 0 or not p.value:
                raise RuntimeError(f"hipMallocManaged rc={rc}")
            ctypes.memmove(p.value, self.arr.ctypes.data, self.arr.nbytes)
            r = timed(p.value)
            r["note"] = "hipMallocManaged without XNACK (demand paging unavailable on this pool)"
            res["managed_no_xnack"] = r
            hip.hipFree(p)
        except Exception as exc:                     # report, never substitute
            res["managed_no_xnack"] = {"error": str(exc)}
        return res


class StreamWorkload:
    """Streaming read-reduce: 8 GiB fp32 host array, 64 KiB pages, 2 GiB pool, 3 passes."""
    name = "stream_reduce_8GiB_f32_64KiB_pages_2GiB_pool_3_passes"
    n_floats, page, pool, passes, block = 1 << 31, 65536, 2 << 30, 3, 1 << 18
    par_baseline = True                              # has an all-cores leg (oracle loops under a parallel-for)
    dtype = "f64"
    kernel = "k_stream_reduce"

    def __init__(self, gv, torch, np, inputs, policy):
        self.gv, self.torch, self.np, self.inputs = gv, torch, np, inputs
        self.arr = gv.pinned_array((self.n_floats,), np.float32)
        ht = torch.from_numpy(self.arr)
        chunk = 1 << 26
        for lo in range(0, self.n_floats, chunk):                 # same values as inputs.f32_uniform
            ht[lo:lo + chunk].copy_(inputs.t_f32_uniform(7, lo, chunk, "cuda"))
        torch.cuda.synchronize()
        self.vm = gv.gpuvm_create(self.arr.ctypes.data, self.arr.nbytes, self.page, self.pool, policy)
        self.nblocks = self.n_floats // self.block
        self.d_s = torch.zeros((self.passes, self.nblocks), dtype=torch.float64, device="cuda")
        self.useful_bytes = 4 * self.n_floats * self.passes

    def launch(self):
        for p in range(self.passes):
            self.gv.gpuvm_run_stream_reduce(self.vm, self.block, self.d_s[p])

    def verify(self, oracle):
        """Every block of every pass against the oracle's sum of the same block
        (the data do not change between passes, so one oracle pass serves all)."""
        np = self.np
        got = self.d_s.cpu().numpy()
        ok = True
        step = 1 << 10                                              # 1024 blocks = 1 GiB at a time
        for b0 in range(0, self.nblocks, step):
            x = self.arr[b0 * self.block:(b0 + step) * self.block]
            want = oracle.stream_reduce(x, self.block, 1)[0]
            scale = oracle.stream_abs(x, self.block)
            ok &= bool(np.all(np.abs(got[:, b0:b0 + step] - want[None, :]) <= 1e-5 * scale[None, :]))
        return ok

    def cpu_baseline(self, oracle, par=False):
        n = 1 << 28                                                  # 1 GiB of the 8 GiB array, one pass
        t0 = time.perf_counter()
        (oracle.par_stream_reduce if par else oracle.stream_reduce)(self.arr[:n], self.block, 1)
        t = time.perf_counter() - t0
        return t * (self.n_floats / n) * self.passes, "1 GiB of the 8 GiB array, one pass, scaled to 3 passes of 8 GiB"

    def config(self):
        return {"floats": self.n_floats, "passes": self.passes, "block_elems": self.block}


class VectorAddWorkload:
    """The paper's vector addition: C = A + B, three fp32 vectors of 2^31 elements
    (8 GiB each) paged from host, 64 KiB pages, 2 GiB pool each; C is flushed."""
    n, page, pool = 1 << 31, 65536, 2 << 30
    dtype = "f32"
    kernel = "k_vector_add"
    name = "vector_add_3x8GiB_f32_64KiB_pages_2GiB_pools_then_flush"

    def __init__(self, gv, torch, np, inputs, policy):
        self.gv, self.torch, self.np = gv, torch, np
        self.arr = gv.pinned_array((self.n,), np.float32)                   # A
        self.barr = gv.pinned_array((self.n,), np.float32)
        self.carr = gv.pinned_array((self.n,), np.float32)
        ha, hb = torch.from_numpy(self.arr), torch.from_numpy(self.barr)
        for lo in range(0, self.n, 1 << 26):
            ha[lo:lo + (1 << 26)].copy_(inputs.t_f32_uniform(1, lo, 1 << 26, "cuda"))
            hb[lo:lo + (1 << 26)].copy_(inputs.t_f32_uniform(2, lo, 1 << 26, "cuda"))
        torch.cuda.synchronize()
        self.vm = gv.gpuvm_create(self.arr.ctypes.data, self.arr.nbytes, self.page, self.pool, policy)
        self.vmb = gv.gpuvm_create(self.barr.ctypes.data, self.barr.nbytes, self.page, self.pool, policy)
        self.vmc = gv.gpuvm_create(self.carr.ctypes.data, self.carr.nbytes, self.page, self.pool, policy)
        self.useful_bytes = 12 * self.n
        self.run = gv.gpuvm_run_vector_add

    def launch(self):
        gv = self.gv
        gv.gpuvm_reset(self.vmb)
        gv.gpuvm_reset(self.vmc)
        self.run(self.vm, self.vmb, self.vmc, self.n)
        gv.gpuvm_flush(self.vmc)
        sb, sc = gv.gpuvm_stats(self.vmb), gv.gpuvm_stats(self.vmc)
        self.stats_w = {k: sb[k] + sc[k] for k in sb}

    def verify(self, oracle):
        np = self.np
        ok = True
        for lo in np.linspace(0, self.n - (1 << 20), 24).astype(np.int64):
            sl = slice(int(lo), int(lo) + (1 << 20))
            ok &= bool(np.array_equal(self.carr[sl], oracle.vector_add(self.arr[sl], self.barr[sl])))
        return ok

    def cpu_baseline(self, oracle):
        k = 1 << 27
        t0 = time.perf_counter()
        oracle.vector_add(self.arr[:k], self.barr[:k])
        return (time.perf_counter() - t0) * (self.n / k), "2^27 of the 2^31 elements, scaled"

    def config(self):
        return {"elements": self.n}


class VectorAddOverwriteWorkload(VectorAddWorkload):
    """The same addition with C's pages installed without a fetch (a wavefront
    stores whole pages of C): 16 GiB cross the link inwards instead of 24."""
    name = "vector_add_3x8GiB_f32_64KiB_pages_2GiB_pools_then_flush_C_not_fetched"

    def __init__(self, gv, torch, np, inputs, policy):
        super().__init__(gv, torch, np, inputs, policy)
        self.run = gv.gpuvm_run_vector_add_overwrite


class BfsWorkload:
    """BFS from vertex 0 on an R-MAT graph (scale 26, edge factor 16): int32 col_idx
    (4 GiB) paged from host in 64 KiB pages, pool = 25 % of col_idx; row_ptr and
    level live in plain HBM."""
    scale, edge_factor, page = 26, 16, 65536
    par_baseline = True                              # has an all-cores leg (oracle loops under a parallel-for)
    dtype = "i32"
    kernel = "k_bfs_level_balanced"
    naive = False                                    # True: vertex-chunk work distribution (plain CSR)

    def __init__(self, gv, torch, np, inputs, policy, scale=None):
        self.gv, self.torch, self.np = gv, torch, np
        if scale:
            self.scale = scale
        self.name = f"bfs_rmat_scale{self.scale}_ef{self.edge_factor}_col_idx_paged_64KiB_pages_pool_25pct"
        self.nv = 1 << self.scale
        self.d_rp, d_ci = inputs.t_rmat_csr(3, self.scale, "cuda", self.edge_factor)
        self.arr = gv.pinned_array((d_ci.numel(),), np.int32)
        torch.from_numpy(self.arr).copy_(d_ci)
        del d_ci
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        self.pool = (self.arr.nbytes // 4 // self.page) * self.page
        self.vm = gv.gpuvm_create(self.arr.ctypes.data, self.arr.nbytes, self.page, self.pool, policy)
        self.d_level = torch.zeros(self.nv, dtype=torch.int32, device="cuda")
        self.levels = 0
        self.useful_bytes = None                      # edges actually traversed * 4, filled by verify

    def launch(self):
        run = self.gv.gpuvm_run_bfs if self.naive else self.gv.gpuvm_run_bfs_balanced
        self.levels = run(self.vm, self.d_rp, self.nv, 0, self.d_level)

    def verify(self, oracle):
        np = self.np
        rp = self.d_rp.cpu().numpy()
        want = oracle.bfs(rp, self.arr, 0)
        got = self.d_level.cpu().numpy()
        deg = np.diff(rp)
        self.useful_bytes = int(deg[want >= 0].sum()) * 4
        self._rp = rp
        return bool(np.array_equal(got, want))

    def cpu_baseline(self, oracle, par=False):
        t0 = time.perf_counter()
        (oracle.par_bfs if par else oracle.bfs)(self._rp, self.arr, 0)
        return time.perf_counter() - t0, ("whole workload (one sweep over the vertices per level)" if par
                                          else "whole workload (queue BFS over the full graph)")

    def config(self):
        return {"vertices": self.nv, "edges": int(self.arr.size), "levels": self.levels}

    def baselines(self, oracle):
        """The same edge-balanced BFS reading col_idx in place in pinned host memory
        (zero-copy: no page table, no frames), and on a copy of col_idx in HBM."""
        if type(self) is not BfsWorkload or self.naive:
            return {}
        gv, torch, np = self.gv, self.torch, self.np
        want = oracle.bfs(self._rp, self.arr, 0)
        res = {}

        def timed(run):
            ts = []
            for _ in range(3):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                run()
                torch.cuda.synchronize()
                ts.append((time.perf_counter() - t0) * 1e3)
            return {"best_ms": round(min(ts), 3), "parity": bool(np.array_equal(self.d_level.cpu().numpy(), want))}

        res["zero_copy_pinned_host"] = timed(lambda: gv.gpuvm_bench_bfs_zero_copy(self.vm, self.d_rp, self.nv, 0, self.d_level))
        res["zero_copy_pinned_host"]["edge_bytes_needed"] = self.useful_bytes
        return res


class CcWorkload(BfsWorkload):
    """Weakly connected components (label propagation, edge-balanced) on the BFS graph."""
    par_baseline = False
    kernel = "k_cc_round_balanced"

    def __init__(self, gv, torch, np, inputs, policy, scale=None):
        super().__init__(gv, torch, np, inputs, policy, scale)
        self.name = self.name.replace("bfs_", "cc_")

    def launch(self):
        self.levels = self.gv.gpuvm_run_cc_balanced(self.vm, self.d_rp, self.nv, self.d_level)

    def verify(self, oracle):
        np = self.np
        self._rp = self.d_rp.cpu().numpy()
        want = oracle.cc(self._rp, self.arr)
        self.useful_bytes = int(self.arr.nbytes) * self.levels          # every round reads every edge
        return bool(np.array_equal(self.d_level.cpu().numpy(), want))

    def cpu_baseline(self, oracle):
        t0 = time.perf_counter()
        oracle.cc(self._rp, self.arr)
        return time.perf_counter() - t0, "whole workload (label propagation to the fixed point)"


class SsspWorkload(BfsWorkload):
    """SSSP from vertex 0 on the BFS graph; col_idx and the uint32 weights (1..64)
    are both paged from host, each with a pool of 25 % of its size."""
    par_baseline = False
    kernel = "k_sssp_round_balanced"

    def __init__(self, gv, torch, np, inputs, policy, scale=None):
        super().__init__(gv, torch, np, inputs, policy, scale)
        self.name = self.name.replace("bfs_", "sssp_") + "_weights_paged"
        n = self.arr.size
        self.warr = gv.pinned_array((n,), np.uint32)
        hw = torch.from_numpy(self.warr.view(np.int32))
        for lo in range(0, n, 1 << 26):
            k = min(1 << 26, n - lo)
            hw[lo:lo + k].copy_(inputs.t_edge_weights(4, lo, k, "cuda"))
        torch.cuda.synchronize()
        self.vmw = gv.gpuvm_create(self.warr.ctypes.data, self.warr.nbytes, self.page, self.pool, policy)

    def launch(self):
        self.gv.gpuvm_reset(self.vmw)
        self.levels = self.gv.gpuvm_run_sssp_balanced(self.vm, self.vmw, self.d_rp, self.nv, 0, self.d_level)
        self.stats_w = self.gv.gpuvm_stats(self.vmw)

    def verify(self, oracle):
        np = self.np
        self._rp = self.d_rp.cpu().numpy()
        want = oracle.sssp(self._rp, self.arr, self.warr, 0)
        self.useful_bytes = None
        return bool(np.array_equal(self.d_level.cpu().numpy().view(np.uint32), want))

    def cpu_baseline(self, oracle):
        t0 = time.perf_counter()
        oracle.sssp(self._rp, self.arr, self.warr, 0)
        return time.perf_counter() - t0, "whole workload (Bellman-Ford sweeps to the fixed point)"


class MatvecTWorkload:
    """y = A^T x, A 32768 x 32768 fp32 (4 GiB) paged from host, one thread per
    column (column-order access), 64 KiB pages, 1 GiB pool."""
    rows, cols, page, pool = 32768, 32768, 65536, 1 << 30
    dtype = "f64"
    kernel = "k_matvec_t"
    name = "matvec_t_32768x32768_f32_column_order_64KiB_pages_1GiB_pool"

    def __init__(self, gv, torch, np, inputs, policy):
        self.gv, self.torch, self.np = gv, torch, np
        n = self.rows * self.cols
        self.arr = gv.pinned_array((self.rows, self.cols), np.float32)
        ht = torch.from_numpy(self.arr).view(-1)
        for lo in range(0, n, 1 << 26):
            ht[lo:lo + (1 << 26)].copy_(inputs.t_f32_uniform(3, lo, 1 << 26, "cuda"))
        torch.cuda.synchronize()
        self.x = inputs.f32_uniform(4, 0, self.rows)
        self.d_x = torch.from_numpy(self.x).cuda()
        self.d_y = torch.zeros(self.cols, dtype=torch.float64, device="cuda")
        self.vm = gv.gpuvm_create(self.arr.ctypes.data, self.arr.nbytes, self.page, self.pool, policy)
        self.useful_bytes = n * 4

    def launch(self):
        self.gv.gpuvm_run_matvec_t(self.vm, self.rows, self.cols, self.d_x, self.d_y)

    def verify(self, oracle):
        np = self.np
        cols = np.linspace(0, self.cols - 64, 16).astype(np.int64)          # sampled column blocks
        got = self.d_y.cpu().numpy()
        ok = True
        for c in cols:
            want, scale = oracle.matvec_t(np.ascontiguousarray(self.arr[:, c:c + 64]), self.x)
            ok &= bool(np.all(np.abs(got[c:c + 64] - want) <= 1e-5 * scale))
        return ok

    def cpu_baseline(self, oracle):
        sub = self.np.ascontiguousarray(self.arr[:, :1024])
        t0 = time.perf_counter()
        oracle.matvec_t(sub, self.x)
        return (time.perf_counter() - t0) * (self.cols / 1024), "1024 of the 32768 columns, scaled"

    def config(self):
        return {"rows": self.rows, "cols": self.cols}


class MatvecWorkload(MatvecTWorkload):
    """y = A x over the same matrix, one thread per row: the 64 lanes of a
    wavefront stand on 64 different pages and walk along their rows."""
    kernel = "k_matvec_rows"
    name = "matvec_32768x32768_f32_row_per_thread_64KiB_pages_1GiB_pool"

    def __init__(self, gv, torch, np, inputs, policy):
        super().__init__(gv, torch, np, inputs, policy)
        self.x = inputs.f32_uniform(4, 0, self.cols)
        self.d_x = torch.from_numpy(self.x).cuda()
        self.d_y = torch.zeros(self.rows, dtype=torch.float64, device="cuda")

    def launch(self):
        self.gv.gpuvm_run_matvec(self.vm, self.rows, self.cols, self.d_x, self.d_y)

    def verify(self, oracle):
        np = self.np
        got = self.d_y.cpu().numpy()
        ok = True
        for r in np.linspace(0, self.rows - 64, 16).astype(np.int64):     # sampled row blocks
            want, scale = oracle.matvec(self.arr[r:r + 64], self.x)
            ok &= bool(np.all(np.abs(got[r:r + 64] - want) <= 1e-5 * scale))
        return ok

    def cpu_baseline(self, oracle):
        t0 = time.perf_counter()
        oracle.matvec(self.arr[:1024], self.x)
        return (time.perf_counter() - t0) * (self.rows / 1024), "1024 of the 32768 rows, scaled"


class FilterWorkload:
    """Filter-then-gather over two uint32 columns of 2^28 rows (1 GiB each), 4 KiB
    pages, 256 MiB pool per column, selectivity 0.08 %."""
    n, page, pool, sel = 1 << 28, 4096, 256 << 20, 0.0008
    dtype = "u32"
    kernel = "k_filter_sum"
    name = "filter_sum_2x1GiB_u32_columns_4KiB_pages_256MiB_pools_selectivity_0.08pct"

    def __init__(self, gv, torch, np, inputs, policy):
        self.gv, self.torch, self.np = gv, torch, np
        self.arr = gv.pinned_array((self.n,), np.uint32)                    # key column
        self.varr = gv.pinned_array((self.n,), np.uint32)
        hk, hv = torch.from_numpy(self.arr.view(np.int32)), torch.from_numpy(self.varr.view(np.int32))
        for lo in range(0, self.n, 1 << 26):
            hk[lo:lo + (1 << 26)].copy_(inputs.t_u32_values(5, lo, 1 << 26, "cuda"))
            hv[lo:lo + (1 << 26)].copy_(inputs.t_u32_values(6, lo, 1 << 26, "cuda"))
        torch.cuda.synchronize()
        self.thr = 0xFFFFFFFF - int(self.sel * 2 ** 32)
        self.vm = gv.gpuvm_create(self.arr.ctypes.data, self.arr.nbytes, self.page, self.pool, policy)
        self.vmw = gv.gpuvm_create(self.varr.ctypes.data, self.varr.nbytes, self.page, self.pool, policy)
        self.d_c = torch.zeros(1, dtype=torch.int64, device="cuda")
        self.d_s = torch.zeros(1, dtype=torch.int64, device="cuda")
        self.useful_bytes = self.n * 4                                       # the scan itself; matches add 8 B each

    def launch(self):
        self.gv.gpuvm_reset(self.vmw)
        self.gv.gpuvm_run_filter_sum(self.vm, self.vmw, self.thr, self.d_c, self.d_s)
        self.gv.gpuvm_check(self.vmw)
        self.stats_w = self.gv.gpuvm_stats(self.vmw)

    def verify(self, oracle):
        np = self.np
        want = oracle.filter_sum(self.arr, self.varr, self.thr)
        got = (int(self.d_c.cpu().numpy().view(np.uint64)[0]), int(self.d_s.cpu().numpy().view(np.uint64)[0]))
        self.matches = want[0]
        return got == want

    def cpu_baseline(self, oracle):
        t0 = time.perf_counter()
        oracle.filter_sum(self.arr, self.varr, self.thr)
        return time.perf_counter() - t0, "whole workload (2^28 rows)"

    def config(self):
        return {"rows": self.n, "selectivity": self.sel, "matches": getattr(self, "matches", None),
                "value_column_faults": self.stats_w["faults"], "value_column_pages": self.n * 4 // self.page}


class EmbeddingWorkload:
    """Embedding-bag lookup: 5e7 x 128 fp32 table (25.6 GB) in host memory, 64 KiB
    pages, 6.4 GB pool, 20 batches of 65536 bags x 32 Zipf(1.05) ids, sum pooling."""
    rows, dim, page, pool = 50_000_000, 128, 65536, 6_400_000_000
    bags, bag_len, batches = 65536, 32, 20
    par_baseline = True                              # has an all-cores leg (oracle loops under a parallel-for)
    dtype = "f32"
    kernel = "k_embedding_bag"
    name = "embedding_bag_5e7x128_f32_64KiB_pages_6.4GB_pool_20x65536x32_zipf1.05"

    def __init__(self, gv, torch, np, inputs, policy):
        self.gv, self.torch, self.np = gv, torch, np
        self.arr = gv.pinned_array((self.rows, self.dim), np.float32)
        ht = torch.from_numpy(self.arr).view(-1)
        chunk = 1 << 26
        total = self.rows * self.dim
        for lo in range(0, total, chunk):
            n = min(chunk, total - lo)
            ht[lo:lo + n].copy_(inputs.t_f32_uniform(11, lo, n, "cuda"))
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        n_ids = self.batches * self.bags * self.bag_len
        self.ids = inputs.bag_row_ids(5, 0, n_ids, self.rows, 1.05).reshape(self.batches, self.bags, self.bag_len)
        self.d_ids = torch.from_numpy(self.ids).cuda()
        self.d_out = torch.zeros((self.batches, self.bags, self.dim), dtype=torch.float32, device="cuda")
        self.vm = gv.gpuvm_create(self.arr.ctypes.data, self.arr.nbytes, self.page, self.pool, policy)
        self.useful_bytes = n_ids * self.dim * 4

    def launch(self):
        for b in range(self.batches):
            self.gv.gpuvm_run_embedding_bag(self.vm, self.dim, self.d_ids[b], self.bags, self.bag_len, self.d_out[b])

    def verify(self, oracle, sample_bags=512, whole_batches=(0, -1)):
        """Bit-exact against the ordered-fp32 oracle: every bag of the first and the
        last batch (cold pool, and the pool after 19 batches of turnover), and
        `sample_bags` evenly spaced bags of each batch in between."""
        np = self.np
        got = self.d_out.cpu().numpy()
        ok = True
        whole = {b % self.batches for b in whole_batches}
        pick = np.linspace(0, self.bags - 1, sample_bags).astype(np.int64)
        for b in range(self.batches):
            if b in whole:
                ok &= bool(np.array_equal(got[b], oracle.embedding_bag_f32(self.arr, np.ascontiguousarray(self.ids[b]))))
            else:
                ids = np.ascontiguousarray(self.ids[b][pick])
                ok &= bool(np.array_equal(got[b][pick], oracle.embedding_bag_f32(self.arr, ids)))
        return ok

    def cpu_baseline(self, oracle, par=False):
        k = 65536 if par else 4096
        ids = np_contig(self.np, self.ids[0][:k])
        t0 = time.perf_counter()
        (oracle.par_embedding_bag_f32 if par else oracle.embedding_bag_f32)(self.arr, ids)
        t = time.perf_counter() - t0
        return t * (self.bags / k) * self.batches, f"{k} bags of batch 0, scaled to 20 x 65536 bags"

    def config(self):
        return {"rows": self.rows, "dim": self.dim, "bags": self.bags, "bag_len": self.bag_len, "batches": self.batches}

    def baselines(self, oracle):
        """Hit path: one batch of bags over the first 2^21 rows of the table (1 GiB)
        with a pool that holds all of it, warm - against the same pooling by torch
        on a copy of those rows in plain HBM."""
        gv, torch, np = self.gv, self.torch, self.np
        rows = 1 << 21
        sub = self.arr[:rows]
        ids = np_contig(np, (self.ids[0].astype(np.int64) % rows).astype(np.int32))
        d_ids = torch.from_numpy(ids).cuda()
        d_out = torch.zeros((self.bags, self.dim), dtype=torch.float32, device="cuda")
        res = {}

        def best_ms(fn, reps=5):
            ts = []
            for _ in range(reps):
                torch.cuda.synchronize()
                e0, e1 = ev_pair(torch)
                e0.record()
                fn()
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            return min(ts)

        vm2 = gv.gpuvm_create(sub.ctypes.data, sub.nbytes, self.page, sub.nbytes, 1)
        try:
            for _ in range(2):
                gv.gpuvm_run_embedding_bag(vm2, self.dim, d_ids, self.bags, self.bag_len, d_out)
            gv.gpuvm_check(vm2)
            f0 = gv.gpuvm_stats(vm2)["faults"]
            ms = best_ms(lambda: gv.gpuvm_run_embedding_bag(vm2, self.dim, d_ids, self.bags, self.bag_len, d_out))
            pick = np.linspace(0, self.bags - 1, 256).astype(np.int64)
            ok = bool(np.array_equal(d_out.cpu().numpy()[pick], oracle.embedding_bag_f32(sub, np_contig(np, ids[pick]))))
            n = self.bags * self.bag_len
            res["gpuvm_all_resident_hits_only"] = {
                "best_ms": round(ms, 4), "new_faults": gv.gpuvm_stats(vm2)["faults"] - f0,
                "G_rows_per_s": round(n / ms / 1e6, 3), "row_GBps": round(n * self.dim * 4 / ms / 1e6, 1), "parity": ok}
        finally:
            gv.gpuvm_destroy(vm2)
        # zero-copy: the whole job (all batches) with the rows read in place in pinned host memory
        def all_batches():
            for bt in range(self.batches):
                gv.gpuvm_bench_embedding_bag_zero_copy(self.vm, self.dim, self.d_ids[bt], self.bags, self.bag_len, self.d_out[bt])
        ms = best_ms(all_batches, reps=2)
        res["zero_copy_pinned_host_whole_job"] = {"best_ms": round(ms, 2), "parity": self.verify(oracle, sample_bags=64, whole_batches=()),
                                                  "row_GBps": round(self.useful_bytes / ms / 1e6, 1)}
        dev_rows = torch.from_numpy(sub).cuda()
        long_ids = d_ids.long()
        ms = best_ms(lambda: torch.nn.functional.embedding_bag(long_ids, dev_rows, mode="sum"))
        res["torch_embedding_bag_rows_in_hbm"] = {"best_ms": round(ms, 4),
                                                  "G_rows_per_s": round(self.bags * self.bag_len / ms / 1e6, 3)}
        return res


def np_contig(np, a):
    return np.ascontiguousarray(a)


class ScatterWorkload:
    """Scatter-increment with write-back: 32 GiB uint64 host array, 64 KiB pages,
    8 GiB pool, 2^28 atomic +1 at Zipf(0.9) indices, then flush."""
    n_elems, n_upd, page, pool = 1 << 32, 1 << 28, 65536, 8 << 30
    par_baseline = True                              # has an all-cores leg (oracle loops under a parallel-for)
    dtype = "u64"
    kernel = "k_scatter_inc"
    name = "scatter_increment_32GiB_u64_64KiB_pages_8GiB_pool_2^28_zipf0.9_then_flush"

    def __init__(self, gv, torch, np, inputs, policy):
        self.gv, self.torch, self.np = gv, torch, np
        self.arr = gv.pinned_array((self.n_elems,), np.uint64)
        ht = torch.from_numpy(self.arr.view(np.int64))
        z = torch.zeros(1 << 27, dtype=torch.int64, device="cuda")
        for lo in range(0, self.n_elems, 1 << 27):
            ht[lo:lo + (1 << 27)].copy_(z)
        torch.cuda.synchronize()
        del z
        self.idx = np.empty(self.n_upd, np.uint32)
        chunk = 1 << 24
        for lo in range(0, self.n_upd, chunk):
            self.idx[lo:lo + chunk] = inputs.scatter_indices(3, lo, chunk, self.n_elems, 0.9)
        self.d_idx = torch.from_numpy(self.idx.view(np.int32)).cuda()
        self.vm = gv.gpuvm_create(self.arr.ctypes.data, self.arr.nbytes, self.page, self.pool, policy)
        self.useful_bytes = 8 * self.n_upd
        self.rounds = 0
        self.accumulates = True                       # steps add up in the host array (no re-zeroing)

    def launch(self):
        self.gv.gpuvm_run_scatter_increment(self.vm, self.d_idx, self.n_upd)
        self.gv.gpuvm_flush(self.vm)
        self.rounds += 1

    def verify(self, oracle):
        """The whole 32 GiB array, without a second one: (1) the hot head of 2^22
        counters against the oracle run on an array of that size; (2) EVERY
        touched position holds its count - the sorted indices, run-length
        encoded, against the array read at those positions; (3) the grand total
        of the unsigned array equals the number of updates, which with (2)
        proves every untouched element zero."""
        np = self.np
        head = 1 << 22
        want = np.zeros(head, np.uint64)
        oracle.scatter_increment(want, self.idx[self.idx < head])
        ok = bool(np.array_equal(self.arr[:head], want * np.uint64(self.rounds)))
        srt = np.sort(self.idx)
        starts = np.flatnonzero(np.concatenate(([True], srt[1:] != srt[:-1])))
        pos = srt[starts]
        cnt = np.diff(np.concatenate((starts, [srt.size]))).astype(np.uint64)
        del srt, starts
        assert int(cnt.sum()) == self.n_upd
        self.touched = int(pos.size)
        for lo in range(0, pos.size, 1 << 24):
            sl = slice(lo, lo + (1 << 24))
            ok &= bool(np.array_equal(self.arr[pos[sl]], cnt[sl] * np.uint64(self.rounds)))
        total = 0
        for lo in range(0, self.n_elems, 1 << 28):
            total += int(self.arr[lo:lo + (1 << 28)].sum(dtype=np.uint64))
        ok &= total == self.rounds * self.n_upd
        return ok

    def cpu_baseline(self, oracle, par=False):
        n = 1 << (24 if par else 22)
        small = self.np.zeros(self.n_elems >> 6, self.np.uint64)
        t0 = time.perf_counter()
        (oracle.par_scatter_increment if par else oracle.scatter_increment)(small, self.idx[:n] >> 6)
        t = time.perf_counter() - t0
        return t * (self.n_upd / n), f"2^{24 if par else 22} of the 2^28 updates on a 1/64-size array, scaled"

    def config(self):
        return {"elements": self.n_elems, "updates": self.n_upd}

    def baselines(self, oracle):
        """Zero-copy form of the same job: every update a system-scope atomic executed
        in place in pinned host memory (no page table).  Adds one more round to the
        host array, which the check accounts for."""
        gv, torch = self.gv, self.torch
        gv.gpuvm_reset(self.vm)                       # the handle steps aside: host memory is all there is
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        gv.gpuvm_bench_scatter_plain(self.arr, self.d_idx, self.n_upd)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3
        self.rounds += 1
        return {"zero_copy_pinned_host_atomics": {"ms": round(ms, 1), "M_updates_per_s": round(self.n_upd / ms / 1e3, 2),
                                                  "parity": self.verify(oracle)}}


WORKLOADS = {"gather": GatherWorkload, "stream": StreamWorkload, "bfs": BfsWorkload, "cc": CcWorkload, "sssp": SsspWorkload,
             "matvec_t": MatvecTWorkload, "matvec": MatvecWorkload, "filter": FilterWorkload, "vector_add": VectorAddWorkload, "vector_add_overwrite": VectorAddOverwriteWorkload,
             "embedding": EmbeddingWorkload, "scatter": ScatterWorkload}
DEFAULT_STEPS = {"gather": (20, 3), "stream": (5, 1), "bfs": (3, 1), "cc": (2, 0), "sssp": (2, 0), "matvec_t": (3, 1), "matvec": (3, 1), "filter": (5, 1), "vector_add": (3, 1), "vector_add_overwrite": (3, 1), "embedding": (2, 1), "scatter": (1, 0)}


def timed_ms(torch, fn, reps=3):
    best = float("inf")
    for _ in range(reps):
        torch.cuda.synchronize()
        e0, e1 = ev_pair(torch)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1))
    return best


def sweep_oversubscription(gv, torch, np, inputs, oracle):
    """Slow-down against memory pressure, level = data / pool - 1 (paper:
    Oversubscription Analysis), levels 0..11, both policies, for the random
    gather (64 MiB, 4 KiB pages) and the edge-balanced BFS (R-MAT scale 24,
    1 GiB of col_idx, 64 KiB pages).  Every point is checked against the oracle."""
    levels = [0, 0.25, 0.5, 1, 2, 3, 5, 7, 9, 11]
    n_elems, n_idx, page = 1 << 24, 1 << 20, 4096
    data = inputs.u32_values(0x9E3779B9, 0, n_elems)
    idx = inputs.u32_indices(1, 0, n_idx, n_elems)
    want, _ = oracle.gather(data, idx)
    arr = gv.pinned_array(data.shape, data.dtype)
    arr[...] = data
    d_idx = torch.from_numpy(idx.view(np.int32)).cuda()
    d_out = torch.zeros(n_idx, dtype=torch.int32, device="cuda")
    for pol_name, pol in (("clock", gv.POLICY_CLOCK), ("clock_one_hand", gv.POLICY_CLOCK), ("clock_hands_6_eighths", gv.POLICY_CLOCK),
                          ("fifo", gv.POLICY_FIFO), ("fifo_wait", gv.POLICY_FIFO_WAIT), ("gclock", gv.POLICY_GCLOCK),
                          ("clock_remote_first", gv.POLICY_CLOCK)):
        base = None
        for lv in levels:
            pool = int(arr.nbytes / (lv + 1)) // page * page
            vm = gv.gpuvm_create(arr.ctypes.data, arr.nbytes, page, pool, pol)
            if pol_name.endswith("remote_first"):
                gv.gpuvm_set_remote_first(vm, 4)          # reads in place until a page has cost its migration
            if pol_name == "clock_one_hand":
                gv.gpuvm_set_clock_hands(vm, 0)
            if pol_name == "clock_hands_6_eighths":
                gv.gpuvm_set_clock_hands(vm, 6)

            def run():
                gv.gpuvm_reset(vm)
                gv.gpuvm_run_gather(vm, d_idx, n_idx, d_out, None)
            ms = timed_ms(torch, run)
            gv.gpuvm_check(vm)
            st = gv.gpuvm_stats(vm)
            ok = bool(np.array_equal(d_out.cpu().numpy().view(np.uint32), want))
            base = base or ms
            print(json.dumps({"sweep": "oversubscription", "workload": "random_gather_64MiB_4KiB_pages", "policy": pol_name,
                              "level": lv, "pool_bytes": pool, "ms": round(ms, 3), "slowdown_vs_level0": round(ms / base, 3),
                              "faults": st["faults"], "passes_per_fault": round(st["alloc_sweeps"] / max(st["faults"], 1), 3),
                              "link_in_GBps": round(st["bytes_in"] / ms / 1e6, 2), "parity": ok}), flush=True)
            gv.gpuvm_destroy(vm)
    gv.free_pinned(arr)
    scale, page = 24, 65536
    d_rp, d_ci = inputs.t_rmat_csr(3, scale, "cuda")
    carr = gv.pinned_array((d_ci.numel(),), np.int32)
    torch.from_numpy(carr).copy_(d_ci)
    del d_ci
    torch.cuda.synchronize()
    nv = 1 << scale
    want = oracle.bfs(d_rp.cpu().numpy(), carr, 0)
    d_level = torch.zeros(nv, dtype=torch.int32, device="cuda")
    for pol_name, pol in (("clock", gv.POLICY_CLOCK), ("fifo", gv.POLICY_FIFO), ("fifo_wait", gv.POLICY_FIFO_WAIT)):
        base = None
        for lv in levels:
            pool = int(carr.nbytes / (lv + 1)) // page * page
            vm = gv.gpuvm_create(carr.ctypes.data, carr.nbytes, page, pool, pol)

            def run():
                gv.gpuvm_reset(vm)
                gv.gpuvm_run_bfs_balanced(vm, d_rp, nv, 0, d_level)
            ms = timed_ms(torch, run)
            st = gv.gpuvm_stats(vm)
            ok = bool(np.array_equal(d_level.cpu().numpy(), want))
            base = base or ms
            print(json.dumps({"sweep": "oversubscription", "workload": "bfs_balanced_rmat24_64KiB_pages", "policy": pol_name,
                              "level": lv, "pool_bytes": pool, "ms": round(ms, 3), "slowdown_vs_level0": round(ms / base, 3),
                              "faults": st["faults"], "link_in_GBps": round(st["bytes_in"] / ms / 1e6, 2), "parity": ok}), flush=True)
            gv.gpuvm_destroy(vm)
    gv.free_pinned(carr)
    # the two matrix-vector products of the paper's transfer-bound applications
    # (access along columns: the case in which its UVM baseline degrades worst)
    n, page = 16384, 65536
    marr = gv.pinned_array((n, n), np.float32)
    torch.from_numpy(marr).view(-1).copy_(inputs.t_f32_uniform(3, 0, n * n, "cuda"))
    torch.cuda.synchronize()
    x = inputs.f32_uniform(4, 0, n)
    d_x = torch.from_numpy(x).cuda()
    d_y = torch.zeros(n, dtype=torch.float64, device="cuda")
    for name, run_fn, ref_fn in (("matvec_t_16384x16384_column_order_64KiB_pages", gv.gpuvm_run_matvec_t, oracle.matvec_t),
                                 ("matvec_16384x16384_row_per_thread_64KiB_pages", gv.gpuvm_run_matvec, oracle.matvec)):
        want, scale = ref_fn(marr, x)
        base = None
        for lv in levels:
            pool = int(marr.nbytes / (lv + 1)) // page * page
            vm = gv.gpuvm_create(marr.ctypes.data, marr.nbytes, page, pool, gv.POLICY_CLOCK)

            def run():
                gv.gpuvm_reset(vm)
                run_fn(vm, n, n, d_x, d_y)
            ms = timed_ms(torch, run)
            gv.gpuvm_check(vm)
            st = gv.gpuvm_stats(vm)
            ok = bool(np.all(np.abs(d_y.cpu().numpy() - want) <= 1e-5 * scale))
            base = base or ms
            print(json.dumps({"sweep": "oversubscription", "workload": name, "policy": "clock",
                              "level": lv, "pool_bytes": pool, "ms": round(ms, 3), "slowdown_vs_level0": round(ms / base, 3),
                              "faults": st["faults"], "link_in_GBps": round(st["bytes_in"] / ms / 1e6, 2), "parity": ok}), flush=True)
            gv.gpuvm_destroy(vm)
    gv.free_pinned(marr)


def sweep_page_size(gv, torch, np, inputs, oracle):
    """Fault throughput against page size, 4 KiB .. 1 MiB (the paper's transfer
    benchmark, Comparison with GPUDirect RDMA: one page per warp, flat from 4 KiB
    up), on a cyclic streaming read (2 GiB fp32, pool 512 MiB, 2 passes: every
    page access faults) and on the random gather (64 MiB)."""
    n_floats, passes = 1 << 29, 2
    arr = gv.pinned_array((n_floats,), np.float32)
    ht = torch.from_numpy(arr)
    for lo in range(0, n_floats, 1 << 26):
        ht[lo:lo + (1 << 26)].copy_(inputs.t_f32_uniform(7, lo, 1 << 26, "cuda"))
    torch.cuda.synchronize()
    block = 1 << 18
    sample = np.linspace(0, n_floats // block - 1, 32).astype(np.int64)
    want = np.array([oracle.stream_reduce(arr[b * block:(b + 1) * block], block, 1)[0, 0] for b in sample])
    scale = np.array([oracle.stream_abs(arr[b * block:(b + 1) * block], block)[0] for b in sample])
    d_s = torch.zeros(n_floats // block, dtype=torch.float64, device="cuda")
    for shift in range(12, 21):
        page = 1 << shift
        vm = gv.gpuvm_create(arr.ctypes.data, arr.nbytes, page, 512 << 20, gv.POLICY_CLOCK)

        def run():
            gv.gpuvm_reset(vm)
            for _ in range(passes):
                gv.gpuvm_run_stream_reduce(vm, block, d_s)
        ms = timed_ms(torch, run)
        gv.gpuvm_check(vm)
        st = gv.gpuvm_stats(vm)
        ok = bool(np.all(np.abs(d_s.cpu().numpy()[sample] - want) <= 1e-5 * scale))
        print(json.dumps({"sweep": "page_size", "workload": "stream_2GiB_pool_512MiB_2_passes", "page_bytes": page,
                          "ms": round(ms, 3), "faults": st["faults"], "faults_per_s": round(st["faults"] / ms * 1e3),
                          "link_in_GBps": round(st["bytes_in"] / ms / 1e6, 2), "waves": gv.gpuvm_max_waves(vm), "parity": ok}), flush=True)
        gv.gpuvm_destroy(vm)
    gv.free_pinned(arr)
    n_elems, n_idx = 1 << 24, 1 << 20
    data = inputs.u32_values(0x9E3779B9, 0, n_elems)
    idx = inputs.u32_indices(1, 0, n_idx, n_elems)
    want, _ = oracle.gather(data, idx)
    garr = gv.pinned_array(data.shape, data.dtype)
    garr[...] = data
    d_idx = torch.from_numpy(idx.view(np.int32)).cuda()
    d_out = torch.zeros(n_idx, dtype=torch.int32, device="cuda")
    for shift in range(12, 19):
        page = 1 << shift
        vm = gv.gpuvm_create(garr.ctypes.data, garr.nbytes, page, 16 << 20, gv.POLICY_CLOCK)

        def run():
            gv.gpuvm_reset(vm)
            gv.gpuvm_run_gather(vm, d_idx, n_idx, d_out, None)
        ms = timed_ms(torch, run)
        gv.gpuvm_check(vm)
        st = gv.gpuvm_stats(vm)
        ok = bool(np.array_equal(d_out.cpu().numpy().view(np.uint32), want))
        print(json.dumps({"sweep": "page_size", "workload": "random_gather_64MiB_pool_16MiB", "page_bytes": page,
                          "ms": round(ms, 3), "faults": st["faults"], "faults_per_s": round(st["faults"] / ms * 1e3),
                          "link_in_GBps": round(st["bytes_in"] / ms / 1e6, 2), "waves": gv.gpuvm_max_waves(vm), "parity": ok}), flush=True)
        gv.gpuvm_destroy(vm)
    gv.free_pinned(garr)
    # edge-balanced BFS (R-MAT scale 24, 1 GiB of col_idx, pool 256 MiB): the paper
    # runs its graph workloads on 8 KiB pages against UVM's 64 KiB
    scale = 24
    d_rp, d_ci = inputs.t_rmat_csr(3, scale, "cuda")
    carr = gv.pinned_array((d_ci.numel(),), np.int32)
    torch.from_numpy(carr).copy_(d_ci)
    del d_ci
    torch.cuda.synchronize()
    nv = 1 << scale
    want = oracle.bfs(d_rp.cpu().numpy(), carr, 0)
    d_level = torch.zeros(nv, dtype=torch.int32, device="cuda")
    for shift in range(12, 21):
        page = 1 << shift
        vm = gv.gpuvm_create(carr.ctypes.data, carr.nbytes, page, 256 << 20, gv.POLICY_CLOCK)

        def run():
            gv.gpuvm_reset(vm)
            gv.gpuvm_run_bfs_balanced(vm, d_rp, nv, 0, d_level)
        ms = timed_ms(torch, run)
        st = gv.gpuvm_stats(vm)
        ok = bool(np.array_equal(d_level.cpu().numpy(), want))
        print(json.dumps({"sweep": "page_size", "workload": "bfs_balanced_rmat24_pool_256MiB", "page_bytes": page,
                          "ms": round(ms, 3), "faults": st["faults"], "faults_per_s": round(st["faults"] / ms * 1e3),
                          "link_in_GBps": round(st["bytes_in"] / ms / 1e6, 2), "link_in_GB": round(st["bytes_in"] / 1e9, 3),
                          "waves": gv.gpuvm_max_waves(vm), "parity": ok}), flush=True)
        gv.gpuvm_destroy(vm)
    gv.free_pinned(carr)


def sweep_policy(gv, torch, np, inputs, oracle):
    """The four eviction policies on a workload that mixes written and read-only
    pages (paper: Comparisons with UVM - write-intensive pages could be kept
    longer than read-intensive ones): a 1 GiB uint64 array, 64 KiB pages, 256 MiB
    pool (4096 frames).  The first eighth of the array is the write region (2048
    pages) in four slices; round r adds 2^16 increments to slice r mod 4 and then
    gathers 512 uniform uint32 elements from the whole array (about 450 faults),
    so a written page is written again a few thousand ring positions later -
    between the second and the third visit of the hand; 256 rounds, then flush.  Checked against the same
    sequence on plain memory."""
    n64, page, pool, rounds, per, reads, slices = 1 << 27, 65536, 256 << 20, 256, 1 << 16, 512, 4
    slice_elems = (n64 >> 3) // slices
    w_idx = [(inputs.u32_indices(100 + r, 0, per, slice_elems) + np.uint32((r % slices) * slice_elems)) for r in range(rounds)]
    r_idx = [inputs.u32_indices(200 + r, 0, reads, n64 << 1) for r in range(rounds)]
    ref = np.zeros(n64, np.uint64)
    want = []
    for r in range(rounds):                                   # the definition, on plain memory
        oracle.scatter_increment(ref, w_idx[r])
        want.append(oracle.gather(ref.view(np.uint32), r_idx[r])[0])
    arr = gv.pinned_array((n64,), np.uint64)
    d_w = [torch.from_numpy(x.view(np.int32)).cuda() for x in w_idx]
    d_r = [torch.from_numpy(x.view(np.int32)).cuda() for x in r_idx]
    d_out = torch.zeros((rounds, reads), dtype=torch.int32, device="cuda")
    for name, pol in (("fifo", gv.POLICY_FIFO), ("fifo_wait", gv.POLICY_FIFO_WAIT), ("clock", gv.POLICY_CLOCK),
                      ("clock_write_aware", gv.POLICY_CLOCK_WRITE_AWARE), ("gclock", gv.POLICY_GCLOCK)):
        arr[...] = 0
        vm = gv.gpuvm_create(arr.ctypes.data, arr.nbytes, page, pool, pol)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for r in range(rounds):
            gv.gpuvm_run_scatter_increment(vm, d_w[r], per)
            gv.gpuvm_run_gather(vm, d_r[r], reads, d_out[r], None)
        gv.gpuvm_flush(vm)
        ms = (time.perf_counter() - t0) * 1e3
        st = gv.gpuvm_stats(vm)
        got = d_out.cpu().numpy().view(np.uint32)
        ok = bool(np.array_equal(arr, ref)) and all(bool(np.array_equal(got[r], want[r])) for r in range(rounds))
        print(json.dumps({"sweep": "policy", "workload": "rotating_increments_and_sparse_gathers_1GiB_u64_64KiB_pages_256MiB_pool",
                          "policy": name, "ms": round(ms, 2), "faults": st["faults"],
                          "writebacks_evict": st["writebacks_evict"], "writebacks_flush": st["writebacks_flush"],
                          "link_in_GB": round(st["bytes_in"] / 1e9, 3), "link_out_GB": round(st["bytes_out"] / 1e9, 3),
                          "alloc_skips": st["alloc_skips"], "alloc_sweeps": st["alloc_sweeps"], "parity": ok}), flush=True)
        gv.gpuvm_destroy(vm)
    gv.free_pinned(arr)


def sweep_writeback(gv, torch, np, inputs, oracle):
    """Faults with a dirty victim, the write-back overlapped with the fetch or
    completed before it (paper: Evaluation, Transfer-bound Applications - the
    synchronous write-back is what its vector addition loses time to).  Uniform
    random increments over a uint64 array much larger than the pool: nearly every
    update faults, and every victim is dirty.  Swept over the page size and the
    number of wavefronts in flight (tiny pools bound it by frames / 2), since the
    overlap shortens one fault and can only pay while the link is not yet full.
    Checked against the histogram."""
    for page, n64, n_upd in ((4096, 1 << 25, 1 << 22), (65536, 1 << 29, 1 << 21)):
        idx = inputs.u32_indices(300, 0, n_upd, n64)
        d_idx = torch.from_numpy(idx.view(np.int32)).cuda()
        arr = gv.pinned_array((n64,), np.uint64)
        quarter = arr.nbytes // 4 // page
        for frames, waves_per_cu, n in ((32, 8, n_upd >> 3), (64, 8, n_upd >> 2), (128, 8, n_upd >> 1), (256, 8, n_upd >> 1),
                                        (quarter, 1, n_upd), (quarter, 4, n_upd), (quarter, 16, n_upd)):
            ref = np.zeros(n64, np.uint64)
            oracle.scatter_increment(ref, idx[:n])
            for name, mode in (("serial", gv.WB_SERIAL), ("overlapped", gv.WB_OVERLAPPED)):
                arr[...] = 0
                vm = gv.gpuvm_create(arr.ctypes.data, arr.nbytes, page, frames * page, gv.POLICY_CLOCK)
                gv.gpuvm_set_writeback_mode(vm, mode)
                gv.gpuvm_set_waves_per_cu(vm, waves_per_cu)
                waves = gv.gpuvm_max_waves_duplex(vm)
                e0, e1 = ev_pair(torch)
                e0.record()
                gv.gpuvm_run_scatter_increment(vm, d_idx, n)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1)
                st = gv.gpuvm_stats(vm)
                gv.gpuvm_flush(vm)
                ok = bool(np.array_equal(arr, ref))
                print(json.dumps({"sweep": "writeback", "workload": f"uniform_increments_u64_{n64 >> 17}MiB",
                                  "page_bytes": page, "frames": frames, "waves": waves, "mode": name, "ms": round(ms, 2),
                                  "faults": st["faults"], "writebacks_evict": st["writebacks_evict"],
                                  "us_per_fault_per_wave": round(ms * 1e3 * waves / max(st["faults"], 1), 2),
                                  "link_in_GBps": round(st["bytes_in"] / ms / 1e6, 2),
                                  "link_out_GBps": round(st["bytes_out"] / ms / 1e6, 2), "parity": ok}), flush=True)
                gv.gpuvm_destroy(vm)
        gv.free_pinned(arr)
        del d_idx


def sweep_remote_first(gv, torch, np, inputs, oracle):
    """How many reads in place before a page migrates?  The rule in
    gpuvm_set_remote_first charges a page for its reads in place and migrates it
    when they have cost one page (rent or buy).  Swept here: the price per read,
    i.e. the number of touches before migration, on the embedding bag (64 KiB
    pages, 512-byte rows: the rule gives 128) and the random gather (4 KiB pages:
    32), from 'migrate at the second touch' to 'never'.  Cold start per point."""
    for cls, points in (("GatherWorkload", (2048, 1024, 512, 256, 128)), ("EmbeddingWorkload", (32768, 8192, 2048, 512, 128))):
        W = globals()[cls](gv, torch, np, inputs, gv.POLICY_CLOCK)
        page = W.page
        for per_touch in (0,) + points + (-1,):
            gv.gpuvm_reset(W.vm)
            if per_touch >= 0:
                gv.gpuvm_set_remote_first(W.vm, per_touch)
                touches = page // max(per_touch, 128) if per_touch else 0
            else:
                # 'never migrate' is the zero-copy kernel of the same workload
                gv.gpuvm_set_remote_first(W.vm, 0)
                base = W.baselines(oracle) if hasattr(W, "baselines") else {}
                zc = base.get("zero_copy_pinned_host_whole_job") or base.get("zero_copy_pinned_host")
                print(json.dumps({"sweep": "remote_first", "workload": W.name, "touches_before_migration": "never (zero-copy kernel)",
                                  "ms": zc.get("best_ms"), "parity": zc.get("parity")}), flush=True)
                continue
            torch.cuda.synchronize()
            e0, e1 = ev_pair(torch)
            e0.record()
            W.launch()
            e1.record()
            torch.cuda.synchronize()
            gv.gpuvm_check(W.vm)
            st = gv.gpuvm_stats(W.vm)
            print(json.dumps({"sweep": "remote_first", "workload": W.name,
                              "touches_before_migration": touches if per_touch else "0 (every miss migrates)",
                              "ms": round(e0.elapsed_time(e1), 2), "pages_migrated": st["faults"], "read_in_place": st["remote_reads"],
                              "link_GB_pages": round(st["bytes_in"] / 1e9, 3), "parity": bool(W.verify(oracle))}), flush=True)
        gv.gpuvm_destroy(W.vm)
        gv.free_pinned(W.arr)
        del W
        torch.cuda.empty_cache()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the paged view is a per-GPU structure: with "
              "several GPUs each would own a frame pool and page table over the same host buffer and "
              "take a slice of the work); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2411_05309_amd as gv
    from paper_2411_05309_amd import inputs
    gv.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    policy = {"clock": gv.POLICY_CLOCK, "fifo": gv.POLICY_FIFO, "fifo_wait": gv.POLICY_FIFO_WAIT,
              "clock_write_aware": gv.POLICY_CLOCK_WRITE_AWARE, "gclock": gv.POLICY_GCLOCK}[args.policy]

    if args.sweep:
        import oracle
        {"oversubscription": sweep_oversubscription, "page_size": sweep_page_size,
         "policy": sweep_policy, "writeback": sweep_writeback, "remote_first": sweep_remote_first}[args.sweep](gv, torch, np, inputs, oracle)
        return
    link = measure_link(gv, torch, np)
    link_peak = max(link["wave_read_4k"], link["wave_read_64k"], link["wave_copy_4k"], link["hipMemcpy_h2d"])

    if args.steps is None:
        args.steps = DEFAULT_STEPS[args.workload][0]
    if args.warmup is None:
        args.warmup = DEFAULT_STEPS[args.workload][1]
    def say(what):                                   # progress of a long run, on stderr
        print(f"[bench {time.strftime('%H:%M:%S')}] {what}", file=sys.stderr, flush=True)

    say(f"host link measured; building the inputs of '{args.workload}'")
    W = WORKLOADS[args.workload](gv, torch, np, inputs, policy)
    say("inputs ready")
    if args.workload == "bfs" and args.bfs_naive:
        W.naive, W.kernel = True, "k_bfs_level"
        W.name += "_vertex_chunks"
    if args.waves_per_cu:
        gv.gpuvm_set_waves_per_cu(W.vm, args.waves_per_cu)
    if args.clock_hands is not None:
        for vm in (W.vm, getattr(W, "vmw", None), getattr(W, "vmb", None), getattr(W, "vmc", None)):
            if vm is not None:
                gv.gpuvm_set_clock_hands(vm, args.clock_hands)
        W.name += f"_clock_hands_{args.clock_hands}_eighths"
    if args.remote_first:
        for vm in (W.vm, getattr(W, "vmw", None)):            # second paged array: the filter's value column
            if vm is not None:
                gv.gpuvm_set_remote_first(vm, args.remote_first)
        W.name += f"_remote_first_{args.remote_first}B_per_touch"

    def step(events=None):
        gv.gpuvm_reset(W.vm)                         # cold start: all INVALID, frames empty
        if events is not None:
            e0, e1 = ev_pair(torch)
            e0.record()
            W.launch()
            e1.record()
            events.append((e0, e1))
        else:
            W.launch()

    for _ in range(args.warmup):
        step()
    gv.gpuvm_check(W.vm)
    torch.cuda.synchronize()
    say(f"{args.warmup} warm-up step(s) done")
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gv.gpuvm_check(W.vm)
    st = gv.gpuvm_stats(W.vm)                        # counters of the last step (reset clears them)
    if hasattr(W, "stats_w"):                        # second paged array (edge weights): add its traffic
        for k in st:
            st[k] += W.stats_w[k]
    kern_s = sum(e0.elapsed_time(e1) for e0, e1 in events) * 1e-3 / len(events)
    step_s = wall / args.steps

    say(f"{args.steps} timed step(s) done, checking against the oracle")
    import oracle
    parity = W.verify(oracle)
    say("checked")

    out = {
        "metric": "effective GB/s (host-link bytes serviced by GPU-thread page faults) at 4x oversubscription",
        "value": round(st["bytes_in"] / step_s / 1e9, 3),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(step_s * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": W.dtype, "data": "synthetic",
        "config": dict({"workload": W.name, "page_bytes": W.page, "frame_pool_bytes": W.pool,
                        "policy": args.policy, "waves_in_flight": (gv.gpuvm_max_waves_duplex if args.workload == "scatter" else
                                            gv.gpuvm_max_waves_streaming if args.workload in ("stream", "embedding") else gv.gpuvm_max_waves)(W.vm),
                        "oversubscription": round(W.arr.nbytes / W.pool, 2)}, **W.config()),
        "faults_per_s": round(st["faults"] / step_s, 1),
        "faults_per_step": st["faults"],
        "evictions_per_step": st["evictions"],
        "useful_GBps": round(W.useful_bytes / step_s / 1e9, 4) if W.useful_bytes else None,
        "io_amplification": round(st["bytes_in"] / W.useful_bytes, 2) if W.useful_bytes else None,
        "frac_of_host_link": round(st["bytes_in"] / step_s / 1e9 / link_peak, 4),
        "link_out_GBps": round(st["bytes_out"] / step_s / 1e9, 3),
        "host_link_measured_GBps": link,
        "parity_vs_oracle": parity,
        "stats_last_step": st,
        "roofline": {
            "bound": "hostlink", "kernel": W.kernel,
            "achieved": round(st["bytes_in"] / kern_s / 1e9, 3),
            "peak": link_peak, "unit": "GB/s",
            "frac": round(st["bytes_in"] / kern_s / 1e9 / link_peak, 4),
            "traffic": None,
            "kernel_ms": round(kern_s * 1e3, 4),
            "peak_source": "measured in this process: best of all-CU wavefront reads of pinned host memory and hipMemcpyAsync H2D",
            "peak_nominal_pcie5_x16": PCIE5_X16_RAW_GBPS,
            "algorithmic_bytes_per_launch": st["bytes_in"],
            "hbm_copy_measured_GBps": link["hbm_copy_rw"],
        },
    }
    tfile = os.path.join(ROOT, "profiles", "traffic_per_launch.txt")
    if os.path.exists(tfile):                       # counters measured with rocprofv3 --pmc, scaled by faults
        for line in open(tfile):
            parts = line.split()
            if len(parts) > 2 and parts[0] == args.workload and parts[1] == W.kernel:
                kv = {k: float(v) for k, v in (p.split("=") for p in parts[2:])}
                scale = st["faults"] / kv["faults"]
                out["roofline"]["traffic"] = int((kv["host_link_read"] + kv.get("host_link_write", 0.0) + kv["hbm_read"] + kv["hbm_write"]) * scale)
                out["roofline"]["traffic_detail"] = {k: int(v * scale) for k, v in kv.items() if k != "faults"}
                out["roofline"]["traffic_source"] = "profiles/traffic_per_launch.txt (rocprofv3 --pmc), scaled by this run's fault count"
    # one more cold step, untimed, with the per-access counters on: what the
    # wavefront dedup and the inter-wave arbitration did (they are off in the
    # timed steps, where they would cost two ballots loops per access)
    if args.workload in ("gather", "filter", "matvec_t", "matvec") and not args.no_baselines:
        gv.gpuvm_configure(W.vm, 0, True)
        step()
        gv.gpuvm_check(W.vm)
        sd = gv.gpuvm_stats(W.vm)
        gv.gpuvm_configure(W.vm, 0, False)
        groups = max(sd["wave_page_groups"], 1)
        out["dedup"] = {
            "lane_accesses": sd["wave_page_groups"] + sd["lanes_coalesced"],
            "wave_page_groups": sd["wave_page_groups"], "lanes_coalesced": sd["lanes_coalesced"],
            "lanes_per_group": round((sd["wave_page_groups"] + sd["lanes_coalesced"]) / groups, 3),
            "hits": sd["hits"], "faults": sd["faults"], "loading_waits": sd["loading_waits"],
            "share_of_groups_that_waited_for_another_wave": round(sd["loading_waits"] / groups, 4),
            "note": "one untimed cold step with access statistics on",
        }
    job = {"gpu_paging": round(step_s, 6)}
    if hasattr(W, "baselines") and not args.no_baselines:
        out["baselines_same_gpu"] = W.baselines(oracle)
        for k, v in out["baselines_same_gpu"].items():
            if isinstance(v, dict) and k.startswith("zero_copy"):
                ms = v.get("best_ms", v.get("ms"))
                if ms:
                    job["gpu_zero_copy"] = round(ms * 1e-3, 6)
    if not args.no_cpu_baseline:
        cpu_s, sample = W.cpu_baseline(oracle)
        useful = W.useful_bytes or 0
        job["cpu_oracle_1_core"] = round(cpu_s, 6)
        out["cpu_baseline"] = {
            "value": round(useful / cpu_s / 1e9, 4) if useful else None, "unit": "useful GB/s",
            "cores": 1, "kind": "oracle", "sample": sample, "job_seconds": round(cpu_s, 6),
            "gpu_useful_GBps": out["useful_GBps"],
            "note": "useful bytes = what the application asked for; the same figure for the GPU path is useful_GBps",
        }
        if getattr(W, "par_baseline", False):
            par_s, par_sample = W.cpu_baseline(oracle, par=True)
            cores = oracle.par_threads()
            job[f"cpu_parallel_for_{cores}_cores"] = round(par_s, 6)
            out["cpu_baseline_all_cores"] = {
                "value": round(useful / par_s / 1e9, 4) if useful else None, "unit": "useful GB/s",
                "cores": cores, "kind": "the oracle's loops under an OpenMP parallel-for (separate build)",
                "sample": par_sample, "job_seconds": round(par_s, 6),
            }
    out["job_seconds"] = job
    if args.workload == "gather" and not args.no_baselines:
        out["hit_path"] = measure_hit_path(gv, torch, np, inputs, oracle, link["hbm_copy_rw"])
    if "gpu_zero_copy" in job:                       # the shortfall (or gain) against reading host memory in place
        out["paging_vs_zero_copy_same_gpu"] = round(job["gpu_zero_copy"] / job["gpu_paging"], 4)
    print(json.dumps(out), flush=True)
    gv.gpuvm_destroy(W.vm)
    gv.free_pinned(W.arr)
    if not parity:
        sys.exit(1)


if __name__ == "__main__":
    main()

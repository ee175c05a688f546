"""CPU oracle for the GPUVM hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``gpuvm_oracle.c`` (plain sequential C, built with
gcc).  Nothing here may be imported by the product package; only ``tests/``,
``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg use it.

Part 1 (``gather``, ``stream_reduce``, ``bfs``, ``cc``, ``sssp``,
``embedding_bag``, ``scatter_increment``): each workload computed directly on ordinary memory --
the definition of the result, since GPUVM's paging is transparent to the
application (paper, System Overview, vector-addition listing).

Part 2 (``PagingSim``): the sequential simulator of the paged memory system
(paper, "Paged Memory System Design" and "Oversubscription Analysis").
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gpuvm_oracle.c")
_LIB = os.path.join(_HERE, "libgpuvm_oracle.so")
_SRC_PAR = os.path.join(_HERE, "gpuvm_oracle_par.c")
_LIB_PAR = os.path.join(_HERE, "libgpuvm_oracle_par.so")

FIFO, CLOCK, CLOCK_WA, GCLOCK = 0, 1, 3, 4
READ, WRITE, ADD = 0, 1, 2
COUNTER_NAMES = ("faults", "hits", "evictions", "writebacks_evict",
                 "writebacks_flush", "skips", "sweeps", "phases")


def build(force=False):
    """Compile the oracle with gcc (no optimisation tricks, no OpenMP), and the
    separate all-cores build of the Part 1 loops that only the benchmark's
    cpu_baseline leg times (the same loops under an OpenMP parallel-for)."""
    if (force or not os.path.exists(_LIB_PAR)
            or os.path.getmtime(_LIB_PAR) < os.path.getmtime(_SRC_PAR)):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", _LIB_PAR, _SRC_PAR])
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared",
                           "-Wall", "-Wextra", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        vp, u64, i64 = C.c_void_p, C.c_uint64, C.c_int64
        L.oracle_gather.argtypes = [vp, vp, u64, vp, vp]
        L.oracle_vector_add.argtypes = [vp, vp, vp, u64]
        L.oracle_stream_reduce.argtypes = [vp, u64, u64, C.c_int, vp]
        L.oracle_stream_abs.argtypes = [vp, u64, u64, vp]
        L.oracle_bfs.argtypes = [vp, vp, i64, i64, vp]
        L.oracle_bfs.restype = C.c_int
        L.oracle_cc.argtypes = [vp, vp, i64, vp]
        L.oracle_cc.restype = C.c_int
        L.oracle_sssp.argtypes = [vp, vp, vp, i64, i64, vp]
        L.oracle_sssp.restype = C.c_int
        for f in (L.oracle_embedding_bag, L.oracle_embedding_bag_f32,
                  L.oracle_embedding_bag_abs):
            f.argtypes = [vp, u64, vp, u64, u64, vp]
        L.oracle_scatter_increment.argtypes = [vp, vp, u64]
        L.oracle_matvec_t.argtypes = [vp, u64, u64, vp, vp, vp]
        L.oracle_matvec.argtypes = [vp, u64, u64, vp, vp, vp]
        L.oracle_filter_sum.argtypes = [vp, vp, u64, C.c_uint32, vp, vp]
        L.sim_create.argtypes = [vp, u64, u64, u64, C.c_int]
        L.sim_create.restype = vp
        L.sim_destroy.argtypes = [vp]
        L.sim_phase.argtypes = [vp, vp, vp, vp, u64, vp]
        L.sim_phase.restype = C.c_int
        L.sim_run.argtypes = [vp, vp, vp, vp, u64, u64, vp]
        L.sim_run.restype = C.c_int
        L.sim_set_spread.argtypes = [vp, u64]
        L.sim_set_spread.restype = C.c_int
        L.sim_flush.argtypes = [vp]
        L.sim_counters.argtypes = [vp, vp]
        L.sim_hand.argtypes = [vp]
        L.sim_hand.restype = u64
        L.sim_state.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        _lib = L
    return _lib


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


# ---------------------------------------------------------------- Part 1

def gather(host, idx):
    """out[k] = host[idx[k]] (uint32) and the uint64 sum of out."""
    host = _arr(host, np.uint32)
    idx = _arr(idx, np.uint32)
    assert idx.size == 0 or int(idx.max()) < host.size
    out = np.empty(idx.size, np.uint32)
    s = np.zeros(1, np.uint64)
    lib().oracle_gather(_p(host), _p(idx), idx.size, _p(out), _p(s))
    return out, int(s[0])


def vector_add(a, b):
    """c[i] = a[i] + b[i] in fp32."""
    a = _arr(a, np.float32)
    b = _arr(b, np.float32)
    assert a.shape == b.shape
    c = np.empty_like(a)
    lib().oracle_vector_add(_p(a), _p(b), _p(c), a.size)
    return c


def stream_reduce(x, block_elems, passes):
    """fp64 sums of consecutive blocks, index order; shape [passes, nblocks]."""
    x = _arr(x, np.float32)
    nb = (x.size + block_elems - 1) // block_elems
    s = np.empty((passes, nb), np.float64)
    lib().oracle_stream_reduce(_p(x), x.size, block_elems, passes, _p(s))
    return s


def stream_abs(x, block_elems):
    x = _arr(x, np.float32)
    nb = (x.size + block_elems - 1) // block_elems
    s = np.empty(nb, np.float64)
    lib().oracle_stream_abs(_p(x), x.size, block_elems, _p(s))
    return s


def bfs(row_ptr, col_idx, src=0):
    """Hop distance from src per vertex, -1 if unreachable (int32)."""
    row_ptr = _arr(row_ptr, np.int64)
    col_idx = _arr(col_idx, np.int32)
    nv = row_ptr.size - 1
    assert 0 <= src < nv and row_ptr[-1] == col_idx.size
    level = np.empty(nv, np.int32)
    rc = lib().oracle_bfs(_p(row_ptr), _p(col_idx), nv, src, _p(level))
    if rc:
        raise MemoryError("oracle_bfs")
    return level


def cc(row_ptr, col_idx):
    """Smallest vertex id of each vertex's weakly connected component (int32)."""
    row_ptr = _arr(row_ptr, np.int64)
    col_idx = _arr(col_idx, np.int32)
    nv = row_ptr.size - 1
    assert row_ptr[-1] == col_idx.size
    label = np.empty(nv, np.int32)
    lib().oracle_cc(_p(row_ptr), _p(col_idx), nv, _p(label))
    return label


def sssp(row_ptr, col_idx, weight, src=0):
    """Shortest-path distance from src with uint32 edge weights; 0xFFFFFFFF = unreachable."""
    row_ptr = _arr(row_ptr, np.int64)
    col_idx = _arr(col_idx, np.int32)
    weight = _arr(weight, np.uint32)
    nv = row_ptr.size - 1
    assert 0 <= src < nv and row_ptr[-1] == col_idx.size == weight.size
    dist = np.empty(nv, np.uint32)
    lib().oracle_sssp(_p(row_ptr), _p(col_idx), _p(weight), nv, src, _p(dist))
    return dist


def _bag_args(table, ids):
    table = _arr(table, np.float32)
    ids = _arr(ids, np.int32)
    assert table.ndim == 2 and ids.ndim == 2
    assert ids.size == 0 or (0 <= int(ids.min()) and int(ids.max()) < table.shape[0])
    return table, ids


def embedding_bag(table, ids):
    """Sum-pooled bags in double precision; shape [bags, dim]."""
    table, ids = _bag_args(table, ids)
    out = np.empty((ids.shape[0], table.shape[1]), np.float64)
    lib().oracle_embedding_bag(_p(table), table.shape[1], _p(ids), ids.shape[0],
                               ids.shape[1], _p(out))
    return out


def embedding_bag_f32(table, ids):
    """Sum-pooled bags added in listed order in fp32; shape [bags, dim]."""
    table, ids = _bag_args(table, ids)
    out = np.empty((ids.shape[0], table.shape[1]), np.float32)
    lib().oracle_embedding_bag_f32(_p(table), table.shape[1], _p(ids),
                                   ids.shape[0], ids.shape[1], _p(out))
    return out


def embedding_bag_abs(table, ids):
    table, ids = _bag_args(table, ids)
    out = np.empty((ids.shape[0], table.shape[1]), np.float64)
    lib().oracle_embedding_bag_abs(_p(table), table.shape[1], _p(ids),
                                   ids.shape[0], ids.shape[1], _p(out))
    return out


def scatter_increment(host, idx):
    """host[idx[k]] += 1 for every k, in place (uint64 array)."""
    assert host.dtype == np.uint64 and host.flags.c_contiguous
    idx = _arr(idx, np.uint32)
    assert idx.size == 0 or int(idx.max()) < host.size
    lib().oracle_scatter_increment(_p(host), _p(idx), idx.size)
    return host


def matvec(A, x):
    """y = A x in double precision (columns ascending) and sum_j |A[i][j] x[j]| per row."""
    A = _arr(A, np.float32)
    x = _arr(x, np.float32)
    assert A.ndim == 2 and x.shape == (A.shape[1],)
    y = np.empty(A.shape[0], np.float64)
    yabs = np.empty(A.shape[0], np.float64)
    lib().oracle_matvec(_p(A), A.shape[0], A.shape[1], _p(x), _p(y), _p(yabs))
    return y, yabs


def matvec_t(A, x):
    """y = A^T x in double precision and sum_i |A[i][j] x[i]| per column."""
    A = _arr(A, np.float32)
    x = _arr(x, np.float32)
    assert A.ndim == 2 and x.shape == (A.shape[0],)
    y = np.empty(A.shape[1], np.float64)
    yabs = np.empty(A.shape[1], np.float64)
    lib().oracle_matvec_t(_p(A), A.shape[0], A.shape[1], _p(x), _p(y), _p(yabs))
    return y, yabs


def filter_sum(key, val, threshold):
    """(#rows with key > threshold, sum of val over them)."""
    key = _arr(key, np.uint32)
    val = _arr(val, np.uint32)
    assert key.shape == val.shape
    c = np.zeros(1, np.uint64)
    s = np.zeros(1, np.uint64)
    lib().oracle_filter_sum(_p(key), _p(val), key.size, threshold, _p(c), _p(s))
    return int(c[0]), int(s[0])


# ---------------------------------------------------------------- Part 1 on all cores (benchmark baseline only)

_par = None


def par_lib():
    global _par
    if _par is None:
        build()
        L = C.CDLL(_LIB_PAR)
        vp, u64, i64 = C.c_void_p, C.c_uint64, C.c_int64
        L.par_threads.restype = C.c_int
        L.par_gather.argtypes = [vp, vp, u64, vp, vp]
        L.par_stream_reduce.argtypes = [vp, u64, u64, C.c_int, vp]
        L.par_bfs.argtypes = [vp, vp, i64, i64, vp]
        L.par_embedding_bag_f32.argtypes = [vp, u64, vp, u64, u64, vp]
        L.par_scatter_increment.argtypes = [vp, vp, u64]
        _par = L
    return _par


def par_threads():
    """Threads the all-cores leg runs on (OpenMP's choice: the cores the process may use)."""
    return int(par_lib().par_threads())


def par_gather(host, idx):
    host = _arr(host, np.uint32)
    idx = _arr(idx, np.uint32)
    assert idx.size == 0 or int(idx.max()) < host.size
    out = np.empty(idx.size, np.uint32)
    s = np.zeros(1, np.uint64)
    par_lib().par_gather(_p(host), _p(idx), idx.size, _p(out), _p(s))
    return out, int(s[0])


def par_stream_reduce(x, block_elems, passes):
    x = _arr(x, np.float32)
    nb = (x.size + block_elems - 1) // block_elems
    s = np.empty((passes, nb), np.float64)
    par_lib().par_stream_reduce(_p(x), x.size, block_elems, passes, _p(s))
    return s


def par_bfs(row_ptr, col_idx, src=0):
    row_ptr = _arr(row_ptr, np.int64)
    col_idx = _arr(col_idx, np.int32)
    nv = row_ptr.size - 1
    assert 0 <= src < nv and row_ptr[-1] == col_idx.size
    level = np.empty(nv, np.int32)
    par_lib().par_bfs(_p(row_ptr), _p(col_idx), nv, src, _p(level))
    return level


def par_embedding_bag_f32(table, ids):
    table, ids = _bag_args(table, ids)
    out = np.empty((ids.shape[0], table.shape[1]), np.float32)
    par_lib().par_embedding_bag_f32(_p(table), table.shape[1], _p(ids), ids.shape[0], ids.shape[1], _p(out))
    return out


def par_scatter_increment(host, idx):
    assert host.dtype == np.uint64 and host.flags.c_contiguous
    idx = _arr(idx, np.uint32)
    assert idx.size == 0 or int(idx.max()) < host.size
    par_lib().par_scatter_increment(_p(host), _p(idx), idx.size)
    return host


# ---------------------------------------------------------------- Part 2

class PagingSim:
    """Sequential simulator of the circular frame buffer with reference
    counters; policy FIFO, CLOCK, CLOCK_WA (write-aware) or GCLOCK (use count
    0..2); ``spread`` > 0 gives the CLOCK policies a front hand that many
    frames ahead of the cursor (two-handed clock).  ``host`` (uint64 array, modified in place by
    write-backs) is optional: without it only the bookkeeping is simulated and
    ``n_words`` gives the size of the address space in 8-byte words."""

    def __init__(self, page_words, n_frames, policy, host=None, n_words=None, spread=0):
        if host is not None:
            assert host.dtype == np.uint64 and host.flags.c_contiguous
            n_words = host.size
        self.host = host
        self.n_words, self.page_words, self.n_frames = n_words, page_words, n_frames
        self.n_pages = (n_words + page_words - 1) // page_words
        self._s = lib().sim_create(_p(host), n_words, page_words, n_frames, policy)
        if not self._s:
            raise ValueError("sim_create failed")
        if spread and lib().sim_set_spread(self._s, spread):
            raise ValueError("a front hand needs a policy with a reference bit")

    def close(self):
        if self._s:
            lib().sim_destroy(self._s)
            self._s = None

    __del__ = close

    def _prep(self, word_idx, op, val):
        word_idx = _arr(word_idx, np.uint64)
        n = word_idx.size
        if op is None:
            op = np.zeros(n, np.uint8)
        elif np.isscalar(op):
            op = np.full(n, op, np.uint8)
        op = _arr(op, np.uint8)
        if val is not None:
            val = _arr(np.broadcast_to(np.asarray(val, np.uint64), (n,)), np.uint64)
        elif np.any(op != READ):
            val = np.ones(n, np.uint64)
        out = np.zeros(n, np.uint64) if self.host is not None else None
        return word_idx, op, val, out

    @staticmethod
    def _check(rc):
        if rc == -1:
            raise IndexError("access outside the address space")
        if rc == -2:
            raise ValueError("a phase touches more distinct pages than frames")
        if rc:
            raise MemoryError("paging simulator")

    def phase(self, word_idx, op=None, val=None):
        word_idx, op, val, out = self._prep(word_idx, op, val)
        self._check(lib().sim_phase(self._s, _p(word_idx), _p(op), _p(val),
                                    word_idx.size, _p(out)))
        return out

    def run(self, word_idx, op=None, val=None, phase_len=1):
        word_idx, op, val, out = self._prep(word_idx, op, val)
        self._check(lib().sim_run(self._s, _p(word_idx), _p(op), _p(val),
                                  word_idx.size, phase_len, _p(out)))
        return out

    def flush(self):
        lib().sim_flush(self._s)

    @property
    def counters(self):
        c = np.zeros(len(COUNTER_NAMES), np.uint64)
        lib().sim_counters(self._s, _p(c))
        return {k: int(v) for k, v in zip(COUNTER_NAMES, c)}

    @property
    def hand(self):
        return int(lib().sim_hand(self._s))

    def state(self):
        owner = np.empty(self.n_frames, np.int64)
        ref = np.empty(self.n_frames, np.uint8)
        dirty = np.empty(self.n_frames, np.uint8)
        pin = np.empty(self.n_frames, np.uint32)
        where = np.empty(self.n_pages, np.int64)
        defer = np.empty(self.n_frames, np.uint8)
        lib().sim_state(self._s, _p(owner), _p(ref), _p(dirty), _p(pin), _p(where), _p(defer))
        return dict(owner=owner, ref=ref, dirty=dirty, pin=pin, where=where, defer=defer)

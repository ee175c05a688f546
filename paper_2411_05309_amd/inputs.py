"""Seeded synthetic inputs for the five GPUVM workloads.

This module only *draws inputs*; it holds none of the method's arithmetic (no
paging, no gather/reduce/BFS/bag/scatter) and is used by the tests and the
benchmark to feed the same arrays to the CPU oracle and to the HIP library.

Every value is a pure function of (seed, position) -- a counter-based
generator -- so an array can be produced in chunks, on the CPU with numpy or on
the GPU with torch integer ops, with identical results.  Integer formulas are
used wherever both back ends must agree bit for bit; the Zipf-like index draw
uses fp64 ``pow`` and therefore exists in numpy only (it is produced once and
handed to both sides).

Shapes follow the paper's irregular workloads (Evaluation: graph traversal on
skewed graphs, vector streaming, sparse query lookups); the recipe for each
configuration is spelled out in the design notes.
"""
import numpy as np

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15


# ------------------------------------------------------------------ numpy

def splitmix64(seed, counter):
    """64-bit mix of (seed, counter); counter is a uint64 numpy array."""
    with np.errstate(over="ignore"):
        z = counter.astype(np.uint64) * np.uint64(_GOLDEN) + np.uint64((seed * 0xD1B54A32D192ED03 + 0x8CB92BA72F3D8DD7) & _M64)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def xorshift64star(seed, counter):
    """One xorshift64* step applied to a Weyl sequence position (never 0)."""
    with np.errstate(over="ignore"):
        x = (counter.astype(np.uint64) + np.uint64(1)) * np.uint64(_GOLDEN) ^ np.uint64(seed & _M64)
        x = np.where(x == 0, np.uint64(_GOLDEN), x)
        x = x ^ (x >> np.uint64(12))
        x = x ^ (x << np.uint64(25))
        x = x ^ (x >> np.uint64(27))
        return x * np.uint64(0x2545F4914F6CDD1D)


def _counter(lo, n):
    return np.arange(lo, lo + n, dtype=np.uint64)


def u32_values(seed, lo, n):
    """uint32 array values (random gather backing store): top half of xorshift64*."""
    return (xorshift64star(seed, _counter(lo, n)) >> np.uint64(32)).astype(np.uint32)


def u32_indices(seed, lo, n, bound):
    """uniform uint32 indices in [0, bound); bound must be a power of two."""
    assert bound & (bound - 1) == 0 and bound <= 1 << 32
    return ((splitmix64(seed, _counter(lo, n)) >> np.uint64(32)) & np.uint64(bound - 1)).astype(np.uint32)


def f32_uniform(seed, lo, n):
    """fp32 values in [-1, 1) on a 2^-23 grid (exact in fp32)."""
    k = (splitmix64(seed, _counter(lo, n)) >> np.uint64(40)).astype(np.int64)
    return ((k - (1 << 23)).astype(np.float32)) * np.float32(2.0 ** -23)


def zipf_ranks(seed, lo, n, n_items, s):
    """Zipf-like ranks in [1, n_items]: inverse transform of a bounded Pareto
    density ~ r^-s (an O(1) approximation of Zipf(s)); fp64, numpy only."""
    assert s != 1.0
    u = (splitmix64(seed, _counter(lo, n)) >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)
    a = 1.0 - s
    r = np.floor((1.0 + u * ((n_items + 1.0) ** a - 1.0)) ** (1.0 / a))
    return np.clip(r, 1, n_items).astype(np.int64)


def bag_row_ids(seed, lo, n, n_rows, s=1.05, scramble=True):
    """Embedding row ids: Zipf-like popularity; with ``scramble`` the rank is
    spread over the table by a multiplicative bijection (the multiplier must be
    coprime to n_rows), like hot rows in a real table."""
    r = zipf_ranks(seed, lo, n, n_rows, s) - 1
    if scramble:
        mult = 2654435761
        assert np.gcd(mult, n_rows) == 1
        r = (r * mult) % n_rows          # < 2^32 * 2^32 never reached: r < n_rows < 2^31
    return r.astype(np.int32)


def scatter_indices(seed, lo, n, n_items, s=0.9):
    """Scatter-increment targets: Zipf-like, hot head contiguous (rank-1)."""
    return (zipf_ranks(seed, lo, n, n_items, s) - 1).astype(np.uint32)


def rmat_edges(seed, lo, n, scale, a=0.57, b=0.19, c=0.19):
    """R-MAT edges number lo..lo+n-1: per edge and per bit level one draw
    picks the quadrant (integer thresholds on a 32-bit draw).  Duplicates and
    self-loops are kept; vertices are not permuted."""
    ta = int(a * 4294967296.0)
    tb = int((a + b) * 4294967296.0)
    tc = int((a + b + c) * 4294967296.0)
    e = _counter(lo, n)
    src = np.zeros(n, np.int64)
    dst = np.zeros(n, np.int64)
    for lvl in range(scale):
        r = (splitmix64(seed + 1000003 * (lvl + 1), e) >> np.uint64(32)).astype(np.int64)
        sbit = (r >= tb).astype(np.int64)                       # quadrants c, d
        dbit = (((r >= ta) & (r < tb)) | (r >= tc)).astype(np.int64)   # b, d
        src = (src << 1) | sbit
        dst = (dst << 1) | dbit
    return src, dst


def edge_weights(seed, lo, n, max_weight=64):
    """uint32 edge weights in [1, max_weight] (max_weight a power of two), by edge position."""
    assert max_weight & (max_weight - 1) == 0
    return ((splitmix64(seed, _counter(lo, n)) >> np.uint64(40)) & np.uint64(max_weight - 1)).astype(np.uint32) + np.uint32(1)


def csr_from_edges(src, dst, n_vertices, scale):
    """CSR of a directed edge list: rows by source, each row's neighbours in
    ascending order (sort of the combined key), duplicates kept."""
    key = np.sort((src << scale) | dst)
    col_idx = (key & ((1 << scale) - 1)).astype(np.int32)
    counts = np.bincount((key >> scale), minlength=n_vertices)
    row_ptr = np.zeros(n_vertices + 1, np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    return row_ptr, col_idx


def rmat_csr(seed, scale, edge_factor=16, a=0.57, b=0.19, c=0.19):
    nv, ne = 1 << scale, edge_factor << scale
    src, dst = rmat_edges(seed, 0, ne, scale, a, b, c)
    return csr_from_edges(src, dst, nv, scale)


# ------------------------------------------------------------------ torch
# The same integer formulas on int64 tensors (two's-complement wrap-around
# equals arithmetic mod 2^64; logical right shifts are emulated with a mask).

def _s64(v):
    v &= _M64
    return v - (1 << 64) if v >= 1 << 63 else v


def _lsr(x, k):
    return (x >> k) & ((1 << (64 - k)) - 1)


def t_splitmix64(seed, counter):
    z = counter * _s64(_GOLDEN) + _s64(seed * 0xD1B54A32D192ED03 + 0x8CB92BA72F3D8DD7)
    z = (z ^ _lsr(z, 30)) * _s64(0xBF58476D1CE4E5B9)
    z = (z ^ _lsr(z, 27)) * _s64(0x94D049BB133111EB)
    return z ^ _lsr(z, 31)


def t_xorshift64star(seed, counter):
    import torch
    x = ((counter + 1) * _s64(_GOLDEN)) ^ _s64(seed)
    x = torch.where(x == 0, torch.full_like(x, _s64(_GOLDEN)), x)
    x = x ^ _lsr(x, 12)
    x = x ^ (x << 25)
    x = x ^ _lsr(x, 27)
    return x * _s64(0x2545F4914F6CDD1D)


def _t_counter(lo, n, device):
    import torch
    return torch.arange(lo, lo + n, dtype=torch.int64, device=device)


def t_u32_values(seed, lo, n, device):
    """torch twin of ``u32_values``; returned as int32 bit patterns."""
    import torch
    return _lsr(t_xorshift64star(seed, _t_counter(lo, n, device)), 32).to(torch.int32)


def t_u32_indices(seed, lo, n, bound, device):
    import torch
    assert bound & (bound - 1) == 0 and bound <= 1 << 32
    return (_lsr(t_splitmix64(seed, _t_counter(lo, n, device)), 32) & (bound - 1)).to(torch.int32)


def t_f32_uniform(seed, lo, n, device):
    import torch
    k = _lsr(t_splitmix64(seed, _t_counter(lo, n, device)), 40)
    return (k - (1 << 23)).to(torch.float32) * (2.0 ** -23)


def t_edge_weights(seed, lo, n, device, max_weight=64):
    import torch
    return ((_lsr(t_splitmix64(seed, _t_counter(lo, n, device)), 40) & (max_weight - 1)) + 1).to(torch.int32)


def t_rmat_edges(seed, lo, n, scale, device, a=0.57, b=0.19, c=0.19):
    import torch
    ta = int(a * 4294967296.0)
    tb = int((a + b) * 4294967296.0)
    tc = int((a + b + c) * 4294967296.0)
    e = _t_counter(lo, n, device)
    src = torch.zeros(n, dtype=torch.int64, device=device)
    dst = torch.zeros(n, dtype=torch.int64, device=device)
    for lvl in range(scale):
        r = _lsr(t_splitmix64(seed + 1000003 * (lvl + 1), e), 32)
        sbit = (r >= tb).to(torch.int64)
        dbit = (((r >= ta) & (r < tb)) | (r >= tc)).to(torch.int64)
        src = (src << 1) | sbit
        dst = (dst << 1) | dbit
    return src, dst


def t_rmat_csr(seed, scale, device, edge_factor=16, chunk=1 << 26, a=0.57, b=0.19, c=0.19):
    """torch twin of ``rmat_csr`` (edges drawn in chunks, one device sort)."""
    import torch
    nv, ne = 1 << scale, edge_factor << scale
    key = torch.empty(ne, dtype=torch.int64, device=device)
    for lo in range(0, ne, chunk):
        n = min(chunk, ne - lo)
        s, d = t_rmat_edges(seed, lo, n, scale, device, a, b, c)
        key[lo:lo + n] = (s << scale) | d
        del s, d
    key = torch.sort(key).values
    col_idx = (key & ((1 << scale) - 1)).to(torch.int32)
    counts = torch.bincount(key >> scale, minlength=nv)
    del key
    row_ptr = torch.zeros(nv + 1, dtype=torch.int64, device=device)
    torch.cumsum(counts, 0, out=row_ptr[1:])
    return row_ptr, col_idx

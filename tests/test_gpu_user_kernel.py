"""A user's own kernel library (tests/user_kernel/vector_add_user.hip: the
paper's vector-addition listing on the array-like view, written against the two
public headers and built separately from the library) gives the oracle's
result: the boundary works from outside the library's sources, and plain
thread-per-element code - divergent tail, operator[] loads and stores - goes
through the fault path unchanged."""
import ctypes
import os

import numpy as np
import pytest

import oracle
import paper_2411_05309_amd as gv
from paper_2411_05309_amd import inputs

from gpu_util import Backing, check_invariants

pytestmark = pytest.mark.gpu
LIB = os.path.join(os.path.dirname(os.path.abspath(__file__)), "user_kernel", "libuser_vector_add.so")


@pytest.fixture(scope="module")
def user():
    gv.load()
    assert os.path.exists(LIB), "build it first: python -c 'import __graft_entry__ as g; g.build()'"
    lib = ctypes.CDLL(LIB)
    lib.user_vector_add.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_size_t, ctypes.c_void_p]
    lib.user_scale.argtypes = [ctypes.c_void_p, ctypes.c_float, ctypes.c_size_t, ctypes.c_void_p]
    lib.user_accumulate.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.user_gather_pairs.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                      ctypes.c_void_p]
    return lib


@pytest.mark.parametrize("n,page,frames", [(100_003, 4096, 16), (1 << 18, 65536, 8), (37, 4096, 8)])
def test_user_vector_add_and_scale(gpu, user, n, page, frames):
    a = inputs.f32_uniform(1, 0, n)
    b = inputs.f32_uniform(2, 0, n)
    with Backing(a, page, frames * page) as ba, Backing(b, page, frames * page) as bb, \
            Backing(np.full(n, -9.0, np.float32), page, frames * page) as bc:
        assert user.user_vector_add(ba.vm, bb.vm, bc.vm, n, None) == 0
        for x in (ba, bb, bc):
            gv.gpuvm_check(x.vm)
        check_invariants(ba, read_only=True, pristine=a)
        check_invariants(bb, read_only=True, pristine=b)
        check_invariants(bc, read_only=False)
        gv.gpuvm_flush(bc.vm)
        want = oracle.vector_add(a, b)
        assert np.array_equal(bc.arr, want)                              # bit-exact fp32
        # in place on the result: every element is loaded and stored by the same lane
        assert user.user_scale(bc.vm, ctypes.c_float(0.5), n, None) == 0
        gv.gpuvm_check(bc.vm)
        gv.gpuvm_flush(bc.vm)
        assert np.array_equal(bc.arr, want * np.float32(0.5))


@pytest.mark.parametrize("n,page,frames", [(100_003, 4096, 16), (1 << 18, 65536, 8), (37, 4096, 8), (1 << 16, 4096, 64)])
def test_user_cursor_walk(gpu, user, n, page, frames):
    """y += x through a pinned cursor per array (loads and stores on the page the
    wave stands on, moves across page boundaries, a pool smaller than the arrays
    and one that holds them whole)."""
    x = inputs.f32_uniform(3, 0, n)
    y = inputs.f32_uniform(4, 0, n)
    with Backing(x, page, frames * page) as bx, Backing(y, page, frames * page) as by:
        for rounds in (1, 2):
            assert user.user_accumulate(bx.vm, by.vm, n, None) == 0
            gv.gpuvm_check(bx.vm)
            gv.gpuvm_check(by.vm)
        check_invariants(bx, read_only=True, pristine=x)
        check_invariants(by, read_only=False)
        gv.gpuvm_flush(by.vm)
        assert np.array_equal(by.arr, oracle.vector_add(x, oracle.vector_add(x, y)))     # bit-exact fp32, two rounds


@pytest.mark.parametrize("n_elems,page,frames,n", [(1 << 18, 4096, 16, 50_001), (1 << 20, 65536, 8, 30_000), (1 << 16, 4096, 16, 4096)])
def test_user_batched_reads(gpu, user, n_elems, page, frames, n):
    """Two reads per lane in one optimistic transaction (gpuvm_load_n), misses included."""
    import torch
    from gpu_util import dev, host
    data = inputs.u32_values(7, 0, n_elems)
    i0 = inputs.u32_indices(8, 0, n, n_elems)
    i1 = inputs.u32_indices(9, 0, n, n_elems)
    want = oracle.gather(data, i0)[0] + oracle.gather(data, i1)[0]       # uint32, wrapping
    with Backing(data, page, frames * page) as b:
        d_out = torch.zeros(n, dtype=torch.int32, device="cuda")
        d0, d1 = dev(i0), dev(i1)
        gv.gpuvm_configure(b.vm, 0, True)
        assert user.user_gather_pairs(b.vm, d0.data_ptr(), d1.data_ptr(), n, d_out.data_ptr(), None) == 0
        gv.gpuvm_check(b.vm)
        assert np.array_equal(host(d_out, np.uint32), want)
        st, *_ = check_invariants(b, read_only=True, pristine=data)
        assert st["wave_page_groups"] + st["lanes_coalesced"] == 2 * n    # every read is a group of its own or rides on one
        assert st["hits"] + st["faults"] == st["wave_page_groups"]

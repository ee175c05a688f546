"""The allocation-free entry point gpuvm_run_matvec_t_noalloc against the entry
point it is a variant of (gpuvm_run_matvec_t), through the C ABI: the same
result to the bit on two calls in a row that share the static scratch array,
the second on a smaller input; the oracle as well; and the stated limit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2411_05309_amd as gv
from paper_2411_05309_amd import inputs

from gpu_util import Backing, check_invariants, dev

pytestmark = pytest.mark.gpu


def _both(rows, cols, page, frames, seed):
    A = inputs.f32_uniform(seed, 0, rows * cols).reshape(rows, cols)
    x = inputs.f32_uniform(seed + 1, 0, rows)
    want, scale = oracle.matvec_t(A, x)
    with Backing(A, page, frames * page) as b:
        d_x = dev(x)
        y_ref = torch.full((cols,), -1.0, dtype=torch.float64, device="cuda")
        y_new = torch.full((cols,), -2.0, dtype=torch.float64, device="cuda")
        gv.gpuvm_run_matvec_t(b.vm, rows, cols, d_x, y_ref)
        gv.gpuvm_check(b.vm)
        gv.gpuvm_reset(b.vm)                                          # the same cold start for the variant
        gv.gpuvm_run_matvec_t_noalloc(b.vm, rows, cols, d_x, y_new)
        gv.gpuvm_check(b.vm)
        ref, new = y_ref.cpu().numpy(), y_new.cpu().numpy()
        assert np.array_equal(new, ref)                               # same kernels, same summation order: bit-exact
        assert np.all(np.abs(new - want) <= 1e-5 * scale)             # the stated bar against the oracle
        assert np.all(np.abs(new - want) <= 1e-12 * scale + 1e-300)
        check_invariants(b, read_only=True, pristine=A)


def test_noalloc_matvec_t_equals_the_allocating_entry_point(gpu):
    # window and fault-ahead helpers on in both calls (so the scratch array is used);
    # the second input is smaller and leaves most of the array's words from the first call behind
    _both(2048, 4096, 4096, 1024, seed=3)          # 64 compute waves
    _both(1024, 320, 4096, 80, seed=5)             # 5 compute waves (8 launched)
    _both(300, 1000, 4096, 16, seed=7)             # window off: the scratch is cleared but not read


def test_noalloc_matvec_t_refuses_what_the_scratch_cannot_hold(gpu):
    rows, cols = 2, 131072 + 64
    A = inputs.f32_uniform(9, 0, rows * cols).reshape(rows, cols)
    with Backing(A, 4096, 64 * 4096) as b:
        d_x = dev(inputs.f32_uniform(10, 0, rows))
        d_y = torch.zeros(cols, dtype=torch.float64, device="cuda")
        with pytest.raises(gv.GpuvmError) as e:
            gv.gpuvm_run_matvec_t_noalloc(b.vm, rows, cols, d_x, d_y)
        assert e.value.code == gv.ERANGE
        gv.gpuvm_run_matvec_t(b.vm, rows, cols, d_x, d_y)             # the allocating entry point takes it
        gv.gpuvm_check(b.vm)
        want, scale = oracle.matvec_t(A, inputs.f32_uniform(10, 0, rows))
        assert np.all(np.abs(d_y.cpu().numpy() - want) <= 1e-12 * scale + 1e-300)

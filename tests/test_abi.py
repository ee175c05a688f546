"""The C-ABI library loads and exports every symbol include/gpuvm.h declares,
and the Python binding covers exactly that set (no GPU needed, no compute)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "gpuvm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"GPUVM_API\s+[\w\s\*]+?\b(gpuvm_\w+)\s*\(", text)


def test_header_declares_the_boundary():
    names = declared_symbols()
    assert len(names) == len(set(names)) >= 20
    for must in ("gpuvm_create", "gpuvm_destroy", "gpuvm_flush", "gpuvm_stats", "gpuvm_reset",
                 "gpuvm_device_handle", "gpuvm_run_gather", "gpuvm_run_stream_reduce", "gpuvm_run_bfs",
                 "gpuvm_run_embedding_bag", "gpuvm_run_scatter_increment"):
        assert must in names


def test_library_exports_every_declared_symbol():
    import paper_2411_05309_amd as gv
    assert os.path.exists(gv.LIB_PATH), "build libgpuvm.so first (python -m paper_2411_05309_amd.build)"
    lib = ctypes.CDLL(gv.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_binding_covers_exactly_the_header():
    import paper_2411_05309_amd as gv
    assert set(gv._SIGNATURES) == set(declared_symbols())
    for name in declared_symbols():
        assert callable(getattr(gv, name)), f"binding lacks {name}"


def test_strerror_and_struct_layouts():
    import paper_2411_05309_amd as gv
    lib = gv.load()
    assert lib.gpuvm_strerror(0) == b"ok"
    for code in range(-6, 0):
        assert b"unknown" not in lib.gpuvm_strerror(code)
    assert b"unknown" in lib.gpuvm_strerror(-99)
    assert ctypes.sizeof(gv.Stats) == 16 * 8
    assert ctypes.sizeof(gv.Dev) == 6 * 8 + 8 + 6 * 4


def test_device_header_constants_match_binding():
    import paper_2411_05309_amd as gv
    text = open(os.path.join(ROOT, "include", "gpuvm_device.h")).read()
    assert int(re.search(r"GPUVM_PTE_STATE_SHIFT\s+(\d+)", text).group(1)) == gv.PTE_STATE_SHIFT
    assert int(re.search(r"GPUVM_PTE_FRAME_SHIFT\s+(\d+)", text).group(1)) == gv.PTE_FRAME_SHIFT
    order = re.search(r"enum \{\s*GPUVM_S_FAULTS = 0,(.*?)GPUVM_S_COUNT", text, re.S).group(1)
    assert len(re.findall(r"GPUVM_S_\w+", order)) + 1 == len(gv.STAT_NAMES)

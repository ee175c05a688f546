"""Protocol stress of the fault path on the CPU (tests/host_model/): the
device header itself, compiled for the host with every wavefront reduced to one
lane run by one thread, under preemptive interleavings, every policy and both
write-back orders.  The library is not involved: this build exists only here."""
import json
import os
import shutil
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CLANG = next((p for p in ("/opt/rocm/llvm/bin/clang++", shutil.which("clang++") or "") if p and os.path.exists(p)), None)

pytestmark = pytest.mark.skipif(CLANG is None, reason="needs clang++ (the __hip_atomic_* builtins)")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    """The header with its two GPU-only lines replaced (the HIP include and the
    s_waitcnt of wait_vm, which becomes a full fence), then the driver."""
    tmp = tmp_path_factory.mktemp("host_model")
    text = open(os.path.join(ROOT, "include", "gpuvm_device.h")).read()
    for old, new in (('#include <hip/hip_runtime.h>\n', ''),
                     ('asm volatile("s_waitcnt vmcnt(0)" ::: "memory");', '__atomic_thread_fence(__ATOMIC_SEQ_CST);')):
        assert text.count(old) == 1, old
        text = text.replace(old, new)
    hdr = tmp / "gpuvm_device_host.h"
    hdr.write_text(text)
    exe = tmp / "driver"
    cmd = [CLANG, "-std=c++17", "-O1", "-g", "-pthread", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-Wno-everything",      # the shim redefines GPU intrinsics as macros on purpose
           f"-DGPUVM_DEVICE_HEADER=\"{hdr}\"", "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "host_model"),
           os.path.join(HERE, "host_model", "driver.cpp"), "-o", str(exe)]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    return str(exe)


POLICIES = {"fifo": 0, "clock": 1, "fifo_wait": 2, "clock_write_aware": 3, "gclock": 4}


@pytest.mark.parametrize("wb_mode,remote_touches,hands", [(0, 0, 4), (1, 0, 4), (0, 3, 4), (0, 40, 0), (0, 0, 0), (1, 0, 7)])
@pytest.mark.parametrize("policy", sorted(POLICIES))
@pytest.mark.parametrize("threads,frames,page,pages,ops,yield_every", [
    (6, 12, 4096, 40, 6000, 7),        # more threads than cores' worth of luck: yields inside the page copies
    (4, 8, 4096, 64, 8000, 0),         # the smallest pool the launchers accept
    (8, 24, 8192, 48, 4000, 3),
])
def test_fault_protocol_under_host_threads(driver, policy, wb_mode, remote_touches, hands, threads, frames, page, pages,
                                           ops, yield_every):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0")
    for seed in (1, 2):
        r = subprocess.run([driver, str(POLICIES[policy]), str(threads), str(frames), str(page), str(pages), str(ops),
                            str(seed), str(wb_mode), str(yield_every), str(remote_touches), str(hands)],
                           capture_output=True, text=True, timeout=300, env=env)
        assert r.returncode == 0, (r.stdout, r.stderr[-2000:])
        out = json.loads(r.stdout.strip().splitlines()[-1])
        assert out["failures"] == 0
        assert out["evictions"] > 0 and out["writebacks_evict"] > 0 and out["increments"] > 0    # the pool really turned over
        assert (out["remote_reads"] > 0) == (remote_touches > 0)                                 # reads in place happened, or not

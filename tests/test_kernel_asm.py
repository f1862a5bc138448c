"""Host-side check of a hand-placed wait in the decode kernel.

The streaming GEMV copies its input row into LDS ahead of the weights and then waits with
`s_waitcnt vmcnt(N)`, N being the number of vector loads that one fill of the weight ring issues, so
that the copies have landed while the weights stay in flight.  N is computed from the format constants;
this test compiles the kernel to assembly and counts the loads the compiler actually placed between
the copies and each such wait.  A mismatch would mean reading LDS before the copy has landed (too
large an N) or stalling on the weights (too small).
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_wait_after_input_copies_counts_the_ring_loads(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    src = os.path.join(ROOT, "paper_2501_07139_amd", "csrc", "fq_gemv.hip")
    out = str(tmp_path / "fq_gemv.s")
    subprocess.check_call([hipcc, "-O3", "--offload-arch=gfx950", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", "-I", os.path.join(ROOT, "paper_2501_07139_amd", "csrc"), "-I",
                           os.path.join(ROOT, "include"), "-S", "--cuda-device-only", src, "-o", out],
                          stderr=subprocess.DEVNULL)
    lines = open(out).read().splitlines()
    mem_op = re.compile(r"\b(global_load_|global_store|buffer_load|buffer_store|scratch_|flat_load|flat_store)")
    kernel, found = None, 0
    for i, ln in enumerate(lines):
        m = re.match(r"^(_ZN\S*gemv_stream_kernel\S*):", ln)
        if m:
            kernel = m.group(1)
        if "s_endpgm" in ln:
            kernel = None
        m = re.search(r"s_waitcnt vmcnt\((\d+)\)\s*$", ln)
        if not (m and kernel and int(m.group(1)) > 0):
            continue
        if "s_barrier" not in " ".join(lines[i + 1:i + 6]):
            continue  # the compiler's own waits are not followed by the barrier
        n, count, j = int(m.group(1)), 0, i - 1
        while j > 0 and not lines[j].startswith("_ZN") and "global_load_lds" not in lines[j]:
            count += bool(mem_op.search(lines[j]))
            j -= 1
        assert "global_load_lds" in lines[j], (kernel, i + 1)
        assert count == n, "%s line %d: vmcnt(%d) but %d loads issued behind the copies" % (kernel, i + 1, n, count)
        found += 1
    # seven input modes x two row counts x (2-bit whole and split, 3-bit whole and split, 4-bit, 8-bit)
    assert found == 7 * 2 * 6

"""Build libfq.so (HIP kernels + C-ABI) for gfx950, in-tree.

    python paper_2501_07139_amd/build.py

The decode kernel (fq_gemv.hip) copies its input row into LDS, waits for the copies, and then fills its
weight ring.  With FQ_GEMV_COUNTED_WAIT=1 in the environment it is built the other way round: the ring is
issued behind the copies and the kernel waits with a counted `s_waitcnt vmcnt(N)`, N the ring's loads, which
may stay in flight.  That count is a property of the compiled code, so such a build compiles the file to
assembly as well, checks every such wait against the loads the compiler actually placed
(`check_gemv_waits`), and fails if one does not match.  Measured gain of the counted form: none on a
7B-shaped block, 0.8 % on a 13B-shaped one, which is why it is not the default.
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libfq.so")

SOURCES = ["fq_host.cpp", "fq_api.hip", "fq_gemv.hip", "fq_decode.hip", "fq_gemm.hip", "fq_dense.hip", "fq_attn.hip", "fq_rowops.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str, extra=(), asm: bool = False) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + (".s" if asm else ".o"))
    mode = ["-S", "--cuda-device-only"] if asm else ["-c"]
    cmd = [_hipcc(), *FLAGS, *extra, "-x", "hip", *mode, os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("is not a recognized feature for this target", "argument unused during compilation")
    err = "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in noise))
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


GEMV_WAIT_SITES = 7 * 2 * 6  # input modes x row counts x (2-bit whole/split, 3-bit whole/split, 4-bit, 8-bit)


def check_gemv_waits(asm_text: str):
    """Every stand-alone `s_waitcnt vmcnt(N)`, N > 0, directly ahead of a barrier in a gemv_stream_kernel must
    have exactly N vector-memory operations between it and the copies into LDS.  Returns the mismatches."""
    lines = asm_text.splitlines()
    mem_op = re.compile(r"\b(global_load_|global_store|buffer_load|buffer_store|scratch_|flat_load|flat_store)")
    kernel, found, bad = None, 0, []
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
        found += 1
        if "global_load_lds" not in lines[j]:
            bad.append("%s line %d: no copy into LDS ahead of the wait" % (kernel, i + 1))
        elif count != n:
            bad.append("%s line %d: vmcnt(%d) but %d loads issued behind the copies" % (kernel, i + 1, n, count))
    if found != GEMV_WAIT_SITES:
        bad.append("found %d counted waits, expected %d" % (found, GEMV_WAIT_SITES))
    return bad


WAIT_MODE = os.path.join(OBJ, "gemv_wait_mode.txt")  # "counted" or "safe": what the last build chose


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    counted = os.environ.get("FQ_GEMV_COUNTED_WAIT", "0") not in ("", "0")
    gemv_flags = ("-DFQ_GEMV_COUNTED_WAIT",) if counted else ()
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        asm_job = ex.submit(_compile, "fq_gemv.hip", gemv_flags, True)
        objs = list(ex.map(lambda src: _compile(src, gemv_flags if src == "fq_gemv.hip" else ()), SOURCES))
        asm = asm_job.result()
    if counted:
        with open(asm) as fh:
            bad = check_gemv_waits(fh.read())
        if bad:
            raise RuntimeError("fq_gemv.hip: the counted wait does not match the compiled code:\n  " + "\n  ".join(bad[:5]))
    with open(WAIT_MODE, "w") as fh:
        fh.write("counted\n" if counted else "safe\n")
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()

"""Host-side check of a hand-placed wait in the decode kernel.

The streaming GEMV copies its input row into LDS, waits for the copies and then fills its weight ring.  As a
build option (FQ_GEMV_COUNTED_WAIT=1) the ring is issued behind the copies instead and the kernel waits with
`s_waitcnt vmcnt(N)`, N being the number of vector loads that one fill of the ring issues, so that the copies
have landed while the weights stay in flight.  Such a build compiles the kernel to assembly, counts the loads
the compiler actually placed between the copies and each such wait, and fails on a mismatch.  This test pins
both halves: the checker finds planted mistakes, and the library on disk is in a mode the check allows (the
default order has no counted wait at all).
"""
import importlib.util
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _build_module():
    spec = importlib.util.spec_from_file_location("fq_build", os.path.join(ROOT, "paper_2501_07139_amd", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _asm(waits, loads_each, site="_ZN12_GLOBAL__N_118gemv_stream_kernelILi0ELi1EEEvNS_9GemvInputEiiNS_8GemvJobsE"):
    out = [site + ":"]
    for n, k in zip(waits, loads_each):
        out.append("\tglobal_load_lds_dwordx4 v1, v[2:3], off")
        out += ["\tglobal_load_dwordx4 v[4:7], v[8:9], off"] * k
        out += ["\ts_waitcnt vmcnt(%d)" % n, "\ts_waitcnt lgkmcnt(0)", "\ts_barrier"]
    out.append("\ts_endpgm")
    return "\n".join(out)


def test_checker_accepts_matching_counts_and_finds_planted_mistakes():
    b = _build_module()
    n = b.GEMV_WAIT_SITES
    assert b.check_gemv_waits(_asm([6] * n, [6] * n)) == []
    assert any("vmcnt(6) but 5 loads" in m for m in b.check_gemv_waits(_asm([6] * n, [6] * (n - 1) + [5])))   # merged loads
    assert any("vmcnt(6) but 7 loads" in m for m in b.check_gemv_waits(_asm([6] * n, [7] + [6] * (n - 1))))   # a spill
    assert any("expected" in m for m in b.check_gemv_waits(_asm([6] * (n - 1), [6] * (n - 1))))              # a lost site
    assert any("no copy into LDS" in m
               for m in b.check_gemv_waits(_asm([6] * n, [6] * n).replace("global_load_lds_dwordx4", "s_nop", 1)))


def test_the_library_on_disk_was_built_with_a_checked_wait():
    b = _build_module()
    if not (os.path.exists(b.WAIT_MODE) and os.path.exists(b.LIB)):
        b.build(verbose=False)  # a fresh tree: build in place rather than skip (needs hipcc; fails loudly without)
    mode = open(b.WAIT_MODE).read().strip()
    assert mode in ("counted", "safe")
    asm = os.path.join(b.OBJ, "fq_gemv.s")
    assert os.path.exists(asm)
    bad = b.check_gemv_waits(open(asm).read())
    if mode == "counted":
        assert bad == [], bad[:3]
    else:  # the default order: no counted wait ahead of a barrier anywhere in the kernel
        assert any("found 0 counted waits" in m for m in bad) and len(bad) == 1, bad[:3]

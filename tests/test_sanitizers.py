"""AddressSanitizer + UndefinedBehaviorSanitizer over the host code of the library (quantizer, packer, size
queries, rotary table) and over the oracle's C functions: tests/sanitize_host.cpp is compiled together with
both sources for the host (clang, which knows the fp16 type the library's host code uses; no device code)
and run; every buffer in it is an exact-size heap block.  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _clang():
    for cand in ("/opt/rocm/llvm/bin/clang", shutil.which("clang")):
        if cand and os.path.exists(cand):
            return cand
    return None


@pytest.mark.skipif(_clang() is None, reason="needs clang")
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    cc = _clang()
    cxx = cc + "++"
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2501_07139_amd", "csrc")]
    objs = []
    for comp, src, std in ((cc, os.path.join(ROOT, "oracle", "fq_oracle.c"), "-std=c11"),
                           (cxx, os.path.join(ROOT, "paper_2501_07139_amd", "csrc", "fq_host.cpp"), "-std=c++17"),
                           (cxx, os.path.join(ROOT, "tests", "sanitize_host.cpp"), "-std=c++17")):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        res = subprocess.run([comp, std, *san, *inc, "-c", src, "-o", obj], capture_output=True, text=True)
        assert res.returncode == 0, res.stderr
        objs.append(obj)
    exe = str(tmp_path / "sanitize_host")
    # clang links its sanitizer runtime statically into the executable, so nothing has to be preloaded
    res = subprocess.run([cxx, *san, *objs, "-o", exe, "-lm", "-lpthread"], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "sanitize_host: ok" in res.stdout

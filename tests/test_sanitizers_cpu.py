"""CPU sanitizer tier: the library's host eigensolver and the whole CPU oracle under AddressSanitizer and
UndefinedBehaviorSanitizer.

`whiten_host.cpp` (product, host side) and `oracle/lpd_oracle.c` (checker) are compiled with
`-fsanitize=address,undefined -fno-sanitize-recover=all` together with `tests/sanitize_driver.cpp`, which drives
every exported function over small seeded inputs and the degenerate shapes.  Any heap overflow, use after free,
leak, signed overflow, misaligned or out-of-range access aborts the run.  GPU code is not covered (device
sanitizers are not available on this machine).
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.mark.skipif(shutil.which("g++") is None, reason="no g++")
def test_host_eigensolver_and_oracle_under_asan_and_ubsan(tmp_path):
    csrc = os.path.join(ROOT, "paper_2207_01016_amd", "csrc")
    objs = []
    for cc, std, src in (("g++", "-std=c++17", os.path.join(csrc, "whiten_host.cpp")),
                         ("gcc", "-std=c11", os.path.join(ROOT, "oracle", "lpd_oracle.c")),
                         ("g++", "-std=c++17", os.path.join(ROOT, "tests", "sanitize_driver.cpp"))):
        obj = tmp_path / (os.path.basename(src) + ".o")
        subprocess.run([cc, std, *SAN, "-fopenmp", "-mavx2", "-mfma", "-Wall", "-c", src, "-o", str(obj)], check=True)
        objs.append(str(obj))
    exe = tmp_path / "sanitize_driver"
    subprocess.run(["g++", *SAN, "-fopenmp", "-static-libasan", *objs, "-o", str(exe), "-lm"], check=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    res = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=600)
    report = res.stdout + res.stderr
    assert res.returncode == 0, report[-4000:]
    assert "sanitize_driver: ok" in res.stdout
    assert "AddressSanitizer" not in report and "runtime error" not in report, report[-4000:]
    # the same executable with a planted heap overflow must be stopped by the sanitizer
    bad = subprocess.run([str(exe), "plant"], env=env, capture_output=True, text=True, timeout=600)
    assert bad.returncode != 0 and "AddressSanitizer" in bad.stderr

"""The CPU oracle, the input generator and the library's host-side C++ (continuous-batching scheduler, credit ledger)
built with AddressSanitizer and UndefinedBehaviorSanitizer and walked by tests/sanitize/driver.cpp: the run must end
cleanly (no invalid access, no leak, no undefined arithmetic)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_oracle_generator_scheduler_and_ledger_under_asan_and_ubsan(tmp_path):
    objs = []
    for src, cc, std in (("oracle/www_oracle.c", "gcc", "-std=c11"),                       # (its OpenMP pragmas are ignored here)
                         ("paper_2603_20661_amd/synth/wwwsynth.c", "gcc", "-std=c11"),
                         ("paper_2603_20661_amd/csrc/sched.cpp", "g++", "-std=c++17"),
                         ("paper_2603_20661_amd/csrc/ledger.cpp", "g++", "-std=c++17"),
                         ("tests/sanitize/driver.cpp", "g++", "-std=c++17")):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.check_call([cc, std, "-Wall", *SAN, "-c", os.path.join(ROOT, src), "-o", obj])
        objs.append(obj)
    exe = str(tmp_path / "driver")
    # the sanitizer runtimes are linked statically: a dynamic one insists on being the first library of the process
    subprocess.check_call(["g++", *SAN, "-static-libasan", "-static-libubsan", *objs, "-o", exe, "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "all paths walked" in r.stdout

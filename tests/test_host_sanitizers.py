"""AddressSanitizer + UndefinedBehaviorSanitizer over the host code: the C oracle and the library's
host-only translation units (offline tuner, selector) are compiled with gcc -fsanitize=address,
undefined into one executable whose driver (tests/sanitize/driver.cpp) walks their entry points
with exactly-sized buffers and edge cases.  CPU only; GPU code is not sanitized here."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2003_06795_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_oracle_tuner_and_selector_are_clean_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    objs = []
    jobs = [(["gcc", "-std=c11", "-ffp-contract=off"], os.path.join(ROOT, "oracle", "gemm_oracle.c")),
            (["g++", "-std=c++17"], os.path.join(CSRC, "tune.cpp")),
            (["g++", "-std=c++17"], os.path.join(CSRC, "selector.cpp")),
            (["g++", "-std=c++17"], os.path.join(ROOT, "tests", "sanitize", "driver.cpp"))]
    for cc, src in jobs:
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.run(cc + san + ["-c", src, "-o", obj], check=True)
        objs.append(obj)
    exe = str(tmp_path / "driver")
    # the sanitizer runtimes are linked statically so that nothing preloaded into the process can
    # come before them
    subprocess.run(["g++"] + san + ["-static-libasan", "-static-libubsan", "-o", exe] + objs + ["-lm"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, "sanitizer run failed:\n" + r.stdout[-2000:] + r.stderr[-6000:]
    assert "sanitize driver: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr

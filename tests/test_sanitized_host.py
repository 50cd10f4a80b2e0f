"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the library's planner
(planner.cpp, compiled alone with the host compiler: it contains no device code) and the C
checker, each driven by the regular host-side tests in a separate process."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fPIC", "-shared"]


def test_planner_and_checker_are_clean_under_asan_and_ubsan(tmp_path):
    planner = str(tmp_path / "libplanner_san.so")
    checker = str(tmp_path / "liboracle_san.so")
    subprocess.check_call(["g++", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"),
                           "-I", os.path.join(ROOT, "paper_2603_28768_amd", "csrc"),
                           os.path.join(ROOT, "paper_2603_28768_amd", "csrc", "planner.cpp"), "-o", planner])
    subprocess.check_call(["gcc", "-fopenmp", *SAN, os.path.join(ROOT, "oracle", "moe_oracle.c"),
                           "-o", checker, "-lm"])
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    env = dict(os.environ)
    # the sanitizer runtime has to come first; whatever is preloaded already stays behind it
    env["LD_PRELOAD"] = ":".join(p for p in (asan, env.get("LD_PRELOAD", "")) if p)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=66"      # the interpreter itself leaks
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    res = subprocess.run([sys.executable, os.path.join(ROOT, "tests", "sanitized_runner.py"), planner, checker],
                         env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "AddressSanitizer" not in res.stdout + res.stderr, tail
    assert "runtime error:" not in res.stdout + res.stderr, tail
    assert " passed" in res.stdout, tail

"""The CPU checker and the host-side launch planner compiled with AddressSanitizer and
UndefinedBehaviorSanitizer and run on small inputs that reach their corner cases (host code only:
no GPU sanitizer is involved)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# sanitizer runtimes linked statically: they then need not come first among the preloaded libraries
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1",
       "-static-libasan", "-static-libubsan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="4")


def _build_and_run(tmp_path, compiler, sources, extra):
    exe = str(tmp_path / "driver")
    cmd = [compiler] + SAN + extra + sources + ["-o", exe, "-lm"]
    subprocess.check_call(cmd)
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    return r.stdout


def test_checker_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    srcs = [os.path.join(ROOT, "oracle", f) for f in
            ("attention_oracle.c", "sampler_oracle.c", "sampler_filtered_oracle.c")]
    out = _build_and_run(tmp_path, "gcc", srcs + [os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c")],
                         ["-fopenmp", "-fno-fast-math"])
    assert out.strip().endswith("ok")


def test_launch_planner_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    out = _build_and_run(tmp_path, "g++", [os.path.join(ROOT, "tests", "sanitize", "plan_driver.cpp")], ["-std=c++17"])
    assert out.startswith("ok")

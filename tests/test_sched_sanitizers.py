"""The host-only scheduler of the C ABI under AddressSanitizer and
UndefinedBehaviorSanitizer (host code, no GPU): a long pseudo-random trace
must run clean and give the same decisions as an unsanitized build."""

import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = [os.path.join(HERE, "sched_sanitizer_driver.cpp"),
       os.path.join(ROOT, "paper_2503_08461_amd", "csrc", "fc_sched.cpp")]


def _build_and_run(tmp_path, name, flags):
    exe = str(tmp_path / name)
    subprocess.run(["g++", "-std=c++17", "-O1", "-g"] + flags + SRC + ["-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stderr[-3000:]
    return r.stdout.strip()


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_scheduler_trace_is_clean_under_asan_and_ubsan(tmp_path):
    plain = _build_and_run(tmp_path, "plain", [])
    checked = _build_and_run(tmp_path, "checked",
                             ["-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                              "-fno-omit-frame-pointer",
                              # runtimes inside the executable: independent of what else is preloaded
                              "-static-libasan", "-static-libubsan"])
    assert plain == checked and plain.isdigit()

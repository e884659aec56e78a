"""The batching server's threading, checked without a GPU: csrc/batcher.cpp is compiled by g++
under ThreadSanitizer against the CPU stand-in for HIP and a stub of the preprocessing handle
(tests/server_stub), then several threads submit into a deliberately small queue while others
collect.  Every request must come back once with its own bytes, and the sanitizer must stay
silent.  The product never uses this build."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
STUB = os.path.join(ROOT, "tests", "server_stub")
BINARY = os.path.join(STUB, "server_tsan")


def build():
    srcs = [os.path.join(ROOT, "paper_2411_19114_amd", "csrc", "batcher.cpp"), os.path.join(STUB, "stub_main.cpp")]
    deps = srcs + [os.path.join(ROOT, "include", "prep.h"), os.path.join(ROOT, "tests", "hip_emulation", "hip", "hip_runtime.h")]
    if os.path.exists(BINARY) and os.path.getmtime(BINARY) >= max(os.path.getmtime(d) for d in deps):
        return
    # this compiler's ThreadSanitizer does not follow the C library's steady-clock wait
    subprocess.run(["g++", "-std=c++20", "-O1", "-g", "-pthread", "-fsanitize=thread",
                    "-DPREP_WAIT_ON_SYSTEM_CLOCK", "-I",
                    os.path.join(ROOT, "tests", "hip_emulation")] + srcs + ["-o", BINARY], check=True)


def test_submitters_and_collectors_race_free_and_nothing_lost():
    build()
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1 exitcode=66")
    r = subprocess.run([BINARY, "4", "400"], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "bad 0" in r.stdout

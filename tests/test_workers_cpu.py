"""The worker pool of the page-cache path's memcpy hop on its own (no GPU), built with ThreadSanitizer: commands
cut into pieces and pushed as the pipeline pushes them, restarts with other thread counts, threads asleep and
awake, idle and never-started pools.  Any data race or lock-order report fails the run."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_worker_pool_under_thread_sanitizer(tmp_path):
    exe = str(tmp_path / "workers_harness")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-Wall", "-Werror", "-fsanitize=thread", "-pthread", "-I",
           os.path.join(ROOT, "paper_2604_26557_amd", "csrc"), os.path.join(ROOT, "tests", "workers_harness.cpp"), "-o", exe]
    try:
        subprocess.check_call(cmd)
    except subprocess.CalledProcessError:
        pytest.skip("g++ cannot link ThreadSanitizer here")
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1 exitcode=66")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip() == "ok", (r.returncode, r.stdout[-500:], r.stderr[-3000:])

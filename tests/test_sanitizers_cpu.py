"""Host-side sanitizer pass (CPU only): the planner / host logic of the library and the C checker are built with
AddressSanitizer + UndefinedBehaviorSanitizer on their host code and the CPU test files are run again against
those builds in a child process.  Device code is not instrumented and nothing here touches a GPU."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/llvm/bin/clang"
OUT = os.path.join(ROOT, "paper_2604_26557_amd", "_build", "san")
FILES = ["tests/test_planner_cpu.py", "tests/test_oracle_plan.py", "tests/test_oracle_layout.py",
         "tests/test_oracle_attention.py"]


def _runtime():
    hits = glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    return hits[0] if hits else None


def _env(rt, **extra):
    env = dict(os.environ)
    # the sanitizer runtime must be in the process before the instrumented libraries are loaded; whatever is
    # preloaded already stays in front of it
    env["LD_PRELOAD"] = ":".join(x for x in (env.get("LD_PRELOAD"), rt) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra)
    return env


@pytest.fixture(scope="module")
def sanitized():
    rt = _runtime()
    if rt is None or not os.path.exists(CLANG):
        pytest.skip("clang's shared AddressSanitizer runtime is not in this image")
    if subprocess.run([sys.executable, "-c", "pass"], env=_env(rt), capture_output=True).returncode != 0:
        pytest.skip("the interpreter does not start with the sanitizer runtime preloaded here")
    sys.path.insert(0, ROOT)
    from paper_2604_26557_amd import build as native_build
    lib = native_build.build_sanitized(OUT)
    orc = os.path.join(OUT, "libkv_oracle_san.so")
    subprocess.check_call([CLANG, "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fsanitize=address",
                           "-fsanitize=undefined", "-fno-gpu-sanitize", "-shared-libsan", "-fno-omit-frame-pointer", "-o", orc,
                           os.path.join(ROOT, "oracle", "kv_oracle.c"), "-lm"])
    return rt, lib, orc


def test_sanitizer_reports_a_planted_overrun(sanitized, tmp_path):
    """The harness itself: a one-line heap overrun in a scrap C file, built and loaded the same way, must be reported."""
    rt, _, _ = sanitized
    src = tmp_path / "overrun.c"
    src.write_text("#include <stdlib.h>\nint poke(int n) { char *p = malloc(8); p[n] = 1; int r = p[0]; free(p); return r; }\n")
    so = tmp_path / "liboverrun.so"
    subprocess.check_call([CLANG, "-O0", "-g", "-fPIC", "-shared", "-fsanitize=address", "-fno-gpu-sanitize", "-shared-libsan", "-o", str(so), str(src)])
    code = f"import ctypes; ctypes.CDLL({str(so)!r}).poke(8)"
    r = subprocess.run([sys.executable, "-c", code], env=_env(rt), capture_output=True, text=True)
    assert r.returncode != 0 and "heap-buffer-overflow" in r.stderr


def test_cpu_suites_are_clean_under_asan_and_ubsan(sanitized):
    rt, lib, orc = sanitized
    env = _env(rt, KVBLADE_LIB=lib, KV_ORACLE_LIB=orc)
    # the child must really run the instrumented builds
    probe = ("from paper_2604_26557_amd import binding; binding.lib(); from oracle import kv_oracle; kv_oracle.lib(); "
             "m = open('/proc/self/maps').read(); print('libkvblade_san.so' in m, 'libkv_oracle_san.so' in m, "
             "'/libkvblade.so' in m, '/libkv_oracle.so' in m)")
    r = subprocess.run([sys.executable, "-c", probe], cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    assert r.stdout.split() == ["True", "True", "False", "False"], r.stdout
    r = subprocess.run([sys.executable, "-m", "pytest", *FILES, "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    text = r.stdout + r.stderr
    assert r.returncode == 0, text[-4000:]
    assert "AddressSanitizer" not in text and "runtime error:" not in text, text[-4000:]

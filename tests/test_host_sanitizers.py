"""The library's host code under sanitizers (CPU only).

kvfs.cpp, desc.cpp, sched.cpp and capi.cpp are compiled with g++ into a host-only build of the
library (the kernel launches replaced by stand-ins that are never called: tests/sanitize/
kernel_stubs.cpp), once with AddressSanitizer + UndefinedBehaviorSanitizer and once with
ThreadSanitizer, and tests/test_host_lib.py (file-system state against the model, descriptors,
error paths, one context used from four threads) is run against each build in a child process
with the sanitizer's runtime preloaded.  Any report fails the run."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2510_25412_amd", "csrc")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def _runtime(name):
    gxx = shutil.which("g++")
    if not gxx:
        return None
    path = subprocess.run([gxx, "-print-file-name=" + name], stdout=subprocess.PIPE, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def _build(tmp, tag, flags):
    out = os.path.join(tmp, f"libsymphony_kv_{tag}.so")
    srcs = [os.path.join(CSRC, f) for f in ("kvfs.cpp", "desc.cpp", "sched.cpp", "capi.cpp")] + [os.path.join(ROOT, "tests", "sanitize", "kernel_stubs.cpp")]
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-w", *flags, "-D__HIP_PLATFORM_AMD__", f"-I{ROCM}/include", f"-I{CSRC}",
           *srcs, f"-L{ROCM}/lib", "-lamdhip64", f"-Wl,-rpath,{ROCM}/lib", "-o", out]
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert p.returncode == 0, p.stdout[-4000:]
    return out


def _run_host_tests(lib, runtime, extra_env, select):
    env = dict(os.environ)
    env["SYMPHONY_KV_LIB"] = lib
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env.update(extra_env)
    # -s: a sanitizer report goes to stderr and ends the process; pytest's capture would swallow it
    p = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_host_lib.py"), "-x", "-q", "-s", "-p", "no:cacheprovider",
                        "-k", select], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    tail = p.stdout[-6000:]
    assert p.returncode == 0, tail
    assert "runtime error" not in p.stdout and "Sanitizer" not in p.stdout, tail
    assert " passed" in p.stdout, tail


@pytest.mark.skipif(_runtime("libasan.so") is None, reason="g++ with libasan is not installed")
def test_host_library_under_address_and_undefined_behavior_sanitizers(tmp_path):
    lib = _build(str(tmp_path), "asan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"])
    # the interpreter itself is not instrumented and "leaks" by design: only the library's errors count
    _run_host_tests(lib, _runtime("libasan.so"), {"ASAN_OPTIONS": "detect_leaks=0:abort_on_error=0", "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"},
                    "not notice_a_wrong_model")


@pytest.mark.skipif(_runtime("libtsan.so") is None, reason="g++ with libtsan is not installed")
def test_host_library_under_thread_sanitizer(tmp_path):
    lib = _build(str(tmp_path), "tsan", ["-fsanitize=thread"])
    _run_host_tests(lib, _runtime("libtsan.so"), {"TSAN_OPTIONS": "halt_on_error=1:report_signal_unsafe=0"},
                    "four_threads or fig1 or staging or random_ops_match or offload")

"""Sanitizer tier for the CPU oracle (CPU only).

The oracle is the definition every GPU result is compared with, so its own C++ must be free of
undefined behaviour and out-of-bounds accesses on the inputs the pins and the workloads feed it.
The file is rebuilt with AddressSanitizer and UndefinedBehaviorSanitizer (first report aborts)
into a temporary directory, and the pin tests run against that build in a child process.
"""
import os
import subprocess
import sys

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    path = subprocess.check_output(["gcc", f"-print-file-name={name}"], text=True).strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def _child_env(so):
    env = dict(os.environ)
    env["QASR_ORACLE_SO"] = so
    # an instrumented shared object inside an uninstrumented interpreter needs the ASan runtime
    # loaded first; whatever the environment already preloads stays in the list
    asan = _runtime("libasan.so")
    assert asan, "no AddressSanitizer runtime beside gcc"
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    return env


@pytest.fixture(scope="module")
def sanitized_so(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("oracle_san") / "libqasr_oracle_san.so")
    return oracle.build(force=True, out=out, sanitize=True)


def test_pins_pass_on_the_sanitized_oracle(sanitized_so):
    cmd = [sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
           "-p", "no:cacheprovider"]
    r = subprocess.run(cmd, cwd=ROOT, env=_child_env(sanitized_so), capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "runtime error" not in r.stdout + r.stderr, tail
    assert " passed" in r.stdout, tail


def test_the_sanitized_build_is_the_one_loaded_and_reports(sanitized_so, tmp_path):
    """The child really runs the instrumented library: a deliberate out-of-range read through the
    oracle's own entry point (a residual array shorter than the output) aborts with a report."""
    code = (
        "import numpy as np, ctypes, oracle\n"
        "L = oracle.lib()\n"
        "x = np.zeros((1, 2, 8), np.int8); w = np.ones((2, 2, 1), np.int8)\n"
        "m = np.full(2, 1 << 30, np.int32); s = np.full(2, 30, np.int32)\n"
        "y = np.zeros((1, 2, 8), np.int8); r = np.zeros(4, np.int8)\n"
        "p = lambda a: a.ctypes.data_as(ctypes.c_void_p)\n"
        "L.qasr_oracle_conv1d_int8(1, 2, 2, 8, 1, 1, 1, 0, 0, 1, 0, 0, 0, p(x), p(w), None, p(m), p(s), p(r), p(y))\n"
        "print('no report')\n")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=_child_env(sanitized_so), capture_output=True,
                       text=True, timeout=300)
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr, (r.returncode, r.stderr[-2000:])

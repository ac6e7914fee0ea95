"""The C oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only): its pin tests
are run once more in a child process that loads a sanitizer build of the same sources
(oracle.build_sanitized) with the sanitizer runtime preloaded.  Any out-of-bounds access,
misaligned access or signed overflow inside the oracle aborts the child.  A second child shows
that the sanitizer is live: handing the library a buffer shorter than the length it is told
must be reported."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_TESTS = ["tests/test_oracle_attention.py", "tests/test_oracle_handoff.py", "tests/test_oracle_append.py",
             "tests/test_oracle_fp8.py"]


def _asan_runtime():
    out = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


@pytest.fixture(scope="module")
def san_env():
    rt = _asan_runtime()
    if rt is None:
        pytest.skip("gcc has no AddressSanitizer runtime here")
    sys.path.insert(0, ROOT)
    import oracle
    lib = oracle.build_sanitized()
    env = dict(os.environ)
    # the sanitizer runtime has to come first among the preloaded libraries; whatever the
    # environment already preloads stays behind it
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=23"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["ORACLE_LIB"] = lib
    env["OMP_NUM_THREADS"] = "4"
    return env


def test_pin_tests_pass_under_the_sanitizers(san_env):
    probe = ("import oracle; oracle.num_threads(); m = open('/proc/self/maps').read(); "
             "assert 'liboracle_san' in m and 'libasan' in m, 'sanitizer build not loaded'")
    r = subprocess.run([sys.executable, "-c", probe], cwd=ROOT, env=san_env, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + PIN_TESTS,
                       cwd=ROOT, env=san_env, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "passed" in r.stdout and "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr


def test_the_sanitizer_is_live(san_env):
    """oracle_e4m3_decode told to read 64 codes from a 16-byte buffer: a heap overflow the
    sanitizer must report (the planted mistake is in this call, on the CPU)."""
    code = ("import ctypes, os, numpy as np\n"
            "lib = ctypes.CDLL(os.environ['ORACLE_LIB'])\n"
            "src = np.zeros(16, np.uint8); dst = np.zeros(64, np.float64)\n"
            "lib.oracle_e4m3_decode(src.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(64), "
            "dst.ctypes.data_as(ctypes.c_void_p))\n"
            "print('not caught')\n")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=san_env, capture_output=True, text=True)
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr and "not caught" not in r.stdout

"""The oracle's C code under the address and undefined-behaviour sanitizers: the whole set of pins runs once more in a
child process that loads the sanitizer build, so that an out-of-bounds access or an overflow in the oracle fails a test
instead of silently shaping an expected value."""
import os
import subprocess
import sys

import pytest

from oracle import tt_oracle as ora

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _env():
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc has no address sanitizer runtime here")
    env = dict(os.environ)
    env["LD_PRELOAD"] = asan + ((":" + env["LD_PRELOAD"]) if env.get("LD_PRELOAD") else "")
    # (python itself is not instrumented: its interned objects would all be reported as leaks)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["TT_ORACLE_SANITIZE"] = "1"
    env["OMP_NUM_THREADS"] = "1"
    return env


def test_sanitizer_build_catches_a_planted_overrun():
    """The sanitizers are really active in such a child: an output array one element short makes ora_decode's last
    store an overrun, and the child dies naming it."""
    ora.build(sanitize=True)
    code = ("import numpy as np, ctypes as C\n"
            "from oracle import tt_oracle as ora\n"
            "l = ora._load()\n"
            "m = (C.c_int64 * 3)(4, 5, 6)\n"
            "idx = np.arange(100, dtype=np.int64)\n"
            "i1 = np.zeros(100, np.int32); i2 = np.zeros(100, np.int32); i3 = np.zeros(99, np.int32)\n"
            "l.ora_decode(m, idx.ctypes.data_as(C.c_void_p), C.c_int64(100), i1.ctypes.data_as(C.c_void_p),\n"
            "             i2.ctypes.data_as(C.c_void_p), i3.ctypes.data_as(C.c_void_p))\n"
            "print('survived')\n")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=_env(), capture_output=True, text=True, timeout=300)
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr and "survived" not in r.stdout, r.stderr[-2000:]


def test_pins_pass_under_the_sanitizers():
    ora.build(sanitize=True)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=_env(), capture_output=True, text=True, timeout=1500)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert " passed" in r.stdout and "failed" not in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
